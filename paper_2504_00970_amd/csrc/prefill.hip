// Prefill kernels: sentence segmentation (Sec. 4.1, Alg. 1 prefilling phase) and per-bucket mean key
// vectors (Eq. 1).  gfx950, wave64.
#include "skv_internal.h"

namespace skv {

// ------------------------------------------------------------------------------------------------
// Segmentation.  A token closes a bucket iff it is a terminator; seg_id is the exclusive prefix sum
// of the terminator flags.  Two launches over blocks of kSegTokPerBlock tokens:
//   seg_count : per block (number of terminators, 1 + position of the last terminator or 0)
//   seg_scan  : block prefix from the preceding blocks' partials, wave-level scan inside the block,
//               then each thread walks its 4 tokens and emits seg_id and, at every bucket end,
//               the bucket's start and length.
// The scan operator on (count, last_end) pairs is (a.count + b.count, max(a.last_end, b.last_end)).
// ------------------------------------------------------------------------------------------------

__device__ __forceinline__ bool is_terminator(const uint32_t* __restrict__ bitmap, int32_t vocab, int32_t id) {
    if (id < 0 || id >= vocab) return false;
    return (bitmap[id >> 5] >> (id & 31)) & 1u;
}

struct SegLocal {
    int flags;   // bit k set: token i0 + k is a terminator
    int cnt;
    int last;    // 1 + position of the thread's last terminator, 0 if none
};

__device__ __forceinline__ SegLocal seg_load(const int32_t* __restrict__ tok, int32_t T,
                                             const uint32_t* __restrict__ bitmap, int32_t vocab, int32_t i0) {
    int32_t t[kSegTokPerThread];
    if (i0 + kSegTokPerThread <= T) {
        const int4 v = *reinterpret_cast<const int4*>(tok + i0);
        t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < kSegTokPerThread; ++k) t[k] = (i0 + k < T) ? tok[i0 + k] : -1;
    }
    SegLocal r{0, 0, 0};
#pragma unroll
    for (int k = 0; k < kSegTokPerThread; ++k) {
        if (i0 + k < T && is_terminator(bitmap, vocab, t[k])) {
            r.flags |= 1 << k;
            r.cnt += 1;
            r.last = i0 + k + 1;
        }
    }
    return r;
}

__device__ __forceinline__ void wave_reduce_sum_max(int& s, int& m) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        s += __shfl_xor(s, off);
        m = max(m, __shfl_xor(m, off));
    }
}

// Block-wide (sum, max) over kSegThreads threads; result valid in every thread.
__device__ __forceinline__ void block_reduce_sum_max(int& s, int& m, int* sh /*[2 * waves]*/) {
    constexpr int kWaves = kSegThreads / kWave;
    wave_reduce_sum_max(s, m);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh[w] = s; sh[kWaves + w] = m; }
    __syncthreads();
    s = 0; m = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) { s += sh[i]; m = max(m, sh[kWaves + i]); }
}

__global__ __launch_bounds__(kSegThreads) void seg_count_kernel(const int32_t* __restrict__ tok, int32_t T,
                                                                const uint32_t* __restrict__ bitmap, int32_t vocab,
                                                                unsigned long long* __restrict__ part) {
    __shared__ int sh[2 * (kSegThreads / kWave)];
    const int32_t i0 = (blockIdx.x * kSegThreads + threadIdx.x) * kSegTokPerThread;
    SegLocal loc = seg_load(tok, T, bitmap, vocab, i0);
    int s = loc.cnt, m = loc.last;
    block_reduce_sum_max(s, m, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = ((unsigned long long)(unsigned)s << 32) | (unsigned)m;
}

__global__ __launch_bounds__(kSegThreads) void seg_scan_kernel(const int32_t* __restrict__ tok, int32_t T,
                                                               const uint32_t* __restrict__ bitmap, int32_t vocab,
                                                               const unsigned long long* __restrict__ part,
                                                               int32_t* __restrict__ seg_id, int32_t* __restrict__ sent_off,
                                                               int32_t* __restrict__ sent_len, int32_t cap_sent,
                                                               int32_t* __restrict__ n_sent) {
    constexpr int kWaves = kSegThreads / kWave;
    __shared__ int sh[2 * kWaves];
    __shared__ int sh_scan[2 * kWaves];
    if (T == 0) {                       // launched with one block
        if (threadIdx.x == 0) { *n_sent = 0; sent_off[0] = 0; }
        return;
    }
    // prefix of the blocks before this one
    int base_cnt = 0, base_last = 0;
    for (int j = threadIdx.x; j < (int)blockIdx.x; j += kSegThreads) {
        const unsigned long long p = part[j];
        base_cnt += (int)(p >> 32);
        base_last = max(base_last, (int)(p & 0xffffffffu));
    }
    block_reduce_sum_max(base_cnt, base_last, sh);

    const int32_t i0 = (blockIdx.x * kSegThreads + threadIdx.x) * kSegTokPerThread;
    const SegLocal loc = seg_load(tok, T, bitmap, vocab, i0);

    // inclusive wave scan of (cnt, last)
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int c = loc.cnt, l = loc.last;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int tc = __shfl_up(c, off), tl = __shfl_up(l, off);
        if (lane >= off) { c += tc; l = max(l, tl); }
    }
    if (lane == 63) { sh_scan[w] = c; sh_scan[kWaves + w] = l; }
    __syncthreads();
    int ec = __shfl_up(c, 1), el = __shfl_up(l, 1);       // exclusive within the wave
    if (lane == 0) { ec = 0; el = 0; }
    for (int i = 0; i < w; ++i) { ec += sh_scan[i]; el = max(el, sh_scan[kWaves + i]); }

    int seg = base_cnt + ec;
    int start = max(base_last, el);
#pragma unroll
    for (int k = 0; k < kSegTokPerThread; ++k) {
        const int32_t i = i0 + k;
        if (i >= T) break;
        seg_id[i] = seg;
        const bool term = (loc.flags >> k) & 1;
        const bool closes = term || i == T - 1;
        if (closes) {
            if (seg < cap_sent) { sent_off[seg] = start; sent_len[seg] = i + 1 - start; }
            if (i == T - 1) {
                *n_sent = seg + 1;
                if (seg + 1 <= cap_sent) sent_off[seg + 1] = T;
            }
            start = i + 1;
            seg += 1;
        }
    }
}

hipError_t launch_segment(Ctx* c, const int32_t* tok, int32_t T, const uint32_t* bitmap, int32_t vocab,
                          int32_t* seg_id, int32_t* sent_off, int32_t* sent_len, int32_t* n_sent_dev) {
    const int nb = (T + kSegTokPerBlock - 1) / kSegTokPerBlock;
    if (nb > 0) {
        hipLaunchKernelGGL(seg_count_kernel, dim3(nb), dim3(kSegThreads), 0, c->stream, tok, T, bitmap, vocab,
                           c->seg_part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(seg_scan_kernel, dim3(nb > 0 ? nb : 1), dim3(kSegThreads), 0, c->stream, tok, T, bitmap, vocab,
                       c->seg_part, seg_id, sent_off, sent_len, c->d.max_sentences, n_sent_dev);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Eq. 1: one wave per (layer * head, bucket).  A bucket's rows are contiguous in the pool, a row is
// D * EB bytes = LPR lanes of 16 bytes, so one wave-wide load instruction covers RPW = 64 / LPR
// consecutive rows fully coalesced.  Four such loads are kept in flight per lane.
// ------------------------------------------------------------------------------------------------

// Nearest E4M3 code (8-bit float of the OCP specification: bias 7, no infinities, largest value 448) of a finite float,
// ties to the even code, magnitudes that do not fit saturate at 448.
__device__ __forceinline__ uint32_t f32_to_e4m3(float f) {
    const uint32_t u = __float_as_uint(f), sign = (u >> 24) & 0x80u, a = u & 0x7fffffffu;
    uint32_t code;
    if (a < 0x3c800000u) {                                   // below 2^-6, the smallest normal: multiples of 2^-9
        code = (uint32_t)__builtin_rintf(__uint_as_float(a) * 512.0f);         // round half to even; 8 is 2^-6 itself
    } else {
        const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);  // 23 -> 3 fraction bits, round half to even
        code = min((r >> 20) - (120u << 3), 0x7eu);          // exponent bias 127 -> 7; 0x7e = 448
    }
    return sign | code;
}

template <int EB, int SVB>     // SVB: bytes per stored element of the table (4 = fp32, 2 = bf16, 1 = E4M3; rounded to nearest even)
__global__ __launch_bounds__(kSemvecWavesPerBlock * kWave) void semvec_kernel(const char* __restrict__ K, int32_t T,
                                                                              const int32_t* __restrict__ sent_off_all,
                                                                              int32_t off_layer_stride, int32_t Hkv,
                                                                              int32_t S, char* __restrict__ semvec) {
    using R = Row<EB>;
    constexpr int kUnroll = 4;
    const int lane = threadIdx.x & 63;
    const int32_t s = blockIdx.x * kSemvecWavesPerBlock + (threadIdx.x >> 6);
    if (s >= S) return;                                   // wave-uniform
    const int64_t lh = blockIdx.y;
    const int32_t* sent_off = sent_off_all + (int64_t)(blockIdx.y / Hkv) * off_layer_stride;   // the layer's table
    const int32_t b = max(sent_off[s], 0), e = min(sent_off[s + 1], T);   // never read outside the pool
    const int r = lane / R::LPR, cc = lane % R::LPR;
    const char* base = K + (lh * T) * (int64_t)(kHeadDim * EB) + (int64_t)cc * 16;

    float acc[R::EPL];
#pragma unroll
    for (int i = 0; i < R::EPL; ++i) acc[i] = 0.f;

    for (int32_t x0 = b + r; x0 < e; x0 += R::RPW * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int32_t x = x0 + u * R::RPW;
            // clamped address + masked value keeps the kUnroll loads independent of the bounds test
            const uint4 t = *reinterpret_cast<const uint4*>(base + (int64_t)min(x, e - 1) * (kHeadDim * EB));
            v[u] = (x < e) ? t : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float f[R::EPL];
            R::unpack(v[u], f);
#pragma unroll
            for (int i = 0; i < R::EPL; ++i) acc[i] += f[i];
        }
    }
#pragma unroll
    for (int off = R::LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int i = 0; i < R::EPL; ++i) acc[i] += __shfl_xor(acc[i], off);
    }
    if (r == 0) {
        const float n = (e > b) ? (float)(e - b) : 1.f;      // a bucket without tokens yields zeros
        const int64_t o = (lh * S + s) * (int64_t)kHeadDim + cc * R::EPL;      // element index of the lane's first output
#pragma unroll
        for (int i = 0; i < R::EPL; i += 4) {
            const float m[4] = {acc[i] / n, acc[i + 1] / n, acc[i + 2] / n, acc[i + 3] / n};
            if (SVB == 4) {
                *reinterpret_cast<float4*>(semvec + (o + i) * 4) = make_float4(m[0], m[1], m[2], m[3]);
            } else if (SVB == 1) {
                *reinterpret_cast<uint32_t*>(semvec + (o + i)) = f32_to_e4m3(m[0]) | (f32_to_e4m3(m[1]) << 8) |
                                                                 (f32_to_e4m3(m[2]) << 16) | (f32_to_e4m3(m[3]) << 24);
            } else {
                uint32_t rb[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t u = __float_as_uint(m[k]);
                    u += 0x7fffu + ((u >> 16) & 1u);               // round to nearest even bf16 (means are finite)
                    rb[k] = u >> 16;
                }
                *reinterpret_cast<uint2*>(semvec + (o + i) * 2) = make_uint2(rb[0] | (rb[1] << 16), rb[2] | (rb[3] << 16));
            }
        }
    }
}

template <int EB>
static void launch_semvec_eb(Ctx* c, dim3 grid, dim3 block, const void* K_pool, int32_t T, const int32_t* sent_off,
                             int32_t off_layer_stride, int32_t S, void* semvec) {
    if (c->d.semvec_dtype == SKV_BF16)
        hipLaunchKernelGGL((semvec_kernel<EB, 2>), grid, block, 0, c->stream, (const char*)K_pool, T, sent_off, off_layer_stride,
                           c->d.n_kv_heads, S, (char*)semvec);
    else if (c->d.semvec_dtype == SKV_FP8_E4M3)
        hipLaunchKernelGGL((semvec_kernel<EB, 1>), grid, block, 0, c->stream, (const char*)K_pool, T, sent_off, off_layer_stride,
                           c->d.n_kv_heads, S, (char*)semvec);
    else
        hipLaunchKernelGGL((semvec_kernel<EB, 4>), grid, block, 0, c->stream, (const char*)K_pool, T, sent_off, off_layer_stride,
                           c->d.n_kv_heads, S, (char*)semvec);
}

hipError_t launch_semvec(Ctx* c, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t off_layer_stride, int32_t S,
                         void* semvec) {
    if (S == 0) return hipSuccess;
    const dim3 grid((S + kSemvecWavesPerBlock - 1) / kSemvecWavesPerBlock, c->d.n_layers * c->d.n_kv_heads);
    const dim3 block(kSemvecWavesPerBlock * kWave);
    if (c->d.kv_dtype == SKV_BF16) launch_semvec_eb<2>(c, grid, block, K_pool, T, sent_off, off_layer_stride, S, semvec);
    else launch_semvec_eb<4>(c, grid, block, K_pool, T, sent_off, off_layer_stride, S, semvec);
    return hipGetLastError();
}

}  // namespace skv
