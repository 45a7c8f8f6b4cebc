// Decode-step kernels (Sec. 4.2, Eq. 3, Alg. 1 decoding phase): bucket scores, ranking + budgeted
// retrieval, K/V row gather, split-K attention with an online-softmax combine.  gfx950, wave64.
#include "skv_internal.h"
#include "skv_device.h"
#include "skv_stamps.h"

#include <type_traits>

#ifdef SKV_PHASE_STAMPS
namespace skv {
__device__ unsigned long long g_stamps[kStampBlocks * kStampSlots];
}
// Copies the stamp table (kStampBlocks x kStampSlots 64-bit ticks of the 100 MHz clock, zero where nothing was
// recorded) to `host` and clears it on the device.  Profiling build only.
extern "C" int skv_stamps_read(unsigned long long* host, int n_words) {
    if (!host || n_words != skv::kStampBlocks * skv::kStampSlots) return -1;
    if (hipDeviceSynchronize() != hipSuccess) return -3;
    if (hipMemcpyFromSymbol(host, HIP_SYMBOL(skv::g_stamps), sizeof(unsigned long long) * n_words) != hipSuccess) return -3;
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(skv::g_stamps)) != hipSuccess) return -3;
    return hipMemset(p, 0, sizeof(unsigned long long) * n_words) == hipSuccess ? 0 : -3;
}
#endif

namespace skv {

// Per-sequence slice of a ragged batch.
struct Seq {
    int32_t tok_base, n_tok_ctx;     // first pool row and number of tokens of the sequence
    int32_t sent_base, n_sent;       // first bucket and number of buckets
    int32_t budget;
};

// Read of an int32 array that the running launch does not write (the caller's cu_tok, cu_sent, budgets; n_tok, which an
// earlier launch of the same call may have written), through
// the constant address space: with a wave-uniform index it is a scalar load whatever else the kernel contains (loads of
// a plain global pointer turn into vector loads once the compiler cannot prove that the kernel leaves the memory alone,
// which an inline asm statement is enough to cause).
__device__ __forceinline__ int32_t ld_const(const int32_t* p, int64_t i) {
    typedef const int32_t __attribute__((address_space(4))) * ConstI32;
    return ((ConstI32)(uintptr_t)p)[i];
}

__device__ __forceinline__ Seq seq_of(const SeqView& v, int b) {
    Seq s;
    if (v.cu_sent) {
        s.sent_base = ld_const(v.cu_sent, b);
        s.n_sent = ld_const(v.cu_sent, b + 1) - s.sent_base;
    } else {
        s.sent_base = 0;
        s.n_sent = v.S_total;
    }
    if (v.cu_tok) {
        s.tok_base = ld_const(v.cu_tok, b);
        s.n_tok_ctx = ld_const(v.cu_tok, b + 1) - s.tok_base;
    } else {
        s.tok_base = 0;
        s.n_tok_ctx = v.T_total;
    }
    s.budget = v.budget_arr ? ld_const(v.budget_arr, b) : v.budget;
    return s;
}

// ------------------------------------------------------------------------------------------------
// Sentence query cache (Eq. 2; Alg. 1 decoding phase): running sum and count per sequence, mean query
// out, state cleared when the generated token ends a sentence.  One thread per 4 elements.
// ------------------------------------------------------------------------------------------------
template <int EB>
__global__ __launch_bounds__(kBlockThreads) void query_update_kernel(const char* __restrict__ q_t, const int32_t* __restrict__ tok_t,
                                                                     const uint32_t* __restrict__ bitmap, int32_t vocab,
                                                                     int32_t per_seq /* Hq * D */, float* __restrict__ q_sum,
                                                                     int32_t* __restrict__ q_cnt, char* __restrict__ q_bar) {
    const int b = blockIdx.x;                                        // one block per sequence
    const int32_t id = tok_t[b];
    const bool term = id >= 0 && id < vocab && ((bitmap[id >> 5] >> (id & 31)) & 1u);
    const int32_t n = q_cnt[b] + 1;
    const float fn = (float)n;
    for (int i4 = threadIdx.x * 4; i4 < per_seq; i4 += kBlockThreads * 4) {
        const int64_t e = (int64_t)b * per_seq + i4;
        float4 s = *reinterpret_cast<const float4*>(q_sum + e);
        float x[4];
        if (EB == 4) {
            const float4 t = *reinterpret_cast<const float4*>(q_t + e * 4);
            x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
        } else {
            const uint2 t = *reinterpret_cast<const uint2*>(q_t + e * 2);
            x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
            x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
        }
        s.x += x[0]; s.y += x[1]; s.z += x[2]; s.w += x[3];
        const float m[4] = {s.x / fn, s.y / fn, s.z / fn, s.w / fn};
        if (EB == 4) {
            *reinterpret_cast<float4*>(q_bar + e * 4) = make_float4(m[0], m[1], m[2], m[3]);
        } else {
            uint32_t r[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {                             // round to nearest even bf16 (inputs are finite)
                uint32_t u = __float_as_uint(m[k]);
                u += 0x7fffu + ((u >> 16) & 1u);
                r[k] = u >> 16;
            }
            *reinterpret_cast<uint2*>(q_bar + e * 2) = make_uint2(r[0] | (r[1] << 16), r[2] | (r[3] << 16));
        }
        *reinterpret_cast<float4*>(q_sum + e) = term ? make_float4(0.f, 0.f, 0.f, 0.f) : s;
    }
    __syncthreads();                                                  // every thread has read q_cnt[b]
    if (threadIdx.x == 0) q_cnt[b] = term ? 0 : n;
}

hipError_t launch_query_update(Ctx* c, int32_t B, const void* q_t, const int32_t* tok_t, const uint32_t* bitmap,
                               int32_t vocab, float* q_sum, int32_t* q_cnt, void* q_bar) {
    const int per_seq = c->d.n_q_heads * kHeadDim;
    const dim3 grid(B), block(kBlockThreads);
    if (c->d.kv_dtype == SKV_BF16)
        hipLaunchKernelGGL(query_update_kernel<2>, grid, block, 0, c->stream, (const char*)q_t, tok_t, bitmap, vocab, per_seq,
                           q_sum, q_cnt, (char*)q_bar);
    else
        hipLaunchKernelGGL(query_update_kernel<4>, grid, block, 0, c->stream, (const char*)q_t, tok_t, bitmap, vocab, per_seq,
                           q_sum, q_cnt, (char*)q_bar);
    return hipGetLastError();
}

// Stores that other blocks of the same launch read (possibly on another XCD, each with its own L2): device-scope
// relaxed atomic accesses go through to the level all XCDs share, so no L2 write-back / invalidate is needed around
// the arrival counters that publish them.
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned int* p, unsigned int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t ld_agent(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned int ld_agent(const unsigned int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_agent64(const float* p) {       // two consecutive floats
    return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// A float and the tag of the launch that produced it, in one 64-bit word written and read with single relaxed
// device-scope atomic accesses.  A reader that finds the tag it expects holds the value that belongs to it: nothing has
// to be ordered against any other location (per-location coherence of atomics is all that is used), so there is no
// arrival counter, no wait for store acknowledgements and no cache maintenance between producer and consumer.
__device__ __forceinline__ void st_tagged(unsigned long long* p, float v, uint32_t tag) {
    __hip_atomic_store(p, ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_tagged(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t tag_of(unsigned long long w) { return (uint32_t)(w >> 32); }
__device__ __forceinline__ float val_of(unsigned long long w) { return __uint_as_float((uint32_t)w); }

// Barrier behind which another thread of the block publishes what this block has stored (an arrival counter).  The
// workgroup barrier by itself does not wait for a wave's outstanding global stores (the waves of a block share their CU's
// cache, so the compiler leaves the store counter alone at workgroup scope): each wave waits for its own first.
// ASSUMPTION (of the kernels that publish with a counter: skv_attend, the two- and three-launch forms of
// skv_decode_step): a device-scope relaxed atomic store that has left the store counter (vmcnt == 0) has reached the
// level all XCDs share, so a device-scope relaxed load issued by any block after it observed the later counter
// increment returns the stored value.  The language's memory model does not promise this for relaxed accesses to
// different locations; it is how write-through stores and the store counter behave on this chip, and it is guarded by
// test_repeated_launches_reproduce_their_results.  The single-launch step does not rely on it: there every word
// carries its own validity tag (st_tagged).
__device__ __forceinline__ void block_sync_after_stores() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}
__device__ __forceinline__ float lo_f(unsigned long long v) { return __uint_as_float((uint32_t)v); }
__device__ __forceinline__ float hi_f(unsigned long long v) { return __uint_as_float((uint32_t)(v >> 32)); }

// ------------------------------------------------------------------------------------------------
// Scores.  score[h][s] = sum_g q[hG+g] . semvec[h][s]  =  (sum_g q[hG+g]) . semvec[h][s].
// A semantic vector is 512 bytes = 32 lanes x float4; a wave covers 2 buckets per load instruction
// and keeps RPWV / 2 loads in flight (RPWV = buckets per wave; 8 measured best from 1.3 k to 26 k
// buckets per head: 4 and 32 were both slower).  The group-summed query lives in registers.
// Blocks are aligned to sequences: block x -> (sequence b, local block) by walking cu_sent.
// ------------------------------------------------------------------------------------------------

// One wave: the RPWV buckets [row_w, row_w + RPWV) of a sequence.  q_grp = the first query of the head's group,
// sv_seq / out_seq = the (head, sequence) slices of the table and of the scores.  TAGGED: out_seq holds 64-bit (score, tag)
// words that other blocks of the same launch read.
template <bool TAGGED>
__device__ __forceinline__ void store_score(void* __restrict__ out_seq, int32_t s, float v, uint32_t tag) {
    if (TAGGED) st_tagged(static_cast<unsigned long long*>(out_seq) + s, v, tag);
    else static_cast<float*>(out_seq)[s] = v;
}

template <int EB, int G, int RPWV, bool TAGGED>
__device__ __forceinline__ void score_wave_f32(const char* __restrict__ q_grp, const float* __restrict__ sv_seq,
                                               int32_t n_sent, int32_t row_w, void* __restrict__ out_seq, uint32_t tag = 0) {
    const int lane = threadIdx.x & 63;
    const int c = lane & 31, half = lane >> 5;
    float qs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const char* qrow = q_grp + ((int64_t)g * kHeadDim + c * 4) * EB;
        if (EB == 4) {
            const float4 t = *reinterpret_cast<const float4*>(qrow);
            qs[0] += t.x; qs[1] += t.y; qs[2] += t.z; qs[3] += t.w;
        } else {
            const uint2 t = *reinterpret_cast<const uint2*>(qrow);
            qs[0] += __uint_as_float(t.x << 16); qs[1] += __uint_as_float(t.x & 0xffff0000u);
            qs[2] += __uint_as_float(t.y << 16); qs[3] += __uint_as_float(t.y & 0xffff0000u);
        }
    }
    constexpr int kIter = RPWV / 2;
    const int32_t row0 = row_w + half;
    const float* base = sv_seq + c * 4;
    // Addresses are clamped into the sequence instead of predicating the loads, so that all of a
    // lane's loads are issued back to back; rows past the end are computed and dropped.
    float4 x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t s = min(row0 + 2 * i, n_sent - 1);
        x[i] = *reinterpret_cast<const float4*>(base + (int64_t)s * kHeadDim);
    }
    float p[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) p[i] = x[i].x * qs[0] + x[i].y * qs[1] + x[i].z * qs[2] + x[i].w * qs[3];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {                     // sum over the 32 lanes of a bucket
        p[i] = dpp_add<0xB1>(p[i]);
        p[i] = dpp_add<0x4E>(p[i]);
        p[i] = dpp_add<0x124>(p[i]);
        p[i] = dpp_add<0x128>(p[i]);
        p[i] += __shfl_xor(p[i], 16);
    }
    if (c == 0) {
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int32_t s = row0 + 2 * i;
            if (s < n_sent) store_score<TAGGED>(out_seq, s, p[i], tag);
        }
    }
}

// The same from a bf16 table: a vector is 256 bytes = 16 lanes x 16 bytes (8 dims per lane), a wave load covers
// 4 buckets, RPWV / 4 loads in flight; the sum over a bucket's 16 lanes stays inside a DPP row.
template <int EB, int G, int RPWV, bool TAGGED>
__device__ __forceinline__ void score_wave_bf16(const char* __restrict__ q_grp, const char* __restrict__ sv_seq,
                                                int32_t n_sent, int32_t row_w, void* __restrict__ out_seq, uint32_t tag = 0) {
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, sub = lane >> 4;
    float qs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const char* qrow = q_grp + ((int64_t)g * kHeadDim + c * 8) * EB;
        if (EB == 4) {
            const float4 t0 = *reinterpret_cast<const float4*>(qrow), t1 = *reinterpret_cast<const float4*>(qrow + 16);
            qs[0] += t0.x; qs[1] += t0.y; qs[2] += t0.z; qs[3] += t0.w;
            qs[4] += t1.x; qs[5] += t1.y; qs[6] += t1.z; qs[7] += t1.w;
        } else {
            float f[8];
            Row<2>::unpack(*reinterpret_cast<const uint4*>(qrow), f);
#pragma unroll
            for (int i = 0; i < 8; ++i) qs[i] += f[i];
        }
    }
    constexpr int kIter = RPWV / 4;
    const int32_t row0 = row_w + sub;
    const char* base = sv_seq + c * 16;
    uint4 x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {                       // clamped addresses: all loads issued back to back
        const int32_t s = min(row0 + 4 * i, n_sent - 1);
        x[i] = *reinterpret_cast<const uint4*>(base + (int64_t)s * (kHeadDim * 2));
    }
    float p[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        float f[8];
        Row<2>::unpack(x[i], f);
        p[i] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) p[i] += f[e] * qs[e];
    }
#pragma unroll
    for (int i = 0; i < kIter; ++i) {                       // sum over the 16 lanes of a bucket
        p[i] = dpp_add<0xB1>(p[i]);
        p[i] = dpp_add<0x4E>(p[i]);
        p[i] = dpp_add<0x124>(p[i]);
        p[i] = dpp_add<0x128>(p[i]);
    }
    if (c == 0) {
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int32_t s = row0 + 4 * i;
            if (s < n_sent) store_score<TAGGED>(out_seq, s, p[i], tag);
        }
    }
}

// The same from an E4M3 table: a vector is 128 bytes = 8 lanes x 16 bytes (16 dims per lane), a wave load covers 8 buckets,
// RPWV / 8 loads in flight; the sum over a bucket's 8 lanes is two quad exchanges and a rotation by 4.
template <int EB, int G, int RPWV, bool TAGGED>
__device__ __forceinline__ void score_wave_e4m3(const char* __restrict__ q_grp, const char* __restrict__ sv_seq,
                                                int32_t n_sent, int32_t row_w, void* __restrict__ out_seq, uint32_t tag = 0) {
    const int lane = threadIdx.x & 63;
    const int c = lane & 7, sub = lane >> 3;
    float qs[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) qs[i] = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const char* qrow = q_grp + ((int64_t)g * kHeadDim + c * 16) * EB;
        if (EB == 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 t = *reinterpret_cast<const float4*>(qrow + 16 * k);
                qs[4 * k] += t.x; qs[4 * k + 1] += t.y; qs[4 * k + 2] += t.z; qs[4 * k + 3] += t.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float f[8];
                Row<2>::unpack(*reinterpret_cast<const uint4*>(qrow + 16 * k), f);
#pragma unroll
                for (int i = 0; i < 8; ++i) qs[8 * k + i] += f[i];
            }
        }
    }
    constexpr int kIter = RPWV / 8;
    const int32_t row0 = row_w + sub;
    const char* base = sv_seq + c * 16;
    uint4 x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {                       // clamped addresses: all loads issued back to back
        const int32_t s = min(row0 + 8 * i, n_sent - 1);
        x[i] = *reinterpret_cast<const uint4*>(base + (int64_t)s * kHeadDim);
    }
    float p[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const uint32_t wd[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
        p[i] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            // v_cvt_pk_f32_fp8: two codes of a dword -> two floats; gfx950 reads them as E4M3 of the OCP specification
            // (a parity test scores a table holding every code against the format's written-out definition)
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)wd[k], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)wd[k], true);
            p[i] += lo[0] * qs[4 * k] + lo[1] * qs[4 * k + 1] + hi[0] * qs[4 * k + 2] + hi[1] * qs[4 * k + 3];
        }
    }
#pragma unroll
    for (int i = 0; i < kIter; ++i) {                       // sum over the 8 lanes of a bucket
        p[i] = dpp_add<0xB1>(p[i]);
        p[i] = dpp_add<0x4E>(p[i]);
        p[i] = dpp_add<0x124>(p[i]);                        // row_ror 4: lanes 4..7 of each group of 8 now hold the group's sum
    }
    if (c == 4) {
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int32_t s = row0 + 8 * i;
            if (s < n_sent) store_score<TAGGED>(out_seq, s, p[i], tag);
        }
    }
}

constexpr int kScoreRowsPerWave16 = 16;
constexpr int kScoreRowsPerWave8 = 32;
enum { kTableF32 = 4, kTableBf16 = 2, kTableE4m3 = 1 };       // bytes per element of the mean-key table

// Scores of one layer: grid (blocks over the S_total buckets of the concatenated batch, KV heads).  A wave owns RPWV
// consecutive buckets of that axis, wherever the sequence boundaries fall, and scores them in runs that belong to one
// sequence, each run with that sequence's queries: one run unless a boundary falls inside the wave's buckets; a sequence
// without buckets has no run.  The sequence of the wave's first bucket r0 is the last b with cu_sent[b] <= r0: bisection
// of cu_sent down to eight candidates (dependent scalar loads), then eight consecutive boundaries in one scalar load,
// which also gives the end of the first run; log2(B / 8) + 1 round trips, whatever the batch size.

// The RPWV buckets [r0, r0 + RPWV) of the concatenated bucket axis, head h, by one wave.  TAGGED: `out` holds 64-bit
// (score, tag) words, tags[pair] being the launch tag of (sequence, head) pair b * Hkv + h.
template <int EB, int G, int SVB, int RPWV, bool TAGGED>
__device__ __forceinline__ void score_group(const char* __restrict__ q, const char* __restrict__ semvec, const SeqView& v,
                                            int32_t Hq, int h, int32_t r0, void* __restrict__ out,
                                            const uint32_t* tags = nullptr) {
    const int32_t r1 = min(r0 + RPWV, v.S_total);
    auto run = [&](int b, int32_t first, int32_t n) {      // buckets [first, first + n) of the batch axis, sequence b
        const char* qg = q + ((int64_t)(b * Hq + h * G) * kHeadDim) * EB;
        const int64_t row = (int64_t)h * v.S_total + first;
        void* dst = TAGGED ? static_cast<void*>(static_cast<unsigned long long*>(out) + row)
                           : static_cast<void*>(static_cast<float*>(out) + row);
        const uint32_t tag = TAGGED ? tags[b * (Hq / G) + h] : 0u;
        if (SVB == kTableF32)
            score_wave_f32<EB, G, RPWV, TAGGED>(qg, reinterpret_cast<const float*>(semvec) + row * kHeadDim, n, 0, dst, tag);
        else if (SVB == kTableBf16)
            score_wave_bf16<EB, G, RPWV, TAGGED>(qg, semvec + row * kHeadDim * 2, n, 0, dst, tag);
        else
            score_wave_e4m3<EB, G, RPWV, TAGGED>(qg, semvec + row * kHeadDim, n, 0, dst, tag);
    };
    if (!v.cu_sent) {                                      // one sequence
        run(0, r0, r1 - r0);
        return;
    }
    auto cu = [&](int i) { return ld_const(v.cu_sent, i); };
    int b = 0, hi = v.B;                                   // cu(b) <= r0 < cu(hi)
    int32_t end;
    if (v.B >= 8) {
        while (hi - b > 8) {
            const int mid = (b + hi) >> 1;
            if (cu(mid) <= r0) b = mid; else hi = mid;
        }
        const int start = min(b + 1, v.B - 7);             // boundaries start .. start + 7 include hi
        int32_t w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = cu(start + j);
        int below = 0;
        end = w[7];
#pragma unroll
        for (int j = 7; j >= 0; --j) {
            below += w[j] <= r0;
            if (w[j] > r0) end = w[j];
        }
        b = start - 1 + below;
    } else {
        while (hi - b > 1) {
            const int mid = (b + hi) >> 1;
            if (cu(mid) <= r0) b = mid; else hi = mid;
        }
        end = cu(b + 1);
    }
    int32_t cur = r0;
    for (;;) {
        end = min(end, r1);
        if (end > cur) {
            run(b, cur, end - cur);
            cur = end;
        }
        if (cur >= r1 || ++b >= v.B) break;
        end = cu(b + 1);
    }
}

template <int EB, int G, int SVB, int RPWV>
__global__ __launch_bounds__(kScoreWavesPerBlock * kWave) void score_kernel(const char* __restrict__ q,
                                                                            const char* __restrict__ semvec, SeqView v,
                                                                            int32_t Hq, float* __restrict__ score) {
    // every argument is demanded here, so the kernel-argument loads go out together; left alone, the compiler loads
    // each one before its first use, a dependent round trip per branch below
    asm volatile("" ::"s"(q), "s"(semvec), "s"(v.cu_sent), "s"(v.S_total), "s"(v.B), "s"(Hq), "s"(score));
    const int32_t r0 = (blockIdx.x * kScoreWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * RPWV;
    if (r0 >= v.S_total) return;
    score_group<EB, G, SVB, RPWV, false>(q, semvec, v, Hq, blockIdx.y, r0, score);
}

template <int EB, int G>
static void launch_score_t(Ctx* c, const char* q, const char* sv, const SeqView& v, float* score) {
    const bool sv16 = c->d.semvec_dtype == SKV_BF16, sv8 = c->d.semvec_dtype == SKV_FP8_E4M3;
    const int rows_per_block = (sv8 ? kScoreRowsPerWave8 : sv16 ? kScoreRowsPerWave16 : kScoreRowsPerWave) * kScoreWavesPerBlock;
    const dim3 grid((v.S_total + rows_per_block - 1) / rows_per_block, c->d.n_kv_heads), block(kScoreWavesPerBlock * kWave);
    if (sv8)
        hipLaunchKernelGGL((score_kernel<EB, G, kTableE4m3, kScoreRowsPerWave8>), grid, block, 0, c->stream, q, sv, v,
                           c->d.n_q_heads, score);
    else if (sv16)
        hipLaunchKernelGGL((score_kernel<EB, G, kTableBf16, kScoreRowsPerWave16>), grid, block, 0, c->stream, q, sv, v,
                           c->d.n_q_heads, score);
    else
        hipLaunchKernelGGL((score_kernel<EB, G, kTableF32, kScoreRowsPerWave>), grid, block, 0, c->stream, q, sv, v,
                           c->d.n_q_heads, score);
}

template <int EB>
static hipError_t launch_score_g(Ctx* c, const void* q, const void* semvec_layer, const SeqView& v, float* score) {
    const char* qp = (const char*)q;
    const char* sv = (const char*)semvec_layer;
    switch (c->G) {
        case 1: launch_score_t<EB, 1>(c, qp, sv, v, score); break;
        case 2: launch_score_t<EB, 2>(c, qp, sv, v, score); break;
        case 4: launch_score_t<EB, 4>(c, qp, sv, v, score); break;
        case 8: launch_score_t<EB, 8>(c, qp, sv, v, score); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_score(Ctx* c, const void* q, const void* semvec_layer, const SeqView& v, float* score) {
    if (v.S_total == 0) return hipSuccess;
    return c->d.kv_dtype == SKV_BF16 ? launch_score_g<2>(c, q, semvec_layer, v, score)
                                     : launch_score_g<4>(c, q, semvec_layer, v, score);
}

// ------------------------------------------------------------------------------------------------
// Selection (Sec. 4.2 ranking + budgeted retrieval) as a block-level routine for kBlockThreads
// threads, used by the stand-alone select kernel (one block per sequence and KV head) and, redundantly
// per block, by the fused attention kernel.
//
// Buckets are ranked by (score descending, id ascending) and taken along the ranking until the first
// one that does not fit.  Because lengths are positive the running total along the ranking is
// increasing, so the retrieved set is {i : (total length ranked before i) + len_i <= budget}.  The
// first bucket that overflows (the "cut") is found without sorting, by a length-weighted radix select
// on an order-preserving 32-bit image of the score: 11 + 11 + 10 bit digits, most significant first.
// Per pass: LDS atomics build a histogram of (count, total length) per digit; thread t owns digits
// 2047-2t and 2046-2t, so a block-wide prefix sum in thread order (DPP wave scan + 16 wave totals) is
// the running total from the top digit down, and exactly one thread sees the budget crossed inside
// its two digits.  The three histograms are zeroed up front.  The search stops as soon as the crossing
// digit holds a single bucket (typically after two passes); buckets with exactly the cut's score are
// resolved in id order by a scan.
//
// The routine is written for few instructions per wave (a wave issues one instruction every 4+
// cycles, so instruction count is latency) and 32-bit arithmetic throughout (token totals < 2^31):
// thread t owns the kpt = ceil(S / 1024) consecutive buckets [t*kpt, (t+1)*kpt); keys, lengths and
// offsets of the first KREG of them live in registers (one global round trip); buckets beyond KREG per
// thread are re-read from memory in every phase.  The blocked ownership makes the id-ordered
// compaction a thread-local walk plus one block scan.
// ------------------------------------------------------------------------------------------------

constexpr int kSelKreg = 6;                                   // 1024 threads x 6 buckets in registers: S <= 6144
constexpr int kBins = 2048;                                   // 11-bit digits (the last pass uses 1024)

struct SelectShared {
    unsigned long long hist[3][kBins];                        // packed (count << 32 | total length) per digit
    uint32_t wave_tot[6][kBlockWaves];                        // one slot per block scan
    int32_t res[3][4];                                        // per pass: crossing digit (-1: none), carry, count
    int32_t poll[3];                                          // tagged scores: [0] set by a thread whose wait ran out
    __attribute__((aligned(16))) uint32_t wmax[kBlockWaves];  // largest key per wave
};

// emit(s, off_s, len_s, sel_pos, tok_pos) is called by the owner thread of every selected bucket,
// sel_pos / tok_pos being the number of selected buckets / tokens with lower ids (sel_pos is only
// computed when COUNT is set, else 0).  Every thread of the block must call this; *n_sel_out /
// *n_tok_out are block-uniform.
// TAGGED: `sc` points at 64-bit (score, tag) words that other blocks of the same launch are writing; every thread reads
// its words again and again until they carry `tag` (at most wait_limit times: *ok_out tells whether they all
// arrived; if not, the selection is made from whatever was read and is meaningless).
template <int KREG, bool COUNT, bool TAGGED, typename Emit>
__device__ __forceinline__ void select_block(const float* __restrict__ sc, const int32_t* __restrict__ len,
                                             const int32_t* __restrict__ off, int32_t S, int32_t budget,
                                             SelectShared& sh, Emit emit, int32_t* n_sel_out, int32_t* n_tok_out,
                                             uint32_t tag = 0, int32_t wait_limit = 0, bool* ok_out = nullptr,
                                             uint32_t* __restrict__ key_lds = nullptr /* TAGGED: KREG * kBlockThreads words */) {
    const int tid = threadIdx.x;
    *n_sel_out = 0;
    *n_tok_out = 0;
    if (ok_out) *ok_out = true;
    if (S <= 0 || budget <= 0) return;
    const int kpt = (S + kBlockThreads - 1) / kBlockThreads;
    const int32_t s0 = tid * kpt;
    const unsigned long long* tw = reinterpret_cast<const unsigned long long*>(sc);
    auto ldsc = [&](int32_t i) -> float { return TAGGED ? val_of(ld_tagged(tw + i)) : sc[i]; };

    uint32_t rkey[KREG];
    int32_t rlen[KREG], roff[KREG];
    static_assert(KREG % 2 == 0, "the register-held buckets are loaded in pairs");
#pragma unroll
    for (int i = 0; i < KREG; ++i) { rkey[i] = 0; rlen[i] = 0; roff[i] = 0; }
    if (KREG > 2 && S >= 2) {
        // Many buckets per thread: they are consecutive, so two per load instruction (8 bytes at 4-byte alignment; with
        // two buckets per thread single loads measured slightly faster).  The pair is moved back so that it ends inside
        // the arrays; a slot past the end gets some in-range value and is dropped below.
        struct __attribute__((aligned(4))) Pair { uint32_t x, y; };
#pragma unroll
        for (int j = 0; j < KREG / 2; ++j) {
            if (2 * j < kpt) {                             // block-uniform; loads unconditional
                const int32_t idx = s0 + 2 * j, bse = min(idx, S - 2);
                Pair k{0u, 0u};
                if (!TAGGED) k = *reinterpret_cast<const Pair*>(sc + bse);
                const Pair l = *reinterpret_cast<const Pair*>(len + bse);
                const Pair o = *reinterpret_cast<const Pair*>(off + bse);
                const bool tail = idx == S - 1;            // the pair was moved back by one: the last bucket sits in .y
                rkey[2 * j] = tail ? k.y : k.x; rkey[2 * j + 1] = k.y;
                rlen[2 * j] = (int32_t)(tail ? l.y : l.x); rlen[2 * j + 1] = (int32_t)l.y;
                roff[2 * j] = (int32_t)(tail ? o.y : o.x); roff[2 * j + 1] = (int32_t)o.y;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            if (i < kpt) {                                 // block-uniform; addresses clamped, loads unconditional
                const int32_t sidx = min(s0 + i, S - 1);
                if (!TAGGED) rkey[i] = __float_as_uint(sc[sidx]);
                rlen[i] = len[sidx];
                roff[i] = off[sidx];
            }
        }
    }
    // zero the histograms while the loads are in flight
    auto zero_hist = [&]() {
        unsigned long long* h = &sh.hist[0][0];
#pragma unroll
        for (int i = 0; i < 3 * kBins / kBlockThreads; ++i) h[i * kBlockThreads + tid] = 0;
        if (tid < 3) sh.res[tid][0] = -1;
    };
    zero_hist();
    if (tid == 0) sh.poll[0] = 0;
    // The largest key of the block (over all buckets read, with or without tokens: an upper bound of the keys that take
    // part is all that is needed): a wave's maximum goes to LDS ahead of a barrier that is there anyway.
    uint32_t my_max = 0;
    auto share_max = [&]() {
        const uint32_t wm = (uint32_t)__builtin_amdgcn_readlane((int)wave_scan_max_u32(my_max), kWave - 1);
        if ((tid & (kWave - 1)) == 0) sh.wmax[tid >> 6] = wm;
    };
    if (!TAGGED) {
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            rkey[i] = score_key(__uint_as_float(rkey[i]));
            if (s0 + i >= S) rlen[i] = 0;                  // slots past the end take part in nothing
            if (i < kpt) my_max = max(my_max, rkey[i]);
        }
        for (int i = KREG; i < kpt; ++i)
            if (s0 + i < S) my_max = max(my_max, score_key(sc[s0 + i]));
        share_max();
        __syncthreads();
    } else {
        __syncthreads();                                   // the flag is clear
        // Every thread reads its own words until all of them carry the tag (bounded), without talking to anyone; the
        // block meets at one barrier afterwards.  A thread whose wait ran out raises the block's flag.
        const bool strided = kpt <= KREG;                  // every bucket of the pair is held in registers
        bool mine = false;
        if (strided) {
            // The words are read with consecutive lanes on consecutive words (thread t: words t, t + 1024, ...: whole
            // cache lines per wave instruction; a thread's own consecutive buckets would cost kpt times the memory
            // requests), and the keys reach their owners through LDS.
            uint32_t kk[KREG];
#pragma unroll
            for (int i = 0; i < KREG; ++i) kk[i] = 0u;
            for (int32_t round = 0; !mine && round < wait_limit; ++round) {
                mine = true;
#pragma unroll
                for (int i = 0; i < KREG; ++i) {
                    if (i < kpt) {
                        const int32_t sidx = min(i * kBlockThreads + tid, S - 1);
                        const unsigned long long wd = ld_tagged(tw + sidx);
                        kk[i] = (uint32_t)wd;
                        mine = mine && tag_of(wd) == tag;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < KREG; ++i) {
                if (i < kpt) {
                    key_lds[i * kBlockThreads + tid] = kk[i];
                    my_max = max(my_max, score_key(__uint_as_float(kk[i])));
                }
            }
        } else {
            for (int32_t round = 0; !mine && round < wait_limit; ++round) {
                mine = true;
#pragma unroll
                for (int i = 0; i < KREG; ++i) {
                    const unsigned long long wd = ld_tagged(tw + min(s0 + i, S - 1));
                    rkey[i] = (uint32_t)wd;
                    mine = mine && tag_of(wd) == tag;
                }
                for (int i = KREG; i < kpt; ++i) {         // buckets beyond the registers are re-read in every phase below
                    if (s0 + i < S) {
                        const unsigned long long wd = ld_tagged(tw + s0 + i);
                        mine = mine && tag_of(wd) == tag;
                        my_max = max(my_max, score_key(val_of(wd)));
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < KREG; ++i) my_max = max(my_max, score_key(__uint_as_float(rkey[i])));
        }
        share_max();
        if (!mine) sh.poll[0] = 1;
        __syncthreads();
        if (sh.poll[0] != 0 && ok_out) *ok_out = false;
        if (strided) {
#pragma unroll
            for (int i = 0; i < KREG; ++i)
                if (i < kpt) rkey[i] = key_lds[s0 + i];    // s0 + i < kpt * 1024 <= KREG * 1024
        }
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            rkey[i] = score_key(__uint_as_float(rkey[i]));
            if (s0 + i >= S) rlen[i] = 0;                  // slots past the end take part in nothing
        }
    }
    uint32_t kmax = 0;
    {
        const uint4* wm4 = reinterpret_cast<const uint4*>(sh.wmax);
#pragma unroll
        for (int q4 = 0; q4 < kBlockWaves / 4; ++q4) {
            const uint4 t = wm4[q4];
            kmax = max(max(kmax, max(t.x, t.y)), max(t.z, t.w));
        }
    }
    SKV_T(1);

    // ---- weighted radix select of the cut ----------------------------------------------------------
    // Two attempts.  The first ranks the buckets by their distance below the best key, r = ~(kmax - key) (the same order
    // as the key), and looks only at those within 2^24 key steps of it (two binades of score; the others cannot be told
    // apart there and stay out of the histograms): digits of 11, 11 and 2 bits from bit 23 down, so that the first
    // histogram already resolves 2^13 key steps and the crossing digit mostly holds a single bucket: one pass instead of
    // two.  If those near buckets all fit the budget, the cut lies further down (or nowhere) and the second attempt runs
    // the plain digits 11, 11, 10 of the key over all buckets.
    uint32_t prefix = 0;        // resolved high bits of the cut's key
    int shift = 32;             // number of unresolved low bits
    int32_t carry = 0;          // total length of the buckets ranked strictly above the current digit range
    int32_t cut_cnt = 0;        // number of buckets sharing the resolved prefix
    bool select_all = false;
    bool near = true;           // first attempt: keys are distances below kmax
    auto to_rank = [&](uint32_t k) -> uint32_t { return near ? ~(kmax - k) : k; };
#pragma unroll
    for (int i = 0; i < KREG; ++i) rkey[i] = ~(kmax - rkey[i]);
    for (int attempt = 0; attempt < 2; ++attempt) {
        bool found_none = false;
        prefix = near ? 0xffu : 0u;
        shift = near ? 24 : 32;
        carry = 0;
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int bits = pass < 2 ? 11 : (near ? 2 : 10), nbins = 1 << bits, nshift = shift - bits;
            unsigned long long* H = sh.hist[pass];
#pragma unroll
            for (int i = 0; i < KREG; ++i) {
                if (i < kpt && rlen[i] > 0 && (shift == 32 || (rkey[i] >> shift) == prefix))
                    atomicAdd(&H[(rkey[i] >> nshift) & (nbins - 1)], (1ull << 32) | (unsigned long long)(uint32_t)rlen[i]);
            }
            for (int i = KREG; i < kpt; ++i) {
                if (s0 + i < S && len[s0 + i] > 0) {           // a bucket without tokens takes part in nothing
                    const uint32_t k = to_rank(score_key(ldsc(s0 + i)));
                    if (shift == 32 || (k >> shift) == prefix)
                        atomicAdd(&H[(k >> nshift) & (nbins - 1)], (1ull << 32) | (unsigned long long)(uint32_t)len[s0 + i]);
                }
            }
            __syncthreads();
            // thread order == descending digit order: thread t owns digits nbins-1-2t and nbins-2-2t
            const int d1 = nbins - 1 - 2 * tid;
            const unsigned long long v1 = d1 >= 0 ? H[d1] : 0ull, v0 = d1 >= 1 ? H[d1 - 1] : 0ull;
            const uint32_t l1 = (uint32_t)v1, l0 = (uint32_t)v0;
            uint32_t total;
            const uint32_t incl = block_scan_u32(l1 + l0, sh.wave_tot[pass], &total);
            const uint32_t above1 = (uint32_t)carry + incl - l1 - l0, above0 = above1 + l1;
            if (l1 > 0 && above1 <= (uint32_t)budget && above1 + l1 > (uint32_t)budget) {
                sh.res[pass][0] = d1; sh.res[pass][1] = (int32_t)above1; sh.res[pass][2] = (int32_t)(v1 >> 32);
            }
            if (l0 > 0 && above0 <= (uint32_t)budget && above0 + l0 > (uint32_t)budget) {
                sh.res[pass][0] = d1 - 1; sh.res[pass][1] = (int32_t)above0; sh.res[pass][2] = (int32_t)(v0 >> 32);
            }
            __syncthreads();
            const int digit = sh.res[pass][0];
            if (digit < 0) { found_none = true; break; }           // the buckets of this attempt all fit (only possible in pass 0)
            prefix = (shift == 32) ? (uint32_t)digit : ((prefix << bits) | (uint32_t)digit);
            carry = sh.res[pass][1];
            cut_cnt = sh.res[pass][2];
            shift = nshift;
            if (cut_cnt == 1) break;                               // the cut is unique: it is the bucket that overflows
        }
        if (!found_none) break;
        if (!near) { select_all = true; break; }                   // every bucket was seen and they all fit: no cut
        // The buckets near the best key all fit: the cut, if there is one, is among the others.
        near = false;
#pragma unroll
        for (int i = 0; i < KREG; ++i) rkey[i] = kmax - ~rkey[i];  // back to the plain keys
        zero_hist();                                               // (every thread is past its reads of the first attempt)
        __syncthreads();
    }
    const bool ties = !select_all && cut_cnt > 1;              // then shift == 0: several buckets share the cut's score
    SKV_T(2);

    // ---- compaction in id order --------------------------------------------------------------------
    // fn(i, s, key, len, off) for every bucket the thread owns, in id order
    auto for_items = [&](auto&& fn) {
#pragma unroll
        for (int i = 0; i < KREG; ++i)
            if (i < kpt && rlen[i] > 0) fn(i, s0 + i, rkey[i], rlen[i], roff[i]);
        for (int i = KREG; i < kpt; ++i)
            if (s0 + i < S && len[s0 + i] > 0) fn(i, s0 + i, to_rank(score_key(ldsc(s0 + i))), len[s0 + i], off[s0 + i]);
    };
    uint32_t tie_run = 0;          // length of tied buckets with lower ids (starts at the thread's base)
    if (ties) {
        uint32_t mine = 0;
        for_items([&](int, int32_t, uint32_t k, int32_t ln, int32_t) { if (k == prefix) mine += (uint32_t)ln; });
        uint32_t tot;
        tie_run = block_scan_u32(mine, sh.wave_tot[3], &tot) - mine;
    }
    auto chosen = [&](uint32_t k, int32_t ln, uint32_t& tie_acc) -> bool {
        if (select_all) return true;
        if ((k >> shift) > prefix) return true;                // shift < 32 here: at least one pass ran
        if (ties && k == prefix) {
            tie_acc += (uint32_t)ln;
            return (uint32_t)carry + tie_acc <= (uint32_t)budget;
        }
        return false;
    };
    // first walk: count; the register-held buckets that are chosen are remembered in a mask, so that the second walk
    // does not evaluate the rule again (buckets beyond the registers, re-read from memory, are evaluated in both walks)
    uint32_t my_tok = 0, my_cnt = 0, sel_mask = 0, tie_after_regs = tie_run;
    {
        uint32_t t = tie_run;
#pragma unroll
        for (int i = 0; i < KREG; ++i)
            if (i < kpt && rlen[i] > 0 && chosen(rkey[i], rlen[i], t)) { my_tok += (uint32_t)rlen[i]; my_cnt += 1; sel_mask |= 1u << i; }
        tie_after_regs = t;
        for (int i = KREG; i < kpt; ++i)
            if (s0 + i < S && len[s0 + i] > 0 && chosen(to_rank(score_key(ldsc(s0 + i))), len[s0 + i], t)) { my_tok += (uint32_t)len[s0 + i]; my_cnt += 1; }
    }
    uint32_t tot_tok, tot_cnt = 0;
    uint32_t pos_tok = block_scan_u32(my_tok, sh.wave_tot[4], &tot_tok) - my_tok;
    uint32_t pos_cnt = 0;
    if (COUNT) pos_cnt = block_scan_u32(my_cnt, sh.wave_tot[5], &tot_cnt) - my_cnt;
    if (my_cnt != 0) {
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            if ((sel_mask >> i) & 1u) {
                emit(s0 + i, roff[i], rlen[i], (int32_t)pos_cnt, (int32_t)pos_tok);
                pos_tok += (uint32_t)rlen[i];
                pos_cnt += 1;
            }
        }
        uint32_t t = tie_after_regs;
        for (int i = KREG; i < kpt; ++i) {
            if (s0 + i < S && len[s0 + i] > 0 && chosen(to_rank(score_key(ldsc(s0 + i))), len[s0 + i], t)) {
                emit(s0 + i, off[s0 + i], len[s0 + i], (int32_t)pos_cnt, (int32_t)pos_tok);
                pos_tok += (uint32_t)len[s0 + i];
                pos_cnt += 1;
            }
        }
    }
    *n_sel_out = (int32_t)tot_cnt;
    *n_tok_out = (int32_t)tot_tok;
    SKV_T(3);
}

// Stand-alone selection: the selected buckets go through an LDS list so that the token positions of
// each bucket are written by a whole wave, coalesced.
constexpr int kSelListCap = 2048;

__global__ __launch_bounds__(kBlockThreads) void select_kernel(const float* __restrict__ score,
                                                               const int32_t* __restrict__ sent_off,
                                                               const int32_t* __restrict__ sent_len, SeqView v,
                                                               int32_t Hkv, int32_t max_sel,
                                                               int32_t* __restrict__ sel_sent, int32_t* __restrict__ n_sel,
                                                               int32_t* __restrict__ tok_idx, int32_t idx_stride,
                                                               int32_t budget_cap, int32_t* __restrict__ n_tok) {
    __shared__ SelectShared sh;
    __shared__ int4 list[kSelListCap];                        // (bucket, offset, length, first output slot)
    const int bh = blockIdx.x, b = bh / Hkv, h = bh % Hkv;
    const Seq sq = seq_of(v, b);
    const int32_t budget = min(sq.budget, min(idx_stride, budget_cap));   // tok_idx holds at most idx_stride positions
    const float* sc = score + (int64_t)h * v.S_total + sq.sent_base;
    const int32_t* len = sent_len + sq.sent_base;
    const int32_t* off = sent_off + sq.sent_base + (v.cu_sent ? b : 0);
    int32_t* my_sel = sel_sent + (int64_t)bh * max_sel;
    int32_t* my_idx = tok_idx + (int64_t)bh * idx_stride;
    int32_t nsel, ntok;
    auto emit = [&](int32_t s, int32_t o, int32_t ln, int32_t sel_pos, int32_t tok_pos) {
        if (sel_pos < max_sel) my_sel[sel_pos] = s;
        if (sel_pos < kSelListCap) {
            list[sel_pos] = make_int4(s, o, ln, tok_pos);
        } else {                                              // list full: the owner writes its bucket's positions itself
            for (int32_t t = 0; t < ln && tok_pos + t < idx_stride; ++t) my_idx[tok_pos + t] = o + t;
        }
    };
    if (sq.n_sent <= 2 * kBlockThreads) select_block<2, true, false>(sc, len, off, sq.n_sent, budget, sh, emit, &nsel, &ntok);
    else select_block<kSelKreg, true, false>(sc, len, off, sq.n_sent, budget, sh, emit, &nsel, &ntok);
    if (threadIdx.x == 0) { n_sel[bh] = min(nsel, max_sel); n_tok[bh] = ntok; }
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int listed = min(nsel, kSelListCap);
    for (int e = w; e < listed; e += kBlockWaves) {
        const int4 it = list[e];
        for (int32_t t = lane; t < it.z && it.w + t < idx_stride; t += kWave) my_idx[it.w + t] = it.y + t;
    }
}

hipError_t launch_select(Ctx* c, const float* score, const int32_t* sent_off, const int32_t* sent_len,
                         const SeqView& v, int32_t* sel_sent, int32_t* n_sel, int32_t* tok_idx, int32_t idx_stride,
                         int32_t budget_cap, int32_t* n_tok) {
    hipLaunchKernelGGL(select_kernel, dim3(v.B * c->d.n_kv_heads), dim3(kBlockThreads), 0, c->stream, score, sent_off,
                       sent_len, v, c->d.n_kv_heads, c->max_sel, sel_sent, n_sel, tok_idx, idx_stride, budget_cap, n_tok);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Gather.  One 16-byte lane chunk per thread per row; a block copies RPB rows of K (blockIdx.z == 0) or V
// (blockIdx.z == 1) of one KV head with all its loads issued before its stores.  The pool pointer may be
// device-mapped pinned host memory: the same loads then cross PCIe.  RPB = 32 for a pool in HBM (16.7 MB per layer
// at a 2048-token budget: 6.3 us against 7.1 with 64 rows and 8.9 with 128), 64 for a host pool (53 GB/s over PCIe
// against 52 with 32 rows and 47 with 16).
// ------------------------------------------------------------------------------------------------
constexpr int kGatherRowsHbm = 32, kGatherRowsHost = kGatherRowsPerBlock;

template <int EB, int RPB>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(const char* __restrict__ Kl, const char* __restrict__ Vl,
                                                                int32_t T, const int32_t* __restrict__ tok_idx,
                                                                const int32_t* __restrict__ n_tok, int32_t budget,
                                                                char* __restrict__ Ks, char* __restrict__ Vs) {
    using R = Row<EB>;
    constexpr int kRowsPerIter = kGatherThreads / R::LPR;
    constexpr int kIter = RPB / kRowsPerIter;
    constexpr int kRowBytes = kHeadDim * EB;
    static_assert(kIter >= 1 && RPB % kRowsPerIter == 0, "block shape of the gather");
    const int h = blockIdx.y;
    const int32_t n = min(n_tok[h], budget);
    const int32_t j0 = blockIdx.x * RPB;
    if (j0 >= n) return;
    const char* src = (blockIdx.z == 0 ? Kl : Vl) + (int64_t)h * T * kRowBytes;
    char* dst = (blockIdx.z == 0 ? Ks : Vs) + (int64_t)h * budget * kRowBytes;
    const int r = threadIdx.x / R::LPR, cc = threadIdx.x % R::LPR;
    if (T <= 0) return;
    // Branch-free: indices and rows are clamped into range so every load can be issued up front
    // (two dependent rounds: all indices, then all rows); only the stores are predicated.
    int32_t x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t j = min(j0 + i * kRowsPerIter + r, n - 1);
        x[i] = tok_idx[(int64_t)h * budget + j];
    }
    uint4 val[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t xc = min(max(x[i], 0), T - 1);
        val[i] = *reinterpret_cast<const uint4*>(src + (int64_t)xc * kRowBytes + cc * 16);
    }
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t j = j0 + i * kRowsPerIter + r;
        if (j < n && x[i] >= 0 && x[i] < T) *reinterpret_cast<uint4*>(dst + (int64_t)j * kRowBytes + cc * 16) = val[i];
    }
}

template <int EB, int RPB>
static hipError_t launch_gather_g(Ctx* c, const void* K_layer, const void* V_layer, int32_t T, const int32_t* tok_idx,
                                  const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel) {
    const dim3 grid((budget + RPB - 1) / RPB, c->d.n_kv_heads, 2), block(kGatherThreads);
    hipLaunchKernelGGL((gather_kernel<EB, RPB>), grid, block, 0, c->stream, (const char*)K_layer, (const char*)V_layer, T, tok_idx,
                       n_tok, budget, (char*)K_sel, (char*)V_sel);
    return hipGetLastError();
}

hipError_t launch_gather(Ctx* c, const void* K_layer, const void* V_layer, int32_t T, bool host_pool, const int32_t* tok_idx,
                         const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel) {
    if (budget == 0) return hipSuccess;
    if (c->d.kv_dtype == SKV_BF16)
        return host_pool ? launch_gather_g<2, kGatherRowsHost>(c, K_layer, V_layer, T, tok_idx, n_tok, budget, K_sel, V_sel)
                         : launch_gather_g<2, kGatherRowsHbm>(c, K_layer, V_layer, T, tok_idx, n_tok, budget, K_sel, V_sel);
    return host_pool ? launch_gather_g<4, kGatherRowsHost>(c, K_layer, V_layer, T, tok_idx, n_tok, budget, K_sel, V_sel)
                     : launch_gather_g<4, kGatherRowsHbm>(c, K_layer, V_layer, T, tok_idx, n_tok, budget, K_sel, V_sel);
}

// ------------------------------------------------------------------------------------------------
// Attention (Eq. 3), split-K flash decoding.  A 1024-thread block (split, sequence*KV head) handles
// kAttChunk = 64 consecutive retrieved tokens for the G query heads of its KV head.
//   FUSED == false: rows come from K_sel/V_sel and n_tok from memory (skv_attend).
//   FUSED == true : the block first runs the selection for its (sequence, head) from the scores
//                   (redundantly with the other splits: the scores are a few KB in L2, and it saves a
//                   launch plus a round trip through tok_idx), keeps the pool rows of its own 64 tokens
//                   in LDS and reads K/V straight from the pool (skv_decode_step).
// Lane mapping: a wave covers RPW consecutive rows; lane = chunk * RPW + row, chunk being the 16-byte
// piece of the row.  The wave's loads still cover whole rows (coalesced), the P.V sum over a wave's
// rows is a DPP quad exchange (no LDS), and the q.k sum over chunks is DPP row rotations plus two
// cross-row shuffles.
//   1. every K and V chunk is requested up front on clamped addresses (no load waits for a bounds test);
//   2. logits for the G heads -> LDS;   3. one wave per query head: max, exp2, sum over the 64 logits;
//   4. P.V in registers, reduced over the wave's rows by DPP and over the 16 waves through LDS;
//   5. the un-normalised partial (m, l, acc) goes to the workspace with write-through stores; the last
//      block to arrive for the (sequence, KV head) -- a device-scope counter, no spinning -- merges the
//      partials with one round of independent loads and an online-softmax merge.
// ------------------------------------------------------------------------------------------------

// Split-K partials travel between blocks inside one kernel through st_agent / ld_agent64 (see above).

// sum over the RPW rows of a wave (lane bits below log2 RPW); every lane gets the total
template <int RPW>
__device__ __forceinline__ float sum_rows(float x) {
    x = dpp_add<0xB1>(x);
    if (RPW == 4) x = dpp_add<0x4E>(x);
    return x;
}
// sum over the LPR chunks of a row (the remaining lane bits); every lane gets the total
template <int RPW>
__device__ __forceinline__ float sum_chunks(float x) {
    if (RPW == 2) x = dpp_add<0x4E>(x);
    x = dpp_add<0x124>(x);
    x = dpp_add<0x128>(x);
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

// ds_read_b64_tr_b16 (gfx950): within each group of 16 lanes, lane i receives element i % 4 of the 8-byte pieces that
// lanes i / 4, i / 4 + 4, i / 4 + 8 and i / 4 + 12 of the group point at, in that order.  With lane s of the group
// pointing at dims 4 (s % 4) .. + 3 of row s / 4 of a row-major 4 x 16 block of bf16, lane i gets column i of the
// block's four rows: the B fragment of a 16x16x16 MFMA whose k index runs over the rows (one read instead of four
// 2-byte reads).
typedef short bf16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4_t lds_read_tr16(const char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((bf16x4_t __attribute__((address_space(3)))*)(p));
}

// q.K^T step on 32 dims: v_mfma_f32_16x16x32_bf16 with a 16-byte row chunk (8 consecutive dims) per lane on both sides
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4_t mfma_qk32(const uint4& k, const uint4& q, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, k), __builtin_bit_cast(bf16x8_t, q), c, 0, 0, 0);
}

// Tag of a launch of the single-launch step for one pair: the pair's epoch after this launch (1 .. 2^26 - 1, never 0, so
// zero-filled memory never looks valid) above the pair's number.  A word of memory carries a pair's current tag only if
// a block of that pair wrote it in this launch: other pairs differ in the low bits, earlier launches in the epoch (which
// repeats after 2^26 - 1 launches of the pair).
__device__ __forceinline__ uint32_t step_tag(uint32_t epoch, int pair) {
    uint32_t e = (epoch + 1u) & ((1u << (32 - kStepPairBits)) - 1u);
    if (e == 0u) e = 1u;
    return (e << kStepPairBits) | (uint32_t)pair;
}

struct AttArgs {
    const char* q;            // [B][Hq][D]
    const char* Kb;           // kDirect: K_sel [B*Hkv][row_stride][D]; else the layer's pool [Hkv][T_total][D]
    const char* Vb;
    const int32_t* n_tok;     // kDirect, kIndirect: [B*Hkv]
    const int32_t* tok_idx;   // kIndirect: [B*Hkv][idx_stride] positions local to the sequence
    int32_t row_stride;       // kDirect
    const float* score;       // kFused: [Hkv][S_total]
    const int32_t* sent_off;  // kFused
    const int32_t* sent_len;  // kFused
    int32_t* tok_idx_out;     // kFused, nullable: [B*Hkv][idx_stride]
    int32_t* n_tok_out;       // kFused, nullable: [B*Hkv]
    int32_t idx_stride;       // kFused, kIndirect: max_budget (positions per pair in tok_idx / tok_idx_out)
    int32_t budget_cap;       // budgets are clamped to this (the context's budget hint, at most max_budget)
    SeqView v;
    int32_t Hkv;
    int32_t max_splits;       // partial slots per query head (counted in 64-token chunks)
    float* part;
    float* ml;
    unsigned int* counter;
    float* out;
    float* lse;
    // kStep: the blocks of a (sequence, head) pair first score the pair's buckets between them
    const char* q_score;      // [B][Hq][D]
    const char* semvec;       // the layer's table [Hkv][S_total][D]
    int32_t sv_bytes;         // bytes per element of the table: 4, 2 or 1
    int32_t lg_parts;         // log2 of the blocks per pair
    unsigned int* step_epoch; // [pairs][kStepEpochStride]: launches of the single-launch step each pair has been through
    unsigned long long* step_score;   // [pairs][score_stride] (score, tag) words
    int32_t score_stride;
    unsigned long long* step_part;    // [blocks][G][kHeadDim + 2] (value, tag) words: a block's partial sums, then (max, normaliser)
    int32_t wait_limit;       // rounds of polling before a block gives up
    unsigned int* err_dev;    // set to 1 by a block that gave up
    unsigned int* err_host;   // the same word in pinned host memory (device address), nullable
};

enum { kDirect = 0, kFused = 1, kIndirect = 2, kStep = 3 };

// Every argument is demanded at this point, so the kernel-argument loads go out in one batch at the top of the kernel;
// left alone, the compiler loads each argument before its first use: one dependent round trip per branch, and a
// scalar-cache miss for each new 64-byte line of the argument block.
__device__ __forceinline__ void demand_args(const AttArgs& a) {
    asm volatile("" ::"s"(a.q), "s"(a.Kb), "s"(a.Vb), "s"(a.n_tok), "s"(a.tok_idx), "s"(a.row_stride), "s"(a.score),
                 "s"(a.sent_off), "s"(a.sent_len), "s"(a.tok_idx_out), "s"(a.n_tok_out), "s"(a.idx_stride), "s"(a.budget_cap), "s"(a.v.cu_tok),
                 "s"(a.v.cu_sent), "s"(a.v.budget_arr), "s"(a.v.T_total), "s"(a.v.S_total), "s"(a.v.budget), "s"(a.v.B),
                 "s"(a.Hkv), "s"(a.max_splits), "s"(a.part), "s"(a.ml), "s"(a.counter), "s"(a.out), "s"(a.lse));
}
__device__ __forceinline__ void demand_step_args(const AttArgs& a) {
    asm volatile("" ::"s"(a.q_score), "s"(a.semvec), "s"(a.sv_bytes), "s"(a.lg_parts), "s"(a.step_epoch), "s"(a.step_score),
                 "s"(a.score_stride), "s"(a.step_part), "s"(a.wait_limit), "s"(a.err_dev), "s"(a.err_host));
}

// CHUNK = retrieved tokens per block: 64 for the latency-bound single-sequence step (most blocks in
// flight), 256 for batches (fewer partials and arrivals per head, more loads in flight per block).
template <int EB, int G, int MODE, int CHUNK>
__global__ __launch_bounds__(kBlockThreads) void attend_kernel(AttArgs a) {
    using R = Row<EB>;
    constexpr int kRowsPerIter = kBlockWaves * R::RPW;        // 64 (bf16) or 32 (fp32)
    constexpr int kIter = CHUNK / kRowsPerIter;
    constexpr int kRowBytes = kHeadDim * EB;
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    constexpr int GH = G > 4 ? 4 : G, NH = G / GH;           // heads are processed GH at a time (register budget)
    constexpr int kTPL = CHUNK / kWave;                       // logits per lane in the softmax
    constexpr bool kMfma = (EB == 2);                         // bf16 runs on the matrix cores
    constexpr int kTiles = CHUNK / 16;                        // 16-token MFMA tiles, one per wave
    constexpr int kRedWaves = kMfma ? kTiles : kBlockWaves;   // waves that leave partial sums in sm_red
    static_assert(kTiles <= kBlockWaves, "one tile per wave");
    constexpr int kOut = G * kHeadDim;                        // outputs of the block
    constexpr int kCol2 = kOut / 2;                           // float pairs over the G heads
    constexpr int kGroups = kBlockThreads / kCol2;            // split groups of the merge: 16, 8, 4, 2 for G = 1, 2, 4, 8
    static_assert(kIter >= 1 && kGroups >= 1 && CHUNK % kWave == 0, "block shape");

    __shared__ float sm_logit[G][CHUNK];
    // Wave partial sums of P.V (wave ww, head g, dim d at sm_red_flat[ww * kRedStride + g * 128 + d], on the MFMA path at
    // [ww * kRedStride + d * G + g]); later the
    // merge scratch.  On the MFMA path each wave's partial sums reuse its own value tile.
    constexpr int kVPitch = 2 * kHeadDim + 16;                // bytes per value row in LDS; +16 spreads row groups over banks
    constexpr int kRedStride = kMfma ? 16 * kVPitch / 4 : G * kHeadDim;
    constexpr int kRedFloats = (kRedWaves * kRedStride > 4 * kBlockThreads) ? kRedWaves * kRedStride : 4 * kBlockThreads;
    static_assert(!kMfma || G * kHeadDim <= kRedStride, "a wave's partial sums fit in its value tile");
    __shared__ __attribute__((aligned(16))) float sm_red_flat[kRedFloats];
    __shared__ int sm_last;
    __shared__ int32_t sm_row[CHUNK];
    // kStep: the pair's scores on their way to the owning threads; later the merging block's scratch
    __shared__ uint32_t sm_keys[MODE == kStep ? kSelKreg * kBlockThreads : 1];

    // kStep: a one-dimensional grid, pair fastest, so that the hardware's round-robin of consecutive blocks over the XCDs
    // keeps the blocks of a pair together whenever the number of pairs is a multiple of the number of XCDs
    constexpr bool kSel = MODE == kFused || MODE == kStep;        // the block runs the selection itself
    const int n_pairs = a.v.B * a.Hkv;
    const int bh = MODE == kStep ? (int)(blockIdx.x % (unsigned)n_pairs) : (int)blockIdx.y;
    const int split = MODE == kStep ? (int)(blockIdx.x / (unsigned)n_pairs) : (int)blockIdx.x;
    const int b = bh / a.Hkv, h = bh % a.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane % R::RPW, cc = lane / R::RPW;
    const int Hq = a.Hkv * G;
    const int64_t qhead0 = (int64_t)b * Hq + (int64_t)h * G;      // first query head of the group
    demand_args(a);
    // kStep: the tag of this launch for this pair.  Every launch of the pair ends with its epoch advanced by one (block 0,
    // after it has seen the partial of every attending block, each of which had seen every score of the pair: so every
    // block whose tag matters has read the epoch by then), and the pair's number makes tags of different pairs differ.
    uint32_t tag = 0;
    if constexpr (MODE == kStep) {
        demand_step_args(a);
        tag = step_tag(ld_agent(a.step_epoch + bh * kStepEpochStride), bh);
    }
    const Seq sq = seq_of(a.v, b);
    const int32_t j0 = split * CHUNK;
    const int slot = split * (CHUNK / kWave);                     // partial slot (slots are counted in 64-token units)
    SKV_T(0);

    // bf16: the query fragments of the tile waves are requested first of all; they are in registers long before the
    // key rows arrive, so the logits wait for the keys only (lane (t16, qd): head t16, dims 32 s + 8 qd .. + 7)
    uint4 qB[kMfma ? 4 : 1];
    if constexpr (kMfma) {
        if (w < kTiles) {
            const int t16 = lane & 15, qd = lane >> 4;
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2)
                qB[s2] = *reinterpret_cast<const uint4*>(a.q + ((qhead0 + min(t16, G - 1)) * kHeadDim) * EB + 64 * s2 + 16 * qd);
        }
    }

    int32_t n;                                                    // retrieved tokens of this (sequence, head)
    bool step_ok = true;                                          // kStep: every wait of this block ended in time
    if constexpr (kSel) {
        __shared__ SelectShared sel_sh;
        const int32_t budget = min(sq.budget, a.budget_cap);
        if constexpr (MODE == kStep) {
            // ---- 0. scores of this block's share of the pair's buckets, published to the pair's other blocks ---------
            // Part `split` of the 2^lg_parts blocks of the pair owns the buckets [split * per, (split + 1) * per); wave
            // w takes RPWV consecutive buckets at a time.  The arithmetic per bucket is that of score_kernel (same
            // lanes, same order), so skv_score returns the very floats that are ranked here.  Each score is stored
            // with the launch tag in one 64-bit word; the blocks that go on read the pair's words until all carry it.
            const int32_t S = sq.n_sent;
            const int32_t per = (S + (1 << a.lg_parts) - 1) >> a.lg_parts;
            const int32_t lo = split * per, hi = min(lo + per, S);
            const char* qg = a.q_score + ((qhead0 * kHeadDim) * EB);
            const int64_t row0 = (int64_t)h * a.v.S_total + sq.sent_base;
            unsigned long long* sc_out = a.step_score + (int64_t)bh * a.score_stride;
            auto score_rows = [&](auto rpwv_tag) {
                constexpr int RPWV = decltype(rpwv_tag)::value;
                for (int32_t rw = lo + w * RPWV; rw < hi; rw += kBlockWaves * RPWV) {
                    if (a.sv_bytes == kTableF32)
                        score_wave_f32<EB, G, RPWV, true>(qg, reinterpret_cast<const float*>(a.semvec) + row0 * kHeadDim, hi, rw, sc_out, tag);
                    else if (a.sv_bytes == kTableBf16)
                        score_wave_bf16<EB, G, (RPWV < 4 ? 4 : RPWV), true>(qg, a.semvec + row0 * kHeadDim * 2, hi, rw, sc_out, tag);
                    else
                        score_wave_e4m3<EB, G, (RPWV < 8 ? 8 : RPWV), true>(qg, a.semvec + row0 * kHeadDim, hi, rw, sc_out, tag);
                }
            };
            // few buckets per block: 4 per wave visit (two loads in flight per lane, all 16 waves busy from 64 buckets on);
            // many: 16 per visit (eight loads in flight per lane)
            if (per <= kBlockWaves * 4) score_rows(std::integral_constant<int, 4>{});
            else score_rows(std::integral_constant<int, 16>{});
            SKV_T(12);
            // Blocks that neither attend (no position of theirs can hold a token: n <= budget) nor merge are done.
            if (split >= G && j0 >= budget) return;
        } else {
            if (split > 0 && j0 >= budget) return;                // n <= budget: nothing for this split
        }
        if (tid < CHUNK) sm_row[tid] = -1;
        int32_t nsel, ntok;
        // Each selected bucket that reaches into this block's positions marks, in every 64-position piece it touches,
        // where it starts there and which pool row that is; one wave per piece then fills the positions in between.
        auto mark = [&](int32_t, int32_t o, int32_t ln, int32_t, int32_t tok_pos) {
#pragma unroll
            for (int pc = 0; pc < CHUNK / kWave; ++pc) {
                const int32_t lo = max(tok_pos, j0 + pc * kWave);
                if (lo < min(tok_pos + ln, j0 + (pc + 1) * kWave)) sm_row[lo - j0] = o + (lo - tok_pos);
            }
        };
        const float* sc = a.score + (int64_t)h * a.v.S_total + sq.sent_base;
        const int32_t* len = a.sent_len + sq.sent_base;
        const int32_t* off = a.sent_off + sq.sent_base + (a.v.cu_sent ? b : 0);
        if constexpr (MODE == kStep) {                            // the scores are being written by the pair's blocks
            const float* tsc = reinterpret_cast<const float*>(a.step_score + (int64_t)bh * a.score_stride);
            if (sq.n_sent <= 2 * kBlockThreads)
                select_block<2, false, true>(tsc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok, tag, a.wait_limit, &step_ok, sm_keys);
            else
                select_block<kSelKreg, false, true>(tsc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok, tag, a.wait_limit, &step_ok, sm_keys);
        } else if (sq.n_sent <= 2 * kBlockThreads) {
            select_block<2, false, false>(sc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok);
        } else {
            select_block<kSelKreg, false, false>(sc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok);
        }
        n = ntok;
        if (split == 0 && tid == 0 && a.n_tok_out) a.n_tok_out[bh] = n;
        __syncthreads();                                          // bucket starts are marked
        if (w < CHUNK / kWave) {
            const int32_t v = sm_row[w * kWave + lane];
            // position of the last bucket start at or before this lane (-1: none): running maximum of lane + 1 over the starts
            const int32_t hp = (int32_t)wave_scan_max_u32(v >= 0 ? (uint32_t)lane + 1u : 0u) - 1;
            const int32_t base = __shfl(v, max(hp, 0));
            const int32_t row = hp >= 0 ? base + (lane - hp) : -1;
            sm_row[w * kWave + lane] = row;
            const int32_t pos = j0 + w * kWave + lane;
            if (a.tok_idx_out && pos < n) a.tok_idx_out[(int64_t)bh * a.idx_stride + pos] = row;
        }
        __syncthreads();                                          // sm_row complete
    } else {
        n = min(ld_const(a.n_tok, bh), MODE == kDirect ? a.row_stride : a.idx_stride);
    }
    // kStep: every block of the pair that ran the selection (and so used the epoch it read at its start) tells block 0 so
    // in the first (max, tag) word of its partial: the attending blocks with their partial, the others as soon as they
    // know that they hold no retrieved tokens.  Block 0 advances the epoch only after it has seen all of them, so that no
    // block of this launch can read the advanced epoch.
    auto presence = [&]() {
        if constexpr (MODE == kStep) {
            if (tid == 0)                                         // a block that gave up publishes nothing valid
                st_tagged(a.step_part + (int64_t)blockIdx.x * G * kStepPartWords + kHeadDim, -INFINITY, step_ok ? tag : 0u);
        }
    };
    // block 0: the words of blocks first .. (blocks of the pair that run the selection) - 1 carry the tag (bounded wait);
    // every thread of the block calls this
    auto others_were_here = [&](int first) -> bool {
        if constexpr (MODE == kStep) {
            const int n_cand = min(1 << a.lg_parts, max(G, (min(sq.budget, a.budget_cap) + CHUNK - 1) / CHUNK));
            if (n_cand <= first) return true;                     // block-uniform: the usual case, the budget is filled
            // the flag lives in the first word of the space the scores came through (thread 0, the only reader of that
            // word in the merge, is past its reads when it clears it)
            volatile uint32_t* missing = sm_keys;
            if (tid == 0) *missing = 0u;
            __syncthreads();
            if (tid >= first && tid < n_cand) {
                const unsigned long long* src = a.step_part + ((int64_t)(tid * n_pairs + bh) * G) * kStepPartWords + kHeadDim;
                bool there = false;
                for (int32_t round = 0; !there && round < a.wait_limit; ++round) there = tag_of(ld_tagged(src)) == tag;
                if (!there) *missing = 1u;
            }
            __syncthreads();
            return *missing == 0u;
        }
        return true;
    };
    if (n <= 0) {
        if (split == 0) {
            step_ok = others_were_here(1) && step_ok;
            for (int i = tid; i < kOut; i += kBlockThreads) a.out[qhead0 * kHeadDim + i] = step_ok ? 0.f : __builtin_nanf("");
            if (a.lse && tid < G) a.lse[qhead0 + tid] = -INFINITY;
            if constexpr (MODE == kStep) {
                if (tid == 0) {
                    st_agent(a.step_epoch + bh * kStepEpochStride, tag >> kStepPairBits);     // this launch of the pair is over
                    if (!step_ok) { st_agent(a.err_dev, 1u); if (a.err_host) st_agent(a.err_host, 1u); }
                }
            }
        } else {
            presence();
        }
        return;
    }
    const int nsplit = (n + CHUNK - 1) / CHUNK;
    // kStep: block g < G merges query head g of the group, whether or not it holds retrieved tokens itself
    const bool has_work = split < nsplit;
    if (!has_work) {
        presence();
        if (!(MODE == kStep && split < G)) return;
    }
    unsigned long long* my_part = nullptr;
    uint32_t part_tag = 0;
    if constexpr (MODE == kStep) {
        my_part = a.step_part + (int64_t)blockIdx.x * G * kStepPartWords;
        part_tag = step_ok ? tag : 0u;                            // a block that gave up publishes nothing valid
    }
    if (has_work) {
        const int32_t cnt = min(CHUNK, n - j0);
        SKV_T(4);

        // ---- 1. issue every load of the chunk ------------------------------------------------------------
        const char* Kh;
        const char* Vh;
        if (MODE == kDirect) {
            Kh = a.Kb + ((int64_t)bh * a.row_stride + j0) * kRowBytes;
            Vh = a.Vb + ((int64_t)bh * a.row_stride + j0) * kRowBytes;
        } else {
            Kh = a.Kb + ((int64_t)h * a.v.T_total + sq.tok_base) * kRowBytes;
            Vh = a.Vb + ((int64_t)h * a.v.T_total + sq.tok_base) * kRowBytes;
        }
        const float scale = kLog2e * rsqrtf((float)kHeadDim);
        if constexpr (kMfma) {
            // ---- bf16: q.K^T (v_mfma_f32_16x16x32_bf16) and P.V (v_mfma_f32_16x16x16_bf16) on the matrix cores ----
            // Wave w owns the 16 tokens [16w, 16w+16) of the chunk.  With t = lane % 16 and qd = lane / 16:
            //  * S^T = K Q^T: A fragment = 8 consecutive dims of token t's key, B fragment = the same 8 dims of head t's
            //    query (heads >= G are zero).  The dimension order inside the contraction is free as long as A and B agree,
            //    so one 16-byte load of a row (dims 32s+8qd .. +7) is one 32-deep MFMA step; four loads cover the row.
            //    The accumulator holds logit(token 4qd+j, head t), j = 0..3.
            //  * O = P V: that accumulator layout IS the A-fragment layout (head t, tokens 4qd+j); the B fragment
            //    V[token 4qd+j][16dt + t] is read from a wave-private LDS copy of the 16 value rows (padded pitch).
            typedef short bf16x4 __attribute__((ext_vector_type(4)));
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            char* sm_v = reinterpret_cast<char*>(sm_red_flat) + (size_t)w * 16 * kVPitch;       // this wave's value tile
            __shared__ float sm_wmax[kTiles][16], sm_wsum[kTiles][16];
            const int t16 = lane & 15, qd = lane >> 4;
            const bool tile = w < kTiles;
            float sj[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            bool lv[4] = {false, false, false, false};
            if (tile) {
                const int jj = 16 * w + t16;
                bool liveK = jj < cnt;
                const int jc = min(jj, cnt - 1);
                int32_t rowK;
                if (MODE == kDirect) {
                    rowK = jc;
                } else {
                    const int32_t x = kSel ? sm_row[jc] : a.tok_idx[(int64_t)bh * a.idx_stride + j0 + jc];
                    liveK = liveK && x >= 0 && x < sq.n_tok_ctx;
                    rowK = min(max(x, 0), max(sq.n_tok_ctx - 1, 0));
                }
                uint4 kA[4], vR[4];
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) kA[s2] = *reinterpret_cast<const uint4*>(Kh + (int64_t)rowK * kRowBytes + 64 * s2 + 16 * qd);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int32_t rowV = __shfl(rowK, 4 * i + qd);     // lane 4i+qd (< 16) holds the row of token 4i+qd
                    vR[i] = *reinterpret_cast<const uint4*>(Vh + (int64_t)rowV * kRowBytes + 16 * t16);
                }
                const unsigned long long vm = __ballot(liveK);        // bit t (t < 16): token t of the tile is real
                SKV_T(5);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) {
                    uint4 qq = qB[s2];
                    if (t16 >= G) qq = make_uint4(0, 0, 0, 0);
                    acc = mfma_qk32(kA[s2], qq, acc);
                }
                float mw = -INFINITY;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    lv[j] = (vm >> (4 * qd + j)) & 1ull;
                    sj[j] = lv[j] ? acc[j] * scale : -INFINITY;
                    mw = fmaxf(mw, sj[j]);
                }
                mw = fmaxf(mw, __shfl_xor(mw, 16));
                mw = fmaxf(mw, __shfl_xor(mw, 32));
                if (qd == 0) sm_wmax[w][t16] = mw;
                // the tile's value rows go to LDS (rows of masked tokens as zeros)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool lr = (vm >> (4 * i + qd)) & 1ull;
                    *reinterpret_cast<uint4*>(sm_v + (4 * i + qd) * kVPitch + 16 * t16) = lr ? vR[i] : make_uint4(0, 0, 0, 0);
                }
            }
            __syncthreads();
            SKV_T(6);
            if (tile) {
                float mb = -INFINITY;
#pragma unroll
                for (int ww = 0; ww < kTiles; ++ww) mb = fmaxf(mb, sm_wmax[ww][t16]);
                unsigned short pb[4];
                float lw = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = (lv[j] && mb > -INFINITY) ? exp2f(sj[j] - mb) : 0.f;
                    uint32_t u = __float_as_uint(p);
                    u += 0x7fffu + ((u >> 16) & 1u);                  // round to nearest even bf16
                    pb[j] = (unsigned short)(u >> 16);
                    lw += __uint_as_float((uint32_t)pb[j] << 16);     // the normaliser sums the rounded weights
                }
                lw += __shfl_xor(lw, 16);
                lw += __shfl_xor(lw, 32);
                if (qd == 0) sm_wsum[w][t16] = lw;
                const bf16x4 pa = {(short)pb[0], (short)pb[1], (short)pb[2], (short)pb[3]};
                // B fragments by the LDS transpose read: this lane points at dims 4 (t16 % 4) .. + 3 of value row 4 qd + t16 / 4
                const char* vtr = sm_v + (4 * qd + (t16 >> 2)) * kVPitch + 8 * (t16 & 3);
                f32x4 o[kHeadDim / 16];
#pragma unroll
                for (int dt = 0; dt < kHeadDim / 16; ++dt) {
                    const bf16x4 vb = lds_read_tr16(vtr + 32 * dt);
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vb, zero, 0, 0, 0);
                }
                // the value tile has been consumed: its space takes the wave's partial sums, head fastest (dim d, head g at
                // red[d * G + g]), so that a lane stores its heads of one dim with a single instruction
                float* red = sm_red_flat + w * kRedStride;
                if (4 * qd < G) {
#pragma unroll
                    for (int dt = 0; dt < kHeadDim / 16; ++dt) {
                        float* dst = red + (16 * dt + t16) * G + 4 * qd;
                        if constexpr (G >= 4) *reinterpret_cast<float4*>(dst) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
                        else if constexpr (G == 2) *reinterpret_cast<float2*>(dst) = make_float2(o[dt][0], o[dt][1]);
                        else dst[0] = o[dt][0];
                    }
                }
            }
            __syncthreads();
            if (tid < G) {                                            // block max and normaliser of head tid
                float mb = -INFINITY, lb = 0.f;
#pragma unroll
                for (int ww = 0; ww < kTiles; ++ww) { mb = fmaxf(mb, sm_wmax[ww][tid]); lb += sm_wsum[ww][tid]; }
                if constexpr (MODE == kStep) {
                    unsigned long long* dst = my_part + tid * kStepPartWords + kHeadDim;
                    st_tagged(dst, mb, part_tag);
                    st_tagged(dst + 1, lb, part_tag);
                } else {
                    float* dst = a.ml + (((qhead0 + tid) * a.max_splits) + slot) * 2;
                    st_agent(dst, mb);
                    st_agent(dst + 1, lb);
                }
            }
        } else {
            // Rows past the chunk's end (and positions outside the sequence) are clamped to a valid row, loaded
            // anyway and masked afterwards, so that all loads are in flight together.
            int32_t rowi[kIter];
            bool live[kIter];
#pragma unroll
            for (int i = 0; i < kIter; ++i) {
                const int jj = i * kRowsPerIter + w * R::RPW + r;
                live[i] = jj < cnt;
                const int jc = min(jj, cnt - 1);
                if (MODE == kDirect) {
                    rowi[i] = jc;
                } else {
                    const int32_t x = kSel ? sm_row[jc] : a.tok_idx[(int64_t)bh * a.idx_stride + j0 + jc];
                    live[i] = live[i] && x >= 0 && x < sq.n_tok_ctx;
                    rowi[i] = min(max(x, 0), max(sq.n_tok_ctx - 1, 0));
                }
            }
            uint4 kraw[kIter], vraw[kIter];
#pragma unroll
            for (int i = 0; i < kIter; ++i) {
                kraw[i] = *reinterpret_cast<const uint4*>(Kh + (int64_t)rowi[i] * kRowBytes + cc * 16);
                vraw[i] = *reinterpret_cast<const uint4*>(Vh + (int64_t)rowi[i] * kRowBytes + cc * 16);
            }
            SKV_T(5);

            // ---- 2. logits ---------------------------------------------------------------------------------
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                float qf[GH][R::EPL];
#pragma unroll
                for (int g = 0; g < GH; ++g) {
                    const uint4 t = *reinterpret_cast<const uint4*>(a.q + ((qhead0 + hh * GH + g) * kHeadDim) * EB + cc * 16);
                    R::unpack(t, qf[g]);
                }
#pragma unroll
                for (int i = 0; i < kIter; ++i) {
                    float kf[R::EPL];
                    R::unpack(kraw[i], kf);
#pragma unroll
                    for (int g = 0; g < GH; ++g) {
                        float acc = 0.f;
#pragma unroll
                        for (int e = 0; e < R::EPL; ++e) acc += qf[g][e] * kf[e];
                        acc = sum_chunks<R::RPW>(acc);
                        if (cc == 0) sm_logit[hh * GH + g][i * kRowsPerIter + w * R::RPW + r] = live[i] ? acc * scale : -INFINITY;
                    }
                }
            }
            __syncthreads();
            SKV_T(6);

            // ---- 3. softmax over the chunk, one wave per query head --------------------------------------------
            if (w < G) {
                const int g = w;
                float x[kTPL];
                float m = -INFINITY;
#pragma unroll
                for (int t = 0; t < kTPL; ++t) { x[t] = sm_logit[g][t * kWave + lane]; m = fmaxf(m, x[t]); }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
                float l = 0.f;
#pragma unroll
                for (int t = 0; t < kTPL; ++t) {
                    const float p = (m == -INFINITY) ? 0.f : exp2f(x[t] - m);
                    sm_logit[g][t * kWave + lane] = p;
                    l += p;
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off);
                if (lane == 0) {
                    if constexpr (MODE == kStep) {
                        unsigned long long* dst = my_part + g * kStepPartWords + kHeadDim;
                        st_tagged(dst, m, part_tag);
                        st_tagged(dst + 1, l, part_tag);
                    } else {
                        float* dst = a.ml + (((qhead0 + g) * a.max_splits) + slot) * 2;
                        st_agent(dst, m);
                        st_agent(dst + 1, l);
                    }
                }
            }
            __syncthreads();

            // ---- 4. P.V -------------------------------------------------------------------------------------
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                float acc[GH][R::EPL];
#pragma unroll
                for (int g = 0; g < GH; ++g)
#pragma unroll
                    for (int e = 0; e < R::EPL; ++e) acc[g][e] = 0.f;
#pragma unroll
                for (int i = 0; i < kIter; ++i) {
                    const int jj = i * kRowsPerIter + w * R::RPW + r;
                    float vf[R::EPL];
                    R::unpack(vraw[i], vf);
                    if (!live[i]) {                                      // masked rows hold a clamped (foreign) row
#pragma unroll
                        for (int e = 0; e < R::EPL; ++e) vf[e] = 0.f;
                    }
#pragma unroll
                    for (int g = 0; g < GH; ++g) {
                        const float p = sm_logit[hh * GH + g][jj];
#pragma unroll
                        for (int e = 0; e < R::EPL; ++e) acc[g][e] += p * vf[e];
                    }
                }
#pragma unroll
                for (int g = 0; g < GH; ++g)
#pragma unroll
                    for (int e = 0; e < R::EPL; ++e) acc[g][e] = sum_rows<R::RPW>(acc[g][e]);
                if (r == 0) {
#pragma unroll
                    for (int g = 0; g < GH; ++g)
#pragma unroll
                        for (int e = 0; e < R::EPL; e += 4)
                            *reinterpret_cast<float4*>(&sm_red_flat[w * kRedStride + (hh * GH + g) * kHeadDim + cc * R::EPL + e]) =
                                make_float4(acc[g][e], acc[g][e + 1], acc[g][e + 2], acc[g][e + 3]);
                }
            }
        }
        if constexpr (!kMfma) __syncthreads();                    // (the matrix-core path met after its partial sums already)
        for (int i = tid; i < kOut; i += kBlockThreads) {
            const int g = i / kHeadDim, d = i % kHeadDim;
            const int src = kMfma ? d * G + g : i;                     // the MFMA path leaves its sums head fastest
            float o = sm_red_flat[src];
#pragma unroll
            for (int ww = 1; ww < kRedWaves; ++ww) o += sm_red_flat[ww * kRedStride + src];
            if constexpr (MODE == kStep) st_tagged(my_part + g * kStepPartWords + d, o, part_tag);
            else st_agent(a.part + (((qhead0 + g) * a.max_splits) + slot) * kHeadDim + d, o);
        }
        SKV_T(7);
    }

    if constexpr (MODE == kStep) {
        // ---- 5'. per-head merge without an arrival counter -------------------------------------------------------
        // Block g < G of the pair merges query head g.  Thread (grp, col) -- a group is two whole waves, so a wave's
        // loads of a partial row are contiguous -- reads dim `col` of the partials of the splits grp, grp + 8, ...
        // (value and tag in one word) and their (max, normaliser) words, again and again until all carry the launch tag
        // (bounded; no barrier, no sleep: a wave leaves as soon as its own words are there), folds them into a running
        // (max, normaliser, output), and the eight groups meet once in LDS.  No block waits for a store
        // acknowledgement and nothing is counted.
        if (split >= G) return;
        constexpr int kGroups8 = kBlockThreads / kHeadDim;               // 8 split groups of 128 threads
        const int g = split, col = tid % kHeadDim, grp = tid / kHeadDim;
        float M = -INFINITY, L = 0.f, o = 0.f;
        bool ok = step_ok;
        for (int base = 0; base < nsplit && ok; base += 4 * kGroups8) {
            unsigned long long pv[4] = {0, 0, 0, 0}, mv[4] = {0, 0, 0, 0}, lv[4] = {0, 0, 0, 0};
            bool mine = false;
            for (int32_t round = 0; !mine && round < a.wait_limit; ++round) {
                mine = true;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sp = base + grp + u * kGroups8;             // wave-uniform
                    if (sp < nsplit) {
                        const unsigned long long* src = a.step_part + ((int64_t)(sp * n_pairs + bh) * G + g) * kStepPartWords;
                        pv[u] = ld_tagged(src + col);
                        mv[u] = ld_tagged(src + kHeadDim);
                        lv[u] = ld_tagged(src + kHeadDim + 1);
                        mine = mine && tag_of(pv[u]) == tag && tag_of(mv[u]) == tag && tag_of(lv[u]) == tag;
                    }
                }
            }
            ok = mine;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (ok && base + grp + u * kGroups8 < nsplit) {
                    const float ms = val_of(mv[u]);
                    if (ms > -INFINITY) {
                        const float nm = fmaxf(M, ms);
                        const float ca = exp2f(M - nm), cb = exp2f(ms - nm);  // M == -inf gives ca == 0
                        L = L * ca + val_of(lv[u]) * cb;
                        o = o * ca + val_of(pv[u]) * cb;
                        M = nm;
                    }
                }
            }
        }
        SKV_T(10);
        // (o, M, L) per thread: 3 x 1024 floats in the space the scores came through; a thread whose wait ran out leaves
        // NaN as its maximum
        float* scratch = reinterpret_cast<float*>(sm_keys);
        scratch[tid] = o; scratch[kBlockThreads + tid] = ok ? M : __builtin_nanf(""); scratch[2 * kBlockThreads + tid] = L;
        __syncthreads();
        SKV_T(11);
        bool bad = false;
        if (tid < kHeadDim) {
            float mg[kGroups8], lg[kGroups8], og[kGroups8];
            float Mx = -INFINITY;
#pragma unroll
            for (int gg = 0; gg < kGroups8; ++gg) {
                og[gg] = scratch[gg * kHeadDim + tid];
                mg[gg] = scratch[kBlockThreads + gg * kHeadDim + tid];
                lg[gg] = scratch[2 * kBlockThreads + gg * kHeadDim + tid];
                bad = bad || mg[gg] != mg[gg];
                Mx = fmaxf(Mx, mg[gg]);
            }
            float Ls = 0.f, os = 0.f;
#pragma unroll
            for (int gg = 0; gg < kGroups8; ++gg) {
                if (mg[gg] > -INFINITY) {
                    const float c = exp2f(mg[gg] - Mx);
                    Ls += c * lg[gg];
                    os += c * og[gg];
                }
            }
            const bool empty = !(Ls > 0.f);                               // every retrieved position was out of range
            float res = empty ? 0.f : os / Ls;
            if (bad) res = __builtin_nanf("");                            // a wait of this launch ran out
            a.out[(qhead0 + g) * kHeadDim + tid] = res;
            if (a.lse && tid == 0) a.lse[qhead0 + g] = empty ? -INFINITY : (Mx + log2f(Ls)) * kLn2;
            if (bad) { st_agent(a.err_dev, 1u); if (a.err_host) st_agent(a.err_host, 1u); }
        }
        // Block 0 ends the pair's launch by advancing its epoch: its threads have seen the partial of every attending
        // block (the barrier above) and now make sure of the word of every other block that ran the selection; all of
        // them, and through the scores they waited for every scoring block, have read the epoch by then.
        if (split == 0) {
            const bool all_here = others_were_here(nsplit);
            if (tid == 0) {
                st_agent(a.step_epoch + bh * kStepEpochStride, tag >> kStepPairBits);
                if (!all_here) { st_agent(a.err_dev, 1u); if (a.err_host) st_agent(a.err_host, 1u); }
            }
        }
        SKV_T(9);
        return;
    }

    // ---- 5. last arrival combines ------------------------------------------------------------------
    // Every wave waits for its own write-through partial stores, then the barrier: only after both does thread 0
    // issue the device-scope increment, so whoever reads nsplit - 1 knows every partial is there.
    block_sync_after_stores();
    if (tid == 0) {
        const unsigned int old = __hip_atomic_fetch_add(&a.counter[bh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = (old == (unsigned int)(nsplit - 1));
    }
    __syncthreads();
    SKV_T(8);
    if (!sm_last) return;
    // A thread owns one pair of output floats and every kGroups-th split: one batch of independent 8-byte
    // loads, merged online (running max M, normaliser L, outputs) in registers; groups merge through LDS.
    float4* scratch = reinterpret_cast<float4*>(sm_red_flat);               // (o0, o1, M, L) per thread
    {
        const int col = tid % kCol2, grp = tid / kCol2;
        const int g = col / (kHeadDim / 2);
        const float* mlg = a.ml + ((qhead0 + g) * a.max_splits) * 2;
        const float* pg = a.part + ((qhead0 + g) * a.max_splits) * kHeadDim + (col % (kHeadDim / 2)) * 2;
        float M = -INFINITY, L = 0.f, o0 = 0.f, o1 = 0.f;
        constexpr int kU = CHUNK >= 2 * kWave ? 4 : 8;       // loads in flight per thread: sized for a 2048-token budget
        for (int s0 = grp; s0 < nsplit; s0 += kGroups * kU) {
            unsigned long long pv[kU], mv[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {                   // clamped, unconditional loads
                const int sidx = min(s0 + u * kGroups, nsplit - 1) * (CHUNK / kWave);
                pv[u] = ld_agent64(pg + (int64_t)sidx * kHeadDim);
                mv[u] = ld_agent64(mlg + 2 * sidx);
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const float ms = (s0 + u * kGroups < nsplit) ? lo_f(mv[u]) : -INFINITY;
                if (ms > -INFINITY) {
                    const float nm = fmaxf(M, ms);
                    const float ca = exp2f(M - nm), cb = exp2f(ms - nm);      // M == -inf gives ca == 0
                    L = L * ca + hi_f(mv[u]) * cb;
                    o0 = o0 * ca + lo_f(pv[u]) * cb;
                    o1 = o1 * ca + hi_f(pv[u]) * cb;
                    M = nm;
                }
            }
        }
        SKV_T(10);
        __syncthreads();                                     // sm_red (partial sums) no longer read by anyone
        scratch[grp * kCol2 + col] = make_float4(o0, o1, M, L);
    }
    __syncthreads();
    SKV_T(11);
    if (tid < kCol2) {
        float M = -INFINITY;
#pragma unroll
        for (int grp = 0; grp < kGroups; ++grp) M = fmaxf(M, scratch[grp * kCol2 + tid].z);
        float L = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
        for (int grp = 0; grp < kGroups; ++grp) {
            const float4 t = scratch[grp * kCol2 + tid];
            if (t.z > -INFINITY) {
                const float c = exp2f(t.z - M);
                L += c * t.w; o0 += c * t.x; o1 += c * t.y;
            }
        }
        const bool empty = !(L > 0.f);                       // every retrieved position was out of range
        const float inv = empty ? 0.f : 1.f / L;
        reinterpret_cast<float2*>(a.out + qhead0 * kHeadDim)[tid] = make_float2(o0 * inv, o1 * inv);
        if (a.lse && (tid % (kHeadDim / 2)) == 0)
            a.lse[qhead0 + tid / (kHeadDim / 2)] = empty ? -INFINITY : (M + log2f(L)) * kLn2;
    }
    if (tid == 0) __hip_atomic_store(&a.counter[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
    SKV_T(9);
}

// ------------------------------------------------------------------------------------------------
// Streaming form of the bf16 attention for batches.  Measured on the 1024-thread kernel above with 16 sequences
// x 8 heads: all blocks start together, load together (memory saturated for 5 us) and then compute together
// (memory idle for 7 us), twice.  Here a wave owns 64 consecutive retrieved tokens and walks them in four 16-token
// MFMA tiles -- the next tile's K and V rows are requested as soon as the current ones have been consumed (K by the
// logit MFMAs, V by its copy to LDS) -- carrying a running (max, normaliser, output) per head as in flash decoding;
// all blocks of the launch are resident at once (16 waves per CU, each with 8 KB in flight).
// Tile arithmetic is that of the kernel above: S^T = K Q^T with K rows as A fragments, P rounded to bf16 with the
// normaliser summing the rounded weights, V through a wave-private LDS tile into B fragments.
// A block is 16 waves and CHUNK = 1024 (or 512, or 2048) retrieved tokens of one (sequence, KV head).  It first runs the
// selection itself from the scores (as the single-sequence kernel does, redundantly with the head's other blocks) and
// keeps the pool rows of its positions in LDS: no selection launch, no tok_idx round trip, two partials per 2048-token
// budget with 1024-token blocks, none when one block covers the budget.
// Measured against select_kernel + a 4-wave form of this kernel that read tok_idx (16 sequences x 8 heads, budget
// 2048): 8.7 + 37.1 us -> 39 us per layer; equal or better from 8 to 48 sequences.
// ------------------------------------------------------------------------------------------------
constexpr int kStreamTiles = 4;                                   // 16-token tiles per wave
constexpr int kStreamWaves = kBlockWaves;                         // the block-level selection needs kBlockThreads threads
constexpr int kStreamChunk = kStreamWaves * kStreamTiles * 16;    // 1024 tokens per block, one position per thread
static_assert(kStreamChunk == kBlockThreads, "the usual block: one retrieved position per thread");

constexpr int kStreamMaxChunk = 2 * kStreamChunk;                 // the largest block: two positions per thread
constexpr int kStreamVPitch = 2 * kHeadDim + 16;                  // bytes per value row in LDS; +16 spreads row groups over banks

struct StreamShared {
    __attribute__((aligned(16))) char v[kStreamWaves][16 * kStreamVPitch];   // value tile, later the wave's partial sums
    __attribute__((aligned(16))) unsigned short q[16][kHeadDim];             // the group's queries, rows >= G zero
    float wmax[kStreamWaves][16], wsum[kStreamWaves][16];
    int32_t row[kStreamMaxChunk];                                            // pool row of every position of the block (-1: none)
    int next_tile;
    int last;
};

// queries of the group -> LDS (16 bytes per thread: 16 rows x 256 bytes); a barrier must follow before they are read
template <int G>
__device__ __forceinline__ void stream_load_queries(const AttArgs& a, StreamShared& ss, int64_t qhead0) {
    const int tid = threadIdx.x;
    if (tid < 256) {
        const int row = tid >> 4, piece = tid & 15;
        uint4 t = make_uint4(0, 0, 0, 0);
        if (row < G) t = *reinterpret_cast<const uint4*>(a.q + ((qhead0 + row) * kHeadDim) * 2 + 16 * piece);
        *reinterpret_cast<uint4*>(&ss.q[row][8 * piece]) = t;
    }
}

// Attention of one block of CHUNK (512, 1024 or 2048) positions once the selection is known: n = retrieved tokens of the
// (sequence, head); ss.row holds the pool row of position split * CHUNK + i at i (-1: no such token) for i < CHUNK.
// The queries are on their way to ss.q.  Every thread of the block calls this.
template <int G, int CHUNK>
__device__ __forceinline__ void stream_attend(const AttArgs& a, StreamShared& ss, int bh, int b, int h, int split, const Seq& sq,
                                              int32_t n) {

    constexpr int NW = kStreamWaves;
    constexpr int kThreads = kBlockThreads;
    constexpr int kRowBytes = kHeadDim * 2;
    constexpr int kVPitch = kStreamVPitch;
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    constexpr int kOut = G * kHeadDim, kCol2 = kOut / 2;
    constexpr int kColsPerThread = (kCol2 + kThreads - 1) / kThreads;
    typedef short bf16x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    static_assert(G * kHeadDim * 4 <= 16 * kVPitch, "a wave's partial sums fit in its value tile");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int t16 = lane & 15, qd = lane >> 4;
    const int64_t qhead0 = (int64_t)b * (a.Hkv * G) + (int64_t)h * G;
    const int32_t j0 = split * CHUNK;
    const int slot = split * (CHUNK / kWave);
    if (n <= 0) {
        if (split == 0) {
            for (int i = tid; i < kOut; i += kThreads) a.out[qhead0 * kHeadDim + i] = 0.f;
            if (a.lse && tid < G) a.lse[qhead0 + tid] = -INFINITY;
        }
        return;
    }
    const int nsplit = (n + CHUNK - 1) / CHUNK;
    if (split >= nsplit) return;
    const int32_t cnt = min(CHUNK, n - j0);

    // The block's positions are walked in 16-token tiles handed out dynamically: a wave starts with tile w and takes the
    // next free one from an LDS counter whenever it finishes one, so the waves that memory serves first do more tiles
    // and all 16 keep loads in flight until the block's last tile (with four fixed tiles per wave the slowest wave ran
    // about 5 us behind the first).  Rows of unreal positions are stored as -1.
    if (tid == 0) ss.next_tile = NW;
    const int ntiles = (cnt + 15) / 16;
    const char* Kh = a.Kb + ((int64_t)h * a.v.T_total + sq.tok_base) * kRowBytes;
    const char* Vh = a.Vb + ((int64_t)h * a.v.T_total + sq.tok_base) * kRowBytes;
    const float scale = kLog2e * rsqrtf((float)kHeadDim);
    __syncthreads();                                              // rows and the tile counter are in LDS
    SKV_T(4);

    uint4 kA[4], vR[4];
    // rows of a tile: lanes with the same t16 hold the row of the tile's token t16 (-1: not real)
    auto rows_of = [&](int tile) { return ss.row[16 * tile + t16]; };
    auto issue = [&](int32_t rowt, uint4* k, uint4* v) {
        // 32-bit byte offsets from the (head, sequence) base: the host only uses this kernel below 2^24 tokens
        const int32_t rc = max(rowt, 0);
        const uint32_t offK = (uint32_t)rc * kRowBytes + 16u * qd;
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) k[s2] = *reinterpret_cast<const uint4*>(Kh + (offK + 64u * s2));
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const uint32_t offV = (uint32_t)__shfl(rc, 4 * ii + qd) * kRowBytes + 16u * t16;
            v[ii] = *reinterpret_cast<const uint4*>(Vh + offV);
        }
    };
    int tile = w;                                                 // wave-uniform
    int32_t row_cur = tile < ntiles ? rows_of(tile) : -1;
    if (tile < ntiles) issue(row_cur, kA, vR);
    SKV_T(5);

    float m_run = -INFINITY, l_run = 0.f;                         // per head t16; l_run covers this lane's tokens only
    f32x4 o[kHeadDim / 16];
#pragma unroll
    for (int dt = 0; dt < kHeadDim / 16; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    char* vt_b = ss.v[w];
    // B fragments of P.V by the LDS transpose read: this lane's address is the 4-dim piece (dims 4 (t16 % 4) .. + 3 of
    // the 16-dim group) of value row 4 qd + t16 / 4
    const char* vtr = vt_b + (4 * qd + (t16 >> 2)) * kVPitch + 8 * (t16 & 3);

    while (tile < ntiles) {
        // the wave's next tile, asked for early so that its rows are known when this tile's registers come free
        int nxt = 0;
        if (lane == 0) nxt = atomicAdd(&ss.next_tile, 1);
        nxt = __builtin_amdgcn_readfirstlane(nxt);
        const unsigned int tm = (unsigned int)__ballot(row_cur >= 0) & 0xffffu;   // bit t: token t of the tile is real
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
            const uint4 qq = *reinterpret_cast<const uint4*>(&ss.q[t16][32 * s2 + 8 * qd]);
            acc = mfma_qk32(kA[s2], qq, acc);
        }
        // the tile's value rows go to the wave's LDS tile (rows of masked tokens as zeros) ...
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const bool lr = (tm >> (4 * ii + qd)) & 1u;
            *reinterpret_cast<uint4*>(vt_b + (4 * ii + qd) * kVPitch + 16 * t16) = lr ? vR[ii] : make_uint4(0, 0, 0, 0);
        }
        // ... which frees the row registers for the next tile: its loads fly during this tile's softmax and P.V
        row_cur = nxt < ntiles ? rows_of(nxt) : -1;
        if (nxt < ntiles) issue(row_cur, kA, vR);
        tile = nxt;
        float sj[4], mt = -INFINITY;
        bool lv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lv[j] = (tm >> (4 * qd + j)) & 1u;
            sj[j] = lv[j] ? acc[j] * scale : -INFINITY;
            mt = fmaxf(mt, sj[j]);
        }
        mt = fmaxf(mt, __shfl_xor(mt, 16));
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        const float m_new = fmaxf(m_run, mt);
        const float alpha = (m_new > -INFINITY) ? exp2f(m_run - m_new) : 1.f;   // m_run == -inf gives 0
        unsigned short pb[4];
        float lw = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = lv[j] ? exp2f(sj[j] - m_new) : 0.f;
            uint32_t u = __float_as_uint(p);
            u += 0x7fffu + ((u >> 16) & 1u);                      // round to nearest even bf16
            pb[j] = (unsigned short)(u >> 16);
            lw += __uint_as_float((uint32_t)pb[j] << 16);         // the normaliser sums the rounded weights
        }
        l_run = l_run * alpha + lw;
        m_run = m_new;
        // running outputs: row 4qd+j of o is head 4qd+j, whose factor sits in lane 4qd+j
        float ar[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) ar[j] = __shfl(alpha, 4 * qd + j);
#pragma unroll
        for (int dt = 0; dt < kHeadDim / 16; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) o[dt][j] *= ar[j];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");    // the tile is private to the wave: order only
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const bf16x4 pa = {(short)pb[0], (short)pb[1], (short)pb[2], (short)pb[3]};
#pragma unroll
        for (int dt = 0; dt < kHeadDim / 16; ++dt) {
            const bf16x4 vb = lds_read_tr16(vtr + 32 * dt);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vb, o[dt], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");    // reads of this tile precede the next tile's writes
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    SKV_T(6);

    // ---- the block's waves combine: common max per head, partial sums through the value tiles ------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (qd == 0) ss.wmax[w][t16] = m_run;
    __syncthreads();
    float mb = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) mb = fmaxf(mb, ss.wmax[ww][t16]);
    const float cw = (m_run > -INFINITY) ? exp2f(m_run - mb) : 0.f;
    if (qd == 0) ss.wsum[w][t16] = l_run * cw;
    {
        float cr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cr[j] = __shfl(cw, 4 * qd + j);
        float* red = reinterpret_cast<float*>(vt_b);
#pragma unroll
        for (int dt = 0; dt < kHeadDim / 16; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * qd + j < G) red[(4 * qd + j) * kHeadDim + 16 * dt + t16] = o[dt][j] * cr[j];
    }
    __syncthreads();
    if (nsplit == 1) {
        // the only block of this (sequence, head): its combined sums are the result, no partials, no arrival, no merge
        for (int i = tid; i < kOut; i += kThreads) {
            const int g = i / kHeadDim;
            float sum = 0.f, lb = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) {
                sum += reinterpret_cast<const float*>(ss.v[ww])[i];
                lb += ss.wsum[ww][g];
            }
            const bool empty = !(lb > 0.f);                       // every retrieved position was out of range
            a.out[qhead0 * kHeadDim + i] = empty ? 0.f : sum / lb;
            if (a.lse && (i % kHeadDim) == 0) {
                float mh = -INFINITY;
#pragma unroll
                for (int ww = 0; ww < NW; ++ww) mh = fmaxf(mh, ss.wmax[ww][g]);
                a.lse[qhead0 + g] = empty ? -INFINITY : (mh + log2f(lb)) * kLn2;
            }
        }
        return;
    }
    if (tid < G) {
        float lb = 0.f, mh = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) { lb += ss.wsum[ww][tid]; mh = fmaxf(mh, ss.wmax[ww][tid]); }
        float* dst = a.ml + (((qhead0 + tid) * a.max_splits) + slot) * 2;
        st_agent(dst, mh);
        st_agent(dst + 1, lb);
    }
    for (int i = tid; i < kOut; i += kThreads) {
        const int g = i / kHeadDim, d = i % kHeadDim;
        float sum = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) sum += reinterpret_cast<const float*>(ss.v[ww])[i];
        st_agent(a.part + (((qhead0 + g) * a.max_splits) + slot) * kHeadDim + d, sum);
    }
    SKV_T(7);

    // ---- last arrival combines (same protocol as attend_kernel) ------------------------------------------------
    block_sync_after_stores();
    if (tid == 0) {
        const unsigned int old = __hip_atomic_fetch_add(&a.counter[bh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ss.last = (old == (unsigned int)(nsplit - 1));
    }
    __syncthreads();
    SKV_T(8);
    if (!ss.last) return;
#pragma unroll
    for (int c = 0; c < kColsPerThread; ++c) {
        const int col = tid + c * kThreads;
        if (col >= kCol2) break;
        const int g = col / (kHeadDim / 2);
        const float* mlg = a.ml + ((qhead0 + g) * a.max_splits) * 2;
        const float* pg = a.part + ((qhead0 + g) * a.max_splits) * kHeadDim + (col % (kHeadDim / 2)) * 2;
        float M = -INFINITY, L = 0.f, o0 = 0.f, o1 = 0.f;
        constexpr int kU = 2;                                     // loads in flight per thread: sized for a 2048-token budget
        for (int s0 = 0; s0 < nsplit; s0 += kU) {
            unsigned long long pv[kU], mv[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {                        // clamped, unconditional loads
                const int sidx = min(s0 + u, nsplit - 1) * (CHUNK / kWave);
                pv[u] = ld_agent64(pg + (int64_t)sidx * kHeadDim);
                mv[u] = ld_agent64(mlg + 2 * sidx);
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const float ms = (s0 + u < nsplit) ? lo_f(mv[u]) : -INFINITY;
                if (ms > -INFINITY) {
                    const float nm = fmaxf(M, ms);
                    const float ca = exp2f(M - nm), cb = exp2f(ms - nm);
                    L = L * ca + hi_f(mv[u]) * cb;
                    o0 = o0 * ca + lo_f(pv[u]) * cb;
                    o1 = o1 * ca + hi_f(pv[u]) * cb;
                    M = nm;
                }
            }
        }
        const bool empty = !(L > 0.f);                            // every retrieved position was out of range
        const float inv = empty ? 0.f : 1.f / L;
        reinterpret_cast<float2*>(a.out + qhead0 * kHeadDim)[col] = make_float2(o0 * inv, o1 * inv);
        if (a.lse && (col % (kHeadDim / 2)) == 0) a.lse[qhead0 + g] = empty ? -INFINITY : (M + log2f(L)) * kLn2;
    }
    if (tid == 0) __hip_atomic_store(&a.counter[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
    SKV_T(9);
}

template <int G, int CHUNK>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void select_attend_stream_kernel(AttArgs a) {
    static_assert(CHUNK % kWave == 0 && CHUNK <= kStreamMaxChunk, "the row table holds kStreamMaxChunk positions");
    __shared__ StreamShared ss;
    const int bh = blockIdx.y, b = bh / a.Hkv, h = bh % a.Hkv, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    demand_args(a);
    const Seq sq = seq_of(a.v, b);
    const int32_t j0 = split * CHUNK;
    SKV_T(0);

    int32_t n;                    // retrieved tokens of this (sequence, head)
    {
        __shared__ SelectShared sel_sh;
        const int32_t budget = min(sq.budget, a.budget_cap);
        if (split > 0 && j0 >= budget) return;                    // n <= budget: nothing for this split
        stream_load_queries<G>(a, ss, (int64_t)b * (a.Hkv * G) + (int64_t)h * G);
        for (int p = tid; p < (CHUNK > kBlockThreads ? CHUNK : kBlockThreads); p += kBlockThreads)
            ss.row[p] = -1;                                       // bucket-start marks first, the rows of all positions later
        // A selected bucket that reaches into this block's positions marks, in every 64-position piece it touches,
        // where it starts there and which pool row that is; each wave then fills the positions of its own piece.
        auto mark = [&](int32_t, int32_t o, int32_t ln, int32_t, int32_t tok_pos) {
            const int32_t hi = min(tok_pos + ln, j0 + CHUNK);
            int32_t lo = max(tok_pos, j0);
            while (lo < hi) {
                ss.row[lo - j0] = o + (lo - tok_pos);
                lo = j0 + (((lo - j0) >> 6) + 1) * kWave;
            }
        };
        const float* sc = a.score + (int64_t)h * a.v.S_total + sq.sent_base;
        const int32_t* len = a.sent_len + sq.sent_base;
        const int32_t* off = a.sent_off + sq.sent_base + (a.v.cu_sent ? b : 0);
        int32_t nsel, ntok;
        if (sq.n_sent <= 2 * kBlockThreads) select_block<2, false, false>(sc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok);
        else select_block<kSelKreg, false, false>(sc, len, off, sq.n_sent, budget, sel_sh, mark, &nsel, &ntok);
        n = ntok;
        if (split == 0 && tid == 0 && a.n_tok_out) a.n_tok_out[bh] = n;
        __syncthreads();                                          // bucket starts are marked, queries are in LDS
        for (int pc = tid >> 6; pc < CHUNK / kWave; pc += kStreamWaves) {    // a wave fills 64-position pieces, in place
            const int32_t v = ss.row[pc * kWave + lane];
            // position of the last bucket start at or before this lane (-1: none): running maximum of lane + 1 over the starts
            const int32_t hp = (int32_t)wave_scan_max_u32(v >= 0 ? (uint32_t)lane + 1u : 0u) - 1;
            const int32_t base = __shfl(v, max(hp, 0));
            const int32_t xi = hp >= 0 ? base + (lane - hp) : -1;
            const int32_t pos = j0 + pc * kWave + lane;
            if (a.tok_idx_out && pos < n) a.tok_idx_out[(int64_t)bh * a.idx_stride + pos] = xi;
            ss.row[pc * kWave + lane] = (pos < n && xi >= 0 && xi < sq.n_tok_ctx) ? xi : -1;
        }
    }
    stream_attend<G, CHUNK>(a, ss, bh, b, h, split, sq, n);
}

template <int CHUNK>
static hipError_t launch_select_attend_stream_g(Ctx* c, const AttArgs& a) {
    int n_splits = (c->budget_cap + CHUNK - 1) / CHUNK;
    if (n_splits < 1) n_splits = 1;       // block 0 still writes the empty-selection result
    const dim3 grid(n_splits, a.v.B * c->d.n_kv_heads), block(kBlockThreads);
    switch (c->G) {
        case 1: hipLaunchKernelGGL((select_attend_stream_kernel<1, CHUNK>), grid, block, 0, c->stream, a); break;
        case 2: hipLaunchKernelGGL((select_attend_stream_kernel<2, CHUNK>), grid, block, 0, c->stream, a); break;
        case 4: hipLaunchKernelGGL((select_attend_stream_kernel<4, CHUNK>), grid, block, 0, c->stream, a); break;
        case 8: hipLaunchKernelGGL((select_attend_stream_kernel<8, CHUNK>), grid, block, 0, c->stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int EB, int MODE, int CHUNK>
static hipError_t launch_attend_g(Ctx* c, const AttArgs& a, int32_t n_splits) {
    const dim3 grid(n_splits, a.v.B * c->d.n_kv_heads), block(kBlockThreads);
    switch (c->G) {
        case 1: hipLaunchKernelGGL((attend_kernel<EB, 1, MODE, CHUNK>), grid, block, 0, c->stream, a); break;
        case 2: hipLaunchKernelGGL((attend_kernel<EB, 2, MODE, CHUNK>), grid, block, 0, c->stream, a); break;
        case 4: hipLaunchKernelGGL((attend_kernel<EB, 4, MODE, CHUNK>), grid, block, 0, c->stream, a); break;
        case 8: hipLaunchKernelGGL((attend_kernel<EB, 8, MODE, CHUNK>), grid, block, 0, c->stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static AttArgs att_common(Ctx* c, const void* q, const void* Kbase, const void* Vbase, const SeqView& v, float* out,
                          float* lse) {
    AttArgs a{};
    a.q = (const char*)q; a.Kb = (const char*)Kbase; a.Vb = (const char*)Vbase;
    a.v = v; a.Hkv = c->d.n_kv_heads; a.max_splits = c->max_splits;
    a.part = c->att_part; a.ml = c->att_ml; a.counter = c->att_counter; a.out = out; a.lse = lse;
    a.budget_cap = c->budget_cap;
    return a;
}

// Batches with many (sequence, head) pairs fill the GPU with 256-token blocks; below that 128-token blocks.
static bool wide_chunks(const Ctx* c, const SeqView& v) { return v.B * c->d.n_kv_heads >= kWideChunkMinHeads; }

hipError_t launch_attend(Ctx* c, const void* q, const void* K_sel, const void* V_sel, int32_t row_stride,
                         const int32_t* n_tok, int32_t budget, const SeqView& v, float* out, float* lse) {
    AttArgs a = att_common(c, q, K_sel, V_sel, v, out, lse);
    a.n_tok = n_tok; a.row_stride = row_stride;
    // Few (sequence, head) pairs: 128-token blocks.  The merging block's uncached reads of the partials cost about
    // 0.1 us per split, more than a 64-token block saves on its K/V rows (budget 2048: 11.0 us with 64-token blocks,
    // 9.2 with 128, 10.8 with 256; from a budget of 4096 on 256-token blocks are ahead).
    const bool wide = wide_chunks(c, v) || budget >= 4096;
    const int chunk = wide ? kAttChunkWide : kAttChunkMid;
    int n_splits = (budget + chunk - 1) / chunk;
    if (n_splits < 1) n_splits = 1;       // block 0 still writes the empty-selection result
    if (wide)
        return c->d.kv_dtype == SKV_BF16 ? launch_attend_g<2, kDirect, kAttChunkWide>(c, a, n_splits)
                                         : launch_attend_g<4, kDirect, kAttChunkWide>(c, a, n_splits);
    return c->d.kv_dtype == SKV_BF16 ? launch_attend_g<2, kDirect, kAttChunkMid>(c, a, n_splits)
                                     : launch_attend_g<4, kDirect, kAttChunkMid>(c, a, n_splits);
}

hipError_t launch_attend_indirect(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const int32_t* tok_idx,
                                  const int32_t* n_tok, const SeqView& v, float* out, float* lse) {
    AttArgs a = att_common(c, q, K_layer, V_layer, v, out, lse);
    a.n_tok = n_tok; a.tok_idx = tok_idx; a.idx_stride = c->d.max_budget;
    const int n_splits = (c->budget_cap + kAttChunkWide - 1) / kAttChunkWide;
    return c->d.kv_dtype == SKV_BF16 ? launch_attend_g<2, kIndirect, kAttChunkWide>(c, a, n_splits)
                                     : launch_attend_g<4, kIndirect, kAttChunkWide>(c, a, n_splits);
}

// Batch form of the fused step (bf16 pools below 2^24 tokens, addressed with 32-bit byte offsets inside a
// (head, sequence) slab): 1024-token blocks that select, then stream.
hipError_t launch_select_attend_stream(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const float* score,
                                       const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                                       float* lse, int32_t* tok_idx_out, int32_t* n_tok_out) {
    if (c->d.kv_dtype != SKV_BF16 || v.T_total >= (1 << 24)) return hipErrorInvalidValue;
    AttArgs a = att_common(c, q, K_layer, V_layer, v, out, lse);
    a.score = score; a.sent_off = sent_off; a.sent_len = sent_len;
    a.tok_idx_out = tok_idx_out; a.n_tok_out = n_tok_out; a.idx_stride = c->d.max_budget;
    // Block size by rounds of blocks (one block per compute unit).  While 512-token blocks still run in one round they
    // are ahead: two tiles per wave instead of four and twice the compute units busy (8 sequences x 8 heads, budget 2048:
    // 36.7 -> 33.0 us per layer); in two rounds they lose (16 sequences: 50.8 -> 58.1).  With several rounds of 1024-token
    // blocks, 2048-token blocks halve the selections and, up to a budget of 2048, need no merge: a round of them takes
    // about 5/3 of a 1024-token round (32 sequences: 94.7 -> 87.0 us, 64: 180.2 -> 166.3; 48: 137.8 either way).
    const int pairs = v.B * c->d.n_kv_heads;
    const int blocks = pairs * ((c->budget_cap + kStreamChunk - 1) / kStreamChunk);
    if (2 * blocks <= c->n_cu) return launch_select_attend_stream_g<kStreamChunk / 2>(c, a);
    const int big_blocks = pairs * ((c->budget_cap + kStreamMaxChunk - 1) / kStreamMaxChunk);
    const int rounds = (blocks + c->n_cu - 1) / c->n_cu, big_rounds = (big_blocks + c->n_cu - 1) / c->n_cu;
    if (5 * big_rounds < 3 * rounds) return launch_select_attend_stream_g<kStreamMaxChunk>(c, a);
    return launch_select_attend_stream_g<kStreamChunk>(c, a);
}

hipError_t launch_select_attend(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const float* score,
                                const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                                float* lse, int32_t* tok_idx_out, int32_t* n_tok_out) {
    AttArgs a = att_common(c, q, K_layer, V_layer, v, out, lse);
    a.score = score; a.sent_off = sent_off; a.sent_len = sent_len;
    a.tok_idx_out = tok_idx_out; a.n_tok_out = n_tok_out; a.idx_stride = c->d.max_budget;
    // Every split block of a head repeats the selection; with thousands of buckets per sequence that repetition
    // (bucket loads from L2, histogram passes) outweighs the shorter K/V phase of 64-token blocks.
    // bf16: one block per compute unit fits (value tiles + selection histograms in LDS), so the block size is the
    // smallest whose blocks all run at once; a second round of blocks costs more than the larger blocks' longer K/V phase
    // (4 sequences of 32K, 8 heads, budget 2048: 25.9 us in 128-token blocks, 17 in 256-token blocks).
    const int pairs = v.B * c->d.n_kv_heads;
    auto blocks = [&](int chunk) { return pairs * ((c->budget_cap + chunk - 1) / chunk); };
    if (c->d.kv_dtype == SKV_BF16 && blocks(kAttChunkMid) > c->n_cu) {
        const int n_splits = (c->budget_cap + kAttChunkWide - 1) / kAttChunkWide;
        return launch_attend_g<2, kFused, kAttChunkWide>(c, a, n_splits);
    }
    // Every split block of a head repeats the selection; with thousands of buckets per sequence that repetition
    // (bucket loads from L2, histogram passes) outweighs the shorter K/V phase of 64-token blocks.
    if (v.S_total / (v.B > 0 ? v.B : 1) > kMidChunkMinSentences || (c->d.kv_dtype == SKV_BF16 && blocks(kAttChunk) > c->n_cu)) {
        const int n_splits = (c->budget_cap + kAttChunkMid - 1) / kAttChunkMid;
        return c->d.kv_dtype == SKV_BF16 ? launch_attend_g<2, kFused, kAttChunkMid>(c, a, n_splits)
                                         : launch_attend_g<4, kFused, kAttChunkMid>(c, a, n_splits);
    }
    const int n_splits = (c->budget_cap + kAttChunk - 1) / kAttChunk;
    return c->d.kv_dtype == SKV_BF16 ? launch_attend_g<2, kFused, kAttChunk>(c, a, n_splits)
                                     : launch_attend_g<4, kFused, kAttChunk>(c, a, n_splits);
}

// Single-launch step.  Blocks per pair: the largest power of two that keeps pairs x blocks within the compute units (every
// block must be resident for the per-pair wait to end: one 1024-thread block per compute unit).  All of them score; the
// first ceil(max_budget / CHUNK) of them attend.
// Blocks of the single-launch kernel a compute unit can hold at once (registers, LDS), asked of the runtime once per
// instantiation: the kernel's waits need every block of the grid resident, so the launcher refuses grids beyond
// compute units x this number.
template <int EB, int G, int CHUNK>
static int step_blocks_per_cu() {
    static int cached = -1;
    if (cached < 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attend_kernel<EB, G, kStep, CHUNK>, kBlockThreads, 0) != hipSuccess) {
            (void)hipGetLastError();
            n = 0;
        }
        cached = n;
    }
    return cached;
}

template <int EB, int CHUNK>
static hipError_t launch_step_g(Ctx* c, const AttArgs& a, int n_blocks, bool* launched) {
    const dim3 grid(n_blocks), block(kBlockThreads);
    int per_cu = 0;
    switch (c->G) {
        case 1: per_cu = step_blocks_per_cu<EB, 1, CHUNK>(); break;
        case 2: per_cu = step_blocks_per_cu<EB, 2, CHUNK>(); break;
        case 4: per_cu = step_blocks_per_cu<EB, 4, CHUNK>(); break;
        case 8: per_cu = step_blocks_per_cu<EB, 8, CHUNK>(); break;
        default: return hipErrorInvalidValue;
    }
    if (per_cu < 1 || n_blocks > c->n_cu * per_cu) return hipSuccess;       // not every block would be resident: other forms
    *launched = true;
    switch (c->G) {
        case 1: hipLaunchKernelGGL((attend_kernel<EB, 1, kStep, CHUNK>), grid, block, 0, c->stream, a); break;
        case 2: hipLaunchKernelGGL((attend_kernel<EB, 2, kStep, CHUNK>), grid, block, 0, c->stream, a); break;
        case 4: hipLaunchKernelGGL((attend_kernel<EB, 4, kStep, CHUNK>), grid, block, 0, c->stream, a); break;
        case 8: hipLaunchKernelGGL((attend_kernel<EB, 8, kStep, CHUNK>), grid, block, 0, c->stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_step(Ctx* c, const void* q_score, const void* q_attn, const void* semvec_layer, const void* K_layer,
                       const void* V_layer, const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                       float* lse, int32_t* tok_idx_out, int32_t* n_tok_out, bool* launched) {
    *launched = false;
    const int pairs = v.B * c->d.n_kv_heads;
    const int max_blocks = c->n_cu < kStepMaxBlocks ? c->n_cu : kStepMaxBlocks;
    if (pairs < 1 || pairs > kStepMaxPairs || pairs > max_blocks || c->step_score_stride <= 0) return hipSuccess;
    if (v.S_total > c->step_score_stride || (int64_t)pairs * c->step_score_stride > c->step_score_words) return hipSuccess;
    int lg = 0;
    while ((pairs << (lg + 1)) <= max_blocks) ++lg;
    const int parts = 1 << lg;
    // attention blocks of 128 tokens, or of 256 when a pair has too few blocks for 128 (three or four sequences of 8 heads)
    int chunk = kAttChunkMid;
    if ((c->budget_cap + chunk - 1) / chunk > parts) chunk = kAttChunkWide;
    const int att_parts = (c->budget_cap + chunk - 1) / chunk;
    if (att_parts > parts || c->G > parts) return hipSuccess;                    // attention blocks or mergers do not fit
    AttArgs a = att_common(c, q_attn, K_layer, V_layer, v, out, lse);
    a.sent_off = sent_off; a.sent_len = sent_len;
    a.tok_idx_out = tok_idx_out; a.n_tok_out = n_tok_out; a.idx_stride = c->d.max_budget;
    a.q_score = (const char*)q_score; a.semvec = (const char*)semvec_layer;
    a.sv_bytes = c->d.semvec_dtype == SKV_BF16 ? kTableBf16 : c->d.semvec_dtype == SKV_FP8_E4M3 ? kTableE4m3 : kTableF32;
    a.lg_parts = lg; a.step_epoch = c->step_epoch; a.step_score = c->step_score; a.score_stride = c->step_score_stride;
    a.step_part = c->step_part; a.wait_limit = c->wait_limit;
    a.err_dev = c->err_dev; a.err_host = c->err_host_dev;
    if (chunk == kAttChunkWide)
        return c->d.kv_dtype == SKV_BF16 ? launch_step_g<2, kAttChunkWide>(c, a, pairs * parts, launched)
                                         : launch_step_g<4, kAttChunkWide>(c, a, pairs * parts, launched);
    return c->d.kv_dtype == SKV_BF16 ? launch_step_g<2, kAttChunkMid>(c, a, pairs * parts, launched)
                                     : launch_step_g<4, kAttChunkMid>(c, a, pairs * parts, launched);
}

// ------------------------------------------------------------------------------------------------
// Merge of two partial attention results over disjoint token sets (Eq. 3 over their union): the retrieved tokens and,
// for instance, a contiguous window of recent tokens attended with skv_attend.  One thread per output pair.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merge_lse_kernel(const float* __restrict__ out_a, const float* __restrict__ lse_a,
                                                        const float* __restrict__ out_b, const float* __restrict__ lse_b,
                                                        int32_t n_heads, float* __restrict__ out, float* __restrict__ lse) {
    const int32_t i = blockIdx.x * 256 + threadIdx.x;                  // pair index: head * (D / 2) + pair
    if (i >= n_heads * (kHeadDim / 2)) return;
    const int32_t j = i / (kHeadDim / 2);
    const float la = lse_a[j], lb = lse_b[j];
    const float m = fmaxf(la, lb);
    float2 r = make_float2(0.f, 0.f);
    float l = -INFINITY;
    if (m > -INFINITY) {
        const float za = expf(la - m), zb = expf(lb - m);              // an empty side has lse = -inf: weight 0
        const float inv = 1.f / (za + zb);
        const float2 a = reinterpret_cast<const float2*>(out_a)[i], b = reinterpret_cast<const float2*>(out_b)[i];
        r.x = ((za > 0.f ? za * a.x : 0.f) + (zb > 0.f ? zb * b.x : 0.f)) * inv;
        r.y = ((za > 0.f ? za * a.y : 0.f) + (zb > 0.f ? zb * b.y : 0.f)) * inv;
        l = m + logf(za + zb);
    }
    reinterpret_cast<float2*>(out)[i] = r;
    if (lse && (i % (kHeadDim / 2)) == 0) lse[j] = l;
}

hipError_t launch_merge_lse(Ctx* c, const float* out_a, const float* lse_a, const float* out_b, const float* lse_b,
                            int32_t n_heads, float* out, float* lse) {
    const int n = n_heads * (kHeadDim / 2);
    hipLaunchKernelGGL(merge_lse_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, out_a, lse_a, out_b, lse_b, n_heads, out,
                       lse);
    return hipGetLastError();
}

}  // namespace skv
