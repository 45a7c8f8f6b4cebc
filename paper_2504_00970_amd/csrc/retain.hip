// Prefill-side token retention (Sec. 4.1 "Token importance measurement", "Token selection within sentence
// buckets"; App. "Effect of Sentence Length"; Alg. 1 prefilling phase): observation-window importance on the
// matrix cores, global top-k of the importance, buckets of the retained tokens, compaction of the K/V pool.
// gfx950, wave64, bf16 and fp32 inputs.
#include "skv_internal.h"
#include "skv_device.h"

namespace skv {

// ------------------------------------------------------------------------------------------------
// Importance.  For one layer and KV head h the window's R = G*N query rows (row = g*N + n: query head
// h*G+g, window token n, contiguous in q_obs) meet all T keys: S^T = K Q^T / sqrt(D) on
// v_mfma_f32_16x16x32_bf16, keys as A fragments straight from 16-byte row loads (lane (t, qd): key t of
// the tile, dims 32s+8qd..+7), query rows as B fragments from an LDS copy.  fp32 inputs are split
// exactly into three bf16 terms -- see Frag -- so that the products keep fp32 accuracy.
//   pass 1 (stats):   per row, max and sum of exp2 over the keys visible to it (positions <= Tp + n), per block
//                     of kKeysPerBlock keys; the partials are combined per row by importance_combine_kernel;
//   pass 2 (colsum):  per KV head, the column sums of exp2(s - m_row) / l_row over the head's rows, for the Tp
//                     prefix keys; importance_sum_heads_kernel adds the heads in ascending order (deterministic).
// A wave owns 16*KT keys per sweep and walks the row tiles; a block makes kImpSubs sweeps, the next sweep's key
// fragments being requested before the current sweep is computed (bf16: two register buffers of 32 VGPRs).
// Each pass covers all layers in one launch (grid z = layer).
// ------------------------------------------------------------------------------------------------
constexpr int kImpThreads = 256;
constexpr int kImpWaves = kImpThreads / kWave;
constexpr int kImpSubs = 4;                                    // sweeps of a block
template <int EB> struct Imp {
    static constexpr int KT = EB == 2 ? 2 : 1;                 // 16-key tiles per wave and sweep
    static constexpr int NB = EB == 2 ? 2 : 1;                 // register buffers of key fragments
    static constexpr int kKeysPerWave = 16 * KT;
    static constexpr int kKeysPerSub = kImpWaves * kKeysPerWave;
    static constexpr int kKeysPerBlock = kKeysPerSub * kImpSubs;
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma_bf16(const uint4& a, const uint4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// 2^x for x <= 0 (a probability): the bare instruction; results below the normal range flush to zero
__device__ __forceinline__ float exp2_neg(float x) { return __builtin_amdgcn_exp2f(x); }

// 8 consecutive elements of a row as bf16 fragments.  bf16 storage: one 16-byte load.  fp32 storage: each value
// is split exactly into three bf16 terms by truncation (8 + 8 + 8 mantissa bits: x = a + b + c), and x*y is evaluated
// as aa' + ab' + ba' + ac' + bb' + ca' by six MFMAs; the dropped terms are below 2^-23 of the product.
template <int EB> struct Frag;
template <> struct Frag<2> {
    uint4 t0;
    __device__ __forceinline__ void load(const char* row, int elem) { t0 = *reinterpret_cast<const uint4*>(row + elem * 2); }
};
template <> struct Frag<4> {
    uint4 t0, t1, t2;
    __device__ __forceinline__ void load(const char* row, int elem) {
        const uint4 lo4 = *reinterpret_cast<const uint4*>(row + elem * 4);
        const uint4 hi4 = *reinterpret_cast<const uint4*>(row + elem * 4 + 16);
        const uint32_t x[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        uint32_t a[8], b[8], c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = x[i] & 0xffff0000u;
            const float r1 = __uint_as_float(x[i]) - __uint_as_float(a[i]);          // exact
            b[i] = __float_as_uint(r1) & 0xffff0000u;
            const float r2 = r1 - __uint_as_float(b[i]);                             // exact, at most 8 significant bits
            c[i] = __float_as_uint(r2) & 0xffff0000u;
        }
        t0 = make_uint4((a[0] >> 16) | a[1], (a[2] >> 16) | a[3], (a[4] >> 16) | a[5], (a[6] >> 16) | a[7]);
        t1 = make_uint4((b[0] >> 16) | b[1], (b[2] >> 16) | b[3], (b[4] >> 16) | b[5], (b[6] >> 16) | b[7]);
        t2 = make_uint4((c[0] >> 16) | c[1], (c[2] >> 16) | c[3], (c[4] >> 16) | c[5], (c[6] >> 16) | c[7]);
    }
};

template <int EB>
__device__ __forceinline__ f32x4 frag_mma(const Frag<EB>& k, const Frag<EB>& q, f32x4 c) {
    if constexpr (EB == 4) {                                  // small terms first
        c = mfma_bf16(k.t2, q.t0, c);
        c = mfma_bf16(k.t1, q.t1, c);
        c = mfma_bf16(k.t0, q.t2, c);
        c = mfma_bf16(k.t1, q.t0, c);
        c = mfma_bf16(k.t0, q.t1, c);
    }
    return mfma_bf16(k.t0, q.t0, c);
}

// Query rows of KV head h -> LDS as fragments' source (rows >= R are zero).  Row pitch padded by 16 bytes.
// All loads are issued before the first LDS write, on clamped addresses (a predicated load in a loop costs one
// full memory latency per iteration).
template <int EB, int ROWS>
__device__ __forceinline__ void stage_queries(const char* __restrict__ q_head /* [R][D] */, int R, char* sm_q) {
    constexpr int kRowBytes = kHeadDim * EB, kPitch = kRowBytes + 16, kPieces = kRowBytes / 16;
    constexpr int kIter = (ROWS * kPieces + kImpThreads - 1) / kImpThreads;
    uint4 t[kIter];
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
        const int i = threadIdx.x + it * kImpThreads, row = i / kPieces, piece = i % kPieces;
        t[it] = *reinterpret_cast<const uint4*>(q_head + (int64_t)min(row, R - 1) * kRowBytes + piece * 16);
    }
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
        const int i = threadIdx.x + it * kImpThreads, row = i / kPieces, piece = i % kPieces;
        if (i < ROWS * kPieces) *reinterpret_cast<uint4*>(sm_q + row * kPitch + piece * 16) = row < R ? t[it] : make_uint4(0, 0, 0, 0);
    }
}

// Key fragments of one sweep of a wave: keys key0 + 16 kt + t16 (clamped to the last valid row: never out of bounds).
template <int EB>
__device__ __forceinline__ void load_keys(Frag<EB> (&kf)[Imp<EB>::KT][4], const char* Kh, int32_t key0, int32_t last, int t16, int qd) {
#pragma unroll
    for (int kt = 0; kt < Imp<EB>::KT; ++kt) {
        const char* row = Kh + (int64_t)min(key0 + 16 * kt + t16, last) * (kHeadDim * EB);
#pragma unroll
        for (int s = 0; s < 4; ++s) kf[kt][s].load(row, 32 * s + 8 * qd);
    }
}

// pass 1.  grid (ceil(T / Imp<EB>::kKeysPerBlock), Hkv, L); part [L][Hkv][chunks][RT*16][2] = (max in log2 units, sum).
template <int EB, int RT>
__global__ __launch_bounds__(kImpThreads) void importance_stats_kernel(const char* __restrict__ q_obs, const char* __restrict__ K_pool,
                                                                     int32_t T, int32_t N, int32_t G, float* __restrict__ part) {
    constexpr int kRowBytes = kHeadDim * EB, kPitch = kRowBytes + 16;
    constexpr int kRows = RT * 16;
    constexpr int KT = Imp<EB>::KT, NB = Imp<EB>::NB;
    constexpr float kLog2e = 1.4426950408889634f;
    extern __shared__ __attribute__((aligned(16))) char sm_dyn[];
    char* sm_q = sm_dyn;                                              // [kRows][kPitch]
    __shared__ float sm_m[kImpWaves][kRows], sm_l[kImpWaves][kRows];

    const int h = blockIdx.y, chunk = blockIdx.x, nchunks = gridDim.x;
    const int64_t lh = (int64_t)blockIdx.z * gridDim.y + h;              // (layer, KV head)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t16 = lane & 15, qd = lane >> 4;
    const int R = G * N, Tp = T - N;
    const char* Kh = K_pool + lh * T * kRowBytes;
    const char* q_layer = q_obs + (int64_t)blockIdx.z * gridDim.y * R * kRowBytes;
    const int32_t wave_key0 = chunk * Imp<EB>::kKeysPerBlock + Imp<EB>::kKeysPerWave * w;
    Frag<EB> kf[NB][KT][4];
    if (NB == 2) load_keys<EB>(kf[0], Kh, wave_key0, T - 1, t16, qd);
    stage_queries<EB, kRows>(q_layer + (int64_t)h * R * kRowBytes, R, sm_q);
    const float scale = kLog2e * rsqrtf((float)kHeadDim);

    // Running statistics are kept per LANE (a lane sees the keys 4qd..4qd+3 of every tile of its row), in raw logit
    // units for the max: the four lanes of a row meet only once, after the last sweep.
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) { m_run[rt] = -INFINITY; l_run[rt] = 0.f; }
    __syncthreads();

#pragma unroll
    for (int sub = 0; sub < kImpSubs; ++sub) {
        const int32_t key0 = wave_key0 + sub * Imp<EB>::kKeysPerSub;
        const int cur = NB == 2 ? (sub & 1) : 0;
        if (NB == 2) { if (sub + 1 < kImpSubs) load_keys<EB>(kf[cur ^ 1], Kh, key0 + Imp<EB>::kKeysPerSub, T - 1, t16, qd); }
        else load_keys<EB>(kf[0], Kh, key0, T - 1, t16, qd);
        if (key0 >= T) continue;                                      // wave-uniform: nothing of this sweep exists
        const bool open = key0 + Imp<EB>::kKeysPerWave <= Tp;         // wave-uniform: every key visible to every row
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            Frag<EB> qf[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) qf[s].load(sm_q + (16 * rt + t16) * kPitch, 32 * s + 8 * qd);
            float sv[KT][4];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) acc = frag_mma<EB>(kf[cur][kt][s], qf[s], acc);
#pragma unroll
                for (int j = 0; j < 4; ++j) sv[kt][j] = acc[j];
            }
            if (!open) {                                              // the sweep touches the window or the end of the prompt
                const int32_t limit = min(Tp + (16 * rt + t16) % N, T - 1);   // last position visible to this lane's row
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (key0 + 16 * kt + 4 * qd + j > limit) sv[kt][j] = -INFINITY;
            }
            float mt = m_run[rt];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) mt = fmaxf(mt, sv[kt][j]);
            if (open || mt > -INFINITY) {                             // per-lane code only: divergence is harmless
                const float ms = mt * scale;
                float sum = 0.f;
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) sum += exp2_neg(sv[kt][j] * scale - ms);     // exp2(-inf) = 0
                l_run[rt] = l_run[rt] * exp2_neg(m_run[rt] * scale - ms) + sum;
                m_run[rt] = mt;
            }
        }
    }
    // the four lanes of a row (qd = 0..3), then the block's waves
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float m = m_run[rt];
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        float l = m_run[rt] > -INFINITY ? l_run[rt] * exp2_neg((m_run[rt] - m) * scale) : 0.f;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (qd == 0) { sm_m[w][16 * rt + t16] = m * scale; sm_l[w][16 * rt + t16] = l; }
    }
    __syncthreads();
    for (int row = tid; row < kRows; row += kImpThreads) {
        float m = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < kImpWaves; ++ww) m = fmaxf(m, sm_m[ww][row]);
        float l = 0.f;
#pragma unroll
        for (int ww = 0; ww < kImpWaves; ++ww)
            if (sm_m[ww][row] > -INFINITY) l += sm_l[ww][row] * exp2_neg(sm_m[ww][row] - m);
        float* dst = part + ((lh * nchunks + chunk) * kRows + row) * 2;
        dst[0] = m;
        dst[1] = l;
    }
}

// Combines the per-chunk partials: rowstat [L * Hkv][rows][2] = (max, 1 / sum).  One wave per row, the chunks
// spread over its lanes.  grid (ceil(L * Hkv * rows / 4)); `Hkv` below counts (layer, head) pairs.
__global__ __launch_bounds__(kImpThreads) void importance_combine_kernel(const float* __restrict__ part, int32_t nchunks, int32_t rows,
                                                                       int32_t Hkv, float* __restrict__ rowstat) {
    const int lane = threadIdx.x & 63;
    const int item = blockIdx.x * kImpWaves + (threadIdx.x >> 6);     // (head, row)
    if (item >= Hkv * rows) return;
    const int h = item / rows, row = item % rows;
    float M = -INFINITY, L = 0.f;
    for (int c = lane; c < nchunks; c += kWave) {
        const float2 p = *reinterpret_cast<const float2*>(part + (((int64_t)h * nchunks + c) * rows + row) * 2);
        if (p.x > -INFINITY) {
            const float nm = fmaxf(M, p.x);
            L = L * exp2_neg(M - nm) + p.y * exp2_neg(p.x - nm);
            M = nm;
        }
    }
    float Mw = M;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) Mw = fmaxf(Mw, __shfl_xor(Mw, o));
    float Lw = M > -INFINITY ? L * exp2_neg(M - Mw) : 0.f;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) Lw += __shfl_xor(Lw, o);
    if (lane == 0) {
        float* dst = rowstat + ((int64_t)h * rows + row) * 2;
        dst[0] = Mw;
        dst[1] = Lw > 0.f ? 1.f / Lw : 0.f;
    }
}

// pass 2.  grid (ceil(Tp / Imp<EB>::kKeysPerBlock), Hkv, L); alpha_h [L][Hkv][Tp].
template <int EB, int RT>
__global__ __launch_bounds__(kImpThreads) void importance_colsum_kernel(const char* __restrict__ q_obs, const char* __restrict__ K_pool,
                                                                      int32_t T, int32_t N, int32_t G,
                                                                      const float* __restrict__ rowstat, float* __restrict__ alpha_h) {
    constexpr int kRowBytes = kHeadDim * EB, kPitch = kRowBytes + 16;
    constexpr int kRows = RT * 16;
    constexpr int KT = Imp<EB>::KT, NB = Imp<EB>::NB;
    constexpr float kLog2e = 1.4426950408889634f;
    extern __shared__ __attribute__((aligned(16))) char sm_dyn[];
    char* sm_q = sm_dyn;
    __shared__ float2 sm_stat[kRows];

    const int h = blockIdx.y;
    const int64_t lh = (int64_t)blockIdx.z * gridDim.y + h;              // (layer, KV head)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t16 = lane & 15, qd = lane >> 4;
    const int R = G * N, Tp = T - N;
    const char* Kh = K_pool + lh * T * kRowBytes;
    const char* q_layer = q_obs + (int64_t)blockIdx.z * gridDim.y * R * kRowBytes;
    const int32_t wave_key0 = blockIdx.x * Imp<EB>::kKeysPerBlock + Imp<EB>::kKeysPerWave * w;
    Frag<EB> kf[NB][KT][4];
    if (NB == 2) load_keys<EB>(kf[0], Kh, wave_key0, Tp - 1, t16, qd);
    stage_queries<EB, kRows>(q_layer + (int64_t)h * R * kRowBytes, R, sm_q);
    for (int row = tid; row < kRows; row += kImpThreads)       // rows >= R: 1 / sum = 0, so they add nothing
        sm_stat[row] = row < R ? *reinterpret_cast<const float2*>(rowstat + (lh * kRows + row) * 2) : make_float2(0.f, 0.f);
    const float scale = kLog2e * rsqrtf((float)kHeadDim);
    __syncthreads();

#pragma unroll
    for (int sub = 0; sub < kImpSubs; ++sub) {
        const int32_t key0 = wave_key0 + sub * Imp<EB>::kKeysPerSub;
        const int cur = NB == 2 ? (sub & 1) : 0;
        if (NB == 2) { if (sub + 1 < kImpSubs) load_keys<EB>(kf[cur ^ 1], Kh, key0 + Imp<EB>::kKeysPerSub, Tp - 1, t16, qd); }
        else load_keys<EB>(kf[0], Kh, key0, Tp - 1, t16, qd);
        if (key0 >= Tp) continue;                                     // wave-uniform
        float ps[KT][4];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) ps[kt][j] = 0.f;
#pragma unroll 2
        for (int rt = 0; rt < RT; ++rt) {
            Frag<EB> qf[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) qf[s].load(sm_q + (16 * rt + t16) * kPitch, 32 * s + 8 * qd);
            const float2 st = sm_stat[16 * rt + t16];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) acc = frag_mma<EB>(kf[cur][kt][s], qf[s], acc);
#pragma unroll
                for (int j = 0; j < 4; ++j) ps[kt][j] += exp2_neg(acc[j] * scale - st.x) * st.y;   // prefix keys: s <= row max
            }
        }
        // sum over the 16 rows of the tile layout (the lanes of a DPP row); lane t16 == 0 stores its four keys
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = ps[kt][j];
                v = dpp_add<0xB1>(v);
                v = dpp_add<0x4E>(v);
                v = dpp_add<0x124>(v);
                v = dpp_add<0x128>(v);
                const int32_t key = key0 + 16 * kt + 4 * qd + j;
                if (t16 == 0 && key < Tp) alpha_h[lh * Tp + key] = v;
            }
    }
}

// alpha[l][i] = sum over the KV heads, in ascending order, of alpha_h[l][h][i].  grid (ceil(Tp / 256), L).
__global__ __launch_bounds__(kImpThreads) void importance_sum_heads_kernel(const float* __restrict__ alpha_h, int32_t Tp, int32_t Hkv,
                                                                         float* __restrict__ alpha) {
    const int32_t i = blockIdx.x * kImpThreads + threadIdx.x;
    const int64_t l = blockIdx.y;
    if (i >= Tp) return;
    float v = 0.f;
    for (int h = 0; h < Hkv; ++h) v += alpha_h[(l * Hkv + h) * Tp + i];
    alpha[l * Tp + i] = v;
}

template <int EB, int RT>
static hipError_t launch_importance_rt(Ctx* c, const char* q_obs, const char* K_pool, int32_t T, int32_t N, float* alpha, float* part,
                                       float* rowstat, float* alpha_h) {
    const int Hkv = c->d.n_kv_heads, L = c->d.n_layers, G = c->G, rows = RT * 16;
    const int nchunks = (T + Imp<EB>::kKeysPerBlock - 1) / Imp<EB>::kKeysPerBlock;
    const size_t lds = (size_t)rows * (kHeadDim * EB + 16);
    static bool raised = false;                                        // dynamic LDS above 64 KB needs the opt-in once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&importance_stats_kernel<EB, RT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&importance_colsum_kernel<EB, RT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int Tp = T - N;
    hipLaunchKernelGGL((importance_stats_kernel<EB, RT>), dim3(nchunks, Hkv, L), dim3(kImpThreads), lds, c->stream, q_obs, K_pool, T, N, G,
                       part);
    hipLaunchKernelGGL(importance_combine_kernel, dim3((L * Hkv * rows + kImpWaves - 1) / kImpWaves), dim3(kImpThreads), 0, c->stream,
                       part, nchunks, rows, L * Hkv, rowstat);
    hipLaunchKernelGGL((importance_colsum_kernel<EB, RT>), dim3((Tp + Imp<EB>::kKeysPerBlock - 1) / Imp<EB>::kKeysPerBlock, Hkv, L),
                       dim3(kImpThreads), lds, c->stream, q_obs, K_pool, T, N, G, rowstat, alpha_h);
    hipLaunchKernelGGL(importance_sum_heads_kernel, dim3((Tp + kImpThreads - 1) / kImpThreads, L), dim3(kImpThreads), 0, c->stream,
                       alpha_h, Tp, Hkv, alpha);
    return hipGetLastError();
}

template <int EB>
static hipError_t launch_importance_eb(Ctx* c, const char* q_obs, const char* K_pool, int32_t T, int32_t N, float* alpha, float* part,
                                       float* rowstat, float* alpha_h) {
    const int R = c->G * N;
    if (R <= 32) return launch_importance_rt<EB, 2>(c, q_obs, K_pool, T, N, alpha, part, rowstat, alpha_h);
    if (R <= 64) return launch_importance_rt<EB, 4>(c, q_obs, K_pool, T, N, alpha, part, rowstat, alpha_h);
    if (R <= 128) return launch_importance_rt<EB, 8>(c, q_obs, K_pool, T, N, alpha, part, rowstat, alpha_h);
    if (R <= 256) return launch_importance_rt<EB, 16>(c, q_obs, K_pool, T, N, alpha, part, rowstat, alpha_h);
    return hipErrorInvalidValue;
}

static int importance_rows(int rows) { return (rows <= 32 ? 2 : rows <= 64 ? 4 : rows <= 128 ? 8 : 16) * 16; }

static int64_t importance_chunks(const Ctx* c, int32_t T) {
    const int per = c->d.kv_dtype == SKV_BF16 ? Imp<2>::kKeysPerBlock : Imp<4>::kKeysPerBlock;
    return (T + per - 1) / per;
}

// work = part [L][Hkv][chunks][rows][2] | rowstat [L][Hkv][rows][2] | alpha_h [L][Hkv][Tp], floats
int64_t importance_work_bytes(const Ctx* c, int32_t T, int32_t N) {
    const int64_t rows = importance_rows(c->G * N), LH = (int64_t)c->d.n_layers * c->d.n_kv_heads;
    return (LH * importance_chunks(c, T) * rows * 2 + LH * rows * 2 + LH * (int64_t)(T - N)) * (int64_t)sizeof(float);
}

// Four launches cover all layers: statistics, their combination, column sums per head, the ordered sum over heads.
hipError_t launch_importance(Ctx* c, const void* q_obs, const void* K_pool, int32_t T, int32_t N, float* alpha, void* work) {
    const int64_t rows = importance_rows(c->G * N), LH = (int64_t)c->d.n_layers * c->d.n_kv_heads;
    float* part = (float*)work;
    float* rowstat = part + LH * importance_chunks(c, T) * rows * 2;
    float* alpha_h = rowstat + LH * rows * 2;
    return c->d.kv_dtype == SKV_BF16
               ? launch_importance_eb<2>(c, (const char*)q_obs, (const char*)K_pool, T, N, alpha, part, rowstat, alpha_h)
               : launch_importance_eb<4>(c, (const char*)q_obs, (const char*)K_pool, T, N, alpha, part, rowstat, alpha_h);
}

// ------------------------------------------------------------------------------------------------
// Retention.  One 1024-thread block per layer: radix select (11 + 11 + 10 bits of the order-preserving
// key) of the k-th largest importance, tokens with equal importance by lower position, compaction of
// the kept positions in ascending order, then the retained buckets: kept tokens of one bucket are
// consecutive in keep_idx (positions ascend, bucket ids do not decrease), so ret_off[s] is the index of
// the first kept token whose bucket id is >= s.
// ------------------------------------------------------------------------------------------------
struct RetainShared {
    uint32_t hist[2048];
    uint32_t wave_tot[8][kBlockWaves];
    int32_t res[3][4];
};

__global__ __launch_bounds__(kBlockThreads) void retain_kernel(const float* __restrict__ alpha_all, int32_t Tp, int32_t k,
                                                               const int32_t* __restrict__ seg_id, int32_t S,
                                                               int32_t* __restrict__ keep_all, int32_t keep_stride,
                                                               int32_t* __restrict__ n_keep, int32_t* __restrict__ ret_off_all,
                                                               int32_t* __restrict__ ret_len_all) {
    __shared__ RetainShared sh;
    const int l = blockIdx.x, tid = threadIdx.x;
    const float* alpha = alpha_all + (int64_t)l * Tp;
    int32_t* keep = keep_all + (int64_t)l * keep_stride;
    int32_t* ret_off = ret_off_all + (int64_t)l * (S + 1);
    int32_t* ret_len = ret_len_all + (int64_t)l * S;
    const int32_t need = max(min(k, Tp), 0);
    if (tid == 0) n_keep[l] = need;
    if (need == 0) {
        for (int s = tid; s <= S; s += kBlockThreads) ret_off[s] = 0;
        for (int s = tid; s < S; s += kBlockThreads) ret_len[s] = 0;
        return;
    }
    const int kpt = (Tp + kBlockThreads - 1) / kBlockThreads;
    const int32_t i0 = tid * kpt, i1 = min(i0 + kpt, Tp);

    // Up to kRetainKreg tokens per thread (prompts up to 32K) keep their keys in registers: one batch of loads on
    // clamped addresses instead of a dependent load per token in each of the six sweeps below.
    constexpr int kRetainKreg = 32;
    const bool in_regs = kpt <= kRetainKreg;                           // block-uniform
    uint32_t rk[kRetainKreg];
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kRetainKreg; ++j) rk[j] = __float_as_uint(alpha[min(i0 + j, Tp - 1)]);
#pragma unroll
        for (int j = 0; j < kRetainKreg; ++j) rk[j] = score_key(__uint_as_float(rk[j]));
    }
    // fn(i, key) for every token the thread owns, in position order
    auto for_keys = [&](auto&& fn) {
        if (in_regs) {
#pragma unroll
            for (int j = 0; j < kRetainKreg; ++j)
                if (i0 + j < i1) fn(i0 + j, rk[j]);
        } else {
            for (int32_t i = i0; i < i1; ++i) fn(i, score_key(alpha[i]));
        }
    };

    // ---- key of the need-th largest importance ---------------------------------------------------------
    uint32_t prefix = 0;
    int shift = 32;
    uint32_t above = 0;                                                // tokens ranked strictly above the current digit range
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int bits = pass < 2 ? 11 : 10, nbins = 1 << bits, nshift = shift - bits;
        for (int i = tid; i < 2048; i += kBlockThreads) sh.hist[i] = 0;
        if (tid == 0) sh.res[pass][0] = -1;
        __syncthreads();
        for_keys([&](int32_t, uint32_t key) {
            if (pass == 0 || (key >> shift) == prefix) atomicAdd(&sh.hist[(key >> nshift) & (nbins - 1)], 1u);
        });
        __syncthreads();
        // thread order == descending digit order: thread t owns digits nbins-1-2t and nbins-2-2t
        const int d1 = nbins - 1 - 2 * tid;
        const uint32_t c1 = d1 >= 0 ? sh.hist[d1] : 0u, c0 = d1 >= 1 ? sh.hist[d1 - 1] : 0u;
        uint32_t total;
        const uint32_t incl = block_scan_u32(c1 + c0, sh.wave_tot[pass], &total);
        const uint32_t above1 = above + incl - c1 - c0, above0 = above1 + c1;
        if (c1 > 0 && above1 < (uint32_t)need && above1 + c1 >= (uint32_t)need) { sh.res[pass][0] = d1; sh.res[pass][1] = (int32_t)above1; }
        if (c0 > 0 && above0 < (uint32_t)need && above0 + c0 >= (uint32_t)need) { sh.res[pass][0] = d1 - 1; sh.res[pass][1] = (int32_t)above0; }
        __syncthreads();
        const int digit = sh.res[pass][0];                             // always found: need <= Tp
        prefix = (pass == 0) ? (uint32_t)digit : ((prefix << bits) | (uint32_t)digit);
        above = (uint32_t)sh.res[pass][1];
        shift = nshift;
    }
    // prefix is the full key of the cut; `above` tokens have a larger key; need - above of the equal ones are kept
    const uint32_t take_equal = (uint32_t)need - above;

    // ---- compaction in position order ------------------------------------------------------------------
    uint32_t my_eq = 0;
    for_keys([&](int32_t, uint32_t key) { my_eq += key == prefix ? 1u : 0u; });
    uint32_t tot;
    uint32_t eq_before = block_scan_u32(my_eq, sh.wave_tot[3], &tot) - my_eq;
    uint32_t my_cnt = 0;
    {
        uint32_t e = eq_before;
        for_keys([&](int32_t, uint32_t key) {
            if (key > prefix) my_cnt += 1;
            else if (key == prefix) { if (e < take_equal) my_cnt += 1; e += 1; }
        });
    }
    uint32_t pos = block_scan_u32(my_cnt, sh.wave_tot[4], &tot) - my_cnt;
    {
        uint32_t e = eq_before;
        for_keys([&](int32_t i, uint32_t key) {
            bool kept = key > prefix;
            if (key == prefix) { kept = e < take_equal; e += 1; }
            if (kept) keep[pos++] = i;
        });
    }
    __syncthreads();                                                   // keep[0 .. need) is written (block-visible)

    // ---- buckets of the retained tokens ------------------------------------------------------------------
    for (int32_t j = tid; j < need; j += kBlockThreads) {
        const int32_t s_cur = min(max(seg_id[keep[j]], 0), S - 1);
        const int32_t s_prev = j > 0 ? min(max(seg_id[keep[j - 1]], 0), S - 1) : -1;
        for (int32_t s = s_prev + 1; s <= s_cur; ++s) ret_off[s] = j;
        if (j == need - 1)
            for (int32_t s = s_cur + 1; s <= S; ++s) ret_off[s] = need;
    }
    __syncthreads();
    for (int s = tid; s < S; s += kBlockThreads) ret_len[s] = ret_off[s + 1] - ret_off[s];
}

hipError_t launch_retain(Ctx* c, const float* alpha, int32_t Tp, int32_t k, const int32_t* seg_id, int32_t S, int32_t* keep_idx,
                         int32_t* n_keep, int32_t* ret_off, int32_t* ret_len) {
    hipLaunchKernelGGL(retain_kernel, dim3(c->d.n_layers), dim3(kBlockThreads), 0, c->stream, alpha, Tp, k, seg_id, S, keep_idx,
                       max(k, 1), n_keep, ret_off, ret_len);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Pool compaction: K_ret/V_ret [L][Hkv][k][D] = rows keep_idx[l][0 .. n_keep[l]) of K/V [L][Hkv][T][D].
// Same branch-free copy as the decode-side gather; the kept positions are shared by the heads of a layer.
// ------------------------------------------------------------------------------------------------
template <int EB>
__global__ __launch_bounds__(kGatherThreads) void compact_pool_kernel(const char* __restrict__ Kp, const char* __restrict__ Vp, int32_t T,
                                                                     const int32_t* __restrict__ keep_all, int32_t k,
                                                                     const int32_t* __restrict__ n_keep, int32_t Hkv,
                                                                     char* __restrict__ Kr, char* __restrict__ Vr) {
    using R = Row<EB>;
    constexpr int kRowsPerIter = kGatherThreads / R::LPR;
    constexpr int kIter = kGatherRowsPerBlock / kRowsPerIter;
    constexpr int kRowBytes = kHeadDim * EB;
    const int lh = blockIdx.y, l = lh / Hkv;
    const int32_t n = min(n_keep[l], k);
    const int32_t j0 = blockIdx.x * kGatherRowsPerBlock;
    if (j0 >= n || T <= 0) return;
    const char* src = (blockIdx.z == 0 ? Kp : Vp) + (int64_t)lh * T * kRowBytes;
    char* dst = (blockIdx.z == 0 ? Kr : Vr) + (int64_t)lh * k * kRowBytes;
    const int32_t* keep = keep_all + (int64_t)l * k;
    const int r = threadIdx.x / R::LPR, cc = threadIdx.x % R::LPR;
    int32_t x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) x[i] = keep[min(j0 + i * kRowsPerIter + r, n - 1)];
    uint4 val[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i)
        val[i] = *reinterpret_cast<const uint4*>(src + (int64_t)min(max(x[i], 0), T - 1) * kRowBytes + cc * 16);
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t j = j0 + i * kRowsPerIter + r;
        if (j < n && x[i] >= 0 && x[i] < T) *reinterpret_cast<uint4*>(dst + (int64_t)j * kRowBytes + cc * 16) = val[i];
    }
}

hipError_t launch_compact_pool(Ctx* c, const void* K_pool, const void* V_pool, int32_t T, const int32_t* keep_idx, int32_t k,
                               const int32_t* n_keep, void* K_ret, void* V_ret) {
    if (k == 0) return hipSuccess;
    const dim3 grid((k + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock, c->d.n_layers * c->d.n_kv_heads, 2), block(kGatherThreads);
    if (c->d.kv_dtype == SKV_BF16)
        hipLaunchKernelGGL(compact_pool_kernel<2>, grid, block, 0, c->stream, (const char*)K_pool, (const char*)V_pool, T, keep_idx, k,
                           n_keep, c->d.n_kv_heads, (char*)K_ret, (char*)V_ret);
    else
        hipLaunchKernelGGL(compact_pool_kernel<4>, grid, block, 0, c->stream, (const char*)K_pool, (const char*)V_pool, T, keep_idx, k,
                           n_keep, c->d.n_kv_heads, (char*)K_ret, (char*)V_ret);
    return hipGetLastError();
}

}  // namespace skv
