// Decode-step kernels (Sec. 4.2, Eq. 3, Alg. 1 decoding phase): bucket scores, ranking + budgeted
// retrieval, K/V row gather, split-K attention with an online-softmax combine.  gfx950, wave64.
#include "skv_internal.h"

namespace skv {

// Per-sequence slice of a ragged batch.
struct Seq {
    int32_t tok_base, n_tok_ctx;     // first pool row and number of tokens of the sequence
    int32_t sent_base, n_sent;       // first bucket and number of buckets
    int32_t budget;
};

__device__ __forceinline__ Seq seq_of(const SeqView& v, int b) {
    Seq s;
    if (v.cu_sent) {
        s.sent_base = v.cu_sent[b];
        s.n_sent = v.cu_sent[b + 1] - s.sent_base;
    } else {
        s.sent_base = 0;
        s.n_sent = v.S_total;
    }
    if (v.cu_tok) {
        s.tok_base = v.cu_tok[b];
        s.n_tok_ctx = v.cu_tok[b + 1] - s.tok_base;
    } else {
        s.tok_base = 0;
        s.n_tok_ctx = v.T_total;
    }
    s.budget = v.budget_arr ? v.budget_arr[b] : v.budget;
    return s;
}

// ------------------------------------------------------------------------------------------------
// Scores.  score[h][s] = sum_g q[hG+g] . semvec[h][s]  =  (sum_g q[hG+g]) . semvec[h][s].
// A semantic vector is 512 bytes = 32 lanes x float4; a wave covers 2 buckets per load instruction
// and keeps kScoreRowsPerWave / 2 loads in flight.  The group-summed query lives in registers.
// Blocks are aligned to sequences: block x -> (sequence b, local block) by walking cu_sent.
// ------------------------------------------------------------------------------------------------
template <int EB, int G>
__global__ __launch_bounds__(kScoreWavesPerBlock * kWave) void score_kernel(const char* __restrict__ q,
                                                                            const float* __restrict__ semvec, SeqView v,
                                                                            int32_t Hq, float* __restrict__ score) {
    int blk = blockIdx.x, b = 0;
    Seq sq{};
    for (; b < v.B; ++b) {
        sq = seq_of(v, b);
        const int nb = (sq.n_sent + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock;
        if (blk < nb) break;
        blk -= nb;
    }
    if (b >= v.B) return;
    const int h = blockIdx.y;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c = lane & 31, half = lane >> 5;

    float qs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const char* qrow = q + ((int64_t)(b * Hq + h * G + g) * kHeadDim + c * 4) * EB;
        if (EB == 4) {
            const float4 t = *reinterpret_cast<const float4*>(qrow);
            qs[0] += t.x; qs[1] += t.y; qs[2] += t.z; qs[3] += t.w;
        } else {
            const uint2 t = *reinterpret_cast<const uint2*>(qrow);
            qs[0] += __uint_as_float(t.x << 16); qs[1] += __uint_as_float(t.x & 0xffff0000u);
            qs[2] += __uint_as_float(t.y << 16); qs[3] += __uint_as_float(t.y & 0xffff0000u);
        }
    }

    constexpr int kIter = kScoreRowsPerWave / 2;
    const int32_t row0 = blk * kScoreRowsPerBlock + w * kScoreRowsPerWave + half;
    const float* base = semvec + ((int64_t)h * v.S_total + sq.sent_base) * kHeadDim + c * 4;
    // Addresses are clamped into the sequence instead of predicating the loads, so that all of a
    // lane's loads are issued back to back; rows past the end are computed and dropped.
    float4 x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int32_t s = min(row0 + 2 * i, sq.n_sent - 1);
        x[i] = *reinterpret_cast<const float4*>(base + (int64_t)s * kHeadDim);
    }
    float p[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) p[i] = x[i].x * qs[0] + x[i].y * qs[1] + x[i].z * qs[2] + x[i].w * qs[3];
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) {
#pragma unroll
        for (int i = 0; i < kIter; ++i) p[i] += __shfl_xor(p[i], off);
    }
    if (c == 0) {
        float* out = score + (int64_t)h * v.S_total + sq.sent_base;
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int32_t s = row0 + 2 * i;
            if (s < sq.n_sent) out[s] = p[i];
        }
    }
}

template <int EB>
static hipError_t launch_score_g(Ctx* c, const void* q, const float* semvec_layer, const SeqView& v, float* score) {
    const int blocks = (v.S_total + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock + v.B;   // bound on sum_b ceil(S_b/R)
    const dim3 grid(blocks, c->d.n_kv_heads), block(kScoreWavesPerBlock * kWave);
    const char* qp = (const char*)q;
    switch (c->G) {
        case 1: hipLaunchKernelGGL((score_kernel<EB, 1>), grid, block, 0, c->stream, qp, semvec_layer, v, c->d.n_q_heads, score); break;
        case 2: hipLaunchKernelGGL((score_kernel<EB, 2>), grid, block, 0, c->stream, qp, semvec_layer, v, c->d.n_q_heads, score); break;
        case 4: hipLaunchKernelGGL((score_kernel<EB, 4>), grid, block, 0, c->stream, qp, semvec_layer, v, c->d.n_q_heads, score); break;
        case 8: hipLaunchKernelGGL((score_kernel<EB, 8>), grid, block, 0, c->stream, qp, semvec_layer, v, c->d.n_q_heads, score); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_score(Ctx* c, const void* q, const float* semvec_layer, const SeqView& v, float* score) {
    if (v.S_total == 0) return hipSuccess;
    return c->d.kv_dtype == SKV_BF16 ? launch_score_g<2>(c, q, semvec_layer, v, score)
                                     : launch_score_g<4>(c, q, semvec_layer, v, score);
}

// ------------------------------------------------------------------------------------------------
// Selection.  One 1024-thread block per (sequence, KV head).
//
// Buckets are ranked by (score descending, id ascending) and taken along the ranking until the first
// one that does not fit.  Because lengths are positive the running total along the ranking is
// increasing, so the retrieved set is {i : (total length ranked before i) + len_i <= budget}.  The
// first bucket that overflows (the "cut") is found without sorting, by a length-weighted radix select
// on an order-preserving 32-bit image of the score: 11 + 11 + 10 bit digits, most significant first;
// per pass a histogram of bucket lengths per digit, a suffix scan from the top digit, and the digit in
// which the running total crosses the budget.  The search stops as soon as the crossing digit holds a
// single bucket.  Buckets with exactly the cut's score are resolved in id order by a scan.
// A final scan in id order compacts the selected ids (ascending) and their token ranges.
// ------------------------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t score_key(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;          // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;                             // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive scan over the block's 1024 threads (thread order).  `sh` holds 16 wave totals.
// Returns the inclusive value; *total receives the block total.  Contains two barriers.
__device__ __forceinline__ unsigned long long block_scan_u64(unsigned long long val, unsigned long long* sh,
                                                             unsigned long long* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned long long x = val;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long t = __shfl_up(x, off);
        if (lane >= off) x += t;
    }
    __syncthreads();                        // previous users of sh are done
    if (lane == 63) sh[w] = x;
    __syncthreads();
    unsigned long long pre = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kSelectThreads / kWave; ++i) {
        const unsigned long long t = sh[i];
        if (i < w) pre += t;
        tot += t;
    }
    *total = tot;
    return x + pre;
}

constexpr int kMaxDigitBits = 11;
constexpr unsigned long long kLenMask = (1ull << 40) - 1;

__global__ __launch_bounds__(kSelectThreads) void select_kernel(const float* __restrict__ score,
                                                                const int32_t* __restrict__ sent_off,
                                                                const int32_t* __restrict__ sent_len, SeqView v,
                                                                int32_t Hkv, int32_t max_sel,
                                                                int32_t* __restrict__ sel_sent, int32_t* __restrict__ tokpos,
                                                                int32_t* __restrict__ n_sel, int32_t* __restrict__ tok_idx,
                                                                int32_t idx_stride, int32_t* __restrict__ n_tok) {
    __shared__ unsigned long long hist[1 << kMaxDigitBits];
    __shared__ unsigned long long sh_wave[kSelectThreads / kWave];
    __shared__ int sh_digit;
    __shared__ long long sh_carry;
    __shared__ int sh_cnt;

    const int bh = blockIdx.x, b = bh / Hkv, h = bh % Hkv;
    const int tid = threadIdx.x;
    const Seq sq = seq_of(v, b);
    const int32_t S = sq.n_sent;
    const long long budget = min(sq.budget, idx_stride);     // tok_idx holds at most idx_stride positions
    const float* sc = score + (int64_t)h * v.S_total + sq.sent_base;
    const int32_t* len = sent_len + sq.sent_base;
    const int32_t* off = sent_off + sq.sent_base + (v.cu_sent ? b : 0);
    sel_sent += (int64_t)bh * max_sel;
    tokpos += (int64_t)bh * max_sel;
    tok_idx += (int64_t)bh * idx_stride;

    if (S <= 0 || budget <= 0) {
        if (tid == 0) { n_sel[bh] = 0; n_tok[bh] = 0; }
        return;
    }

    // ---- weighted radix select of the cut --------------------------------------------------------
    uint32_t prefix = 0;        // resolved high bits of the cut's key
    int shift = 32;             // number of unresolved low bits
    long long carry = 0;        // total length of the buckets ranked strictly above the current digit range
    int cut_cnt = 0;            // number of buckets sharing the resolved prefix
    bool select_all = false;
    const int pass_bits[3] = {11, 11, 10};
    for (int pass = 0; pass < 3; ++pass) {
        const int bits = pass_bits[pass], nbins = 1 << bits, nshift = shift - bits;
        for (int i = tid; i < nbins; i += kSelectThreads) hist[i] = 0;
        if (tid == 0) sh_digit = -1;
        __syncthreads();
        for (int32_t s = tid; s < S; s += kSelectThreads) {
            const uint32_t k = score_key(sc[s]);
            if (shift == 32 || (k >> shift) == prefix) {
                const int d = (k >> nshift) & (nbins - 1);
                atomicAdd(&hist[d], (1ull << 40) | (unsigned long long)(uint32_t)len[s]);
            }
        }
        __syncthreads();
        // thread t owns digits nbins-1-2t and nbins-2-2t: thread order == descending digit order
        const int d1 = nbins - 1 - 2 * tid, d0 = d1 - 1;
        const unsigned long long v1 = d1 >= 0 ? hist[d1] : 0ull, v0 = d0 >= 0 ? hist[d0] : 0ull;
        const long long l1 = (long long)(v1 & kLenMask), l0 = (long long)(v0 & kLenMask);
        unsigned long long total;
        const long long incl = (long long)block_scan_u64((unsigned long long)(l1 + l0), sh_wave, &total);
        const long long before1 = carry + incl - l1 - l0, after1 = before1 + l1, after0 = after1 + l0;
        if (l1 > 0 && before1 <= budget && after1 > budget) { sh_digit = d1; sh_carry = before1; sh_cnt = (int)(v1 >> 40); }
        if (l0 > 0 && after1 <= budget && after0 > budget) { sh_digit = d0; sh_carry = after1; sh_cnt = (int)(v0 >> 40); }
        __syncthreads();
        const int digit = sh_digit;
        if (digit < 0) { select_all = true; break; }          // everything fits (only possible in pass 0)
        prefix = (shift == 32) ? (uint32_t)digit : ((prefix << bits) | (uint32_t)digit);
        carry = sh_carry;
        cut_cnt = sh_cnt;
        shift = nshift;
        __syncthreads();                                       // sh_* are rewritten by the next pass
        if (cut_cnt == 1) break;                               // the cut is unique: it is the bucket that overflows
    }
    const bool ties = !select_all && cut_cnt > 1;              // then shift == 0: several buckets share the cut's score

    // ---- compaction in id order ---------------------------------------------------------------------
    long long tie_run = 0;          // length of tied buckets with lower ids
    int run_cnt = 0;                // selected buckets so far
    long long run_tok = 0;          // selected tokens so far
    for (int32_t base = 0; base < S; base += kSelectThreads) {
        const int32_t s = base + tid;
        const bool live = s < S;
        const uint32_t k = live ? score_key(sc[s]) : 0u;
        const int32_t ln = live ? len[s] : 0;
        bool sel = false;
        if (live) {
            if (select_all) sel = true;
            else sel = (shift >= 32 ? 0u : (k >> shift)) > prefix;
        }
        if (ties) {
            const bool tied = live && k == prefix;
            unsigned long long tot;
            const long long cum = (long long)block_scan_u64(tied ? (unsigned long long)(uint32_t)ln : 0ull, sh_wave, &tot);
            if (tied && carry + tie_run + cum <= budget) sel = true;
            tie_run += (long long)tot;
        }
        unsigned long long tot;
        const unsigned long long mine = sel ? ((1ull << 40) | (unsigned long long)(uint32_t)ln) : 0ull;
        const unsigned long long incl = block_scan_u64(mine, sh_wave, &tot);
        if (sel) {
            const unsigned long long excl = incl - mine;
            const int pos = run_cnt + (int)(excl >> 40);
            if (pos < max_sel) {
                sel_sent[pos] = s;
                tokpos[pos] = (int32_t)(run_tok + (long long)(excl & kLenMask));
            }
        }
        run_cnt += (int)(tot >> 40);
        run_tok += (long long)(tot & kLenMask);
    }
    const int nsel = min(run_cnt, max_sel);
    if (tid == 0) { n_sel[bh] = nsel; n_tok[bh] = (int32_t)run_tok; }
    __syncthreads();                                           // sel_sent / tokpos visible to the block

    // ---- token positions of the selected buckets, ascending --------------------------------------------
    const int32_t ntok = (int32_t)min(run_tok, (long long)idx_stride);
    for (int32_t j = tid; j < ntok; j += kSelectThreads) {
        int lo = 0, hi = nsel - 1;                             // last i with tokpos[i] <= j
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tokpos[mid] <= j) lo = mid; else hi = mid - 1;
        }
        tok_idx[j] = off[sel_sent[lo]] + (j - tokpos[lo]);
    }
}

hipError_t launch_select(Ctx* c, const float* score, const int32_t* sent_off, const int32_t* sent_len,
                         const SeqView& v, int32_t* sel_sent, int32_t* tokpos, int32_t* n_sel, int32_t* tok_idx,
                         int32_t idx_stride, int32_t* n_tok) {
    hipLaunchKernelGGL(select_kernel, dim3(v.B * c->d.n_kv_heads), dim3(kSelectThreads), 0, c->stream, score, sent_off,
                       sent_len, v, c->d.n_kv_heads, c->max_sel, sel_sent, tokpos, n_sel, tok_idx, idx_stride, n_tok);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Gather.  One 16-byte lane chunk per thread per row; a block copies kGatherRowsPerBlock rows of K
// (blockIdx.z == 0) or V (blockIdx.z == 1) of one KV head with all its loads issued before its stores.
// The pool pointer may be device-mapped pinned host memory: the same loads then cross PCIe.
// ------------------------------------------------------------------------------------------------
template <int EB>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(const char* __restrict__ Kl, const char* __restrict__ Vl,
                                                                int32_t T, const int32_t* __restrict__ tok_idx,
                                                                const int32_t* __restrict__ n_tok, int32_t budget,
                                                                char* __restrict__ Ks, char* __restrict__ Vs) {
    using R = Row<EB>;
    constexpr int kRowsPerIter = kGatherThreads / R::LPR;
    constexpr int kIter = kGatherRowsPerBlock / kRowsPerIter;
    constexpr int kRowBytes = kHeadDim * EB;
    const int h = blockIdx.y;
    const int32_t n = min(n_tok[h], budget);
    const int32_t j0 = blockIdx.x * kGatherRowsPerBlock;
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

hipError_t launch_gather(Ctx* c, const void* K_layer, const void* V_layer, int32_t T, const int32_t* tok_idx,
                         const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel) {
    if (budget == 0) return hipSuccess;
    const dim3 grid((budget + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock, c->d.n_kv_heads, 2), block(kGatherThreads);
    if (c->d.kv_dtype == SKV_BF16)
        hipLaunchKernelGGL(gather_kernel<2>, grid, block, 0, c->stream, (const char*)K_layer, (const char*)V_layer, T,
                           tok_idx, n_tok, budget, (char*)K_sel, (char*)V_sel);
    else
        hipLaunchKernelGGL(gather_kernel<4>, grid, block, 0, c->stream, (const char*)K_layer, (const char*)V_layer, T,
                           tok_idx, n_tok, budget, (char*)K_sel, (char*)V_sel);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Attention (Eq. 3), split-K flash decoding.  Block (split, sequence*KV head) handles kAttChunk = 64
// consecutive retrieved tokens for the G query heads of its KV head:
//   1. every K and V lane chunk of the chunk is requested up front (16-byte loads, RPW rows per wave
//      instruction), either from K_sel/V_sel or straight from the pool through tok_idx;
//   2. logits for the G heads: per-lane partial dot products, reduced over the LPR lanes of a row;
//   3. one wave per query head: max, exp2, sum over the 64 logits (softmax in log2 units);
//   4. P.V with per-lane accumulators, reduced over the rows of a wave and over the 4 waves in LDS;
//   5. the un-normalised partial (m, l, acc) goes to the workspace; the last block to arrive for the
//      (sequence, KV head) -- a device-scope counter, no spinning -- rescales and sums the partials.
// ------------------------------------------------------------------------------------------------
template <int EB, int G, bool IND>
__global__ __launch_bounds__(kAttThreads) void attend_kernel(const char* __restrict__ q, const char* __restrict__ Kb,
                                                             const char* __restrict__ Vb, const int32_t* __restrict__ tok_idx,
                                                             int32_t idx_stride, int32_t row_stride,
                                                             const int32_t* __restrict__ n_tok, SeqView v, int32_t Hkv,
                                                             int32_t max_splits, float* __restrict__ part,
                                                             float* __restrict__ ml, unsigned int* __restrict__ counter,
                                                             float* __restrict__ out, float* __restrict__ lse) {
    using R = Row<EB>;
    constexpr int kWaves = kAttThreads / kWave;
    constexpr int kRowsPerIter = kWaves * R::RPW;
    constexpr int kIter = kAttChunk / kRowsPerIter;
    constexpr int kRowBytes = kHeadDim * EB;
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

    __shared__ float sm_logit[G][kAttChunk];
    constexpr int kRedFloats = (kWaves * G * kHeadDim > 1024) ? kWaves * G * kHeadDim : 1024;
    __shared__ __attribute__((aligned(16))) float sm_red_flat[kRedFloats];
    float (*sm_red)[G][kHeadDim] = reinterpret_cast<float (*)[G][kHeadDim]>(sm_red_flat);
    __shared__ int sm_last;

    const int bh = blockIdx.y, b = bh / Hkv, h = bh % Hkv, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane / R::LPR, cc = lane % R::LPR;
    const int Hq = Hkv * G;
    const int64_t qhead0 = (int64_t)b * Hq + (int64_t)h * G;      // first query head of the group
    const Seq sq = seq_of(v, b);

    int32_t n = n_tok[bh];
    n = min(n, IND ? idx_stride : row_stride);
    if (n <= 0) {
        if (split == 0) {
            for (int i = tid; i < G * kHeadDim; i += kAttThreads) out[qhead0 * kHeadDim + i] = 0.f;
            if (lse && tid < G) lse[qhead0 + tid] = -INFINITY;
        }
        return;
    }
    const int nsplit = (n + kAttChunk - 1) / kAttChunk;
    if (split >= nsplit) return;
    const int32_t j0 = split * kAttChunk;
    const int32_t cnt = min(kAttChunk, n - j0);

    // ---- 1. issue every load of the chunk ------------------------------------------------------------
    const char* Kh;
    const char* Vh;
    if (IND) {
        Kh = Kb + ((int64_t)h * v.T_total + sq.tok_base) * kRowBytes;
        Vh = Vb + ((int64_t)h * v.T_total + sq.tok_base) * kRowBytes;
    } else {
        Kh = Kb + ((int64_t)bh * row_stride + j0) * kRowBytes;
        Vh = Vb + ((int64_t)bh * row_stride + j0) * kRowBytes;
    }
    // Branch-free loads: rows past the chunk's end (and indices outside the sequence) are clamped to a
    // valid row, loaded anyway and masked afterwards, so that all loads are in flight together.
    int32_t rowi[kIter];
    bool live[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        const int jj = i * kRowsPerIter + w * R::RPW + r;
        live[i] = jj < cnt;
        const int jc = min(jj, cnt - 1);
        if (IND) {
            const int32_t x = tok_idx[(int64_t)bh * idx_stride + j0 + jc];
            live[i] = live[i] && x >= 0 && x < sq.n_tok_ctx;
            rowi[i] = min(max(x, 0), max(sq.n_tok_ctx - 1, 0));
        } else {
            rowi[i] = jc;
        }
    }
    uint4 kraw[kIter], vraw[kIter];
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        kraw[i] = *reinterpret_cast<const uint4*>(Kh + (int64_t)rowi[i] * kRowBytes + cc * 16);
        vraw[i] = *reinterpret_cast<const uint4*>(Vh + (int64_t)rowi[i] * kRowBytes + cc * 16);
    }
    float qf[G][R::EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 t = *reinterpret_cast<const uint4*>(q + ((qhead0 + g) * kHeadDim) * EB + cc * 16);
        R::unpack(t, qf[g]);
    }

    // ---- 2. logits ---------------------------------------------------------------------------------
    const float scale = kLog2e * rsqrtf((float)kHeadDim);
#pragma unroll
    for (int i = 0; i < kIter; ++i) {
        float kf[R::EPL];
        R::unpack(kraw[i], kf);
        float s[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float a = 0.f;
#pragma unroll
            for (int e = 0; e < R::EPL; ++e) a += qf[g][e] * kf[e];
            s[g] = a;
        }
#pragma unroll
        for (int off = R::LPR / 2; off >= 1; off >>= 1) {
#pragma unroll
            for (int g = 0; g < G; ++g) s[g] += __shfl_xor(s[g], off);
        }
        if (cc == 0) {
            const int jj = i * kRowsPerIter + w * R::RPW + r;
#pragma unroll
            for (int g = 0; g < G; ++g) sm_logit[g][jj] = live[i] ? s[g] * scale : -INFINITY;
        }
    }
    __syncthreads();

    // ---- 3. softmax over the chunk, one wave per query head --------------------------------------------
    for (int g = w; g < G; g += kWaves) {
        const float x = sm_logit[g][lane];
        float m = x;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
        const float p = (m == -INFINITY) ? 0.f : exp2f(x - m);
        float l = p;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off);
        sm_logit[g][lane] = p;
        if (lane == 0) {
            float* dst = ml + (((qhead0 + g) * max_splits) + split) * 2;
            dst[0] = m; dst[1] = l;
        }
    }
    __syncthreads();

    // ---- 4. P.V -------------------------------------------------------------------------------------
    float acc[G][R::EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
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
        for (int g = 0; g < G; ++g) {
            const float p = sm_logit[g][jj];
#pragma unroll
            for (int e = 0; e < R::EPL; ++e) acc[g][e] += p * vf[e];
        }
    }
#pragma unroll
    for (int off = R::LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < R::EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], off);
    }
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < R::EPL; ++e) sm_red[w][g][cc * R::EPL + e] = acc[g][e];
    }
    __syncthreads();
    for (int i = tid; i < G * kHeadDim; i += kAttThreads) {
        const int g = i / kHeadDim, d = i % kHeadDim;
        float a = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) a += sm_red[ww][g][d];
        part[(((qhead0 + g) * max_splits) + split) * kHeadDim + d] = a;
    }

    // ---- 5. last arrival combines ------------------------------------------------------------------
    // The barrier orders the block's partial stores before thread 0's device-scope acq_rel increment
    // (which publishes them); the second barrier hands thread 0's acquire to the rest of the block.
    __syncthreads();
    if (tid == 0) {
        const unsigned int old = __hip_atomic_fetch_add(&counter[bh], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = (old == (unsigned int)(nsplit - 1));
    }
    __syncthreads();
    if (!sm_last) return;
    // (a) per query head: global max, normaliser, and each split's weight (stored over its max);
    //     one wave per head, lanes stride over the splits so their loads are independent.
    for (int g = w; g < G; g += kWaves) {
        float* mlg = ml + ((qhead0 + g) * max_splits) * 2;
        float M = -INFINITY;
        for (int s = lane; s < nsplit; s += kWave) M = fmaxf(M, mlg[2 * s]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
        float L = 0.f;
        for (int s = lane; s < nsplit; s += kWave) {
            const float ms = mlg[2 * s];
            L += (ms == -INFINITY) ? 0.f : exp2f(ms - M) * mlg[2 * s + 1];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) L += __shfl_xor(L, off);
        const bool empty = !(L > 0.f);                       // every retrieved index was out of range
        const float inv = empty ? 0.f : 1.f / L;
        for (int s = lane; s < nsplit; s += kWave) {
            const float ms = mlg[2 * s];
            mlg[2 * s] = (ms == -INFINITY) ? 0.f : exp2f(ms - M) * inv;
        }
        if (lse && lane == 0) lse[qhead0 + g] = empty ? -INFINITY : (M + log2f(L)) * kLn2;
    }
    __syncthreads();
    // (b) out[g][:] = sum_s weight[g][s] * partial[g][s][:].  A thread owns one float4 column of one head
    //     and every kGroups-th split; the groups are then summed through LDS.
    constexpr int kCol4 = G * (kHeadDim / 4);                // float4 columns over the G heads
    constexpr int kGroups = kAttThreads / kCol4;             // 8, 4, 2, 1 for G = 1, 2, 4, 8
    {
        const int col = tid % kCol4, grp = tid / kCol4;
        const int g = col / (kHeadDim / 4), d4 = col % (kHeadDim / 4);
        const float* mlg = ml + ((qhead0 + g) * max_splits) * 2;
        const float4* pg = reinterpret_cast<const float4*>(part + ((qhead0 + g) * max_splits) * kHeadDim) + d4;
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
        constexpr int kU = 8;
        for (int s0 = grp; s0 < nsplit; s0 += kGroups * kU) {
            float4 v[kU];
            float wgt[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {                   // clamped, unconditional loads
                const int sidx = min(s0 + u * kGroups, nsplit - 1);
                v[u] = pg[(int64_t)sidx * (kHeadDim / 4)];
                wgt[u] = (s0 + u * kGroups < nsplit) ? mlg[2 * sidx] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                o.x += wgt[u] * v[u].x; o.y += wgt[u] * v[u].y; o.z += wgt[u] * v[u].z; o.w += wgt[u] * v[u].w;
            }
        }
        reinterpret_cast<float4*>(sm_red_flat)[grp * kCol4 + col] = o;
    }
    __syncthreads();
    if (tid < kCol4) {
        float4 o = reinterpret_cast<const float4*>(sm_red_flat)[tid];
#pragma unroll
        for (int grp = 1; grp < kGroups; ++grp) {
            const float4 t = reinterpret_cast<const float4*>(sm_red_flat)[grp * kCol4 + tid];
            o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
        }
        reinterpret_cast<float4*>(out + qhead0 * kHeadDim)[tid] = o;
    }
    if (tid == 0) counter[bh] = 0;          // ready for the next call on this stream
}

template <int EB>
static hipError_t launch_attend_g(Ctx* c, const void* q, const void* Kbase, const void* Vbase, const int32_t* tok_idx,
                                  int32_t idx_stride, int32_t row_stride, const int32_t* n_tok, int32_t n_splits,
                                  const SeqView& v, float* out, float* lse) {
    const dim3 grid(n_splits, v.B * c->d.n_kv_heads), block(kAttThreads);
#define SKV_ATT_I(GG, IND)                                                                                            \
    hipLaunchKernelGGL((attend_kernel<EB, GG, IND>), grid, block, 0, c->stream, (const char*)q, (const char*)Kbase,   \
                       (const char*)Vbase, tok_idx, idx_stride, row_stride, n_tok, v, c->d.n_kv_heads, c->max_splits, \
                       c->att_part, c->att_ml, c->att_counter, out, lse)
#define SKV_ATT(GG)                    \
    do {                               \
        if (tok_idx) SKV_ATT_I(GG, true); \
        else SKV_ATT_I(GG, false);     \
    } while (0)
    switch (c->G) {
        case 1: SKV_ATT(1); break;
        case 2: SKV_ATT(2); break;
        case 4: SKV_ATT(4); break;
        case 8: SKV_ATT(8); break;
        default: return hipErrorInvalidValue;
    }
#undef SKV_ATT
#undef SKV_ATT_I
    return hipGetLastError();
}

hipError_t launch_attend(Ctx* c, const void* q, const void* Kbase, const void* Vbase, const int32_t* tok_idx,
                         int32_t idx_stride, int32_t row_stride, const int32_t* n_tok, int32_t n_splits,
                         const SeqView& v, float* out, float* lse) {
    if (n_splits < 1) n_splits = 1;       // block 0 still writes the empty-selection result
    return c->d.kv_dtype == SKV_BF16
               ? launch_attend_g<2>(c, q, Kbase, Vbase, tok_idx, idx_stride, row_stride, n_tok, n_splits, v, out, lse)
               : launch_attend_g<4>(c, q, Kbase, Vbase, tok_idx, idx_stride, row_stride, n_tok, n_splits, v, out, lse);
}

}  // namespace skv
