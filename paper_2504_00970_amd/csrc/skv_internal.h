// Internal declarations shared by the translation units of libsentencekv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sentencekv.h"

namespace skv {

constexpr int kHeadDim = 128;
constexpr int kWave = 64;

// ---- launch geometry (host and device must agree; the host checks shapes against these) ----------
constexpr int kSegThreads = 256;
constexpr int kSegTokPerThread = 4;
constexpr int kSegTokPerBlock = kSegThreads * kSegTokPerThread;      // 1024 tokens per block

constexpr int kSemvecWavesPerBlock = 4;                               // one wave per (layer*head, bucket)

constexpr int kScoreRowsPerWave = 8;          // buckets per wave (32 per block)
constexpr int kScoreWavesPerBlock = 4;

constexpr int kBlockThreads = 1024;   // select, attention and the fused select+attention kernel: 16 waves per block

constexpr int kGatherRowsPerBlock = 64;
constexpr int kGatherThreads = 256;

constexpr int kAttChunk = 64;         // tokens per split-K block, single-sequence step (one wave-width of logits)
constexpr int kAttChunkMid = 128;     // tokens per split-K block of the single-sequence step when a sequence has many buckets
constexpr int kMidChunkMinSentences = 1024;
constexpr int kAttChunkWide = 256;    // tokens per split-K block when many (sequence, head) pairs fill the GPU
constexpr int kWideChunkMinHeads = 64;   // (sequences x KV heads) from which the fp32 batch path is used
constexpr int kComputeUnits = 256;       // MI355X; the context takes the device's own count when it can be read
// single-launch decode step: at most kStepMaxPairs (sequence, head) pairs and kStepMaxBlocks blocks per launch
constexpr int kStepPairBits = 6;
constexpr int kStepMaxPairs = 1 << kStepPairBits;
constexpr int kStepMaxBlocks = 256;
constexpr int kStepEpochStride = 16;     // 32-bit words between the epoch counters of two pairs (one 64-byte line each)
constexpr int kStepPartWords = kHeadDim + 2;   // 64-bit words per query head of a block's partial: D sums, max, normaliser
constexpr int kStepWaitLimit = 200000;   // default bound on the polling rounds of a waiting block (a round is about a microsecond)
// bf16 decode step: the fused kernel's block size (64, 128, 256 tokens) is the smallest whose blocks, (sequence, KV head)
// pairs x ceil(max_budget / size), all fit the chip at once (one block per compute unit); if even the 256-token blocks do
// not, the streaming kernel's 512- or 1024-token blocks

struct Ctx {
    skv_desc d;
    hipStream_t stream;
    int device;
    int n_cu;               // compute units of the device
    int G;
    int max_sel;            // min(max_sentences, max_budget)
    int max_splits;         // ceil(max_budget / kAttChunk)
    int budget_cap;         // the largest budget the decode step plans for: max_budget, or the caller's hint below it
    char* ws;               // one device allocation, carved below
    size_t ws_bytes;
    unsigned long long* seg_part;  // [ceil(max_tokens / kSegTokPerBlock)] packed (count << 32 | last_end)
    float* att_part;        // [max_batch * Hq][max_splits][D] un-normalised partial outputs
    float* att_ml;          // [max_batch * Hq][max_splits][2] (running max in log2 units, sum)
    unsigned int* att_counter;  // [max_batch * Hkv] arrivals per (sequence, KV head); zero between calls
    float* f_score;         // [Hkv][max_sentences] scores of the fused path
    int32_t* f_sel_sent;    // [max_batch * Hkv][max_sel]     selection of the batch path
    int32_t* f_n_sel;       // [max_batch * Hkv]
    int32_t* f_n_tok;       // [max_batch * Hkv]
    int32_t* f_tok_idx;     // [max_batch * Hkv][max_budget]
    unsigned int* step_epoch;    // [kStepMaxPairs][kStepEpochStride] launches of the single-launch step per pair; never reset
    unsigned long long* step_score;  // [pairs][step_score_stride] (score, tag) words
    int32_t step_score_stride;   // words per pair (max_sentences)
    int64_t step_score_words;    // words in step_score: a launch needs pairs * step_score_stride of them
    unsigned long long* step_part;   // [kStepMaxBlocks][G][kStepPartWords] (value, tag) words
    unsigned int* err_dev;       // [1] set by a block of the single-launch step that gave up waiting
    unsigned int* err_host;      // the same flag in pinned host memory (host address; null: none)
    unsigned int* err_host_dev;  // device address of err_host
    int wait_limit;              // polling rounds before a waiting block gives up
    bool single_launch;          // skv_decode_step may take the single-launch form
};

// Ragged-batch view handed to the decode kernels.  For single-sequence calls cu_tok / cu_sent /
// budget_arr are null and the scalar fields apply.
struct SeqView {
    const int32_t* cu_tok;      // [B+1] or null
    const int32_t* cu_sent;     // [B+1] or null
    const int32_t* budget_arr;  // [B] or null
    int32_t T_total;
    int32_t S_total;
    int32_t budget;             // scalar budget when budget_arr is null
    int32_t B;
};

// ---- launchers (defined in prefill.hip / decode.hip); each returns the hipError_t of its launch -----
hipError_t launch_segment(Ctx* c, const int32_t* tok, int32_t T, const uint32_t* bitmap, int32_t vocab,
                          int32_t* seg_id, int32_t* sent_off, int32_t* sent_len, int32_t* n_sent_dev);
// off_layer_stride: 0 = one offset table for all layers, else the distance (in entries) between the layers' tables
hipError_t launch_semvec(Ctx* c, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t off_layer_stride, int32_t S,
                         void* semvec);
// prefill-side token retention (retain.hip)
constexpr int kImportanceMaxRows = 256;   // query rows (G * window tokens) per KV head
int64_t importance_work_bytes(const Ctx* c, int32_t T, int32_t N);
hipError_t launch_importance(Ctx* c, const void* q_obs, const void* K_pool, int32_t T, int32_t N, float* alpha, void* work);
hipError_t launch_retain(Ctx* c, const float* alpha, int32_t Tp, int32_t k, const int32_t* seg_id, int32_t S, int32_t* keep_idx,
                         int32_t* n_keep, int32_t* ret_off, int32_t* ret_len);
hipError_t launch_compact_pool(Ctx* c, const void* K_pool, const void* V_pool, int32_t T, const int32_t* keep_idx, int32_t k,
                               const int32_t* n_keep, void* K_ret, void* V_ret);
hipError_t launch_query_update(Ctx* c, int32_t B, const void* q_t, const int32_t* tok_t, const uint32_t* bitmap,
                               int32_t vocab, float* q_sum, int32_t* q_cnt, void* q_bar);
hipError_t launch_score(Ctx* c, const void* q, const void* semvec_layer, const SeqView& v, float* score);
hipError_t launch_select(Ctx* c, const float* score, const int32_t* sent_off, const int32_t* sent_len,
                         const SeqView& v, int32_t* sel_sent, int32_t* n_sel, int32_t* tok_idx, int32_t idx_stride,
                         int32_t budget_cap, int32_t* n_tok);
hipError_t launch_gather(Ctx* c, const void* K_layer, const void* V_layer, int32_t T, bool host_pool, const int32_t* tok_idx,
                         const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel);
// Attention over K_sel/V_sel [B*Hkv][row_stride][D] with n_tok [B*Hkv] from memory.
hipError_t launch_attend(Ctx* c, const void* q, const void* K_sel, const void* V_sel, int32_t row_stride,
                         const int32_t* n_tok, int32_t budget, const SeqView& v, float* out, float* lse);
// Attention over the layer's pool [Hkv][T_total][D] through tok_idx [B*Hkv][max_budget] (batch path).
hipError_t launch_attend_indirect(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const int32_t* tok_idx,
                                  const int32_t* n_tok, const SeqView& v, float* out, float* lse);
// Selection from `score` fused with attention over the layer's pool (single-sequence / small-batch path).
hipError_t launch_select_attend(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const float* score,
                                const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                                float* lse, int32_t* tok_idx_out, int32_t* n_tok_out);

// The whole step in one launch (scores by the blocks of each pair, a per-pair ticket barrier, selection, attention) when
// its grid fits the chip at once; *launched is false (and nothing was launched) when the shapes do not allow it.
hipError_t launch_step(Ctx* c, const void* q_score, const void* q_attn, const void* semvec_layer, const void* K_layer,
                       const void* V_layer, const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                       float* lse, int32_t* tok_idx_out, int32_t* n_tok_out, bool* launched);

// The same for batches with bf16 pools of fewer than 2^24 tokens: 1024-token blocks, streaming attention.
hipError_t launch_select_attend_stream(Ctx* c, const void* q, const void* K_layer, const void* V_layer, const float* score,
                                       const int32_t* sent_off, const int32_t* sent_len, const SeqView& v, float* out,
                                       float* lse, int32_t* tok_idx_out, int32_t* n_tok_out);

hipError_t launch_merge_lse(Ctx* c, const float* out_a, const float* lse_a, const float* out_b, const float* lse_b,
                            int32_t n_heads, float* out, float* lse);

// A K/V row is D * EB bytes = LPR lanes of 16 bytes, so one wave-wide 128-bit load covers RPW
// consecutive rows; each lane holds EPL elements of its row.
template <int EB> struct Row;
template <> struct Row<2> {          // bf16: 8 elements per 16-byte lane chunk
    static constexpr int LPR = 16, RPW = 4, EPL = 8;
    __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};
template <> struct Row<4> {          // fp32: 4 elements per 16-byte lane chunk
    static constexpr int LPR = 32, RPW = 2, EPL = 4;
    __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
};

}  // namespace skv

struct skv_ctx {
    skv::Ctx c;
};
