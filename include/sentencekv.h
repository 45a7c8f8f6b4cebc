/*
 * sentencekv.h -- C ABI of the MI355X (gfx950) SentenceKV hot path (arxiv 2504.00970).
 *
 * The library implements, as hand-written HIP kernels, the data-parallel work SentenceKV does
 *   - once per prompt (prefill):  sentence buckets and their mean key vectors (Sec. 4.1, Eq. 1);
 *   - at every decode step, per layer: similarity scores of every bucket against the (mean) query,
 *     ranking and budgeted retrieval of whole buckets, loading the retrieved tokens' K/V, and
 *     attention over them (Sec. 4.2, Eq. 3, Alg. 1 decoding phase).
 *
 * Conventions
 *   - Every function returns an int: SKV_OK (0) or a negative skv_status.  Nothing aborts, throws
 *     or prints.  Argument checks are done on the host before anything is launched.
 *   - "dev" pointers are device memory (HBM) unless stated otherwise, "host" pointers host memory.
 *     All are caller-owned, 16-byte aligned, and must stay valid until the work queued on the
 *     context's stream has finished.  The library owns only the context and its workspace, which
 *     is sized from skv_desc at skv_create; no call after skv_create allocates.
 *   - All tensors are dense, row-major, innermost dimension last.  head_dim D is 128.
 *     K/V/q element type is skv_desc.kv_dtype (fp32 or bf16); semantic vectors, scores, attention
 *     outputs and log-sum-exps are fp32; every index, length and count is int32.
 *   - Grouped-query attention: query head j reads KV head j / G, G = n_q_heads / n_kv_heads.
 *     One bucket selection is made per KV head (and per layer, per sequence); the score of a bucket
 *     is the sum over the group's G query heads of q_j^T k-bar (the paper states the score per
 *     attention head and is silent on GQA).
 *   - Decode calls are asynchronous on the context's stream and never block the host.  Calls on one
 *     context must come from one host thread at a time and execute in stream order; they share the
 *     context's workspace, so two contexts are needed for concurrent streams (and skv_set_single_launch(ctx, 0)
 *     on both when their decode steps may overlap on one GPU).
 */
#ifndef SENTENCEKV_H
#define SENTENCEKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SKV_OK = 0,
    SKV_EINVAL = -1,     /* null / misaligned pointer, negative size, shape not matching the descriptor */
    SKV_ECAPACITY = -2,  /* tokens, sentences, budget or batch exceed the maxima given at skv_create */
    SKV_EHIP = -3,       /* a HIP runtime call or kernel launch failed (no usable GPU included) */
    SKV_ENOMEM = -4      /* workspace allocation failed */
} skv_status;

typedef enum { SKV_F32 = 0, SKV_BF16 = 1, SKV_FP8_E4M3 = 2 /* semantic-vector table only */ } skv_dtype;

typedef struct {
    int32_t n_layers;       /* L: leading dimension of the K/V pools and of the semantic-vector table */
    int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads; G = Hq / Hkv must be 1, 2, 4 or 8 */
    int32_t n_kv_heads;     /* Hkv */
    int32_t head_dim;       /* D, must be 128 */
    int32_t kv_dtype;       /* skv_dtype of K, V and the queries */
    int32_t max_tokens;     /* largest T (T_total for a ragged batch) any call will pass */
    int32_t max_sentences;  /* largest S (S_total for a ragged batch) any call will pass */
    int32_t max_budget;     /* largest per-sequence token budget tau any call will pass.  skv_decode_step sizes its grid and
                               picks its kernel from this value, not from the budgets of a call (see there): a context
                               made for 8192 runs a 2048-token step in larger blocks than a context made for 2048 would
                               (measured: up to 2x slower for one sequence), so keep it close to the budgets in use, or
                               tell the context the budgets in use with skv_set_budget_hint */
    int32_t max_batch;      /* largest number of sequences in one skv_decode_step (>= 1, <= 4096, max_batch * Hkv <= 65535) */
    int32_t semvec_dtype;   /* skv_dtype of the semantic-vector table: SKV_F32, or SKV_BF16 / SKV_FP8_E4M3 = the fp32 mean
                               rounded once to nearest even (the mixed-precision sentence vectors of the paper's "Future
                               Work"; a half / a quarter of the bytes the scoring step reads).  E4M3 is the 8-bit format of
                               the OCP specification (bias 7, no infinities, largest value 448); larger means saturate */
} skv_desc;

typedef struct skv_ctx skv_ctx;   /* opaque */

/* Creates a context on the current HIP device.  `hip_stream` (a hipStream_t, may be NULL for the
 * default stream) is borrowed, not owned.  Fails with SKV_EINVAL on a bad descriptor (checked before
 * the GPU is touched), SKV_EHIP / SKV_ENOMEM if the device or its memory is unavailable. */
int skv_create(skv_ctx** out, const skv_desc* desc, void* hip_stream);
void skv_destroy(skv_ctx* ctx);
int skv_set_stream(skv_ctx* ctx, void* hip_stream);
const char* skv_strerror(int status);
/* Bytes of device workspace the context holds (0 for a NULL context). */
int64_t skv_workspace_bytes(const skv_ctx* ctx);
/* skv_decode_step plans its launches (kernel, block size, grid) for the largest budget it may meet.  That is the
 * descriptor's max_budget unless the caller gives a tighter bound here: `budget` = the largest per-sequence budget the
 * following skv_decode_step calls on this context will use (0 restores max_budget).  Budgets above the hint are
 * treated as the hint.  Array shapes (tok_idx_out is [B][Hkv][max_budget]) do not change.  A context created for
 * max_budget = 8192 and hinted 2048 runs a 2048-token step exactly as a context created for 2048 does.
 * Errors: SKV_EINVAL (NULL context, budget < 0), SKV_ECAPACITY (budget > max_budget). */
int skv_set_budget_hint(skv_ctx* ctx, int32_t budget);
/* skv_decode_step with few (sequence, head) pairs runs as ONE launch whose blocks wait, inside the kernel, for the bucket
 * scores and the partial attention results that the other blocks of their pair produce (see skv_decode_step).  Every
 * such wait is bounded: `polls` is the number of times a thread reads the words it waits for before it gives up (a
 * read takes about a microsecond; default 200000; with 0 nothing is read and every waiting block gives up at once: the
 * kernel still ends normally).  A give-up turns the outputs of that call into NaN and makes every later skv_decode_step
 * on the context return SKV_EHIP until this function is called again, which also clears the condition (it waits for
 * the stream).
 * Errors: SKV_EINVAL (NULL context, polls < 0). */
int skv_set_wait_limit(skv_ctx* ctx, int32_t polls);
/* The single-launch form needs every block of its grid on the GPU at the same time: the library launches it only when
 * the grid fits the compute units of an otherwise idle GPU.  Work that other streams, contexts or processes run on the
 * same GPU at the same moment can keep part of the grid waiting for a compute unit while the blocks that did start
 * wait for it: the bounded waits then run out and the step fails as described above.  A caller that overlaps steps of
 * several contexts, or other kernels, on one GPU turns the form off (`enable` = 0): skv_decode_step then always uses
 * the forms of two or three launches, which wait for nothing.  On by default.
 * Errors: SKV_EINVAL (NULL context). */
int skv_set_single_launch(skv_ctx* ctx, int32_t enable);

/* ---------------------------------------------------------------------------------------------
 * (1) Prefill.  Sec. 4.1 first paragraph and Alg. 1 prefilling phase: the prompt is split into
 * sentence buckets at punctuation.  Which token ids are punctuation is data: bit (id % 32) of word
 * (id / 32) of `term_bitmap` is set for a terminator; ids outside [0, vocab) are never terminators.
 *
 * A bucket ends WITH its terminator; tokens after the last terminator form a final bucket; every
 * terminator of a run closes a (length-1) bucket.  Hence
 *     seg_id[i]   = number of terminators among tok[0..i)         (exclusive prefix sum)
 *     S           = seg_id[T-1] + 1  (0 when T == 0)
 *     sent_off[s] = first position of bucket s, sent_off[S] = T;  sent_len[s] = sent_off[s+1] - sent_off[s]
 *
 * tok          dev  [T]                      seg_id      dev [T]
 * term_bitmap  dev  [ceil(vocab / 32)]       sent_off    dev [max_sentences + 1]
 * n_sent_dev   dev  [1], receives S          sent_len    dev [max_sentences]
 * n_sent_host  host [1] or NULL.  Non-NULL: the call waits for the stream, stores S there and returns
 *              SKV_ECAPACITY if S > max_sentences.  Buckets beyond max_sentences are never written
 *              (n_sent_dev still receives the true S).  NULL: fully asynchronous.
 * Errors: SKV_EINVAL (null pointers, T < 0, vocab <= 0), SKV_ECAPACITY (T > max_tokens). */
int skv_segment(skv_ctx* ctx, const int32_t* tok, int32_t T, const uint32_t* term_bitmap, int32_t vocab,
                int32_t* seg_id, int32_t* sent_off, int32_t* sent_len, int32_t* n_sent_dev,
                int32_t* n_sent_host);

/* Eq. 1: semvec[l][h][s][:] = mean over the tokens x of bucket s of K_pool[l][h][x][:], accumulated
 * in fp32.  The pool holds the full context, so the set S_s of Eq. 1 is the whole bucket.
 * K_pool  dev [L][Hkv][T][D] kv_dtype          sent_off  dev [S + 1] (as produced by skv_segment)
 * semvec  dev [L][Hkv][S][D] semvec_dtype
 * Errors: SKV_EINVAL, SKV_ECAPACITY (T > max_tokens or S > max_sentences).  S == 0 is a no-op. */
int skv_build_semvec(skv_ctx* ctx, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t S,
                     void* semvec);

/* Eq. 1 over a retained pool: as skv_build_semvec, but every layer has its own offset table (the retained
 * tokens differ per layer) and a bucket may hold no token (its vector is stored as zeros; skv_select and
 * skv_decode_step never list a bucket of length 0).
 * K_pool dev [L][Hkv][T][D] kv_dtype      sent_off dev [L][S + 1]      semvec dev [L][Hkv][S][D] semvec_dtype
 * Errors: SKV_EINVAL, SKV_ECAPACITY (T > max_tokens or S > max_sentences). */
int skv_build_semvec_layers(skv_ctx* ctx, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t S, void* semvec);

/* ---------------------------------------------------------------------------------------------
 * Prefill-side token retention: Sec. 4.1 "Token importance measurement" and "Token selection within sentence
 * buckets", App. "Effect of Sentence Length", Alg. 1 prefilling phase.
 *
 * skv_token_importance: the last N tokens of the T-token prompt are the observation window (Tp = T - N tokens
 * precede it).  Window query n of query head j attends, as in the model's forward pass, to the keys of positions
 * 0 .. Tp + n of KV head floor(j / G) with softmax(q k^T / sqrt(D)); alpha[l][i], i < Tp, is the sum over all N window
 * queries and all Hq heads of the probability token i receives.  One importance per token and layer.
 * q_obs  dev [L][Hq][N][D] kv_dtype    K_pool dev [L][Hkv][T][D] kv_dtype    alpha dev [L][Tp] fp32
 * work   dev scratch of at least skv_token_importance_work_bytes(ctx, T, N) bytes (caller-owned; nothing is kept in
 *        it between calls).  G * N <= 256.  Asynchronous.
 * Errors: SKV_EINVAL (null / misaligned pointers, N < 1, N >= T, work too small), SKV_ECAPACITY (T > max_tokens,
 * G * N > 256).  skv_token_importance_work_bytes returns -1 for arguments the call would reject. */
int64_t skv_token_importance_work_bytes(const skv_ctx* ctx, int32_t T, int32_t N);
int skv_token_importance(skv_ctx* ctx, const void* q_obs, const void* K_pool, int32_t T, int32_t N, float* alpha, void* work,
                         int64_t work_bytes);

/* skv_retain: per layer, the k = floor(r tau) tokens with the highest importance over the whole prefix are retained,
 * regardless of bucket boundaries (equal importance: lower position first; NaN last).  The buckets of the retained
 * pool keep the prompt's numbering.
 * alpha    dev [L][Tp] fp32               seg_id  dev [>= Tp] bucket id per token (as produced by skv_segment)
 * keep_idx dev [L][max(k,1)] retained positions, ascending; n_keep dev [L] = min(k, Tp)
 * ret_len  dev [L][S] retained tokens per bucket (0: the bucket vanished)
 * ret_off  dev [L][S + 1] exclusive prefix sum of ret_len = first row of the bucket in the compacted pool.
 * Errors: SKV_EINVAL (null / misaligned pointers, Tp < 1, k < 0, S < 1), SKV_ECAPACITY (Tp > max_tokens, S > max_sentences). */
int skv_retain(skv_ctx* ctx, const float* alpha, int32_t Tp, int32_t k, const int32_t* seg_id, int32_t S, int32_t* keep_idx,
               int32_t* n_keep, int32_t* ret_off, int32_t* ret_len);

/* skv_compact_pool: K_ret[l][h][j] = K_pool[l][h][keep_idx[l][j]] for j < n_keep[l], same for V (the pool the paper
 * offloads; here it stays in HBM).  Rows j >= n_keep[l] are not written.
 * K_pool, V_pool dev [L][Hkv][T][D]      K_ret, V_ret dev [L][Hkv][k][D]      keep_idx dev [L][max(k,1)], n_keep dev [L]
 * The retained pool is then used with T = k, sent_off = ret_off + l * (S + 1) and sent_len = ret_len + l * S in
 * skv_build_semvec_layers, skv_select, skv_gather and skv_decode_step. */
int skv_compact_pool(skv_ctx* ctx, const void* K_pool, const void* V_pool, int32_t T, const int32_t* keep_idx, int32_t k,
                     const int32_t* n_keep, void* K_ret, void* V_ret);

/* ---------------------------------------------------------------------------------------------
 * Sec. 4.2 "Sentence-level query aggregation", Eq. 2, and Alg. 1 decoding phase (append q_t to Q_s, compute
 * q-bar, reset Q_s at a sentence boundary).  The sentence cache Q_s is kept as a running sum and a count per
 * sequence (one state per layer, owned by the caller, zero-initialised).  One call per generated token and layer:
 *     q_sum[b] += q_t[b];  q_cnt[b] += 1;  q_bar[b] = q_sum[b] / q_cnt[b]   (fp32, rounded once to kv_dtype)
 *     then, if the generated token tok_t[b] is a terminator (same bitmap convention as skv_segment), the state
 *     of sequence b is cleared, so the next token starts a new sentence.  q_bar still includes the terminator's query.
 * q_t    dev [B][Hq][D] kv_dtype      tok_t  dev [B] int32       term_bitmap dev [ceil(vocab/32)]
 * q_sum  dev [B][Hq][D] fp32 (in/out)  q_cnt  dev [B] int32 (in/out)
 * q_bar  dev [B][Hq][D] kv_dtype (out; pass it as q_score of the calls below).  Asynchronous.
 * Errors: SKV_EINVAL (null / misaligned pointers, B < 1, vocab <= 0), SKV_ECAPACITY (B > max_batch). */
int skv_query_update(skv_ctx* ctx, int32_t B, const void* q_t, const int32_t* tok_t, const uint32_t* term_bitmap,
                     int32_t vocab, float* q_sum, int32_t* q_cnt, void* q_bar);

/* ---------------------------------------------------------------------------------------------
 * (2) Sec. 4.2 "Semantic similarity and token retrieval": score[h][s] = sum over the G query heads j
 * of KV head h of q_score[j]^T semvec[layer][h][s].  No scaling, no normalisation.  q_score is the
 * mean query q-bar of Eq. 2 (or the current query: the choice is the caller's).
 * q_score dev [Hq][D] kv_dtype;  semvec dev [L][Hkv][S][D] semvec_dtype (whole table; `layer` selects the slice);
 * score   dev [Hkv][S] fp32. */
int skv_score(skv_ctx* ctx, int32_t layer, const void* q_score, const void* semvec, int32_t S, float* score);

/* (3) Sec. 4.2 ranking and budgeted retrieval, App. "Effect of Sentence Length": per KV head, buckets
 * are ranked by score (descending; equal scores by ascending id; NaN last; -0 == +0) and whole buckets
 * are taken along the ranking until the first one that does not fit the remaining budget.
 * score    dev [Hkv][S]         sent_off dev [S+1]      sent_len dev [S]
 * sel_sent dev [Hkv][max_sel]   selected bucket ids, ascending; max_sel = min(max_sentences, max_budget)
 * n_sel    dev [Hkv]            tok_idx  dev [Hkv][budget] token positions of the selected buckets, ascending
 * n_tok    dev [Hkv]            (n_tok[h] <= budget).  Entries past n_sel[h] / n_tok[h] are not written.
 * Errors: SKV_EINVAL (budget < 0 ...), SKV_ECAPACITY (S > max_sentences, budget > max_budget). */
int skv_select(skv_ctx* ctx, const float* score, const int32_t* sent_off, const int32_t* sent_len, int32_t S,
               int32_t budget, int32_t* sel_sent, int32_t* n_sel, int32_t* tok_idx, int32_t* n_tok);

/* (4) Alg. 1, decoding phase, the K/V load step: K_sel[h][j][:] = K_pool[layer][h][tok_idx[h][j]][:] for
 * j < n_tok[h], same for V.  Rows j >= n_tok[h] are not written.
 * K_pool, V_pool  [L][Hkv][T][D] kv_dtype, in HBM (pool_in_host == 0) or in pinned, device-mapped host
 *                 memory (pool_in_host == 1: the paper's CPU-offloaded store; the kernel reads it over
 *                 PCIe and the pointer passed is the host pointer).
 * tok_idx dev [Hkv][budget], n_tok dev [Hkv];  K_sel, V_sel dev [Hkv][budget][D] kv_dtype.
 * A tok_idx entry outside [0, T) is skipped, never dereferenced. */
int skv_gather(skv_ctx* ctx, int32_t layer, const void* K_pool, const void* V_pool, int32_t T, int pool_in_host,
               const int32_t* tok_idx, const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel);

/* (5) Eq. 3: out[j] = softmax(q_attn[j] K_sel[h]^T / sqrt(D)) V_sel[h] over the first n_tok[h] rows,
 * h = j / G; lse[j] = log sum_i exp(logit_i) (natural log).  n_tok[h] == 0 gives out = 0 and lse = -inf.
 * Arithmetic: logits, maxima, normalisers and all sums are fp32.  With fp32 K/V the softmax weights stay fp32.  With
 * bf16 K/V the products run on the matrix cores: the weights exp(logit - max) are rounded to bf16 (nearest even)
 * before P.V, and the normaliser sums those rounded weights, so out is exactly the weighted mean the rounded weights
 * define (max-abs error against fp32 weights below 2e-2 for unit-variance values; the same holds for skv_decode_step).
 * q_attn dev [Hq][D] kv_dtype;  K_sel, V_sel dev [Hkv][budget][D];  out dev [Hq][D] fp32;
 * lse dev [Hq] fp32 or NULL. */
int skv_attend(skv_ctx* ctx, const void* q_attn, const void* K_sel, const void* V_sel, const int32_t* n_tok,
               int32_t budget, float* out, float* lse);

/* ---------------------------------------------------------------------------------------------
 * One call per layer for the whole decode chain of Alg. 1 (score -> rank/retrieve -> attend), for a
 * batch of B sequences concatenated along the token axis and the bucket axis.  The retrieved tokens
 * are read straight from the HBM pool (no K_sel/V_sel copy).  Results equal skv_score + skv_select +
 * skv_gather + skv_attend run per sequence: the selection bit for bit, out / lse up to the order of the
 * floating-point sums.
 * Launches per call (P = B * Hkv pairs of sequence and KV head, all sizes from the descriptor's max_budget):
 *   - ONE, when P <= 64 and P * 2^k blocks (2^k the largest power of two with P * 2^k <= 256 compute units) cover the
 *     budget in attention blocks of 128 or 256 tokens (2^k * 256 >= max_budget) and 2^k >= G: the blocks first score the buckets of their pair
 *     between them, pass the scores and later the partial attention results to each other inside the kernel, select
 *     and attend.  The waits inside the kernel are bounded, see skv_set_wait_limit;
 *   - TWO otherwise for bf16 pools (scores; selection + attention in 256-token blocks, or in streaming blocks of 512,
 *     1024 or 2048 tokens when P * ceil(max_budget / 256) exceeds the compute units);
 *   - THREE for fp32 pools with P >= 64 (scores; selection; attention through the positions).
 * In the streaming kernel the order of the floating-point sums can depend on how the hardware schedules a block's
 * waves, so the last bits of out / lse can differ between two identical calls; all other forms are reproducible.
 * q_score, q_attn  dev [B][Hq][D] kv_dtype (may alias)
 * K_pool, V_pool   dev [L][Hkv][T_total][D]        semvec dev [L][Hkv][S_total][D]
 * cu_tok   dev [B+1]  token offset of each sequence in the pool (cu_tok[0] == 0, cu_tok[B] == T_total)
 * cu_sent  dev [B+1]  bucket offset of each sequence (cu_sent[0] == 0, cu_sent[B] == S_total)
 * sent_off dev [S_total + B]  per sequence b, S_b + 1 positions local to the sequence, stored at
 *                             sent_off + cu_sent[b] + b;   sent_len dev [S_total]
 * budget   dev [B]   per-sequence token budget, each <= max_budget
 * out dev [B][Hq][D] fp32;  lse dev [B][Hq] or NULL
 * tok_idx_out dev [B][Hkv][max_budget] or NULL: positions (local to the sequence) of the retrieved
 *             tokens;  n_tok_out dev [B][Hkv] or NULL. */
int skv_decode_step(skv_ctx* ctx, int32_t layer, int32_t B, const void* q_score, const void* q_attn,
                    const void* K_pool, const void* V_pool, int32_t T_total, const void* semvec, int32_t S_total,
                    const int32_t* cu_tok, const int32_t* cu_sent, const int32_t* sent_off, const int32_t* sent_len,
                    const int32_t* budget, float* out, float* lse, int32_t* tok_idx_out, int32_t* n_tok_out);

/* skv_decode_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as skv_decode_step, but no context: the
 * descriptor and the stream are passed with every call, and the workspace (scores, split-K partials, arrival counters)
 * is a static array of SKV_NOALLOC_SCRATCH_BYTES of device memory inside the library, which every GPU the library runs
 * on holds until the process ends.  The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library
 * routine) and never blocks the host; it queues two small clearing kernels (arrival counters, error word) ahead of the
 * kernels of skv_decode_step.  A give-up of the single-launch form (see skv_set_single_launch for what can cause one:
 * other work on the GPU at the same moment) shows as NaN outputs only: there is no context to report it.  The address
 * of the array is looked up once per device, at skv_create or at the first call here on that device (a symbol lookup:
 * make that first call outside graph capture).
 * desc        host; the maxima only need to cover this call (max_tokens is not used for sizing).  The workspace a
 *             descriptor needs is 3.2 MB that every descriptor shares (the tagged words and epochs of the single-launch
 *             form, never cleared) plus about  max_batch * Hq * ceil(max_budget / 64) * 520  +  Hkv * max_sentences * 4
 *             + max_batch * Hkv * (max_budget + min(max_sentences, max_budget)) * 4  bytes
 *             (0.7 MB for 32/8 heads, 2048-token budget, 1332 buckets, one sequence).  The single-launch form is used
 *             when Hkv * max_batch * max_sentences <= 131072; otherwise the call takes the two-launch form.
 * Errors: as skv_decode_step, plus SKV_EINVAL for a bad descriptor and SKV_ECAPACITY when the descriptor needs more
 * than SKV_NOALLOC_SCRATCH_BYTES.
 * All calls on one GPU share the one array, on whatever stream: calls that overlap in time on the same GPU race
 * (order them on one stream or by events).  skv_decode_step with a context is unaffected. */
#define SKV_NOALLOC_SCRATCH_BYTES (8 * 1024 * 1024)
int skv_decode_step_noalloc(const skv_desc* desc, void* hip_stream, int32_t layer, int32_t B, const void* q_score,
                            const void* q_attn, const void* K_pool, const void* V_pool, int32_t T_total, const void* semvec,
                            int32_t S_total, const int32_t* cu_tok, const int32_t* cu_sent, const int32_t* sent_off,
                            const int32_t* sent_len, const int32_t* budget, float* out, float* lse, int32_t* tok_idx_out,
                            int32_t* n_tok_out);

/* Eq. 3 over the union of two disjoint token sets from the two partial results (each side's `out` and `lse` as
 * written by skv_attend or skv_decode_step): out = (Z_a out_a + Z_b out_b) / (Z_a + Z_b), lse = log(Z_a + Z_b),
 * Z = exp(lse).  The paper's Eq. 3 sees the retrieved prompt tokens only; a caller that also keeps a contiguous
 * window of recent tokens resident attends it with skv_attend (K_sel/V_sel = the window's rows) and merges here.
 * A side with lse = -inf is empty and its `out` is ignored; both empty gives out = 0, lse = -inf.
 * n_heads = number of query heads covered (e.g. B * Hq);  out_a, out_b, out dev [n_heads][D] fp32 (out may alias
 * either input);  lse_a, lse_b dev [n_heads];  lse dev [n_heads] or NULL.  Asynchronous.
 * Errors: SKV_EINVAL (null / misaligned pointers, n_heads < 1), SKV_ECAPACITY (n_heads > max_batch * Hq). */
int skv_merge_lse(skv_ctx* ctx, int32_t n_heads, const float* out_a, const float* lse_a, const float* out_b, const float* lse_b,
                  float* out, float* lse);

#ifdef __cplusplus
}
#endif
#endif /* SENTENCEKV_H */
