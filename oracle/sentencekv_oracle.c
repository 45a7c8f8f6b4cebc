/*
 * SentenceKV CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded implementation of what the SentenceKV hot path computes,
 * written from the paper's definitions (arxiv 2504.00970).  It exists only so that the HIP
 * kernels can be checked against it; nothing in the product path may call it.  It shares no
 * source, header, table or helper with the HIP library.
 *
 * Arithmetic: REAL (float unless built with -DSKVO_REAL=double), one operation at a time in the
 * order written (build with -ffp-contract=off, no -ffast-math).  bf16 inputs are widened exactly.
 * Semantic vectors and scores are stored as float in both builds.
 *
 * Steps (names follow the paper's notation):
 *   skvo_segment  sentence buckets from a token stream          (Sec. 4.1 "split ... into sentences
 *                                                                according to punctuation"; Alg. 1 prefill)
 *   skvo_token_importance  alpha_i from the observation window  (Sec. 4.1 "Token importance measurement")
 *   skvo_retain   global top floor(r tau) tokens and the buckets of the retained tokens
 *                                                               (Sec. 4.1 "Token selection within sentence buckets";
 *                                                                App. "Effect of Sentence Length")
 *   skvo_semvec   mean key vector k-bar_{s,h} per bucket, head  (Eq. 1)
 *   skvo_query_cache_step  sentence cache Q_s and its mean query q-bar  (Sec. 4.2 "Sentence-level query aggregation",
 *                                                                Eq. 2; Alg. 1 decoding phase)
 *   skvo_score    S(q-bar, k-bar_{s,h}) = q-bar^T k-bar_{s,h}   (Sec. 4.2 "Semantic similarity and token retrieval")
 *   skvo_select   rank buckets by score, take whole buckets in descending order until the token
 *                 budget tau is reached                        (Sec. 4.2; App. "Effect of Sentence Length")
 *   skvo_gather   K_tau, V_tau = rows of the selected tokens    (Sec. 4.2 retrieval; Alg. 1, decoding phase, K/V load step)
 *   skvo_attend   O = softmax(q K_tau^T / sqrt(d)) V_tau        (Eq. 3)
 *   skvo_merge_lse  Eq. 3 over the union of two disjoint token sets from the two partial results
 *
 * Readings taken where the paper is silent (each is a documented constant of this oracle):
 *   - the terminator set is input data (a bitmap over the vocabulary);
 *   - a sentence ends WITH its terminator; trailing tokens after the last terminator form a
 *     final sentence; a terminator at the last position opens no empty sentence; every
 *     terminator closes a sentence (runs of terminators give length-1 sentences);
 *   - S_s of Eq. 1 is the whole sentence (the KV pool is the full context);
 *   - with grouped-query attention one selection is made per KV head and the bucket score is
 *     the sum over the G query heads of the group of q-bar_j^T k-bar_{s,h}; query head j uses
 *     KV head floor(j / G);
 *   - no scaling or normalisation of the score;
 *   - buckets are taken in (score descending, id ascending) order and the walk stops at the
 *     first bucket that does not fit the remaining budget (no skipping ahead, no partial
 *     bucket); NaN scores rank lowest; -0 == +0;
 *   - gathered tokens are in ascending position order;
 *   - an empty selection gives O = 0 and lse = -inf;
 *   - observation window: the window queries see every earlier token and, causally, the window itself (the
 *     attention of the model's forward pass); alpha_i is defined for the tokens before the window only and sums the
 *     probabilities over the window's queries and over ALL query heads, so one set of tokens is retained per layer;
 *     no pooling of alpha; the window's own tokens are not part of the retained pool;
 *   - a bucket none of whose tokens is retained does not exist: its length is 0, its mean key vector is stored as
 *     zeros, and the selection never lists it;
 *   - the query of the token that ends a generated sentence still belongs to that sentence: Q_s is
 *     reset after q-bar of that step has been formed; q-bar is rounded once to the storage type.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (hand-built streams,
 * float64 brute force from raw keys, an independent O(S^2) characterisation of the selection,
 * dense softmax attention in float64 when tau >= T).  The readings listed above are fixed by
 * this file and its documentation only: the paper prints no worked numerical example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef SKVO_REAL
#define SKVO_REAL float
#endif
typedef SKVO_REAL real;

enum { SKVO_F32 = 0, SKVO_BF16 = 1, SKVO_FP8 = 2 };   /* FP8 = the 8-bit E4M3 format of the OCP specification */

/* E4M3 (1 sign, 4 exponent bits with bias 7, 3 fraction bits; no infinities, 0x7f / 0xff are NaN, largest finite value
 * 448): the value of a code, written out from the format's definition. */
static float from_e4m3(uint8_t code) {
    int e = (code >> 3) & 15, m = code & 7;
    float mag;
    if (e == 0) mag = (float)m * 0.001953125f;                       /* subnormal: m * 2^-9 */
    else {
        mag = 1.0f + (float)m * 0.125f;
        for (int i = 7; i < e; ++i) mag *= 2.0f;                     /* 2^(e-7), exact */
        for (int i = e; i < 7; ++i) mag *= 0.5f;
    }
    return (code & 0x80) ? -mag : mag;
}

/* nearest E4M3 value to a finite float, ties to the even code, magnitudes beyond the format saturate at 448 */
static uint8_t to_e4m3(float f) {
    uint8_t sign = f < 0.0f || (f == 0.0f && 1.0f / f < 0.0f) ? 0x80 : 0x00;
    float a = f < 0.0f ? -f : f;
    uint8_t lo = 0, best = 0;
    /* the codes 0x00..0x7e are increasing in value: find the last one not above a (bisection), then compare with its
     * successor */
    int first = 0, last = 0x7e;
    while (first < last) {
        int mid = (first + last + 1) / 2;
        if (from_e4m3((uint8_t)mid) <= a) first = mid; else last = mid - 1;
    }
    lo = (uint8_t)first;
    if (lo == 0x7e) best = lo;                                       /* at or beyond 448 */
    else {
        float below = from_e4m3(lo), above = from_e4m3((uint8_t)(lo + 1));
        float d0 = a - below, d1 = above - a;                        /* exact: neighbouring values, a between them */
        if (d0 < d1) best = lo;
        else if (d0 > d1) best = (uint8_t)(lo + 1);
        else best = (lo & 1) ? (uint8_t)(lo + 1) : lo;
    }
    return (uint8_t)(sign | best);
}

/* exact widening of one stored element to REAL */
static real load_elt(const void* base, int dtype, int64_t i) {
    if (dtype == SKVO_F32) return (real)((const float*)base)[i];
    if (dtype == SKVO_FP8) return (real)from_e4m3(((const uint8_t*)base)[i]);
    uint32_t bits = ((uint32_t)((const uint16_t*)base)[i]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (real)f;
}

static size_t elt_size(int dtype) { return dtype == SKVO_F32 ? 4u : dtype == SKVO_FP8 ? 1u : 2u; }

static int is_terminator(const uint32_t* bitmap, int32_t vocab, int32_t id) {
    if (id < 0 || id >= vocab) return 0;
    return (int)((bitmap[id >> 5] >> (id & 31)) & 1u);
}

/* nearest bf16 to a finite float, ties to the even bit pattern */
static uint16_t to_bf16(float f) {
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    uint32_t below = bits & 0xffff0000u;             /* neighbour towards zero */
    uint32_t above = below + 0x00010000u;            /* neighbour away from zero */
    uint32_t rest = bits & 0x0000ffffu;              /* distance from `below`, in units of 2^-16 bf16 ulp */
    uint32_t pick;
    if (rest < 0x8000u) pick = below;
    else if (rest > 0x8000u) pick = above;
    else pick = ((below >> 16) & 1u) ? above : below;
    return (uint16_t)(pick >> 16);
}

/* Sec. 4.1 / Alg. 1 prefill: sentence buckets.  seg_id[i] = number of terminators strictly before i.
 * sent_off has room for cap_sent + 1 entries, sent_len for cap_sent.  *n_sent receives S even if
 * S > cap_sent (then only the first cap_sent buckets are written and -1 is returned). */
int skvo_segment(const int32_t* tok, int32_t T, const uint32_t* bitmap, int32_t vocab,
                 int32_t* seg_id, int32_t* sent_off, int32_t* sent_len, int32_t cap_sent, int32_t* n_sent) {
    int32_t seg = 0, start = 0;
    for (int32_t i = 0; i < T; ++i) {
        seg_id[i] = seg;
        int closes = is_terminator(bitmap, vocab, tok[i]) || i == T - 1;
        if (closes) {
            if (seg < cap_sent) {
                sent_off[seg] = start;
                sent_len[seg] = i + 1 - start;
            }
            start = i + 1;
            seg++;
        }
    }
    *n_sent = seg;
    if (seg <= cap_sent) sent_off[seg] = T;
    return seg <= cap_sent ? 0 : -1;
}

/* The two conversions on arrays, for the tests that pin them. */
void skvo_e4m3_encode(const float* x, int64_t n, uint8_t* code) { for (int64_t i = 0; i < n; ++i) code[i] = to_e4m3(x[i]); }
void skvo_e4m3_decode(const uint8_t* code, int64_t n, float* x) { for (int64_t i = 0; i < n; ++i) x[i] = from_e4m3(code[i]); }

/* Eq. 1: semvec[l][h][s][:] = (1/|S_s|) sum_{x in S_s} k_{x,h}, S_s = the tokens of bucket s in the pool.
 * sv_dtype selects the storage of the table: float, or bf16 or E4M3 (the float mean rounded once, to nearest even: the
 * mixed-precision sentence vectors the paper names as future work). */
void skvo_semvec_to(const void* K, int dtype, int32_t L, int32_t Hkv, int32_t T, int32_t D,
                    const int32_t* sent_off, int32_t S, int sv_dtype, void* semvec) {
    real* acc = (real*)malloc(sizeof(real) * (size_t)D);
    for (int32_t l = 0; l < L; ++l)
        for (int32_t h = 0; h < Hkv; ++h)
            for (int32_t s = 0; s < S; ++s) {
                int32_t b = sent_off[s], e = sent_off[s + 1];
                for (int32_t d = 0; d < D; ++d) acc[d] = 0;
                for (int32_t x = b; x < e; ++x) {
                    int64_t row = (((int64_t)l * Hkv + h) * T + x) * D;
                    for (int32_t d = 0; d < D; ++d) acc[d] = acc[d] + load_elt(K, dtype, row + d);
                }
                real n = (real)(e - b);
                int64_t o = (((int64_t)l * Hkv + h) * S + s) * D;
                for (int32_t d = 0; d < D; ++d) {
                    float mean = e > b ? (float)(acc[d] / n) : 0.0f;   /* no retained token: no bucket */
                    if (sv_dtype == SKVO_F32) ((float*)semvec)[o + d] = mean;
                    else if (sv_dtype == SKVO_FP8) ((uint8_t*)semvec)[o + d] = to_e4m3(mean);
                    else ((uint16_t*)semvec)[o + d] = to_bf16(mean);
                }
            }
    free(acc);
}

void skvo_semvec(const void* K, int dtype, int32_t L, int32_t Hkv, int32_t T, int32_t D,
                 const int32_t* sent_off, int32_t S, float* semvec) {
    skvo_semvec_to(K, dtype, L, Hkv, T, D, sent_off, S, SKVO_F32, semvec);
}

/* Sec. 4.2 "Sentence-level query aggregation", Eq. 2, Alg. 1 decoding phase.  Q_s is kept literally: a list of
 * the query vectors of the tokens generated since the last sentence boundary (cache is [cap][per], *n_cached
 * entries used; per = Hq * D elements of one token's queries).  One call = one generated token:
 *   append q_t to Q_s;  q-bar = (1/|Q_s|) sum_{t in Q_s} q_t, summed in the order of generation;
 *   if the generated token is a terminator, Q_s is emptied for the next sentence.
 * qbar_real receives the mean as float; qbar_store (nullable) the same rounded to the storage type.
 * Returns -1 (and changes nothing) if Q_s is full. */
int skvo_query_cache_step(const void* q_t, int dtype, int32_t per, int32_t tok, const uint32_t* bitmap, int32_t vocab,
                          float* cache, int32_t cap, int32_t* n_cached, float* qbar_real, void* qbar_store) {
    int32_t n = *n_cached;
    if (n >= cap) return -1;
    for (int32_t i = 0; i < per; ++i) cache[(int64_t)n * per + i] = (float)load_elt(q_t, dtype, i);
    n = n + 1;
    for (int32_t i = 0; i < per; ++i) {
        real sum = 0;
        for (int32_t t = 0; t < n; ++t) sum = sum + (real)cache[(int64_t)t * per + i];
        float mean = (float)(sum / (real)n);
        qbar_real[i] = mean;
        if (qbar_store) {
            if (dtype == SKVO_F32) ((float*)qbar_store)[i] = mean;
            else ((uint16_t*)qbar_store)[i] = to_bf16(mean);
        }
    }
    *n_cached = is_terminator(bitmap, vocab, tok) ? 0 : n;
    return 0;
}

/* Sec. 4.2: score[h][s] = sum_{g<G} q[hG+g]^T semvec[h][s]  (one layer; semvec is [Hkv][S][D], float or bf16). */
void skvo_score_from(const void* q, int dtype, int32_t Hq, int32_t Hkv, int32_t D,
                     const void* semvec, int sv_dtype, int32_t S, float* score) {
    int32_t G = Hq / Hkv;
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t s = 0; s < S; ++s) {
            int64_t kbar = ((int64_t)h * S + s) * D;
            real acc = 0;
            for (int32_t g = 0; g < G; ++g)
                for (int32_t d = 0; d < D; ++d) {
                    real prod = load_elt(q, dtype, (int64_t)(h * G + g) * D + d) * load_elt(semvec, sv_dtype, kbar + d);
                    acc = acc + prod;
                }
            score[(int64_t)h * S + s] = (float)acc;
        }
}

void skvo_score(const void* q, int dtype, int32_t Hq, int32_t Hkv, int32_t D,
                const float* semvec, int32_t S, float* score) {
    skvo_score_from(q, dtype, Hq, Hkv, D, semvec, SKVO_F32, S, score);
}

/* ranking order of the buckets: higher score first, NaN last, equal scores by lower id */
typedef struct { float score; int32_t id; } ranked;

static int rank_before(const void* pa, const void* pb) {
    const ranked* a = (const ranked*)pa;
    const ranked* b = (const ranked*)pb;
    int an = isnan(a->score), bn = isnan(b->score);
    if (an != bn) return an ? 1 : -1;
    if (!an) {
        if (a->score > b->score) return -1;
        if (a->score < b->score) return 1;
    }
    return (a->id > b->id) - (a->id < b->id);
}

static int by_id(const void* pa, const void* pb) {
    int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
    return (a > b) - (a < b);
}

/* Sec. 4.2 ranking + budgeted retrieval, per KV head.  score is [Hkv][S].  Outputs per head h:
 * sel_sent[h][0..n_sel[h]) selected bucket ids ascending (row stride max_sel), tok_idx[h][0..n_tok[h])
 * their token positions ascending (row stride budget_stride). */
void skvo_select(const float* score, const int32_t* sent_off, const int32_t* sent_len, int32_t S,
                 int32_t Hkv, int32_t budget, int32_t* sel_sent, int32_t max_sel, int32_t* n_sel,
                 int32_t* tok_idx, int32_t budget_stride, int32_t* n_tok) {
    ranked* order = (ranked*)malloc(sizeof(ranked) * (size_t)(S > 0 ? S : 1));
    int32_t* chosen = (int32_t*)malloc(sizeof(int32_t) * (size_t)(S > 0 ? S : 1));
    for (int32_t h = 0; h < Hkv; ++h) {
        for (int32_t s = 0; s < S; ++s) {
            order[s].score = score[(int64_t)h * S + s];
            order[s].id = s;
        }
        qsort(order, (size_t)S, sizeof(ranked), rank_before);
        int32_t used = 0, cnt = 0;
        for (int32_t r = 0; r < S; ++r) {
            int32_t len = sent_len[order[r].id];
            if (len <= 0) continue;                  /* a bucket without retained tokens does not exist */
            if (used + len > budget) break;          /* first bucket that does not fit ends the walk */
            used += len;
            chosen[cnt++] = order[r].id;
        }
        qsort(chosen, (size_t)cnt, sizeof(int32_t), by_id);
        int32_t w = 0;
        for (int32_t c = 0; c < cnt; ++c) {
            int32_t s = chosen[c];
            if (c < max_sel) sel_sent[(int64_t)h * max_sel + c] = s;
            for (int32_t x = sent_off[s]; x < sent_off[s] + sent_len[s]; ++x)
                tok_idx[(int64_t)h * budget_stride + w++] = x;
        }
        n_sel[h] = cnt;
        n_tok[h] = w;
    }
    free(order);
    free(chosen);
}

/* Sec. 4.1 "Token importance measurement" for one layer.  The last N tokens of the prompt (positions Tp .. T-1,
 * Tp = T - N) are the observation window.  Window query n of query head j (KV head floor(j/G)) attends, as in the
 * model's forward pass, to the keys of positions 0 .. Tp + n with softmax(q k / sqrt(D)); alpha_i, i < Tp, is the
 * sum of the probabilities token i receives from all N window queries of all Hq heads.
 * q_obs [Hq][N][D], K [Hkv][T][D] (dtype), alpha [Tp] float. */
void skvo_token_importance(const void* q_obs, const void* K, int dtype, int32_t Hq, int32_t Hkv, int32_t T,
                           int32_t N, int32_t D, float* alpha) {
    int32_t Tp = T - N, G = Hq / Hkv;
    if (Tp <= 0) return;
    real* total = (real*)calloc((size_t)Tp, sizeof(real));
    real* logit = (real*)malloc(sizeof(real) * (size_t)T);
    real inv_sqrt_d = (real)1 / (real)sqrt((double)D);
    for (int32_t j = 0; j < Hq; ++j) {
        int32_t h = j / G;
        for (int32_t n = 0; n < N; ++n) {
            int32_t visible = Tp + n + 1;                      /* keys of positions 0 .. Tp + n */
            real m = -INFINITY;
            for (int32_t x = 0; x < visible; ++x) {
                real dot = 0;
                for (int32_t d = 0; d < D; ++d) {
                    real prod = load_elt(q_obs, dtype, ((int64_t)j * N + n) * D + d) * load_elt(K, dtype, ((int64_t)h * T + x) * D + d);
                    dot = dot + prod;
                }
                logit[x] = dot * inv_sqrt_d;
                if (logit[x] > m) m = logit[x];
            }
            real z = 0;
            for (int32_t x = 0; x < visible; ++x) z = z + (real)exp((double)(logit[x] - m));
            for (int32_t i = 0; i < Tp; ++i) total[i] = total[i] + (real)exp((double)(logit[i] - m)) / z;
        }
    }
    for (int32_t i = 0; i < Tp; ++i) alpha[i] = (float)total[i];
    free(total);
    free(logit);
}

/* Sec. 4.1 "Token selection within sentence buckets", App. "Effect of Sentence Length": the floor(r tau) = k tokens
 * with the highest alpha over the whole prefix are retained, regardless of sentence boundaries (equal alpha: lower
 * position first; NaN last).  keep_idx [min(k, Tp)] receives their positions in ascending order.  The buckets of
 * the retained pool keep the numbering of the prompt's buckets: ret_len[s] = retained tokens of bucket s (0 for a
 * bucket that vanished), ret_off[s] = retained tokens of all earlier buckets, ret_off[S] = n_keep.
 * seg_id [>= Tp] as produced by skvo_segment. */
void skvo_retain(const float* alpha, int32_t Tp, int32_t k, const int32_t* seg_id, int32_t S,
                 int32_t* keep_idx, int32_t* n_keep, int32_t* ret_off, int32_t* ret_len) {
    int32_t keep = k < Tp ? k : Tp;
    if (keep < 0) keep = 0;
    ranked* order = (ranked*)malloc(sizeof(ranked) * (size_t)(Tp > 0 ? Tp : 1));
    for (int32_t i = 0; i < Tp; ++i) { order[i].score = alpha[i]; order[i].id = i; }
    qsort(order, (size_t)(Tp > 0 ? Tp : 0), sizeof(ranked), rank_before);
    for (int32_t r = 0; r < keep; ++r) keep_idx[r] = order[r].id;
    qsort(keep_idx, (size_t)keep, sizeof(int32_t), by_id);
    for (int32_t s = 0; s < S; ++s) ret_len[s] = 0;
    for (int32_t r = 0; r < keep; ++r) ret_len[seg_id[keep_idx[r]]] += 1;
    ret_off[0] = 0;
    for (int32_t s = 0; s < S; ++s) ret_off[s + 1] = ret_off[s] + ret_len[s];
    *n_keep = keep;
    free(order);
}

/* Alg. 1, decoding phase, the K/V load step: row copy.
 * pool is one layer [Hkv][T][D]; dst is [Hkv][budget_stride][D]; rows >= n_tok[h] are left untouched. */
void skvo_gather(const void* pool, int dtype, int32_t Hkv, int32_t T, int32_t D,
                 const int32_t* tok_idx, int32_t budget_stride, const int32_t* n_tok, void* dst) {
    size_t row = (size_t)D * elt_size(dtype);
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t j = 0; j < n_tok[h]; ++j) {
            int32_t x = tok_idx[(int64_t)h * budget_stride + j];
            memcpy((char*)dst + ((size_t)h * budget_stride + j) * row,
                   (const char*)pool + ((size_t)h * T + x) * row, row);
        }
}

/* Eq. 3 for every query head j (KV head floor(j/G)): two-pass softmax over the gathered tokens.
 * K_sel, V_sel are [Hkv][budget_stride][D]; out is [Hq][D]; lse (nullable) is [Hq]. */
void skvo_attend(const void* q, const void* K_sel, const void* V_sel, int dtype,
                 int32_t Hq, int32_t Hkv, int32_t D, const int32_t* n_tok, int32_t budget_stride,
                 float* out, float* lse) {
    int32_t G = Hq / Hkv;
    int32_t max_n = 0;
    for (int32_t h = 0; h < Hkv; ++h) if (n_tok[h] > max_n) max_n = n_tok[h];
    real* logit = (real*)malloc(sizeof(real) * (size_t)(max_n > 0 ? max_n : 1));
    real* acc = (real*)malloc(sizeof(real) * (size_t)D);
    real scale = sizeof(real) == sizeof(float) ? (real)(1.0f / sqrtf((float)D)) : (real)(1.0 / sqrt((double)D));
    for (int32_t j = 0; j < Hq; ++j) {
        int32_t h = j / G, n = n_tok[h];
        if (n <= 0) {
            for (int32_t d = 0; d < D; ++d) out[(int64_t)j * D + d] = 0.0f;
            if (lse) lse[j] = -INFINITY;
            continue;
        }
        real m = -INFINITY;
        for (int32_t i = 0; i < n; ++i) {
            int64_t row = ((int64_t)h * budget_stride + i) * D;
            real dot = 0;
            for (int32_t d = 0; d < D; ++d) {
                real prod = load_elt(q, dtype, (int64_t)j * D + d) * load_elt(K_sel, dtype, row + d);
                dot = dot + prod;
            }
            logit[i] = dot * scale;
            if (logit[i] > m) m = logit[i];
        }
        real denom = 0;
        for (int32_t d = 0; d < D; ++d) acc[d] = 0;
        for (int32_t i = 0; i < n; ++i) {
            int64_t row = ((int64_t)h * budget_stride + i) * D;
            real p = sizeof(real) == sizeof(float) ? (real)expf((float)(logit[i] - m))
                                                   : (real)exp((double)(logit[i] - m));
            denom = denom + p;
            for (int32_t d = 0; d < D; ++d) {
                real prod = p * load_elt(V_sel, dtype, row + d);
                acc[d] = acc[d] + prod;
            }
        }
        for (int32_t d = 0; d < D; ++d) out[(int64_t)j * D + d] = (float)(acc[d] / denom);
        if (lse)
            lse[j] = sizeof(real) == sizeof(float) ? (float)m + logf((float)denom)
                                                   : (float)((double)m + log((double)denom));
    }
    free(logit);
    free(acc);
}

/* Eq. 3 over the union of two disjoint token sets A and B, given each side's output and log-sum-exp:
 * softmax over A u B weights side A by Z_A / (Z_A + Z_B) with Z = exp(lse).  A side with lse = -inf is empty.
 * out_a, out_b, out are [n_heads][D]; lse_a, lse_b, lse are [n_heads]. */
void skvo_merge_lse(const float* out_a, const float* lse_a, const float* out_b, const float* lse_b, int32_t n_heads,
                    int32_t D, float* out, float* lse) {
    for (int32_t j = 0; j < n_heads; ++j) {
        real la = (real)lse_a[j], lb = (real)lse_b[j];
        real m = la > lb ? la : lb;
        if (!(m > -INFINITY)) {                       /* both sides empty */
            for (int32_t d = 0; d < D; ++d) out[(int64_t)j * D + d] = 0.0f;
            lse[j] = -INFINITY;
            continue;
        }
        real za = (real)exp((double)(la - m)), zb = (real)exp((double)(lb - m));   /* exp(-inf) = 0 */
        real z = za + zb;
        for (int32_t d = 0; d < D; ++d) {
            real a = za > 0 ? za * (real)out_a[(int64_t)j * D + d] : 0;
            real b = zb > 0 ? zb * (real)out_b[(int64_t)j * D + d] : 0;
            out[(int64_t)j * D + d] = (float)((a + b) / z);
        }
        lse[j] = (float)(m + (real)log((double)z));
    }
}

/* size of REAL in this build (4 = float, 8 = double), so a loader can tell the two libraries apart */
int skvo_real_bytes(void) { return (int)sizeof(real); }
