// C ABI of libsentencekv: context management, host-side argument checks, and the launch sequence of
// every entry point declared in sentencekv.h.  All checks run before anything touches the GPU.
#include <mutex>
#include <new>

#include "skv_internal.h"

using skv::Ctx;
using skv::SeqView;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad_ptr(const void* p) { return p == nullptr || !aligned16(p); }
inline size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

int check_desc(const skv_desc* d) {
    if (!d) return SKV_EINVAL;
    if (d->n_layers < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1) return SKV_EINVAL;
    if (d->head_dim != skv::kHeadDim) return SKV_EINVAL;
    if (d->kv_dtype != SKV_F32 && d->kv_dtype != SKV_BF16) return SKV_EINVAL;
    if (d->semvec_dtype != SKV_F32 && d->semvec_dtype != SKV_BF16 && d->semvec_dtype != SKV_FP8_E4M3) return SKV_EINVAL;
    if (d->n_q_heads % d->n_kv_heads != 0) return SKV_EINVAL;
    const int G = d->n_q_heads / d->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return SKV_EINVAL;
    if (d->max_tokens < 1 || d->max_sentences < 1 || d->max_budget < 1 || d->max_batch < 1) return SKV_EINVAL;
    if (d->max_batch > 4096) return SKV_EINVAL;
    if ((int64_t)d->max_batch * d->n_kv_heads > 65535) return SKV_EINVAL;    // (sequence, head) pairs are a grid dimension
    return SKV_OK;
}

inline int hip_status(hipError_t e) {
    if (e == hipSuccess) return SKV_OK;
    return e == hipErrorOutOfMemory ? SKV_ENOMEM : SKV_EHIP;
}

// The context belongs to one device; refuse calls made with another device current.
int check_ctx(const skv_ctx* ctx) {
    if (!ctx) return SKV_EINVAL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SKV_EHIP;
    return dev == ctx->c.device ? SKV_OK : SKV_EINVAL;
}

inline int64_t layer_elems(const Ctx& c, int64_t rows) { return (int64_t)c.d.n_kv_heads * rows * skv::kHeadDim; }
inline int elt_bytes(const Ctx& c) { return c.d.kv_dtype == SKV_BF16 ? 2 : 4; }
inline int sv_bytes(const Ctx& c) { return c.d.semvec_dtype == SKV_BF16 ? 2 : c.d.semvec_dtype == SKV_FP8_E4M3 ? 1 : 4; }


// ---- workspace: one block of device memory, carved the same way whether skv_create allocated it or it is the static
// scratch array of skv_decode_step_noalloc ---------------------------------------------------------------------------
constexpr int kWsParts = 14;
// Fixed sizes of the tagged area (epochs, tagged scores, tagged partials) in the static scratch of
// skv_decode_step_noalloc: that area must hold tagged words only, whatever descriptor a call brings (a word of some
// other array could look like a valid tag), so it has the same extent for every descriptor.
constexpr size_t kFixedEpochBytes = (size_t)skv::kStepMaxPairs * skv::kStepEpochStride * sizeof(unsigned int);
constexpr size_t kFixedScoreWords = 128 * 1024;
constexpr size_t kFixedPartBytes = (size_t)skv::kStepMaxBlocks * 8 * skv::kStepPartWords * sizeof(unsigned long long);

// fixed_tagged: the static-scratch form.  *score_stride receives the words per pair of the tagged scores.
size_t workspace_layout(const skv_desc& d, int max_splits, int max_sel, bool fixed_tagged, size_t sz[kWsParts], int32_t* score_stride) {
    const size_t BH = (size_t)d.max_batch * d.n_kv_heads, BQ = (size_t)d.max_batch * d.n_q_heads;
    const size_t n_seg = (size_t)(d.max_tokens + skv::kSegTokPerBlock - 1) / skv::kSegTokPerBlock;
    const size_t step_pairs = BH < (size_t)skv::kStepMaxPairs ? BH : (size_t)skv::kStepMaxPairs;
    const int G = d.n_q_heads / d.n_kv_heads;
    *score_stride = d.max_sentences;
    sz[0] = kFixedEpochBytes;                                                      // step_epoch
    if (fixed_tagged) {
        sz[1] = kFixedScoreWords * sizeof(unsigned long long);                     // step_score
        sz[2] = kFixedPartBytes;                                                   // step_part
    } else {
        sz[1] = round256(step_pairs * (size_t)d.max_sentences * sizeof(unsigned long long));
        sz[2] = round256((size_t)skv::kStepMaxBlocks * G * skv::kStepPartWords * sizeof(unsigned long long));
    }
    sz[3] = round256(n_seg * sizeof(unsigned long long));                          // seg_part
    sz[4] = round256(BQ * max_splits * skv::kHeadDim * sizeof(float));             // att_part
    sz[5] = round256(BQ * max_splits * 2 * sizeof(float));                         // att_ml
    sz[6] = round256(BH * sizeof(unsigned int));                                   // att_counter
    sz[7] = round256((size_t)d.n_kv_heads * d.max_sentences * sizeof(float));      // f_score
    sz[8] = round256(BH * max_sel * sizeof(int32_t));                              // f_sel_sent
    sz[9] = round256(BH * sizeof(int32_t));                                        // f_n_sel
    sz[10] = round256(BH * sizeof(int32_t));                                       // f_n_tok
    sz[11] = round256(BH * d.max_budget * sizeof(int32_t));                        // f_tok_idx
    sz[12] = 256;                                                                  // err_dev
    sz[13] = 0;
    size_t total = 0;
    for (int i = 0; i < kWsParts; ++i) total += sz[i];
    return total;
}

void carve_workspace(Ctx& c, char* base, const size_t sz[kWsParts], int32_t score_stride) {
    char* p = base;
    c.step_epoch = reinterpret_cast<unsigned int*>(p); p += sz[0];
    c.step_score = reinterpret_cast<unsigned long long*>(p); p += sz[1];
    c.step_part = reinterpret_cast<unsigned long long*>(p); p += sz[2];
    c.step_score_stride = score_stride;
    c.step_score_words = (int64_t)(sz[1] / sizeof(unsigned long long));
    c.seg_part = reinterpret_cast<unsigned long long*>(p); p += sz[3];
    c.att_part = reinterpret_cast<float*>(p); p += sz[4];
    c.att_ml = reinterpret_cast<float*>(p); p += sz[5];
    c.att_counter = reinterpret_cast<unsigned int*>(p); p += sz[6];
    c.f_score = reinterpret_cast<float*>(p); p += sz[7];
    c.f_sel_sent = reinterpret_cast<int32_t*>(p); p += sz[8];
    c.f_n_sel = reinterpret_cast<int32_t*>(p); p += sz[9];
    c.f_n_tok = reinterpret_cast<int32_t*>(p); p += sz[10];
    c.f_tok_idx = reinterpret_cast<int32_t*>(p); p += sz[11];
    c.err_dev = reinterpret_cast<unsigned int*>(p); p += sz[12];
}

void fill_context(Ctx& c, const skv_desc& d, hipStream_t stream, int dev) {
    c.d = d;
    c.stream = stream;
    c.device = dev;
    c.n_cu = skv::kComputeUnits;
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n_cu > 0) c.n_cu = n_cu;
    c.G = d.n_q_heads / d.n_kv_heads;
    c.max_sel = d.max_sentences < d.max_budget ? d.max_sentences : d.max_budget;
    c.max_splits = (d.max_budget + skv::kAttChunk - 1) / skv::kAttChunk;
    c.budget_cap = d.max_budget;
    c.wait_limit = skv::kStepWaitLimit;
    c.single_launch = true;
}

// ---- static scratch of skv_decode_step_noalloc -----------------------------------------------------------------------
// Device memory that exists from the moment the code object is loaded on a GPU until the process ends: nothing is
// allocated for it at run time.  Every GPU holds its own copy at its own address; `scratch` below is only the host-side
// handle of the symbol and must never be used as an address.  static_scratch() resolves the address once per device
// (with that device current) and every use goes through the pointer it returns.
constexpr size_t kStaticScratchBytes = (size_t)SKV_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices];      // per device; null until resolved

// Device address of the scratch array on device `dev`, which must be the current device.  out may be null.
int static_scratch(int dev, char** out) {
    if (dev < 0 || dev >= kMaxDevices) return SKV_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SKV_EHIP;
        }
        g_scratch_ptr[dev] = static_cast<char*>(p);
    }
    if (out) *out = g_scratch_ptr[dev];
    return SKV_OK;
}

// Clears `n` 32-bit words (a kernel rather than a memset node: the call may be recorded into a HIP graph).
__global__ void clear_words_kernel(unsigned int* __restrict__ p, int32_t n) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace

extern "C" {

const char* skv_strerror(int status) {
    switch (status) {
        case SKV_OK: return "ok";
        case SKV_EINVAL: return "invalid argument";
        case SKV_ECAPACITY: return "size exceeds the capacity (the maxima given at skv_create, or the static scratch of skv_decode_step_noalloc)";
        case SKV_EHIP: return "HIP runtime error";
        case SKV_ENOMEM: return "out of device memory";
        default: return "unknown status";
    }
}

int skv_create(skv_ctx** out, const skv_desc* desc, void* hip_stream) {
    if (!out) return SKV_EINVAL;
    *out = nullptr;
    const int rc = check_desc(desc);
    if (rc != SKV_OK) return rc;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SKV_EHIP;

    skv_ctx* ctx = new (std::nothrow) skv_ctx();
    if (!ctx) return SKV_ENOMEM;
    Ctx& c = ctx->c;
    fill_context(c, *desc, static_cast<hipStream_t>(hip_stream), dev);

    size_t sz[kWsParts];
    int32_t score_stride = 0;
    const size_t total = workspace_layout(*desc, c.max_splits, c.max_sel, false, sz, &score_stride);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c.ws), total);
    if (e != hipSuccess) { delete ctx; return hip_status(e); }
    e = hipMemset(c.ws, 0, total);
    if (e != hipSuccess) { (void)hipFree(c.ws); delete ctx; return hip_status(e); }
    c.ws_bytes = total;
    carve_workspace(c, c.ws, sz, score_stride);
    // a word of pinned host memory the kernels can reach: a block of the single-launch step that gives up waiting sets
    // it, and the next skv_decode_step on this context reports it
    void* eh = nullptr;
    e = hipHostMalloc(&eh, sizeof(unsigned int), hipHostMallocMapped);
    if (e == hipSuccess) {
        void* ed = nullptr;
        *static_cast<unsigned int*>(eh) = 0u;
        if (hipHostGetDevicePointer(&ed, eh, 0) == hipSuccess) {
            c.err_host = static_cast<unsigned int*>(eh);
            c.err_host_dev = static_cast<unsigned int*>(ed);
        } else {
            (void)hipGetLastError();
            (void)hipHostFree(eh);
        }
    } else {
        (void)hipGetLastError();           // without the word errors are still visible as NaN outputs
    }
    (void)static_scratch(dev, nullptr);     // set-up call with the device current: resolve the static scratch too (best effort)
    *out = ctx;
    return SKV_OK;
}

void skv_destroy(skv_ctx* ctx) {
    if (!ctx) return;
    if (ctx->c.ws) {
        (void)hipStreamSynchronize(ctx->c.stream);
        (void)hipFree(ctx->c.ws);
    }
    if (ctx->c.err_host) (void)hipHostFree(ctx->c.err_host);
    delete ctx;
}

int skv_set_stream(skv_ctx* ctx, void* hip_stream) {
    if (!ctx) return SKV_EINVAL;
    ctx->c.stream = static_cast<hipStream_t>(hip_stream);
    return SKV_OK;
}

int64_t skv_workspace_bytes(const skv_ctx* ctx) { return ctx ? (int64_t)ctx->c.ws_bytes : 0; }

int skv_set_budget_hint(skv_ctx* ctx, int32_t budget) {
    if (!ctx || budget < 0) return SKV_EINVAL;
    if (budget > ctx->c.d.max_budget) return SKV_ECAPACITY;
    ctx->c.budget_cap = budget == 0 ? ctx->c.d.max_budget : budget;
    return SKV_OK;
}

int skv_set_single_launch(skv_ctx* ctx, int32_t enable) {
    if (!ctx) return SKV_EINVAL;
    ctx->c.single_launch = enable != 0;
    return SKV_OK;
}

int skv_set_wait_limit(skv_ctx* ctx, int32_t polls) {
    if (!ctx || polls < 0) return SKV_EINVAL;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    Ctx& c = ctx->c;
    c.wait_limit = polls;
    // a reported give-up is cleared: the device word in stream order, the host word once the stream has drained
    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, c.stream, c.err_dev, 1);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(c.stream) != hipSuccess) return SKV_EHIP;
    if (c.err_host) *c.err_host = 0u;
    return SKV_OK;
}

int skv_segment(skv_ctx* ctx, const int32_t* tok, int32_t T, const uint32_t* term_bitmap, int32_t vocab,
                int32_t* seg_id, int32_t* sent_off, int32_t* sent_len, int32_t* n_sent_dev, int32_t* n_sent_host) {
    if (!ctx) return SKV_EINVAL;
    if (T < 0 || vocab <= 0) return SKV_EINVAL;
    if (bad_ptr(tok) || bad_ptr(term_bitmap) || bad_ptr(seg_id) || bad_ptr(sent_off) || bad_ptr(sent_len) ||
        bad_ptr(n_sent_dev))
        return SKV_EINVAL;
    if (T > ctx->c.d.max_tokens) return SKV_ECAPACITY;
    int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    rc = hip_status(skv::launch_segment(&ctx->c, tok, T, term_bitmap, vocab, seg_id, sent_off, sent_len, n_sent_dev));
    if (rc != SKV_OK || !n_sent_host) return rc;
    hipError_t e = hipMemcpyAsync(n_sent_host, n_sent_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->c.stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->c.stream);
    if (e != hipSuccess) return SKV_EHIP;
    return *n_sent_host > ctx->c.d.max_sentences ? SKV_ECAPACITY : SKV_OK;
}

int skv_build_semvec(skv_ctx* ctx, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t S, void* semvec) {
    if (!ctx) return SKV_EINVAL;
    if (T < 0 || S < 0) return SKV_EINVAL;
    if (S > 0 && (bad_ptr(K_pool) || bad_ptr(sent_off) || bad_ptr(semvec))) return SKV_EINVAL;
    if (S > T) return SKV_EINVAL;                       // every bucket holds at least one token
    if (T > ctx->c.d.max_tokens || S > ctx->c.d.max_sentences) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_semvec(&ctx->c, K_pool, T, sent_off, 0, S, semvec));
}

int skv_build_semvec_layers(skv_ctx* ctx, const void* K_pool, int32_t T, const int32_t* sent_off, int32_t S, void* semvec) {
    if (!ctx) return SKV_EINVAL;
    if (T < 0 || S < 0) return SKV_EINVAL;
    if (S > 0 && (bad_ptr(K_pool) || bad_ptr(sent_off) || bad_ptr(semvec))) return SKV_EINVAL;
    if (T > ctx->c.d.max_tokens || S > ctx->c.d.max_sentences) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_semvec(&ctx->c, K_pool, T, sent_off, S + 1, S, semvec));
}

int64_t skv_token_importance_work_bytes(const skv_ctx* ctx, int32_t T, int32_t N) {
    if (!ctx || T < 1 || N < 1 || N >= T || ctx->c.G * N > skv::kImportanceMaxRows) return -1;
    return (int64_t)round256((size_t)skv::importance_work_bytes(&ctx->c, T, N));
}

int skv_token_importance(skv_ctx* ctx, const void* q_obs, const void* K_pool, int32_t T, int32_t N, float* alpha, void* work,
                         int64_t work_bytes) {
    if (!ctx) return SKV_EINVAL;
    if (T < 1 || N < 1 || N >= T) return SKV_EINVAL;
    if (ctx->c.G * N > skv::kImportanceMaxRows) return SKV_ECAPACITY;
    if (bad_ptr(q_obs) || bad_ptr(K_pool) || bad_ptr(alpha) || bad_ptr(work)) return SKV_EINVAL;
    if (T > ctx->c.d.max_tokens) return SKV_ECAPACITY;
    if (work_bytes < skv::importance_work_bytes(&ctx->c, T, N)) return SKV_EINVAL;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_importance(&ctx->c, q_obs, K_pool, T, N, alpha, work));
}

int skv_retain(skv_ctx* ctx, const float* alpha, int32_t Tp, int32_t k, const int32_t* seg_id, int32_t S, int32_t* keep_idx,
               int32_t* n_keep, int32_t* ret_off, int32_t* ret_len) {
    if (!ctx) return SKV_EINVAL;
    if (Tp < 1 || k < 0 || S < 1) return SKV_EINVAL;
    if (bad_ptr(alpha) || bad_ptr(seg_id) || bad_ptr(keep_idx) || bad_ptr(n_keep) || bad_ptr(ret_off) || bad_ptr(ret_len))
        return SKV_EINVAL;
    if (Tp > ctx->c.d.max_tokens || S > ctx->c.d.max_sentences) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_retain(&ctx->c, alpha, Tp, k, seg_id, S, keep_idx, n_keep, ret_off, ret_len));
}

int skv_compact_pool(skv_ctx* ctx, const void* K_pool, const void* V_pool, int32_t T, const int32_t* keep_idx, int32_t k,
                     const int32_t* n_keep, void* K_ret, void* V_ret) {
    if (!ctx) return SKV_EINVAL;
    if (T < 1 || k < 0) return SKV_EINVAL;
    if (k > 0 && (bad_ptr(K_pool) || bad_ptr(V_pool) || bad_ptr(keep_idx) || bad_ptr(n_keep) || bad_ptr(K_ret) || bad_ptr(V_ret)))
        return SKV_EINVAL;
    if (T > ctx->c.d.max_tokens) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_compact_pool(&ctx->c, K_pool, V_pool, T, keep_idx, k, n_keep, K_ret, V_ret));
}

int skv_query_update(skv_ctx* ctx, int32_t B, const void* q_t, const int32_t* tok_t, const uint32_t* term_bitmap,
                     int32_t vocab, float* q_sum, int32_t* q_cnt, void* q_bar) {
    if (!ctx) return SKV_EINVAL;
    if (B < 1 || vocab <= 0) return SKV_EINVAL;
    if (bad_ptr(q_t) || bad_ptr(tok_t) || bad_ptr(term_bitmap) || bad_ptr(q_sum) || bad_ptr(q_cnt) || bad_ptr(q_bar))
        return SKV_EINVAL;
    if (B > ctx->c.d.max_batch) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_query_update(&ctx->c, B, q_t, tok_t, term_bitmap, vocab, q_sum, q_cnt, q_bar));
}

int skv_score(skv_ctx* ctx, int32_t layer, const void* q_score, const void* semvec, int32_t S, float* score) {
    if (!ctx) return SKV_EINVAL;
    if (layer < 0 || layer >= ctx->c.d.n_layers || S < 0) return SKV_EINVAL;
    if (S > 0 && (bad_ptr(q_score) || bad_ptr(semvec) || bad_ptr(score))) return SKV_EINVAL;
    if (S > ctx->c.d.max_sentences) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    const SeqView v{nullptr, nullptr, nullptr, 0, S, 0, 1};
    const char* sv = (const char*)semvec + (int64_t)layer * layer_elems(ctx->c, S) * sv_bytes(ctx->c);
    return hip_status(skv::launch_score(&ctx->c, q_score, sv, v, score));
}

int skv_select(skv_ctx* ctx, const float* score, const int32_t* sent_off, const int32_t* sent_len, int32_t S,
               int32_t budget, int32_t* sel_sent, int32_t* n_sel, int32_t* tok_idx, int32_t* n_tok) {
    if (!ctx) return SKV_EINVAL;
    if (S < 0 || budget < 0) return SKV_EINVAL;
    if (bad_ptr(n_sel) || bad_ptr(n_tok)) return SKV_EINVAL;
    if (S > 0 && budget > 0 &&
        (bad_ptr(score) || bad_ptr(sent_off) || bad_ptr(sent_len) || bad_ptr(sel_sent) || bad_ptr(tok_idx)))
        return SKV_EINVAL;
    if (S > ctx->c.d.max_sentences || budget > ctx->c.d.max_budget) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    const SeqView v{nullptr, nullptr, nullptr, 0, S, budget, 1};
    return hip_status(skv::launch_select(&ctx->c, score, sent_off, sent_len, v, sel_sent, n_sel, tok_idx, budget, budget, n_tok));
}

int skv_gather(skv_ctx* ctx, int32_t layer, const void* K_pool, const void* V_pool, int32_t T, int pool_in_host,
               const int32_t* tok_idx, const int32_t* n_tok, int32_t budget, void* K_sel, void* V_sel) {
    if (!ctx) return SKV_EINVAL;
    if (layer < 0 || layer >= ctx->c.d.n_layers || T < 0 || budget < 0) return SKV_EINVAL;
    if (pool_in_host != 0 && pool_in_host != 1) return SKV_EINVAL;
    if (budget > 0 && (bad_ptr(K_pool) || bad_ptr(V_pool) || bad_ptr(tok_idx) || bad_ptr(n_tok) || bad_ptr(K_sel) ||
                       bad_ptr(V_sel)))
        return SKV_EINVAL;
    if (T > ctx->c.d.max_tokens || budget > ctx->c.d.max_budget) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    if (budget == 0) return SKV_OK;
    const void* Kd = K_pool;
    const void* Vd = V_pool;
    if (pool_in_host) {      // device-visible address of the pinned host allocation
        void *kd = nullptr, *vd = nullptr;
        if (hipHostGetDevicePointer(&kd, const_cast<void*>(K_pool), 0) != hipSuccess ||
            hipHostGetDevicePointer(&vd, const_cast<void*>(V_pool), 0) != hipSuccess) {
            (void)hipGetLastError();
            return SKV_EINVAL;
        }
        Kd = kd;
        Vd = vd;
    }
    const int64_t off = (int64_t)layer * layer_elems(ctx->c, T) * elt_bytes(ctx->c);
    return hip_status(skv::launch_gather(&ctx->c, (const char*)Kd + off, (const char*)Vd + off, T, pool_in_host != 0, tok_idx, n_tok, budget,
                                         K_sel, V_sel));
}

int skv_attend(skv_ctx* ctx, const void* q_attn, const void* K_sel, const void* V_sel, const int32_t* n_tok,
               int32_t budget, float* out, float* lse) {
    if (!ctx) return SKV_EINVAL;
    if (budget < 0) return SKV_EINVAL;
    if (bad_ptr(q_attn) || bad_ptr(n_tok) || bad_ptr(out)) return SKV_EINVAL;
    if (lse && !aligned16(lse)) return SKV_EINVAL;
    if (budget > 0 && (bad_ptr(K_sel) || bad_ptr(V_sel))) return SKV_EINVAL;
    if (budget > ctx->c.d.max_budget) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    const SeqView v{nullptr, nullptr, nullptr, 0, 0, budget, 1};
    return hip_status(skv::launch_attend(&ctx->c, q_attn, K_sel, V_sel, budget, n_tok, budget, v, out, lse));
}

// Host-side checks of skv_decode_step (nothing has touched the GPU yet).
static int decode_step_check(const Ctx& c, int32_t layer, int32_t B, const void* q_score, const void* q_attn, const void* K_pool,
                             const void* V_pool, int32_t T_total, const void* semvec, int32_t S_total, const int32_t* cu_tok,
                             const int32_t* cu_sent, const int32_t* sent_off, const int32_t* sent_len, const int32_t* budget,
                             float* out, float* lse, int32_t* tok_idx_out, int32_t* n_tok_out) {
    if (layer < 0 || layer >= c.d.n_layers || B < 1 || T_total < 0 || S_total < 0) return SKV_EINVAL;
    if (bad_ptr(q_score) || bad_ptr(q_attn) || bad_ptr(cu_tok) || bad_ptr(cu_sent) || bad_ptr(sent_off) ||
        bad_ptr(budget) || bad_ptr(out))
        return SKV_EINVAL;
    if (S_total > 0 && (bad_ptr(semvec) || bad_ptr(sent_len))) return SKV_EINVAL;
    if (T_total > 0 && (bad_ptr(K_pool) || bad_ptr(V_pool))) return SKV_EINVAL;
    if ((lse && !aligned16(lse)) || (tok_idx_out && !aligned16(tok_idx_out)) || (n_tok_out && !aligned16(n_tok_out)))
        return SKV_EINVAL;
    if (B > c.d.max_batch || T_total > c.d.max_tokens || S_total > c.d.max_sentences) return SKV_ECAPACITY;
    return SKV_OK;
}

// Launch sequence of skv_decode_step on a checked argument set; `c` holds the workspace pointers to use.
static int decode_step_launch(Ctx& c, int32_t layer, int32_t B, const void* q_score, const void* q_attn, const void* K_pool,
                              const void* V_pool, int32_t T_total, const void* semvec, int32_t S_total, const int32_t* cu_tok,
                              const int32_t* cu_sent, const int32_t* sent_off, const int32_t* sent_len, const int32_t* budget,
                              float* out, float* lse, int32_t* tok_idx_out, int32_t* n_tok_out) {

    // A single sequence spans the whole pool (cu_tok = {0, T_total}, cu_sent = {0, S_total}): the kernels then take the
    // sizes from the arguments instead of loading them, one dependent memory round trip less per launch.
    const SeqView v = B == 1 ? SeqView{nullptr, nullptr, budget, T_total, S_total, 0, 1}
                             : SeqView{cu_tok, cu_sent, budget, T_total, S_total, 0, B};
    const char* sv = (const char*)semvec + (int64_t)layer * layer_elems(c, S_total) * sv_bytes(c);
    const int64_t pool_off = (int64_t)layer * layer_elems(c, T_total) * elt_bytes(c);

    const char* Kl = (const char*)K_pool + pool_off;
    const char* Vl = (const char*)V_pool + pool_off;
    const int pairs = B * c.d.n_kv_heads;
    hipError_t e;
    // Few (sequence, head) pairs: the whole step in one launch, when its attention blocks (128 or 256 tokens) fit the
    // chip at once beside each other; launch_step decides.
    if (c.single_launch && pairs <= skv::kStepMaxPairs && S_total > 0) {
        bool launched = false;
        e = skv::launch_step(&c, q_score, q_attn, sv, Kl, Vl, sent_off, sent_len, v, out, lse, tok_idx_out, n_tok_out, &launched);
        if (launched || e != hipSuccess) return hip_status(e);
    }
    e = skv::launch_score(&c, q_score, sv, v, c.f_score);
    if (e != hipSuccess) return hip_status(e);
    const bool can_stream = c.d.kv_dtype == SKV_BF16 && T_total < (1 << 24);
    const int wide_blocks = pairs * ((c.budget_cap + skv::kAttChunkWide - 1) / skv::kAttChunkWide);
    if (can_stream ? wide_blocks > c.n_cu : pairs >= skv::kWideChunkMinHeads) {
        if (can_stream)
            return hip_status(skv::launch_select_attend_stream(&c, q_attn, Kl, Vl, c.f_score, sent_off, sent_len, v, out, lse,
                                                               tok_idx_out, n_tok_out));
        // batch path: the selection runs once per (sequence, head); attention reads the pool through tok_idx
        int32_t* tok_idx = tok_idx_out ? tok_idx_out : c.f_tok_idx;
        int32_t* n_tok = n_tok_out ? n_tok_out : c.f_n_tok;
        e = skv::launch_select(&c, c.f_score, sent_off, sent_len, v, c.f_sel_sent, c.f_n_sel, tok_idx, c.d.max_budget, c.budget_cap, n_tok);
        if (e != hipSuccess) return hip_status(e);
        return hip_status(skv::launch_attend_indirect(&c, q_attn, Kl, Vl, tok_idx, n_tok, v, out, lse));
    }
    // latency path: every attention block derives the selection itself (no launch, no tok_idx round trip)
    e = skv::launch_select_attend(&c, q_attn, Kl, Vl, c.f_score, sent_off, sent_len, v, out, lse, tok_idx_out, n_tok_out);
    return hip_status(e);
}

int skv_decode_step(skv_ctx* ctx, int32_t layer, int32_t B, const void* q_score, const void* q_attn,
                    const void* K_pool, const void* V_pool, int32_t T_total, const void* semvec, int32_t S_total,
                    const int32_t* cu_tok, const int32_t* cu_sent, const int32_t* sent_off, const int32_t* sent_len,
                    const int32_t* budget, float* out, float* lse, int32_t* tok_idx_out, int32_t* n_tok_out) {
    if (!ctx) return SKV_EINVAL;
    int rc = decode_step_check(ctx->c, layer, B, q_score, q_attn, K_pool, V_pool, T_total, semvec, S_total, cu_tok, cu_sent,
                               sent_off, sent_len, budget, out, lse, tok_idx_out, n_tok_out);
    if (rc != SKV_OK) return rc;
    rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    if (ctx->c.err_host && *static_cast<volatile unsigned int*>(ctx->c.err_host) != 0u) return SKV_EHIP;   // an earlier step gave up waiting
    return decode_step_launch(ctx->c, layer, B, q_score, q_attn, K_pool, V_pool, T_total, semvec, S_total, cu_tok, cu_sent,
                              sent_off, sent_len, budget, out, lse, tok_idx_out, n_tok_out);
}

int skv_decode_step_noalloc(const skv_desc* desc, void* hip_stream, int32_t layer, int32_t B, const void* q_score,
                            const void* q_attn, const void* K_pool, const void* V_pool, int32_t T_total, const void* semvec,
                            int32_t S_total, const int32_t* cu_tok, const int32_t* cu_sent, const int32_t* sent_off,
                            const int32_t* sent_len, const int32_t* budget, float* out, float* lse, int32_t* tok_idx_out,
                            int32_t* n_tok_out) {
    int rc = check_desc(desc);
    if (rc != SKV_OK) return rc;
    Ctx c{};
    // sizes first: everything below is host arithmetic until the scratch address is needed
    c.d = *desc;
    c.G = desc->n_q_heads / desc->n_kv_heads;
    c.max_sel = desc->max_sentences < desc->max_budget ? desc->max_sentences : desc->max_budget;
    c.max_splits = (desc->max_budget + skv::kAttChunk - 1) / skv::kAttChunk;
    rc = decode_step_check(c, layer, B, q_score, q_attn, K_pool, V_pool, T_total, semvec, S_total, cu_tok, cu_sent, sent_off,
                           sent_len, budget, out, lse, tok_idx_out, n_tok_out);
    if (rc != SKV_OK) return rc;
    skv_desc d0 = *desc;
    d0.max_tokens = 1;                                    // the prefill partials are not part of this call
    size_t sz[kWsParts];
    int32_t score_stride = 0;
    if (workspace_layout(d0, c.max_splits, c.max_sel, true, sz, &score_stride) > kStaticScratchBytes) return SKV_ECAPACITY;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SKV_EHIP;
    char* base = nullptr;
    rc = static_scratch(dev, &base);
    if (rc != SKV_OK) return rc;
    fill_context(c, *desc, static_cast<hipStream_t>(hip_stream), dev);
    carve_workspace(c, base, sz, score_stride);
    c.ws = base;
    c.ws_bytes = kStaticScratchBytes;
    // the arrival counters must start at zero; the array keeps whatever the last call on this GPU left there
    // (the tagged area at the start of the array -- epochs, tagged scores, tagged partials of the single-launch step --
    // is never cleared: its words are only ever valid for the launch that wrote them)
    const int32_t n_words = (int32_t)(sz[6] / sizeof(uint32_t));
    hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, c.stream, c.att_counter, n_words);
    if (hipGetLastError() != hipSuccess) return SKV_EHIP;
    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, c.stream, c.err_dev, 1);
    if (hipGetLastError() != hipSuccess) return SKV_EHIP;
    return decode_step_launch(c, layer, B, q_score, q_attn, K_pool, V_pool, T_total, semvec, S_total, cu_tok, cu_sent,
                              sent_off, sent_len, budget, out, lse, tok_idx_out, n_tok_out);
}

int skv_merge_lse(skv_ctx* ctx, int32_t n_heads, const float* out_a, const float* lse_a, const float* out_b, const float* lse_b,
                  float* out, float* lse) {
    if (!ctx) return SKV_EINVAL;
    if (n_heads < 1) return SKV_EINVAL;
    if (bad_ptr(out_a) || bad_ptr(lse_a) || bad_ptr(out_b) || bad_ptr(lse_b) || bad_ptr(out)) return SKV_EINVAL;
    if (lse && !aligned16(lse)) return SKV_EINVAL;
    if (n_heads > ctx->c.d.max_batch * ctx->c.d.n_q_heads) return SKV_ECAPACITY;
    const int rc = check_ctx(ctx);
    if (rc != SKV_OK) return rc;
    return hip_status(skv::launch_merge_lse(&ctx->c, out_a, lse_a, out_b, lse_b, n_heads, out, lse));
}

}  // extern "C"
