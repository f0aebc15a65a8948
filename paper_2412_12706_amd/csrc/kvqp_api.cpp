// Host side of the C ABI: argument validation, size queries, launch order.
// Every entry point validates on the host before anything is enqueued, so a
// bad call can never reach a kernel with shapes it does not expect.
#include <hip/hip_runtime.h>

#include "kvqp_internal.h"

namespace kvqp {
namespace {

bool is_pow2_group(int g) { return g == 32 || g == 64 || g == 128; }

// Checks of the fields every entry point reads.
int check_common(const kvqp_cfg* c) {
    if (!c) return KVQP_ERR_INVALID_ARG;
    if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1) return KVQP_ERR_INVALID_ARG;
    if (c->n_q_heads % c->n_kv_heads) return KVQP_ERR_INVALID_ARG;
    if (!(c->bits == 2 || c->bits == 4 || c->bits == 8 || c->bits == 16)) return KVQP_ERR_INVALID_ARG;
    if (c->key_axis != KVQP_KEY_PER_CHANNEL && c->key_axis != KVQP_KEY_PER_TOKEN) return KVQP_ERR_INVALID_ARG;
    if (c->decode_splits < 0) return KVQP_ERR_INVALID_ARG;
    if (c->bits != 16) {
        if (c->group_size < 1 || c->head_dim % c->group_size) return KVQP_ERR_INVALID_ARG;
    }
    if (!(c->sm_scale > 0.0f) || c->sm_scale > 3.0e38f) return KVQP_ERR_INVALID_ARG;   /* positive and finite */
    if (!(c->outlier_threshold >= 0.0f) || c->outlier_threshold > 3.0e38f) return KVQP_ERR_INVALID_ARG;
    if (c->outlier_threshold > 0.0f && c->bits == 16) return KVQP_ERR_INVALID_ARG;   /* nothing is quantized at 16 bits */
    if (c->decode_cache_hint < KVQP_CACHE_AUTO || c->decode_cache_hint > KVQP_CACHE_KEEP) return KVQP_ERR_INVALID_ARG;
    if (c->outlier_overflow_cap < 0 || c->outlier_overflow_cap > (1 << 28)) return KVQP_ERR_INVALID_ARG;
    const int gq = c->n_q_heads / c->n_kv_heads;
    if (c->head_dim != kHeadDim) return KVQP_ERR_UNSUPPORTED;
    if (!(gq == 1 || gq == 2 || gq == 4 || gq == 8)) return KVQP_ERR_UNSUPPORTED;
    if (c->bits != 16 && !is_pow2_group(c->group_size)) return KVQP_ERR_UNSUPPORTED;
    if ((long long)c->batch * c->n_kv_heads > 65535) return KVQP_ERR_UNSUPPORTED;   // (batch, kv head) is the y index of every launch
    return KVQP_OK;
}

// Checks of the prompt-side fields (compress, quantize_selected, sizes).
int check_prompt(const kvqp_cfg* c) {
    if (c->seq_len < 1 || c->window < 1 || c->window > c->seq_len) return KVQP_ERR_INVALID_ARG;
    if (c->pool_kernel < 1 || c->pool_kernel % 2 == 0) return KVQP_ERR_INVALID_ARG;
    if (c->budget < 0) return KVQP_ERR_INVALID_ARG;
    const int gq = c->n_q_heads / c->n_kv_heads;
    if (c->window * gq > 256 || c->pool_kernel > 63) return KVQP_ERR_UNSUPPORTED;
    if (c->seq_len - c->window > 131072) return KVQP_ERR_UNSUPPORTED;   // selection sweeps at most 128 rows of 1024 candidates
    return KVQP_OK;
}

int n_kept_of(const kvqp_cfg* c) {
    const int P = c->seq_len - c->window;
    return c->budget < P ? c->budget : P;
}

// Any count is fine: a partly filled last block and a short last key group are part of the format.
int check_n_kept(const kvqp_cfg* c, int n_kept) {
    (void)c;
    return n_kept < 0 ? KVQP_ERR_INVALID_ARG : KVQP_OK;
}

// A non-zero capacity must hold the tokens and keep every head's buffers aligned.
int check_cap(const kvqp_cfg* c, int n_cap, int n_kept) {
    if (n_cap == 0) return KVQP_OK;
    if (n_cap < n_kept || n_cap % 64) return KVQP_ERR_INVALID_ARG;
    if (c->bits != 16 && n_cap % c->group_size) return KVQP_ERR_INVALID_ARG;
    return KVQP_OK;
}

int fill_sizes(const kvqp_cfg* cfg, int n_tok, int32_t tail_cap, size_t sizes_out[8]) {
    const size_t heads = (size_t)cfg->batch * cfg->n_kv_heads;
    const size_t km = k_meta_elems(n_tok, cfg->bits, cfg->group_size, cfg->key_axis) * 2 * heads;
    const size_t vm = v_meta_elems(n_tok, cfg->bits, cfg->group_size) * 2 * heads;
    const size_t tail = heads * (size_t)tail_cap * kHeadDim * 2;
    sizes_out[0] = k_code_words(n_tok, cfg->bits) * 4 * heads;
    sizes_out[1] = v_code_words(n_tok, cfg->bits) * 4 * heads;
    sizes_out[2] = km; sizes_out[3] = km;
    sizes_out[4] = vm; sizes_out[5] = vm;
    sizes_out[6] = tail; sizes_out[7] = tail;
    return KVQP_OK;
}

int check_cache_ptrs(const kvqp_cfg* c, const kvqp_cache* cache, int n_kept, bool need_tail) {
    if (!cache) return KVQP_ERR_INVALID_ARG;
    if (check_cap(c, cache->n_cap, n_kept)) return KVQP_ERR_INVALID_ARG;
    if (n_kept > 0) {
        if (!cache->k_codes || !cache->v_codes) return KVQP_ERR_INVALID_ARG;
        if (c->bits != 16 && (!cache->k_scale || !cache->k_zero || !cache->v_scale || !cache->v_zero))
            return KVQP_ERR_INVALID_ARG;
        if (outliers_on(*c) && (!cache->k_out || !cache->v_out || !cache->k_ovf || !cache->v_ovf)) return KVQP_ERR_INVALID_ARG;
    }
    if (need_tail && (!cache->tail_k || !cache->tail_v)) return KVQP_ERR_INVALID_ARG;
    return KVQP_OK;
}

}  // namespace
}  // namespace kvqp

using namespace kvqp;

extern "C" {

int kvqp_version(void) { return 500; }

const char* kvqp_strerror(int code) {
    switch (code) {
        case KVQP_OK: return "ok";
        case KVQP_ERR_INVALID_ARG: return "invalid argument";
        case KVQP_ERR_UNSUPPORTED: return "configuration not supported by this build";
        case KVQP_ERR_WORKSPACE: return "workspace missing or too small";
        case KVQP_ERR_HIP: return "HIP runtime error";
        default: return "unknown error code";
    }
}

int kvqp_cache_sizes(const kvqp_cfg* cfg, int32_t tail_cap, size_t sizes_out[8]) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if ((rc = check_prompt(cfg))) return rc;
    if (!sizes_out || tail_cap < cfg->window) return KVQP_ERR_INVALID_ARG;
    const int n_kept = n_kept_of(cfg);
    if ((rc = check_n_kept(cfg, n_kept))) return rc;
    return fill_sizes(cfg, n_kept, tail_cap, sizes_out);
}

int kvqp_cache_sizes_cap(const kvqp_cfg* cfg, int32_t n_cap, int32_t tail_cap, size_t sizes_out[8]) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!sizes_out || tail_cap < 0 || n_cap < 0) return KVQP_ERR_INVALID_ARG;
    if (n_cap > 0 && (rc = check_cap(cfg, n_cap, 0))) return rc;
    return fill_sizes(cfg, n_cap, tail_cap, sizes_out);
}

int kvqp_outlier_sizes(const kvqp_cfg* cfg, int32_t n_cap, size_t sizes_out[4]) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!sizes_out || n_cap < 0) return KVQP_ERR_INVALID_ARG;
    int n = n_cap;
    if (n == 0) {
        if ((rc = check_prompt(cfg))) return rc;
        n = n_kept_of(cfg);
    }
    const size_t heads = (size_t)cfg->batch * cfg->n_kv_heads;
    const size_t bytes = outliers_on(*cfg) ? heads * (size_t)rows32(n) * KVQP_OUTLIER_SLOTS * sizeof(uint32_t) : 0;
    const size_t list = outliers_on(*cfg) ? heads * ovf_words(n, cfg->outlier_overflow_cap) * sizeof(uint32_t) : 0;
    sizes_out[0] = bytes; sizes_out[1] = bytes;
    sizes_out[2] = list; sizes_out[3] = list;
    return KVQP_OK;
}

int kvqp_workspace_bytes(const kvqp_cfg* cfg, size_t* compress_bytes, size_t* decode_bytes) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if ((rc = check_prompt(cfg))) return rc;
    const int n_kept = n_kept_of(cfg);
    if ((rc = check_n_kept(cfg, n_kept))) return rc;
    if (compress_bytes) *compress_bytes = plan_compress(*cfg).total;
    // decode: covers every token count, so a cache that grows by appended tokens never outgrows it
    if (decode_bytes) *decode_bytes = decode_ws_bound(*cfg);
    return KVQP_OK;
}

// Host check of head-level counts against their bound.
static int check_head_counts(const kvqp_cfg* cfg, const int32_t* counts, int bound) {
    const int heads = cfg->batch * cfg->n_kv_heads;
    for (int h = 0; h < heads; ++h)
        if (counts[h] < 0 || counts[h] > bound) return KVQP_ERR_INVALID_ARG;
    return KVQP_OK;
}

static int quantize_selected_impl(const kvqp_cfg* cfg, const void* k, const void* v, const int32_t* idx, int32_t n_kept,
                                  const int32_t* head_count, kvqp_cache* cache, void* hip_stream) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if ((rc = check_prompt(cfg))) return rc;
    if ((rc = check_n_kept(cfg, n_kept))) return rc;
    if (!k || !v || (n_kept > 0 && !idx)) return KVQP_ERR_INVALID_ARG;
    if (n_kept > cfg->seq_len - cfg->window) return KVQP_ERR_INVALID_ARG;
    if ((rc = check_cache_ptrs(cfg, cache, n_kept, true))) return rc;
    if (cache->tail_cap < cfg->window) return KVQP_ERR_INVALID_ARG;
    if ((head_count != nullptr) != (cache->head_n_kept != nullptr)) return KVQP_ERR_INVALID_ARG;
    if (head_count && (rc = check_head_counts(cfg, head_count, n_kept))) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (head_count && upload_counts(cache->head_n_kept, head_count, cfg->batch * cfg->n_kv_heads, stream) != hipSuccess)
        return KVQP_ERR_HIP;
    if (launch_quant_pack(*cfg, k, v, idx, n_kept, cache->head_n_kept, *cache, stream) != hipSuccess) return KVQP_ERR_HIP;
    cache->n_kept = n_kept;
    cache->tail_len = cfg->window;
    return KVQP_OK;
}

int kvqp_quantize_selected(const kvqp_cfg* cfg, const void* k, const void* v, const int32_t* idx, int32_t n_kept,
                           kvqp_cache* cache, void* hip_stream) {
    return quantize_selected_impl(cfg, k, v, idx, n_kept, nullptr, cache, hip_stream);
}

int kvqp_quantize_selected_ragged(const kvqp_cfg* cfg, const void* k, const void* v, const int32_t* idx, int32_t n_kept,
                                  const int32_t* head_count, kvqp_cache* cache, void* hip_stream) {
    if (!head_count) return KVQP_ERR_INVALID_ARG;
    return quantize_selected_impl(cfg, k, v, idx, n_kept, head_count, cache, hip_stream);
}

// Both forms of compression: head_budget == NULL is the uniform one.
static int compress_impl(const kvqp_cfg* cfg, const void* q_obs, const void* k, const void* v, const int32_t* head_budget,
                         kvqp_cache* cache, int32_t* idx_out, int32_t* unrefined_out, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if ((rc = check_prompt(cfg))) return rc;
    const int n_kept = n_kept_of(cfg);
    if ((rc = check_n_kept(cfg, n_kept))) return rc;
    if (!q_obs || !k || !v) return KVQP_ERR_INVALID_ARG;
    if ((rc = check_cache_ptrs(cfg, cache, n_kept, true))) return rc;
    if (cache->tail_cap < cfg->window) return KVQP_ERR_INVALID_ARG;
    if ((head_budget != nullptr) != (cache->head_n_kept != nullptr)) return KVQP_ERR_INVALID_ARG;
    const int heads = cfg->batch * cfg->n_kv_heads;
    bool score = n_kept < cfg->seq_len - cfg->window;
    if (head_budget) {
        if ((rc = check_head_counts(cfg, head_budget, n_kept))) return rc;
        score = false;
        for (int h = 0; h < heads; ++h)
            if (head_budget[h] > 0 && head_budget[h] < cfg->seq_len - cfg->window) score = true;
    }
    const CompressPlan plan = plan_compress(*cfg);
    if (!workspace || workspace_bytes < plan.total) return KVQP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15) != 0) return KVQP_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    int32_t* idx = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + plan.off_idx);
    if (head_budget && upload_counts(cache->head_n_kept, head_budget, heads, stream) != hipSuccess) return KVQP_ERR_HIP;
    if (n_kept == 0 && unrefined_out && upload_counts(unrefined_out, nullptr, heads, stream) != hipSuccess) return KVQP_ERR_HIP;   // nothing is cut
    if (n_kept > 0) {
        if (launch_select(*cfg, q_obs, k, idx, unrefined_out, workspace, plan, cache->head_n_kept, score, stream) != hipSuccess) return KVQP_ERR_HIP;
        if (idx_out) {
            const size_t bytes = (size_t)heads * n_kept * sizeof(int32_t);
            if (hipMemcpyAsync(idx_out, idx, bytes, hipMemcpyDeviceToDevice, stream) != hipSuccess) return KVQP_ERR_HIP;
        }
    }
    if (launch_quant_pack(*cfg, k, v, idx, n_kept, cache->head_n_kept, *cache, stream) != hipSuccess) return KVQP_ERR_HIP;
    cache->n_kept = n_kept;
    cache->tail_len = cfg->window;
    return KVQP_OK;
}

int kvqp_compress(const kvqp_cfg* cfg, const void* q_obs, const void* k, const void* v, kvqp_cache* cache,
                  int32_t* idx_out, int32_t* unrefined_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return compress_impl(cfg, q_obs, k, v, nullptr, cache, idx_out, unrefined_out, workspace, workspace_bytes, hip_stream);
}

int kvqp_compress_ragged(const kvqp_cfg* cfg, const void* q_obs, const void* k, const void* v, const int32_t* head_budget,
                         kvqp_cache* cache, int32_t* idx_out, int32_t* unrefined_out, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    if (!head_budget) return KVQP_ERR_INVALID_ARG;
    return compress_impl(cfg, q_obs, k, v, head_budget, cache, idx_out, unrefined_out, workspace, workspace_bytes, hip_stream);
}

// Both forms of the decode-time update: head_count == NULL is the uniform one.
static int append_impl(const kvqp_cfg* cfg, kvqp_cache* cache, int32_t n_tokens, const int32_t* head_count, void* hip_stream) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!cache || n_tokens < 1) return KVQP_ERR_INVALID_ARG;
    if (cache->n_kept < 0 || cache->tail_len < 0 || cache->tail_len > cache->tail_cap) return KVQP_ERR_INVALID_ARG;
    if (n_tokens > cache->tail_len) return KVQP_ERR_INVALID_ARG;
    // whole value superblocks and, for per-channel keys, whole key groups
    int quantum = cfg->bits == 2 ? 64 : 32;
    if (cfg->bits != 16 && cfg->key_axis == KVQP_KEY_PER_CHANNEL && cfg->group_size > quantum) quantum = cfg->group_size;
    if (n_tokens % quantum || cache->n_kept % quantum) return KVQP_ERR_INVALID_ARG;
    const int cap = cache->n_cap > 0 ? cache->n_cap : cache->n_kept;
    if (cache->n_kept + n_tokens > cap) return KVQP_ERR_INVALID_ARG;
    if ((rc = check_cache_ptrs(cfg, cache, cache->n_kept + n_tokens, true))) return rc;
    const int heads = cfg->batch * cfg->n_kv_heads;
    if (head_count) {
        for (int h = 0; h < heads; ++h)
            if (head_count[h] < 0 || head_count[h] > cache->n_kept || head_count[h] % quantum) return KVQP_ERR_INVALID_ARG;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    if (launch_append_tail(*cfg, *cache, n_tokens, head_count ? quantum : 0, stream) != hipSuccess) return KVQP_ERR_HIP;
    // (the new counts are stored after the quantizer, which takes its positions from the old ones)
    if (head_count && upload_counts(cache->head_n_kept, head_count, heads, stream, n_tokens) != hipSuccess) return KVQP_ERR_HIP;
    cache->n_kept += n_tokens;
    cache->tail_len -= n_tokens;
    return KVQP_OK;
}

int kvqp_append_tail(const kvqp_cfg* cfg, kvqp_cache* cache, int32_t n_tokens, void* hip_stream) {
    if (cache && cache->head_n_kept) return KVQP_ERR_UNSUPPORTED;   // head-level counts: kvqp_append_tail_ragged
    return append_impl(cfg, cache, n_tokens, nullptr, hip_stream);
}

int kvqp_append_tail_ragged(const kvqp_cfg* cfg, kvqp_cache* cache, int32_t n_tokens, const int32_t* head_count,
                            void* hip_stream) {
    if (!head_count || !cache || !cache->head_n_kept) return KVQP_ERR_INVALID_ARG;
    return append_impl(cfg, cache, n_tokens, head_count, hip_stream);
}

// Checks shared by both decode entry points; the plan comes back through *plan.
static int check_decode(const kvqp_cfg* cfg, const void* q, const kvqp_cache* cache, const void* out, DecodePlan* plan) {
    int rc = check_common(cfg);
    if (rc) return rc;
    if (!q || !out || !cache) return KVQP_ERR_INVALID_ARG;
    if (cache->n_kept < 0 || cache->tail_len < 0 || cache->tail_len > cache->tail_cap) return KVQP_ERR_INVALID_ARG;
    if (cache->n_kept + cache->tail_len < 1) return KVQP_ERR_INVALID_ARG;
    if (cache->head_n_kept && cache->tail_len < 1) return KVQP_ERR_INVALID_ARG;   // a head may hold no packed token at all
    if ((rc = check_n_kept(cfg, cache->n_kept))) return rc;
    if ((rc = check_cache_ptrs(cfg, cache, cache->n_kept, cache->tail_len > 0))) return rc;
    *plan = plan_decode(*cfg, cache->n_kept, cache->tail_len);
    return KVQP_OK;
}

int kvqp_decode_attn(const kvqp_cfg* cfg, const void* q, const kvqp_cache* cache, void* out, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
    DecodePlan plan;
    const int rc = check_decode(cfg, q, cache, out, &plan);
    if (rc) return rc;
    if (!workspace || workspace_bytes < plan.ws_bytes) return KVQP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15) != 0) return KVQP_ERR_INVALID_ARG;
    if (launch_decode(*cfg, q, *cache, out, workspace, plan, (hipStream_t)hip_stream) != hipSuccess) return KVQP_ERR_HIP;
    return KVQP_OK;
}

int kvqp_decode_attn_static(const kvqp_cfg* cfg, const void* q, const kvqp_cache* cache, void* out, void* hip_stream) {
    DecodePlan plan;
    const int rc = check_decode(cfg, q, cache, out, &plan);
    if (rc) return rc;
    if (plan.ws_bytes > kStaticScratchBytes) return KVQP_ERR_WORKSPACE;   // beyond the library's array: use kvqp_decode_attn
    void* ws = nullptr;
    if (static_scratch(*cfg, &ws, (hipStream_t)hip_stream) != hipSuccess) return KVQP_ERR_HIP;
    if (launch_decode(*cfg, q, *cache, out, ws, plan, (hipStream_t)hip_stream) != hipSuccess) return KVQP_ERR_HIP;
    return KVQP_OK;
}

int kvqp_decode_workspace_init(const kvqp_cfg* cfg, void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = check_common(cfg);
    if (rc) return rc;
    if (!workspace || workspace_bytes < decode_ws_header_bytes(*cfg)) return KVQP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15) != 0) return KVQP_ERR_INVALID_ARG;
    if (launch_ws_init(*cfg, workspace, (hipStream_t)hip_stream) != hipSuccess) return KVQP_ERR_HIP;
    return KVQP_OK;
}

}  // extern "C"
