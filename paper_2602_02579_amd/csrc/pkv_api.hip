// C ABI of the library: host-side argument checks and dispatch to the kernel
// launchers.  Nothing here touches device memory or synchronises.
#include "pkv_common.h"

#include <cmath>
#include <cstdint>

using namespace pkv;

namespace {

constexpr int64_t kMaxTokens = (int64_t)1 << 30;  // indices are int32

pkv_status check_cfg(const pkv_layer_cfg* cfg) {
    if (!cfg) return PKV_ERR_NULL;
    if (cfg->dtype != PKV_F32 && cfg->dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0 ||
        cfg->hidden <= 0)
        return PKV_ERR_SHAPE;
    if (cfg->n_q_heads % cfg->n_kv_heads) return PKV_ERR_SHAPE;
    if (cfg->head_dim % 16 || cfg->head_dim > 2 * kMaxHalfDim) return PKV_ERR_UNSUPPORTED;
    if (cfg->hidden % 8) return PKV_ERR_UNSUPPORTED;
    if (cfg->n_q_heads + 2 * cfg->n_kv_heads > 65535) return PKV_ERR_UNSUPPORTED;
    if (!(cfg->rope_theta > 0.f) || !std::isfinite(cfg->rope_theta)) return PKV_ERR_SHAPE;
    return PKV_OK;
}

float resolve_scale(float s, int head_dim) {
    return s == 0.f ? 1.0f / std::sqrt((float)head_dim) : s;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" {

pkv_status pkv_rope_restore(const pkv_layer_cfg* cfg, const void* k_in,
                            void* k_out, const int32_t* pos, int64_t pos_base,
                            int64_t n, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (n < 0 || n > kMaxTokens) return PKV_ERR_SHAPE;
    if (n == 0) return PKV_OK;
    if (!k_in || !k_out) return PKV_ERR_NULL;
    if (!pos && (pos_base < -kMaxTokens || pos_base > kMaxTokens)) return PKV_ERR_SHAPE;
    return launch_rope_restore(*cfg, k_in, k_out, pos, pos_base, n, (hipStream_t)stream);
}

pkv_status pkv_query_score(const pkv_layer_cfg* cfg, const void* q, const void* k,
                           float* score, int64_t nq, int64_t n_ctx,
                           float softmax_scale, int accumulate, void* ws,
                           size_t ws_bytes, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (nq <= 0 || n_ctx <= 0 || n_ctx > kMaxTokens || nq > (1 << 20)) return PKV_ERR_SHAPE;
    // the kernels count (query token, head) columns in 32-bit integers
    if (nq * (int64_t)cfg->n_q_heads > INT32_MAX) return PKV_ERR_UNSUPPORTED;
    if (!q || !k || !score) return PKV_ERR_NULL;
    if (!std::isfinite(softmax_scale) || softmax_scale < 0.f) return PKV_ERR_SHAPE;
    const size_t need = align256(query_score_ws_bytes(*cfg, n_ctx, nq));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_query_score(*cfg, q, k, score, nq, n_ctx,
                              resolve_scale(softmax_scale, cfg->head_dim), accumulate,
                              ws, (hipStream_t)stream);
}

pkv_status pkv_query_score_lse(const pkv_layer_cfg* cfg, const void* q, const void* k,
                               const float* lse, const int32_t* row_pos, float* score,
                               int64_t nq, int64_t n_ctx, float softmax_scale,
                               int accumulate, void* ws, size_t ws_bytes, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (nq <= 0 || n_ctx <= 0 || n_ctx > kMaxTokens || nq > kMaxTokens) return PKV_ERR_SHAPE;
    if (nq * (int64_t)cfg->n_q_heads > INT32_MAX) return PKV_ERR_UNSUPPORTED;
    if (!q || !k || !lse || !score) return PKV_ERR_NULL;
    if (!std::isfinite(softmax_scale) || softmax_scale < 0.f) return PKV_ERR_SHAPE;
    const size_t need = align256(query_score_ws_bytes(*cfg, n_ctx, nq));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_query_score_lse(*cfg, q, k, lse, row_pos, score, nq, n_ctx,
                                  resolve_scale(softmax_scale, cfg->head_dim), accumulate,
                                  ws, (hipStream_t)stream);
}

pkv_status pkv_topk_select(const float* score, int64_t n, int64_t k,
                           int32_t* idx_out, void* ws, size_t ws_bytes,
                           void* stream) {
    if (n < 0 || n > kMaxTokens || k < 0 || k > n) return PKV_ERR_SHAPE;
    if (k == 0) return PKV_OK;
    if (!score || !idx_out) return PKV_ERR_NULL;
    // the workspace is optional here: without it long vectors take a one-workgroup kernel
    return launch_topk_select(score, n, k, idx_out, ws, ws ? ws_bytes : 0, (hipStream_t)stream);
}

pkv_status pkv_gather_qkv_proj_ex(const pkv_layer_cfg* cfg, const void* hidden,
                                  const int32_t* row_idx, const int32_t* row_pos,
                                  const void* wq, const void* wk, const void* wv,
                                  const pkv_proj_variant* variant, void* q_out, void* k_out,
                                  void* v_out, int64_t m, void* ws, size_t ws_bytes,
                                  void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (m < 0 || m > kMaxTokens) return PKV_ERR_SHAPE;
    if (variant) {
        if ((variant->q_norm == nullptr) != (variant->k_norm == nullptr)) return PKV_ERR_NULL;
        if (variant->q_norm && (!(variant->norm_eps >= 0.f) || !std::isfinite(variant->norm_eps)))
            return PKV_ERR_SHAPE;
    }
    if (m == 0) return PKV_OK;
    if (!hidden || !row_pos) return PKV_ERR_NULL;
    if ((k_out == nullptr) != (v_out == nullptr)) return PKV_ERR_NULL;
    if (!q_out && !k_out) return PKV_ERR_NULL;
    if (q_out && !wq) return PKV_ERR_NULL;
    if (k_out && (!wk || !wv)) return PKV_ERR_NULL;
    const size_t need = align256(gather_qkv_proj_ws_bytes(*cfg, m));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_gather_qkv_proj(*cfg, hidden, row_idx, row_pos, wq, wk, wv, variant, nullptr,
                                  q_out, k_out, v_out, m, ws, (hipStream_t)stream);
}

pkv_status pkv_gather_qkv_proj_scatter(const pkv_layer_cfg* cfg, const void* hidden,
                                       const int32_t* row_idx, const int32_t* row_pos,
                                       const void* wq, const void* wk, const void* wv,
                                       const pkv_proj_variant* variant, void* q_out,
                                       void* k_cache, void* v_cache, const int32_t* dst_row,
                                       int64_t m, int64_t n_cache, void* ws, size_t ws_bytes,
                                       void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (m < 0 || m > kMaxTokens || n_cache < 0 || n_cache > kMaxTokens || m > n_cache)
        return PKV_ERR_SHAPE;
    if (variant) {
        if ((variant->q_norm == nullptr) != (variant->k_norm == nullptr)) return PKV_ERR_NULL;
        if (variant->q_norm && (!(variant->norm_eps >= 0.f) || !std::isfinite(variant->norm_eps)))
            return PKV_ERR_SHAPE;
    }
    if (m == 0) return PKV_OK;
    if (!hidden || !row_pos || !wk || !wv || !k_cache || !v_cache || !dst_row)
        return PKV_ERR_NULL;
    if (q_out && !wq) return PKV_ERR_NULL;
    const size_t need = align256(gather_qkv_proj_ws_bytes(*cfg, m));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_gather_qkv_proj(*cfg, hidden, row_idx, row_pos, wq, wk, wv, variant, dst_row,
                                  q_out, k_cache, v_cache, m, ws, (hipStream_t)stream);
}

pkv_status pkv_gather_qkv_proj(const pkv_layer_cfg* cfg, const void* hidden,
                               const int32_t* row_idx, const int32_t* row_pos,
                               const void* wq, const void* wk, const void* wv,
                               void* q_out, void* k_out, void* v_out, int64_t m,
                               void* ws, size_t ws_bytes, void* stream) {
    return pkv_gather_qkv_proj_ex(cfg, hidden, row_idx, row_pos, wq, wk, wv, nullptr, q_out,
                                  k_out, v_out, m, ws, ws_bytes, stream);
}

pkv_status pkv_scatter_kv(const pkv_layer_cfg* cfg, const void* k_new,
                          const void* v_new, const int32_t* dst_row, void* k_cache,
                          void* v_cache, int64_t m, int64_t n_cache, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (m < 0 || n_cache < 0 || n_cache > kMaxTokens || m > n_cache) return PKV_ERR_SHAPE;
    if (m == 0) return PKV_OK;
    if (!k_new || !v_new || !dst_row || !k_cache || !v_cache) return PKV_ERR_NULL;
    return launch_scatter_kv(*cfg, k_new, v_new, dst_row, k_cache, v_cache, m,
                             (hipStream_t)stream);
}

pkv_status pkv_sparse_row_attn(const pkv_layer_cfg* cfg, const void* q,
                               const void* k_cache, const void* v_cache,
                               const int32_t* row_pos, void* out, float* lse_out,
                               int64_t m, int64_t n_keys, float softmax_scale,
                               void* ws, size_t ws_bytes, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (m < 0 || m > kMaxTokens || n_keys <= 0 || n_keys > kMaxTokens) return PKV_ERR_SHAPE;
    // byte offsets inside one kv head's K rows and transposed V rows are 32-bit in the
    // matrix-core kernels: head_dim * (keys rounded up to 64) * 2 bytes must fit
    if (cfg->dtype == PKV_BF16 &&
        (int64_t)cfg->head_dim * ((n_keys + 63) / 64 * 64) * 2 >= ((int64_t)1 << 32))
        return PKV_ERR_UNSUPPORTED;
    if (m * (int64_t)cfg->n_q_heads > INT32_MAX) return PKV_ERR_UNSUPPORTED;
    if (m == 0) return PKV_OK;
    if (!q || !k_cache || !v_cache || !row_pos || !out) return PKV_ERR_NULL;
    if (!std::isfinite(softmax_scale) || softmax_scale < 0.f) return PKV_ERR_SHAPE;
    const size_t need = align256(sparse_row_attn_ws_bytes(*cfg, n_keys, m));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_sparse_row_attn(*cfg, q, k_cache, v_cache, row_pos, out, lse_out, m,
                                  n_keys, resolve_scale(softmax_scale, cfg->head_dim),
                                  ws, (hipStream_t)stream);
}

pkv_status pkv_sparse_row_attn_ctx_lse(const pkv_layer_cfg* cfg, const void* q,
                                       const void* k_cache, const void* v_cache,
                                       const int32_t* row_pos, void* out, float* lse_out,
                                       float* lse_ctx_out, int64_t m, int64_t n_keys,
                                       int64_t n_ctx, float softmax_scale, void* ws,
                                       size_t ws_bytes, void* stream) {
    pkv_status st = check_cfg(cfg);
    if (st != PKV_OK) return st;
    if (m < 0 || m > kMaxTokens || n_keys <= 0 || n_keys > kMaxTokens || n_ctx <= 0 ||
        n_ctx > n_keys)
        return PKV_ERR_SHAPE;
    if (cfg->dtype == PKV_BF16 &&
        (int64_t)cfg->head_dim * ((n_keys + 63) / 64 * 64) * 2 >= ((int64_t)1 << 32))
        return PKV_ERR_UNSUPPORTED;
    if (m * (int64_t)cfg->n_q_heads > INT32_MAX) return PKV_ERR_UNSUPPORTED;
    if (m == 0) return PKV_OK;
    if (!sparse_row_attn_ctx_lse_supported(*cfg, n_keys, m, n_ctx)) return PKV_ERR_UNSUPPORTED;
    if (!q || !k_cache || !v_cache || !row_pos || !out || !lse_ctx_out) return PKV_ERR_NULL;
    if (!std::isfinite(softmax_scale) || softmax_scale < 0.f) return PKV_ERR_SHAPE;
    const size_t need = align256(sparse_row_attn_ws_bytes(*cfg, n_keys, m, n_ctx));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_sparse_row_attn(*cfg, q, k_cache, v_cache, row_pos, out, lse_out, m, n_keys,
                                  resolve_scale(softmax_scale, cfg->head_dim), ws,
                                  (hipStream_t)stream, n_ctx, lse_ctx_out);
}

size_t pkv_sparse_row_attn_ctx_lse_workspace_bytes(const pkv_layer_cfg* cfg, int64_t n_keys,
                                                   int64_t n_ctx, int64_t m) {
    if (check_cfg(cfg) != PKV_OK || n_keys <= 0 || n_ctx <= 0 || m <= 0 || n_ctx > n_keys ||
        n_keys > kMaxTokens || m > kMaxTokens)
        return 0;
    if (!sparse_row_attn_ctx_lse_supported(*cfg, n_keys, m, n_ctx)) return 0;
    return align256(sparse_row_attn_ws_bytes(*cfg, n_keys, m, n_ctx));
}

pkv_status pkv_rmsnorm_rows(int32_t dtype, const void* h, const int32_t* row_idx,
                            const void* weight, float eps, void* y, int64_t m,
                            int64_t hidden, void* stream) {
    if (dtype != PKV_F32 && dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (m < 0 || m > kMaxTokens || hidden <= 0) return PKV_ERR_SHAPE;
    if (hidden % 8 || hidden > 16384) return PKV_ERR_UNSUPPORTED;
    if (!(eps >= 0.f) || !std::isfinite(eps)) return PKV_ERR_SHAPE;
    if (m == 0) return PKV_OK;
    if (!h || !weight || !y) return PKV_ERR_NULL;
    return launch_rmsnorm_rows(dtype, h, row_idx, weight, eps, y, m, hidden,
                               (hipStream_t)stream);
}

pkv_status pkv_gather_rows(int32_t dtype, const void* src, const int32_t* row_idx, void* dst,
                           int64_t m, int64_t width, void* stream) {
    if (dtype != PKV_F32 && dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (m < 0 || m > kMaxTokens || width <= 0 || width > kMaxTokens) return PKV_ERR_SHAPE;
    if (width % 8) return PKV_ERR_UNSUPPORTED;
    if (m == 0) return PKV_OK;
    if (!src || !row_idx || !dst) return PKV_ERR_NULL;
    return launch_gather_rows(dtype, src, row_idx, dst, m, width, (hipStream_t)stream);
}

static pkv_status linear_checked(int32_t dtype, bool gated, const void* x, const void* w0,
                                 const void* w1, const void* residual, void* y, int64_t m,
                                 int64_t k_in, int64_t n_out, void* ws, size_t ws_bytes,
                                 void* stream) {
    if (dtype != PKV_F32 && dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (m < 0 || m > kMaxTokens || k_in <= 0 || n_out <= 0 || k_in > kMaxTokens ||
        n_out > kMaxTokens)
        return PKV_ERR_SHAPE;
    if (k_in % 8 || n_out % 8) return PKV_ERR_UNSUPPORTED;
    if (m == 0) return PKV_OK;
    if (!x || !w0 || !y || (gated && !w1)) return PKV_ERR_NULL;
    const size_t need = align256(glue_ws_bytes(dtype, m, k_in, n_out));
    if (need && (!ws || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    return launch_linear_rows(dtype, gated, x, w0, w1, residual, y, m, k_in, n_out, ws,
                              (hipStream_t)stream);
}

pkv_status pkv_linear_rows(int32_t dtype, const void* x, const void* w, const void* residual,
                           void* y, int64_t m, int64_t k_in, int64_t n_out, void* ws,
                           size_t ws_bytes, void* stream) {
    return linear_checked(dtype, false, x, w, nullptr, residual, y, m, k_in, n_out, ws,
                          ws_bytes, stream);
}

pkv_status pkv_swiglu_rows(int32_t dtype, const void* x, const void* w_gate, const void* w_up,
                           void* y, int64_t m, int64_t k_in, int64_t n_out, void* ws,
                           size_t ws_bytes, void* stream) {
    return linear_checked(dtype, true, x, w_gate, w_up, nullptr, y, m, k_in, n_out, ws,
                          ws_bytes, stream);
}

size_t pkv_glue_workspace_bytes(int32_t dtype, int64_t m, int64_t k_in, int64_t n_out) {
    if ((dtype != PKV_F32 && dtype != PKV_BF16) || m <= 0 || k_in <= 0 || n_out <= 0 ||
        m > kMaxTokens || k_in > kMaxTokens || n_out > kMaxTokens)
        return 0;
    return align256(glue_ws_bytes(dtype, m, k_in, n_out));
}

size_t pkv_workspace_bytes(int which_call, const pkv_layer_cfg* cfg, int64_t n,
                           int64_t m) {
    if (check_cfg(cfg) != PKV_OK || n < 0 || m < 0) return 0;
    switch (which_call) {
        case PKV_CALL_QUERY_SCORE:
            return align256(query_score_ws_bytes(*cfg, n, m));
        case PKV_CALL_TOPK_SELECT:
            return align256(topk_select_ws_bytes(n));
        case PKV_CALL_GATHER_QKV_PROJ:
            return align256(gather_qkv_proj_ws_bytes(*cfg, m));
        case PKV_CALL_SPARSE_ROW_ATTN:
            return align256(sparse_row_attn_ws_bytes(*cfg, n, m));
        default:
            return 0;
    }
}

const char* pkv_status_string(pkv_status status) {
    switch (status) {
        case PKV_OK: return "ok";
        case PKV_ERR_NULL: return "a required pointer is NULL";
        case PKV_ERR_SHAPE: return "a size argument is negative or inconsistent";
        case PKV_ERR_UNSUPPORTED: return "dtype, head_dim or head geometry not supported";
        case PKV_ERR_WORKSPACE: return "workspace missing or too small";
        case PKV_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int pkv_version(void) { return 100; }

}  // extern "C"
