/*
 * pkv.h - C ABI of the ProphetKV selective-recomputation hot path for
 *         AMD MI355X (gfx950).
 *
 * ProphetKV (arXiv 2602.02579) reuses chunk-wise precomputed KV caches in
 * RAG prefill and repairs them by recomputing only the context tokens the
 * user query attends to.  Per transformer layer the hot path is:
 *
 *   1. pkv_rope_restore     put positions back on the assembled,
 *                           position-free chunk keys
 *   2. pkv_query_score      attention of the user-query tokens to every
 *                           context token, averaged over heads and query
 *                           tokens, summed over layers
 *   3. pkv_topk_select      the top p-fraction of context tokens
 *   4. pkv_gather_qkv_proj  Q/K/V projection + rotation of the selected and
 *      pkv_scatter_kv       the query rows; new K/V replace the cache rows
 *   5. pkv_sparse_row_attn  causal attention of those rows over the cache
 *
 * Conventions shared by every call
 * --------------------------------
 * Pointers: `cfg` is a host pointer, read during the call only.  Every other
 *   pointer is a DEVICE pointer to memory owned by the caller; the library
 *   allocates nothing, frees nothing and keeps no pointer after the call
 *   returns.  Scratch memory is caller-provided (`ws`, `ws_bytes`), sized by
 *   pkv_workspace_bytes(), 256-byte aligned, and may be reused between calls
 *   on the same stream.  Calls that can be in flight at the same time
 *   (different streams) need workspaces of their own: the kernels keep
 *   partial results, flags and work counters there.
 * Layout: token-major, contiguous.  Keys/values [tokens, n_kv_heads,
 *   head_dim]; queries/outputs [rows, n_q_heads, head_dim]; hidden states
 *   [tokens, hidden]; weights [out_features, hidden] (row-major, so both
 *   GEMM operands have the contraction dimension contiguous).  Element type
 *   is cfg->dtype (fp32 or bf16) for every tensor typed `void*`; scores and
 *   log-sum-exp are always fp32, indices and positions int32.
 * Heads: query head h reads kv head h / (n_q_heads / n_kv_heads).
 * Rotary embedding: element i < D/2 of a head is paired with element
 *   i + D/2 and turned by position * rope_theta^(-2i/D); no frequency
 *   scaling.
 * Streams: `stream` is a hipStream_t passed as void* (NULL = the null
 *   stream).  Calls enqueue kernels on it and return without synchronising;
 *   nothing else is enqueued (no memset or copy nodes), so a sequence of
 *   calls can be recorded into a HIP graph and replayed.
 * Errors: arguments that the host can check (null pointers, non-positive or
 *   inconsistent sizes, unsupported dtype or head_dim, workspace too small)
 *   give an error code and enqueue nothing.  A failed launch gives
 *   PKV_ERR_LAUNCH.  Not checked (undefined results, but no out-of-bounds
 *   access is made on their account unless stated): non-finite inputs.
 *   Index arrays (row_idx, dst_row, row_pos) are read on the device, so
 *   their VALUES cannot be checked by the host: out-of-range values there
 *   are undefined behaviour and are the caller's responsibility.
 * Alignment: tensors are expected at 16-byte aligned addresses (any device
 *   allocator gives 256).  The kernels issue 16-byte accesses; where a call
 *   says so it accepts less (pkv_topk_select, pkv_linear_rows,
 *   pkv_swiglu_rows fall back to narrower accesses) or refuses
 *   (pkv_rmsnorm_rows, pkv_gather_rows).
 * Supported shapes: head_dim even, a multiple of 16 and <= 256;
 *   n_q_heads a multiple of n_kv_heads; hidden a multiple of 8.  Token counts
 *   up to 2^30.  pkv_sparse_row_attn (bf16) and pkv_query_score further need
 *   head_dim * (n_keys rounded up to 64) * 2 < 2^32 and rows * n_q_heads
 *   (query tokens * n_q_heads) < 2^31; beyond that they return
 *   PKV_ERR_UNSUPPORTED.
 * Environment: three variables change HOW pkv_sparse_row_attn (bf16, head_dim
 *   128) works, never what it computes; they exist for measurements and
 *   tests.  PKV_ATTN_WAVES=4 (read once per process): workgroups of four
 *   waves instead of eight.  PKV_ATTN_VT=1 / 0 (read at every call): always
 *   / never make a transposed copy of the value cache in the workspace
 *   before the main kernel (unset: decided by problem size).
 *   PKV_ATTN_RANGES=n (read once): process the keys of every row tile in n
 *   ranges (unset: decided by problem size).  Workspace sizes do not depend
 *   on the first two; set the third before asking for sizes.
 */
#ifndef PKV_H
#define PKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PKV_OK = 0,
    PKV_ERR_NULL = 1,        /* a required pointer is NULL               */
    PKV_ERR_SHAPE = 2,       /* a size is negative / inconsistent        */
    PKV_ERR_UNSUPPORTED = 3, /* dtype / head_dim / geometry not built    */
    PKV_ERR_WORKSPACE = 4,   /* ws is NULL or ws_bytes is too small      */
    PKV_ERR_LAUNCH = 5       /* the HIP runtime refused a launch         */
} pkv_status;

typedef enum { PKV_F32 = 0, PKV_BF16 = 1 } pkv_dtype;

typedef struct {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t hidden;
    float   rope_theta;
    int32_t dtype;           /* pkv_dtype: storage type of all void* tensors */
} pkv_layer_cfg;

/* which_call values for pkv_workspace_bytes */
enum {
    PKV_CALL_ROPE_RESTORE = 1,
    PKV_CALL_QUERY_SCORE = 2,
    PKV_CALL_TOPK_SELECT = 3,
    PKV_CALL_GATHER_QKV_PROJ = 4,
    PKV_CALL_SCATTER_KV = 5,
    PKV_CALL_SPARSE_ROW_ATTN = 6
};

/*
 * Step 1 - rotary position restore (paper: Sec. 1 footnote on
 * position-independent caches; Appendix E, closing paragraph: positions are
 * applied to the old key cache exactly once, before cache replacement;
 * Algorithm 1, concatenation of the chunk caches).
 *
 * k_out[t, g, :] = R(p_t) k_in[t, g, :] for t < n, every kv head g, where
 * p_t = pos[t] if pos != NULL else pos_base + t.  Positions may be negative
 * (the inverse rotation).  k_out may alias k_in exactly (in place); partial
 * overlap is not allowed.  The result is rounded once to cfg->dtype.
 * n == 0 is a no-op.
 */
pkv_status pkv_rope_restore(const pkv_layer_cfg* cfg,
                            const void* k_in,   /* [n, Hkv, D] */
                            void* k_out,        /* [n, Hkv, D] */
                            const int32_t* pos, /* [n] or NULL */
                            int64_t pos_base, int64_t n, void* stream);

/*
 * Step 2 - query-driven value function (paper: Algorithm 1, first stage:
 * alpha_l = Softmax(Q_s K'^T / sqrt(d_k)); Sec. 4.2: average over the query
 * tokens; Appendix E: mean over heads; Algorithm 1 second stage / Eq. 7:
 * fusion over layers is a sum).
 *
 * score[t] (+)= 1/(Hq*nq) * sum_{h, q} softmax_t(q[q,h] . k[t,g(h)] * scale)
 * with the softmax running over the n_ctx context keys only.  `q` holds the
 * rotated user-query queries, `k` the restored context keys.  With
 * accumulate == 0 the score is overwritten, otherwise the new layer is added
 * to it (fp32).  softmax_scale == 0 means 1/sqrt(D).  Deterministic: the
 * same inputs give the same bits.
 */
pkv_status pkv_query_score(const pkv_layer_cfg* cfg,
                           const void* q,      /* [nq, Hq, D]     */
                           const void* k,      /* [n_ctx, Hkv, D] */
                           float* score,       /* [n_ctx]         */
                           int64_t nq, int64_t n_ctx, float softmax_scale,
                           int accumulate, void* ws, size_t ws_bytes,
                           void* stream);

/*
 * pkv_query_score for callers that cannot allocate device memory or pass a
 * workspace: code recorded into a HIP graph, tight serving loops, harnesses that
 * forbid allocation.  Same arguments, kernels and results (bit for bit) as
 * pkv_query_score, without `ws`: the scratch is a PKV_STATIC_SCRATCH_BYTES array
 * inside the library, one copy per GPU, held until the process ends.  The call
 * allocates nothing and frees nothing.  A problem that needs more scratch than
 * that - pkv_workspace_bytes(PKV_CALL_QUERY_SCORE, cfg, n_ctx, nq) tells - returns
 * PKV_ERR_WORKSPACE and enqueues nothing (16 MiB cover 32k context keys with 128
 * query tokens of 32 heads; 128k keys with 256 query tokens need 68 MB and are
 * refused).  The first call on a device looks the array's address up
 * (make it outside a graph capture); the device must be current.  All calls on one
 * GPU share the array: calls that can overlap there (different streams, or graphs
 * replayed concurrently) race on it - order them, or use pkv_query_score with
 * workspaces of their own.
 */
#define PKV_STATIC_SCRATCH_BYTES (16u << 20)
pkv_status pkv_query_score_static(const pkv_layer_cfg* cfg,
                                  const void* q,      /* [nq, Hq, D]     */
                                  const void* k,      /* [n_ctx, Hkv, D] */
                                  float* score,       /* [n_ctx]         */
                                  int64_t nq, int64_t n_ctx, float softmax_scale,
                                  int accumulate, void* stream);

/*
 * Step 3 - top-p selection (paper: Eq. 4, TOP_p of the value function;
 * Algorithm 1 "Select token indices"; Sec. 4.3: one set for all layers).
 *
 * idx_out receives the indices of the k largest scores in ascending index
 * order.  Among equal scores the lower index is taken first, so the result
 * is unique.  -0.0 and +0.0 compare equal.  k == 0 writes nothing; k == n
 * writes 0..n-1.  Scores must be finite.  The workspace is optional: vectors of
 * up to 24576 scores need none; longer ones (up to 2^22) are selected by many
 * workgroups when `ws` holds pkv_workspace_bytes(PKV_CALL_TOPK_SELECT, cfg, n, 0)
 * bytes, and by one workgroup (1.4x slower at 32k scores, 8x at 128k) when it is
 * NULL or smaller.  The result is the same either way.
 */
pkv_status pkv_topk_select(const float* score, /* [n] */
                           int64_t n, int64_t k,
                           int32_t* idx_out,   /* [k] */
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Step 4a - gather, project, rotate (paper: Algorithm 1 "Recompute KV cache
 * at layer l" and "Calculate user query KV cache"; Appendix E, third step:
 * hidden states and positions are pruned to the selected tokens).
 *
 * For i < m: x = hidden[row_idx ? row_idx[i] : i, :];
 *   q_out[i] = R(row_pos[i]) (Wq x),  k_out[i] = R(row_pos[i]) (Wk x),
 *   v_out[i] = Wv x,
 * fp32 accumulation, one rounding to cfg->dtype after the rotation.
 * q_out may be NULL (then only K and V are produced); k_out and v_out may
 * both be NULL (then only Q is produced).  row_idx values must lie in
 * [0, n_hidden_rows) (checked only against negative m / null pointers on
 * the host).  Scratch: pkv_workspace_bytes(PKV_CALL_GATHER_QKV_PROJ, cfg, 0, m)
 * bytes (a cos/sin table of the m row positions).  m == 0 is a no-op.
 */
pkv_status pkv_gather_qkv_proj(const pkv_layer_cfg* cfg,
                               const void* hidden,     /* [n_hidden_rows, hidden] */
                               const int32_t* row_idx, /* [m] or NULL */
                               const int32_t* row_pos, /* [m] */
                               const void* wq,         /* [Hq*D, hidden]  */
                               const void* wk,         /* [Hkv*D, hidden] */
                               const void* wv,         /* [Hkv*D, hidden] */
                               void* q_out,            /* [m, Hq, D]  */
                               void* k_out,            /* [m, Hkv, D] */
                               void* v_out,            /* [m, Hkv, D] */
                               int64_t m, void* ws, size_t ws_bytes,
                               void* stream);

/*
 * Step 4a for the other public model families the paper evaluates (Sec. 5.1 names
 * Qwen models besides Llama; the paper does not describe their blocks, so these
 * are the public architectures, not something the paper defines):
 *   bq, bk, bv      additive biases of the three projections ([Hq*D], [Hkv*D],
 *                   [Hkv*D], element type cfg->dtype), each may be NULL;
 *   q_norm, k_norm  gains [D] of an RMS normalisation over head_dim applied to
 *                   every head of Q and of K after projection and bias and BEFORE
 *                   the rotation: y = x / sqrt(mean(x^2) + norm_eps) * gain.
 *                   Both or neither.  V is never normalised.
 * Everything runs in fp32 on the fp32 accumulators; there is still exactly one
 * rounding to cfg->dtype, after the rotation.  `variant` is a HOST pointer read
 * during the call (NULL = plain pkv_gather_qkv_proj); the pointers inside it are
 * device pointers.  Same scratch, errors and no-op rules as pkv_gather_qkv_proj.
 */
typedef struct {
    const void* bq;
    const void* bk;
    const void* bv;
    const void* q_norm;
    const void* k_norm;
    float norm_eps;
} pkv_proj_variant;

pkv_status pkv_gather_qkv_proj_ex(const pkv_layer_cfg* cfg,
                                  const void* hidden, const int32_t* row_idx,
                                  const int32_t* row_pos, const void* wq,
                                  const void* wk, const void* wv,
                                  const pkv_proj_variant* variant,
                                  void* q_out, void* k_out, void* v_out, int64_t m,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * Steps 4a + 4b in one call (Algorithm 1: the recomputed K/V of the selected and
 * the query rows replace the cache rows): as pkv_gather_qkv_proj_ex, but K and V of
 * output row i are written straight to row dst_row[i] of k_cache / v_cache
 * ([n_cache, Hkv, D]) instead of to separate [m, Hkv, D] buffers followed by
 * pkv_scatter_kv.  q_out ([m, Hq, D], may be NULL) is written as before.  dst_row
 * values must be distinct and lie in [0, n_cache) (device data, not checked);
 * the caches must not overlap hidden or the weights.  variant may be NULL.
 */
pkv_status pkv_gather_qkv_proj_scatter(const pkv_layer_cfg* cfg,
                                       const void* hidden, const int32_t* row_idx,
                                       const int32_t* row_pos, const void* wq,
                                       const void* wk, const void* wv,
                                       const pkv_proj_variant* variant,
                                       void* q_out, void* k_cache, void* v_cache,
                                       const int32_t* dst_row, int64_t m,
                                       int64_t n_cache, void* ws, size_t ws_bytes,
                                       void* stream);

/*
 * Step 4b - cache update (paper: Algorithm 1 "Update layer-wise KV cache":
 * rows in T_p take the recomputed K/V, all other rows are reused as they
 * are; the user-query K/V are appended after the context).
 *
 * k_cache[dst_row[i]] = k_new[i], v_cache[dst_row[i]] = v_new[i] for i < m.
 * dst_row values must be unique and lie in [0, n_cache).  No other cache row
 * is touched.  m == 0 is a no-op.
 */
pkv_status pkv_scatter_kv(const pkv_layer_cfg* cfg,
                          const void* k_new,      /* [m, Hkv, D] */
                          const void* v_new,      /* [m, Hkv, D] */
                          const int32_t* dst_row, /* [m] */
                          void* k_cache,          /* [n_cache, Hkv, D] */
                          void* v_cache,          /* [n_cache, Hkv, D] */
                          int64_t m, int64_t n_cache, void* stream);

/*
 * Step 5 - attention of the recomputed rows over the whole updated cache
 * (paper: Sec. 4.3 Stage II: complete recomputation across all layers, but
 * only for the selected tokens; Sec. 5.3: this attention dominates the
 * cost; Eq. 1 for the attention output).
 *
 * out[i, h] = sum_{t <= row_pos[i]} softmax_t(q[i,h] . k_cache[t,g(h)] * scale)
 *             * v_cache[t, g(h)],
 * i < m, fp32 softmax and accumulation, one rounding to cfg->dtype.
 * row_pos[i] must lie in [0, n_keys); rows need not be sorted, but sorted
 * rows (the order step 3 returns) give balanced tiles.  lse_out, if not
 * NULL, receives the natural-log normaliser per (row, head).
 * softmax_scale == 0 means 1/sqrt(D).  m == 0 is a no-op.
 */
pkv_status pkv_sparse_row_attn(const pkv_layer_cfg* cfg,
                               const void* q,          /* [m, Hq, D] */
                               const void* k_cache,    /* [n_keys, Hkv, D] */
                               const void* v_cache,    /* [n_keys, Hkv, D] */
                               const int32_t* row_pos, /* [m] */
                               void* out,              /* [m, Hq, D] */
                               float* lse_out,         /* [m, Hq] or NULL */
                               int64_t m, int64_t n_keys, float softmax_scale,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * Fused variants for the first stage (paper: Sec. 4.2 - the user query is run through
 * the model against the imprecise cache, and its attention to the context is the value
 * function; Algorithm 1, first stage).  The query rows' attention pass and the score
 * form the same exponentials of the same Q K^T; these two calls let the attention emit
 * the normaliser the score needs, so that the score reads the keys once, not twice.
 *
 * pkv_sparse_row_attn_ctx_lse: pkv_sparse_row_attn that also writes
 *   lse_ctx_out[i, h] = log sum_{t < n_ctx, t <= row_pos[i]} exp(q[i,h] . k[t,g(h)] * scale),
 * the log-sum-exp over the CONTEXT keys alone (the first n_ctx rows of the cache; the
 * softmax of Algorithm 1's value function runs over exactly those).  out and lse_out
 * (may be NULL) are those of pkv_sparse_row_attn.  Built for bf16 with head_dim 128,
 * n_ctx a multiple of 64 and at most 32 n_ctx >= n_keys; anything else returns
 * PKV_ERR_UNSUPPORTED (use pkv_query_score then).  It is meant for launches of few rows
 * (the user-query rows): the keys are always processed in ranges with partial results
 * in `ws`.  Scratch: pkv_sparse_row_attn_ctx_lse_workspace_bytes(cfg, n_keys, n_ctx, m)
 * (0 = not supported).
 *
 * pkv_query_score_lse: the column sums of pkv_query_score with the normalisers given:
 *   score[t] (+)= 1/(Hq*nq) * sum_{h, q : t <= row_pos[q]} exp(q[q,h] . k[t,g(h)] * scale
 *                                                             - lse[q, h]),  t < n_ctx.
 * row_pos == NULL: every query row counts for every key; with lse = lse_ctx_out of the
 * call above this is pkv_query_score exactly (up to rounding).  row_pos != NULL ([nq],
 * device): row q counts for the keys it sees only; with lse = lse_out of
 * pkv_sparse_row_attn over all rows of a prompt this is the attention each key RECEIVES
 * from the whole prompt (the global column sum that Appendix B, Tab. 3 lists as the
 * first factor of a comparison method's criterion; used by the diagnostics only).
 * Any dtype and geometry pkv_query_score takes.  Scratch: as pkv_query_score.
 */
pkv_status pkv_sparse_row_attn_ctx_lse(const pkv_layer_cfg* cfg,
                                       const void* q,          /* [m, Hq, D] */
                                       const void* k_cache,    /* [n_keys, Hkv, D] */
                                       const void* v_cache,    /* [n_keys, Hkv, D] */
                                       const int32_t* row_pos, /* [m] */
                                       void* out,              /* [m, Hq, D] */
                                       float* lse_out,         /* [m, Hq] or NULL */
                                       float* lse_ctx_out,     /* [m, Hq] */
                                       int64_t m, int64_t n_keys, int64_t n_ctx,
                                       float softmax_scale, void* ws, size_t ws_bytes,
                                       void* stream);

size_t pkv_sparse_row_attn_ctx_lse_workspace_bytes(const pkv_layer_cfg* cfg, int64_t n_keys,
                                                   int64_t n_ctx, int64_t m);

pkv_status pkv_query_score_lse(const pkv_layer_cfg* cfg,
                               const void* q,          /* [nq, Hq, D]     */
                               const void* k,          /* [n_ctx, Hkv, D] */
                               const float* lse,       /* [nq, Hq]        */
                               const int32_t* row_pos, /* [nq] or NULL    */
                               float* score,           /* [n_ctx]         */
                               int64_t nq, int64_t n_ctx, float softmax_scale,
                               int accumulate, void* ws, size_t ws_bytes, void* stream);

/*
 * Scratch bytes the given call needs for a problem with `n` cache/context
 * tokens and `m` rows (query tokens for PKV_CALL_QUERY_SCORE).  Pure host
 * function; returns 0 for calls that need none and for invalid arguments.
 */
size_t pkv_workspace_bytes(int which_call, const pkv_layer_cfg* cfg,
                           int64_t n, int64_t m);

/*
 * ---- Layer glue for the carried rows -----------------------------------
 *
 * Between two runs of the hot path the rows that ProphetKV carries through
 * the model (Sec. 4.2: the user query, run against the imprecise cache to
 * obtain its attention to the context; Sec. 4.3 and Appendix E: the selected
 * and the query rows, through every layer) pass through the rest of a decoder
 * layer.  The paper evaluates Llama-3.1-8B and Qwen models (Sec. 5.1) and does
 * not restate their block; the three calls below are the public pre-norm
 * Llama block, not something the paper defines:
 *
 *     x  = rmsnorm(h, w_in)            -> pkv_gather_qkv_proj, ..., attention a
 *     h' = h + a Wo^T                  (pkv_linear_rows with a residual)
 *     y  = rmsnorm(h', w_post)
 *     g  = silu(y Wg^T) * (y Wu^T)     (pkv_swiglu_rows)
 *     h''= h' + g Wd^T                 (pkv_linear_rows with a residual)
 *
 * They take no pkv_layer_cfg: `dtype` is a pkv_dtype and the matrix sizes are
 * arguments.  Rounding: every tensor these calls write is rounded once to
 * `dtype`; where a residual is added the product is rounded first and the sum
 * again, and pkv_swiglu_rows rounds the gate product, its activation, the up
 * product and the final product separately - the values a framework that
 * keeps each of these tensors in `dtype` would hold.  Accumulation is fp32.
 */

/*
 * y[i, :] = h[row_idx[i], :] / sqrt(mean_j h[row_idx[i], j]^2 + eps) * weight
 * for i < m; row_idx == NULL means row i.  The mean of squares and the scaling
 * are fp32.  hidden must be a multiple of 8 and at most 16384; h, weight and y
 * must be 16-byte aligned (PKV_ERR_UNSUPPORTED otherwise).  y must not overlap
 * h.  m == 0 is a no-op.
 */
pkv_status pkv_rmsnorm_rows(int32_t dtype,
                            const void* h,          /* [>= max row + 1, hidden] */
                            const int32_t* row_idx, /* [m] or NULL */
                            const void* weight,     /* [hidden] */
                            float eps,
                            void* y,                /* [m, hidden] */
                            int64_t m, int64_t hidden, void* stream);

/*
 * dst[i, :] = src[row_idx[i], :] for i < m: the hidden states of the carried
 * rows at the first layer (Appendix E: the hidden states are pruned to the
 * selected tokens).  `width` elements per row, a multiple of 8; src, dst
 * 16-byte aligned and not overlapping.  m == 0 is a no-op.
 */
pkv_status pkv_gather_rows(int32_t dtype,
                           const void* src,        /* [>= max row + 1, width] */
                           const int32_t* row_idx, /* [m] */
                           void* dst,              /* [m, width] */
                           int64_t m, int64_t width, void* stream);

/*
 * y = round(x W^T), then, if residual != NULL, y = round(y + residual).
 * y may be the same buffer as residual (each element is read before it is
 * written, by the same thread); it must not overlap x or w.  k_in and n_out
 * must be multiples of 8.  Any alignment of the element type is accepted;
 * 16-byte aligned bf16 operands with k_in a multiple of 32 and n_out a
 * multiple of 256 take the matrix-core kernel.  Scratch: pkv_glue_workspace_bytes(dtype, m, k_in,
 * n_out); its contents are garbage afterwards.  m == 0 is a no-op.
 */
pkv_status pkv_linear_rows(int32_t dtype,
                           const void* x,        /* [m, k_in] */
                           const void* w,        /* [n_out, k_in] */
                           const void* residual, /* [m, n_out] or NULL */
                           void* y,              /* [m, n_out] */
                           int64_t m, int64_t k_in, int64_t n_out,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * y = round(round(silu(round(x Wg^T))) * round(x Wu^T)), silu(a) = a / (1 + e^-a).
 * Same size rules, scratch and aliasing rules as pkv_linear_rows (n_out is
 * the intermediate size; the scratch of pkv_glue_workspace_bytes covers both
 * calls for the same m, k_in and n_out).
 */
pkv_status pkv_swiglu_rows(int32_t dtype,
                           const void* x,        /* [m, k_in] */
                           const void* w_gate,   /* [n_out, k_in] */
                           const void* w_up,     /* [n_out, k_in] */
                           void* y,              /* [m, n_out] */
                           int64_t m, int64_t k_in, int64_t n_out,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Scratch bytes pkv_linear_rows and pkv_swiglu_rows need for these sizes
 * (the larger of the two).  Pure host function; 0 for invalid arguments or
 * when none is needed.
 */
size_t pkv_glue_workspace_bytes(int32_t dtype, int64_t m, int64_t k_in,
                                int64_t n_out);

/* Static, never-NULL description of a status code. */
const char* pkv_status_string(pkv_status status);

/* Library version as major*10000 + minor*100 + patch. */
int pkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PKV_H */
