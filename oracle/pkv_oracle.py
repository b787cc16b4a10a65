"""CPU oracle for the ProphetKV selective-recomputation hot path.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  This module is a plain, slow,
double-precision restatement of what the paper's method computes per layer.
It exists only so that the GPU library can be checked against something that
a reader can compare with the paper by eye.  Nothing in the product package
imports it; it imports nothing from the product package; the two share no
helpers, tables or constants.  Only the test-suite, the smoke check and the
CPU-baseline leg of the benchmark may call it.

Conventions
-----------
* All arrays are ``numpy.float64``.  A "storage dtype" (``"f32"`` or
  ``"bf16"``) names the precision in which the real system keeps a tensor in
  memory; wherever the method stores a tensor (restored keys, projected
  Q/K/V, the score vector, the attention output) the oracle rounds the fp64
  value to that precision with round-to-nearest-even and carries on in fp64
  with the rounded value.  Between two storage points nothing is rounded.
* Tensors are token-major: keys/values ``[tokens, kv_heads, head_dim]``,
  queries ``[rows, q_heads, head_dim]``, hidden states ``[tokens, hidden]``,
  weights ``[out_features, in_features]``.
* Grouped-query attention: query head ``h`` reads kv head
  ``h // (n_q_heads // n_kv_heads)``.
* Token ``t`` of the assembled context sits at position ``t``; user-query
  token ``j`` sits at position ``N + j`` (the query closes the prompt,
  Sec. 3.2).

Readings of the paper where it is silent (each is listed in the design
notes of the repository): softmax in the score runs over the context keys
only, exactly as written in Algorithm 1; scores are averaged over query
tokens (Sec. 4.2) and over heads (Appendix E); layer fusion is the plain sum
of Algorithm 1; rotary embedding uses the half-split pairing
``(i, i + D/2)`` with ``inv_freq_i = theta ** (-2 i / D)``; top-p ties go to
the lower index and the index set is returned ascending.

Parity status: every function below is pinned by tests that do not use the
oracle to check itself (closed forms, library routines, brute force); none
is "parity unpinned".  Behaviour on NaN/Inf scores is undefined on both
sides and is not tested.
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "round_to_storage",
    "rope_inv_freq",
    "rope_rotate",
    "rope_restore",
    "project_qkv_rows",
    "query_score",
    "fuse_score",
    "topk_select",
    "scatter_kv",
    "sparse_row_attn",
    "selective_recompute_layer",
    "prophetkv_stack",
]


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------

def round_to_storage(x, dtype: str):
    """Round fp64 values to the storage precision, return them as fp64.

    ``"f64"`` keeps the value, ``"f32"`` rounds to IEEE binary32, ``"bf16"``
    rounds *directly* from binary64 to bfloat16 (8 exponent bits, 7 stored
    mantissa bits) with round-to-nearest, ties-to-even, so that there is no
    double rounding through binary32.
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f64":
        return x.copy()
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype != "bf16":
        raise ValueError(f"unknown storage dtype {dtype!r}")

    out = np.empty_like(x)
    flat_in = np.ascontiguousarray(x).reshape(-1)
    flat_out = out.reshape(-1)
    a = np.abs(flat_in)
    tiny = a < 2.0 ** -126          # bfloat16 subnormal range (and zero)
    special = ~np.isfinite(flat_in)
    normal = ~(tiny | special)

    # Normal range: keep the top 7 of the 52 stored mantissa bits.  Adding
    # half of the dropped field (minus one, plus the bit that will become the
    # new least significant bit) and then clearing the dropped field is
    # round-half-to-even; a mantissa carry moves into the exponent by itself.
    bits = flat_in[normal].view(np.uint64)
    drop = np.uint64(45)
    lsb = (bits >> drop) & np.uint64(1)
    bits = bits + (np.uint64((1 << 44) - 1) + lsb)
    bits = bits & ~np.uint64((1 << 45) - 1)
    r = bits.view(np.float64)
    # anything that rounded past the largest finite bfloat16 becomes inf
    bf16_max = (2.0 - 2.0 ** -7) * 2.0 ** 127
    r = np.where(np.abs(r) > bf16_max, np.copysign(np.inf, r), r)
    flat_out[normal] = r

    # Subnormal range: fixed quantum 2**-133, numpy's rint is ties-to-even.
    q = 2.0 ** -133
    flat_out[tiny] = np.rint(flat_in[tiny] / q) * q
    flat_out[special] = flat_in[special]
    return out


# --------------------------------------------------------------------------
# step 1: rotary position restore (Sec. 1 footnote; Appendix E, last
# paragraph: applied to the old key cache once, before replacement)
# --------------------------------------------------------------------------

def rope_inv_freq(head_dim: int, theta: float):
    """``theta ** (-2 i / D)`` for ``i = 0 .. D/2 - 1``."""
    if head_dim % 2:
        raise ValueError("head_dim must be even")
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(theta) ** (-2.0 * i / head_dim)


def rope_rotate(x, pos, theta: float):
    """Rotate ``x [n, heads, D]`` by the rotary angles of ``pos [n]``.

    Element ``i < D/2`` is paired with element ``i + D/2``; the pair is
    turned by ``phi = pos * inv_freq_i``:
    ``(a, b) -> (a cos phi - b sin phi, b cos phi + a sin phi)``.
    Negative positions turn the other way (the inverse rotation).
    No rounding happens here.
    """
    x = np.asarray(x, dtype=np.float64)
    pos = np.asarray(pos, dtype=np.float64)
    n, _, d = x.shape
    if pos.shape != (n,):
        raise ValueError("pos must have one entry per token")
    half = d // 2
    phi = pos[:, None] * rope_inv_freq(d, theta)[None, :]      # [n, D/2]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    a = x[:, :, :half]
    b = x[:, :, half:]
    out = np.empty_like(x)
    out[:, :, :half] = a * c - b * s
    out[:, :, half:] = b * c + a * s
    return out


def rope_restore(k_nope, pos, theta: float, dtype: str):
    """Restore positions on the assembled, position-free keys; round to storage."""
    return round_to_storage(rope_rotate(k_nope, pos, theta), dtype)


# --------------------------------------------------------------------------
# step 4a: gather hidden rows, project Q/K/V, rotate Q and K
# (Algorithm 1, "Recompute KV cache" and "Calculate user query KV cache";
#  Appendix E: hidden states and positions are pruned to the chosen rows)
# --------------------------------------------------------------------------

def project_qkv_rows(hidden, rows, row_pos, wq, wk, wv,
                     n_q_heads: int, n_kv_heads: int, head_dim: int,
                     theta: float, dtype: str, bq=None, bk=None, bv=None,
                     q_norm=None, k_norm=None, norm_eps: float = 1e-6):
    """Q, K, V for the hidden rows ``rows`` at rotary positions ``row_pos``.

    ``hidden [tokens, hid]``, ``wq [Hq*D, hid]``, ``wk, wv [Hkv*D, hid]``.
    Returns ``q [m, Hq, D]``, ``k [m, Hkv, D]``, ``v [m, Hkv, D]``, each
    rounded to the storage dtype after the rotation (V is not rotated).

    Variants of the public model families the paper evaluates besides Llama
    (Sec. 5.1; the paper itself does not describe them): ``bq, bk, bv`` are
    additive biases of the three projections (Qwen2.5); ``q_norm, k_norm [D]``
    are the gains of an RMS normalisation over head_dim applied to every head of
    Q and of K after the projection and before the rotation (Qwen3).  Everything
    up to the single rounding at the end is exact arithmetic here.
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    m = rows.shape[0]
    xr = hidden[rows, :]                                        # [m, hid]

    def proj(w, b, heads, gain):
        y = xr @ np.asarray(w, np.float64).T
        if b is not None:
            y = y + np.asarray(b, np.float64)[None, :]
        y = y.reshape(m, heads, head_dim)
        if gain is not None:
            ms = (y * y).mean(axis=2, keepdims=True)
            y = y / np.sqrt(ms + norm_eps) * np.asarray(gain, np.float64)[None, None, :]
        return y

    q = rope_rotate(proj(wq, bq, n_q_heads, q_norm), row_pos, theta)
    k = rope_rotate(proj(wk, bk, n_kv_heads, k_norm), row_pos, theta)
    v = proj(wv, bv, n_kv_heads, None)
    return (round_to_storage(q, dtype), round_to_storage(k, dtype),
            round_to_storage(v, dtype))


# --------------------------------------------------------------------------
# step 2: query-driven score (Algorithm 1, first stage; Sec. 4.2 average
# over query tokens; Appendix E mean over heads)
# --------------------------------------------------------------------------

def query_score(q_s, k_ctx, scale=None):
    """``alpha[t] = mean_{h, q} softmax_t(q_s[q, h] . k_ctx[t, g(h)] * scale)``.

    ``q_s [Qn, Hq, D]`` are the rotated user-query queries, ``k_ctx
    [N, Hkv, D]`` the restored context keys.  The softmax runs over the N
    context keys only.  Returns fp64 ``alpha [N]`` (not rounded).
    """
    q_s = np.asarray(q_s, dtype=np.float64)
    k_ctx = np.asarray(k_ctx, dtype=np.float64)
    qn, hq, d = q_s.shape
    n, hkv, d2 = k_ctx.shape
    if d != d2 or hq % hkv:
        raise ValueError("head geometry mismatch")
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    group = hq // hkv
    alpha = np.zeros(n, dtype=np.float64)
    for h in range(hq):
        g = h // group
        s = (q_s[:, h, :] @ k_ctx[:, g, :].T) * scale          # [Qn, N]
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        alpha += p.sum(axis=0)
    return alpha / (hq * qn)


def fuse_score(score_f32, alpha):
    """One step of the layer fusion sum: ``score <- fp32(score + alpha_l)``.

    The fused score lives in fp32 memory, so it is rounded after each layer
    is added (Algorithm 1, second stage, taken in layer order).
    """
    return round_to_storage(np.asarray(score_f32, np.float64) + alpha, "f32")


# --------------------------------------------------------------------------
# step 3: top-p selection (Eq. 4; Algorithm 1 "Select token indices")
# --------------------------------------------------------------------------

def topk_select(score, k: int):
    """Indices of the ``k`` largest scores, ties to the lower index, ascending."""
    score = np.asarray(score, dtype=np.float64)
    n = score.shape[0]
    if not 0 <= k <= n:
        raise ValueError("k out of range")
    idx = np.arange(n, dtype=np.int64)
    # last key is the primary one: descending score, then ascending index
    order = np.lexsort((idx, -score))
    return np.sort(order[:k]).astype(np.int32)


# --------------------------------------------------------------------------
# step 4b: cache update (Algorithm 1 "Update layer-wise KV cache")
# --------------------------------------------------------------------------

def scatter_kv(k_cache, v_cache, k_new, v_new, dst_rows):
    """Return copies of the caches with rows ``dst_rows`` replaced."""
    dst_rows = np.asarray(dst_rows, dtype=np.int64)
    if np.unique(dst_rows).shape[0] != dst_rows.shape[0]:
        raise ValueError("destination rows must be unique")
    k_out = np.array(k_cache, dtype=np.float64, copy=True)
    v_out = np.array(v_cache, dtype=np.float64, copy=True)
    k_out[dst_rows] = k_new
    v_out[dst_rows] = v_new
    return k_out, v_out


# --------------------------------------------------------------------------
# step 5: causal attention of the chosen rows against the whole cache
# (Sec. 4.3 Stage II: complete recomputation, only for the selected tokens;
#  Eq. 1 for what an attention output is)
# --------------------------------------------------------------------------

def sparse_row_attn(q, k_cache, v_cache, row_pos, scale=None, dtype="f64"):
    """``out[i, h] = sum_{t <= row_pos[i]} softmax_t(q[i,h].k[t,g]*scale) v[t,g]``.

    ``q [m, Hq, D]``; caches ``[n_keys, Hkv, D]``; row ``i`` sees keys
    ``0 .. row_pos[i]`` inclusive.  Returns ``(out [m, Hq, D]`` rounded to
    ``dtype``, ``lse [m, Hq]`` natural-log normaliser, fp64``)``.
    """
    q = np.asarray(q, dtype=np.float64)
    k_cache = np.asarray(k_cache, dtype=np.float64)
    v_cache = np.asarray(v_cache, dtype=np.float64)
    row_pos = np.asarray(row_pos, dtype=np.int64)
    m, hq, d = q.shape
    n_keys, hkv, _ = k_cache.shape
    if m and (row_pos.min() < 0 or row_pos.max() >= n_keys):
        raise ValueError("row_pos outside the cache")
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    group = hq // hkv
    out = np.zeros((m, hq, d), dtype=np.float64)
    lse = np.zeros((m, hq), dtype=np.float64)
    visible = np.arange(n_keys)[None, :] <= row_pos[:, None]    # [m, n_keys]
    for h in range(hq):
        g = h // group
        s = (q[:, h, :] @ k_cache[:, g, :].T) * scale          # [m, n_keys]
        s = np.where(visible, s, -np.inf)
        top = s.max(axis=1, keepdims=True)
        p = np.exp(s - top)
        z = p.sum(axis=1, keepdims=True)
        out[:, h, :] = (p @ v_cache[:, g, :]) / z
        lse[:, h] = (top + np.log(z))[:, 0]
    return round_to_storage(out, dtype), lse


# --------------------------------------------------------------------------
# one layer of Stage II, and the whole two-stage method over a layer stack
# --------------------------------------------------------------------------

def selective_recompute_layer(k_rope, v_ctx, hidden, wq, wk, wv, sel, n_query,
                              n_q_heads, n_kv_heads, head_dim, theta, dtype):
    """Stage II for one layer, given the already-restored context keys.

    ``k_rope, v_ctx [N, Hkv, D]``; ``hidden [N + Qn, hid]``; ``sel`` the
    ascending selected context indices.  Rows recomputed are
    ``sel ++ [N .. N+Qn-1]``, each at the position equal to its row index.
    Returns a dict with the projected ``q, k_new, v_new``, the updated
    caches ``k_cache, v_cache [N + Qn, Hkv, D]``, ``rows``, and the
    attention ``out`` and ``lse``.
    """
    n = k_rope.shape[0]
    rows = np.concatenate([np.asarray(sel, np.int64),
                           np.arange(n, n + n_query, dtype=np.int64)])
    q, k_new, v_new = project_qkv_rows(hidden, rows, rows, wq, wk, wv,
                                       n_q_heads, n_kv_heads, head_dim,
                                       theta, dtype)
    k_cache = np.zeros((n + n_query, n_kv_heads, head_dim), np.float64)
    v_cache = np.zeros_like(k_cache)
    k_cache[:n] = k_rope
    v_cache[:n] = v_ctx
    k_cache, v_cache = scatter_kv(k_cache, v_cache, k_new, v_new, rows)
    out, lse = sparse_row_attn(q, k_cache, v_cache, rows, dtype=dtype)
    return dict(rows=rows, q=q, k_new=k_new, v_new=v_new,
                k_cache=k_cache, v_cache=v_cache, out=out, lse=lse)


def prophetkv_stack(layers, n_query, k, n_score_layers,
                    n_q_heads, n_kv_heads, head_dim, theta, dtype):
    """Algorithm 1 over a stack of layers with supplied per-layer hidden states.

    ``layers`` is a list of dicts with ``k_nope, v [N, Hkv, D]``,
    ``hidden [N + Qn, hid]``, ``wq, wk, wv``.  Stage I runs over the first
    ``n_score_layers`` layers (the paper uses all of them), Stage II over all.
    Returns ``(sel, fused_score_f32, [per-layer result dicts])``.
    """
    n = layers[0]["k_nope"].shape[0]
    ctx_pos = np.arange(n)
    q_rows = np.arange(n, n + n_query)
    k_rope = [rope_restore(l["k_nope"], ctx_pos, theta, dtype) for l in layers]

    score = np.zeros(n, dtype=np.float64)
    for li in range(n_score_layers):
        l = layers[li]
        q_s, _, _ = project_qkv_rows(l["hidden"], q_rows, q_rows,
                                     l["wq"], l["wk"], l["wv"],
                                     n_q_heads, n_kv_heads, head_dim,
                                     theta, dtype)
        score = fuse_score(score, query_score(q_s, k_rope[li]))
    sel = topk_select(score, k)

    results = []
    for li, l in enumerate(layers):
        results.append(selective_recompute_layer(
            k_rope[li], round_to_storage(l["v"], dtype), l["hidden"],
            l["wq"], l["wk"], l["wv"], sel, n_query,
            n_q_heads, n_kv_heads, head_dim, theta, dtype))
    return sel, score, results
