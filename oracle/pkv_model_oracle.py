"""CPU oracle for the layer glue around the selective-recomputation hot path.

TEST INFRASTRUCTURE, NOT PRODUCT CODE (same rules as ``pkv_oracle``: plain fp64
numpy, imported only by the tests, the smoke check and the benchmark's CPU leg).

What it adds: the parts of a decoder layer that sit between two runs of the hot
path when ProphetKV carries only the selected and the user-query rows through the
model (paper: Sec. 4.2, the query is run through the model against the imprecise
cache to obtain the attention it pays to the context; Sec. 4.3 and Appendix E, the
hidden states, positions and mask are pruned to the selected tokens and go through
every layer).  The paper names Llama-3.1-8B and Qwen models (Sec. 5.1) and does
not restate their block, so the block below is the public Llama one, stated here,
not derived from the paper:

    x = RMSNorm(h, w_in)                  y = RMSNorm(h', w_post)
    a = Attention(x Wq, x Wk, x Wv)       h'' = h' + (silu(y Wg^T) * (y Wu^T)) Wd^T
    h' = h + a Wo^T

Rounding points (a tensor kept in memory in the storage dtype is rounded there, as
a bf16 framework would): the normalised rows x and y; Q, K, V; the attention
output; every linear output BEFORE a residual is added, and the sum after; the
gate activation silu(.), the up projection, and their product.

Parity status: pinned against torch's CPU ``rms_norm``/``linear``/``silu`` on fp64
inputs, closed forms and the hot-path oracle (tests/test_model_oracle_pins.py);
none is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

from . import pkv_oracle as O

__all__ = ["rmsnorm_rows", "linear_rows", "swiglu_up", "attention_block_tail",
           "mlp_block", "prophetkv_model"]


def rmsnorm_rows(h, rows, weight, eps: float, dtype: str):
    """``y[i] = h[rows[i]] / sqrt(mean(h[rows[i]]^2) + eps) * weight``, rounded.

    ``h [tokens, hid]``; ``rows`` indices or ``None`` for all rows in order."""
    h = np.asarray(h, dtype=np.float64)
    x = h if rows is None else h[np.asarray(rows, dtype=np.int64)]
    ms = (x * x).mean(axis=1, keepdims=True)
    return O.round_to_storage(x / np.sqrt(ms + eps) * np.asarray(weight, np.float64), dtype)


def linear_rows(x, w, residual, dtype: str):
    """``round(x W^T)``, then, if a residual is given, ``round(. + residual)``.

    ``x [m, k]``, ``w [n, k]``, ``residual [m, n]`` or ``None``."""
    y = O.round_to_storage(np.asarray(x, np.float64) @ np.asarray(w, np.float64).T, dtype)
    if residual is not None:
        y = O.round_to_storage(y + np.asarray(residual, np.float64), dtype)
    return y


def swiglu_up(x, w_gate, w_up, dtype: str):
    """``round(round(silu(round(x Wg^T))) * round(x Wu^T))``; silu(a) = a / (1 + e^-a)."""
    x = np.asarray(x, np.float64)
    a = O.round_to_storage(x @ np.asarray(w_gate, np.float64).T, dtype)
    b = O.round_to_storage(x @ np.asarray(w_up, np.float64).T, dtype)
    s = O.round_to_storage(a / (1.0 + np.exp(-a)), dtype)
    return O.round_to_storage(s * b, dtype)


def attention_block_tail(h_rows, attn_out, wo, dtype: str):
    """``h' = h + attn_out Wo^T`` for rows already gathered; ``attn_out [m, Hq, D]``."""
    m = attn_out.shape[0]
    return linear_rows(attn_out.reshape(m, -1), wo, h_rows, dtype)


def mlp_block(h_rows, w_post, eps, w_gate, w_up, w_down, dtype: str):
    """``h'' = h' + (silu(y Wg^T) * (y Wu^T)) Wd^T`` with ``y = RMSNorm(h', w_post)``."""
    y = rmsnorm_rows(h_rows, None, w_post, eps, dtype)
    g = swiglu_up(y, w_gate, w_up, dtype)
    return linear_rows(g, w_down, h_rows, dtype)


def prophetkv_model(embed, layers, n_query, k, n_score_layers,
                    n_q_heads, n_kv_heads, head_dim, theta, eps, dtype, sel=None):
    """Both stages of Algorithm 1 with the hidden states carried through the layers.

    ``embed [N + Qn, hid]``: the layer-0 hidden state of every prompt token (context
    then query).  ``layers``: dicts with the precomputed position-free chunk caches
    ``k_nope, v [N, Hkv, D]`` of that layer and its weights ``w_in, wq, wk, wv, wo,
    w_post, w_gate, w_up, w_down``; optional ``bq, bk, bv`` (projection biases) and
    ``q_norm, k_norm`` (per-head RMS-norm gains, with the block's ``eps``).

    Stage I (Sec. 4.2): only the Qn query rows go through the first
    ``n_score_layers`` layers; in each, their attention to the restored context keys
    gives alpha_l (summed over layers), and their own attention output - over the
    imprecise cache plus their own causal keys - feeds the next layer.
    Stage II (Sec. 4.3, Appendix E): the rows ``T_p ++ query`` go through every
    layer; their K/V replace the cache rows before they attend to the cache.

    ``sel``: if given, Stage II uses this selection instead of the one Stage I finds
    (Stage I is still run and its score returned).  Returns ``(sel, score, out)``
    with ``out`` a dict: ``h_final [M, hid]``, ``rows``, per-layer lists ``k_cache``,
    ``v_cache``, ``attn`` and ``h`` (hidden of the rows after each layer), and
    ``stage1_h`` (query hidden after each scoring layer).
    """
    embed = np.asarray(embed, np.float64)
    n = layers[0]["k_nope"].shape[0]
    ctx_pos = np.arange(n)
    q_rows = np.arange(n, n + n_query)
    k_rope = [O.rope_restore(l["k_nope"], ctx_pos, theta, dtype) for l in layers]
    v_ctx = [O.round_to_storage(l["v"], dtype) for l in layers]

    def run_rows(h, rows, li, want_score):
        """One layer for the gathered rows ``h [m, hid]`` at positions ``rows``."""
        l = layers[li]
        x = rmsnorm_rows(h, None, l["w_in"], eps, dtype)
        q, k_new, v_new = O.project_qkv_rows(
            x, np.arange(len(rows)), rows, l["wq"], l["wk"], l["wv"], n_q_heads, n_kv_heads,
            head_dim, theta, dtype, bq=l.get("bq"), bk=l.get("bk"), bv=l.get("bv"),
            q_norm=l.get("q_norm"), k_norm=l.get("k_norm"), norm_eps=eps)
        alpha = None
        if want_score:   # the rows are exactly the query rows here
            alpha = O.query_score(q, k_rope[li])
        k_cache = np.zeros((n + n_query, n_kv_heads, head_dim), np.float64)
        v_cache = np.zeros_like(k_cache)
        k_cache[:n] = k_rope[li]
        v_cache[:n] = v_ctx[li]
        k_cache, v_cache = O.scatter_kv(k_cache, v_cache, k_new, v_new, rows)
        attn, _ = O.sparse_row_attn(q, k_cache, v_cache, rows, dtype=dtype)
        h1 = attention_block_tail(h, attn, l["wo"], dtype)
        h2 = mlp_block(h1, l["w_post"], eps, l["w_gate"], l["w_up"], l["w_down"], dtype)
        return h2, alpha, k_cache, v_cache, attn

    # ---- Stage I: the query rows alone, against the imprecise cache ---------------
    score = np.zeros(n, dtype=np.float64)
    hq = O.round_to_storage(embed[q_rows], dtype)
    stage1_h = []
    for li in range(n_score_layers):
        hq, alpha, _, _, _ = run_rows(hq, q_rows, li, True)
        score = O.fuse_score(score, alpha)
        stage1_h.append(hq)
    found = O.topk_select(score, k)
    if sel is None:
        sel = found

    # ---- Stage II: the selected and the query rows through every layer -------------
    rows = np.concatenate([np.asarray(sel, np.int64), q_rows])
    h = O.round_to_storage(embed[rows], dtype)
    out = dict(rows=rows, k_cache=[], v_cache=[], attn=[], h=[], stage1_h=stage1_h,
               selection_found=found)
    for li in range(len(layers)):
        h, _, kc, vc, attn = run_rows(h, rows, li, False)
        out["k_cache"].append(kc)
        out["v_cache"].append(vc)
        out["attn"].append(attn)
        out["h"].append(h)
    out["h_final"] = h
    return sel, score, out
