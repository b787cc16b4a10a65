"""CPU oracle for the paper's selection diagnostics on synthetic models.

TEST INFRASTRUCTURE, NOT PRODUCT CODE (same rules as ``pkv_oracle``: plain fp64
numpy, imported only by the tests, the smoke check and the benchmark's CPU leg).

What it restates (each from the paper, on models with random weights, since neither
the paper's datasets nor trained weights are available):

* the producer of the method's input: chunk-wise *isolated* precomputation of the
  KV cache (Sec. 2: every chunk is prefilled by itself, its keys stored without
  positions) and the ordinary full prefill it approximates;
* the ground truth of Sec. 3.1 / Fig. 2: ``G`` = the context tokens that the user
  query attends to most under full prefill, and the overlap ratio ``|S n G| / |G|``
  of a selected set ``S`` with it;
* the global column-sum criterion of Appendix B, Tab. 3 (the attention a token
  receives from ALL rows of the prompt, the first factor of the KVShare row), for the
  crowding-out contrast of Sec. 3.1: tokens that everything attends to fill the
  budget although the user query does not care for them;
* the chunk-size sweep of Sec. 5.5 (smaller chunks lose more cross-chunk attention).

Parity status: pinned in tests/test_diag_oracle_pins.py against brute force, closed
forms (one chunk = full prefill; the first layer's chunk-isolated K/V are exact) and the
model oracle; none is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

from . import pkv_model_oracle as MO
from . import pkv_oracle as O

__all__ = ["overlap_ratio", "column_sum_score", "prefill_rows", "chunk_isolated_cache",
           "full_prefill_cache", "query_attention_score", "selection_diagnostics"]


def overlap_ratio(selected, ground_truth) -> float:
    """``|S n G| / |G|`` (Sec. 3.1, Fig. 2) for two index sets."""
    g = np.unique(np.asarray(ground_truth, dtype=np.int64))
    s = np.unique(np.asarray(selected, dtype=np.int64))
    if g.size == 0:
        raise ValueError("empty ground-truth set")
    return float(np.intersect1d(s, g).size) / float(g.size)


def column_sum_score(q, k_cache, row_pos, scale=None):
    """Attention each key RECEIVES from all rows (Appendix B, Tab. 3: sum_n Phi_{n,t}).

    ``q [m, Hq, D]`` are the rotated queries of m rows, row ``i`` seeing keys
    ``0 .. row_pos[i]`` of ``k_cache [n_keys, Hkv, D]``; ``Phi`` is the causal softmax
    of every (row, head).  Returns ``beta [n_keys]`` = the mean over rows and heads of
    ``Phi[i, h, t]`` (zero where a row does not see the key) - rank-equivalent to the
    plain sum.
    """
    q = np.asarray(q, np.float64)
    k_cache = np.asarray(k_cache, np.float64)
    row_pos = np.asarray(row_pos, np.int64)
    m, hq, d = q.shape
    n_keys, hkv, _ = k_cache.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    group = hq // hkv
    visible = np.arange(n_keys)[None, :] <= row_pos[:, None]
    beta = np.zeros(n_keys)
    for h in range(hq):
        s = (q[:, h, :] @ k_cache[:, h // group, :].T) * scale
        s = np.where(visible, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        beta += p.sum(axis=0)
    return beta / (hq * m)


def prefill_rows(embed_rows, layers, positions, n_q_heads, n_kv_heads, head_dim, theta,
                 eps, dtype):
    """Ordinary causal forward of a token sequence through the block stack.

    ``embed_rows [T, hid]`` at rotary positions ``positions [T]`` (ascending).  Returns
    per-layer lists ``k`` (rotated keys), ``v``, and the final hidden states.  Every
    row attends to the rows before it and itself; nothing is reused.
    """
    h = O.round_to_storage(np.asarray(embed_rows, np.float64), dtype)
    t = h.shape[0]
    positions = np.asarray(positions, np.int64)
    order = np.arange(t)
    ks, vs = [], []
    for l in layers:
        x = MO.rmsnorm_rows(h, None, l["w_in"], eps, dtype)
        q, k, v = O.project_qkv_rows(x, order, positions, l["wq"], l["wk"], l["wv"],
                                     n_q_heads, n_kv_heads, head_dim, theta, dtype,
                                     bq=l.get("bq"), bk=l.get("bk"), bv=l.get("bv"),
                                     q_norm=l.get("q_norm"), k_norm=l.get("k_norm"),
                                     norm_eps=eps)
        attn, _ = O.sparse_row_attn(q, k, v, order, dtype=dtype)   # row i sees rows 0..i
        h = MO.attention_block_tail(h, attn, l["wo"], dtype)
        h = MO.mlp_block(h, l["w_post"], eps, l["w_gate"], l["w_up"], l["w_down"], dtype)
        ks.append(k)
        vs.append(v)
    return ks, vs, h


def _position_free(k_rot, positions, theta, dtype):
    """Stored form of precomputed keys: the inverse rotation, rounded to storage."""
    return O.rope_restore(k_rot, -np.asarray(positions, np.int64), theta, dtype)


def chunk_isolated_cache(embed, layers, n_ctx, chunk_len, **geo):
    """Per-layer ``(k_nope, v) [n_ctx, Hkv, D]`` from prefilling every chunk by itself.

    Chunk ``c`` holds tokens ``c * chunk_len ..`` (the last one may be shorter), runs
    through the whole stack alone at positions ``0 .. len - 1`` and so misses all
    attention to earlier chunks from the second layer on (Sec. 2)."""
    theta, dtype = geo["theta"], geo["dtype"]
    k_nope = [[] for _ in layers]
    v_all = [[] for _ in layers]
    for a in range(0, n_ctx, chunk_len):
        b = min(a + chunk_len, n_ctx)
        pos = np.arange(b - a)
        ks, vs, _ = prefill_rows(embed[a:b], layers, pos, **geo)
        for li in range(len(layers)):
            k_nope[li].append(_position_free(ks[li], pos, theta, dtype))
            v_all[li].append(vs[li])
    return [np.concatenate(x) for x in k_nope], [np.concatenate(x) for x in v_all]


def full_prefill_cache(embed, layers, n_ctx, **geo):
    """The same storage form for an ordinary prefill of the whole context."""
    return chunk_isolated_cache(embed, layers, n_ctx, n_ctx, **geo)


def query_attention_score(embed, layers, k_nope, v, n_query, n_score_layers, **geo):
    """Fused user-query attention to the context (Algorithm 1, first stage) over the
    given per-layer caches: with the chunk-isolated ones this is ProphetKV's value
    function, with the full-prefill ones the ground truth G of Sec. 3.1 is its top
    part (the query rows' hidden states are then those of a full prefill)."""
    with_cache = [dict(l, k_nope=k_nope[li], v=v[li]) for li, l in enumerate(layers)]
    _, score, _ = MO.prophetkv_model(embed, with_cache, n_query, 0, n_score_layers,
                                     geo["n_q_heads"], geo["n_kv_heads"], geo["head_dim"],
                                     geo["theta"], geo["eps"], geo["dtype"])
    return score


def selection_diagnostics(embed, layers, n_ctx, n_query, chunk_len, ratios, **geo):
    """Overlap ratios with the full-prefill ground truth (Sec. 3.1) for three criteria
    at each selection ratio: the fused query-attention score over all layers, the
    first layer's alone (Sec. 4.3's ablation), and the global column sum of the first
    layer's attention over the assembled chunk caches (Appendix B, Tab. 3).

    Returns a dict ``{name: [overlap per ratio]}`` plus the score vectors."""
    n_layers = len(layers)
    kc, vc = chunk_isolated_cache(embed, layers, n_ctx, chunk_len, **geo)
    kf, vf = full_prefill_cache(embed, layers, n_ctx, **geo)
    truth = query_attention_score(embed, layers, kf, vf, n_query, n_layers, **geo)
    fused = query_attention_score(embed, layers, kc, vc, n_query, n_layers, **geo)
    first = query_attention_score(embed, layers, kc, vc, n_query, 1, **geo)
    # global column sum at the first layer: every prompt row's attention over the
    # assembled cache (context keys restored to their positions, query keys appended)
    l0 = layers[0]
    theta, dtype = geo["theta"], geo["dtype"]
    pos = np.arange(n_ctx + n_query)
    x = MO.rmsnorm_rows(O.round_to_storage(embed, dtype), None, l0["w_in"], geo["eps"], dtype)
    q_all, k_q, _ = O.project_qkv_rows(x, pos, pos, l0["wq"], l0["wk"], l0["wv"],
                                       geo["n_q_heads"], geo["n_kv_heads"], geo["head_dim"],
                                       theta, dtype)
    k_asm = np.concatenate([O.rope_restore(kc[0], np.arange(n_ctx), theta, dtype),
                            k_q[n_ctx:]])
    colsum = column_sum_score(q_all, k_asm, pos)[:n_ctx]
    out = dict(fused=[], first_layer=[], column_sum=[], scores=dict(
        truth=truth, fused=fused, first_layer=first, column_sum=colsum))
    for r in ratios:
        k = int(np.floor(r * n_ctx + 1e-9))
        g = O.topk_select(truth, k)
        out["fused"].append(overlap_ratio(O.topk_select(fused, k), g))
        out["first_layer"].append(overlap_ratio(O.topk_select(first, k), g))
        out["column_sum"].append(overlap_ratio(O.topk_select(colsum, k), g))
    return out
