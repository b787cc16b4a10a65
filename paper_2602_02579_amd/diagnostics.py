"""Selection diagnostics of the paper on synthetic models, through the C ABI.

Orchestration only, like ``pipeline`` and ``model``: torch buffers and sequences of
library calls; the set arithmetic of the overlap ratio is host bookkeeping on the
downloaded index lists.

* ``chunk_isolated_cache`` / ``full_prefill_cache``: the producer of the method's input
  (Sec. 2: every chunk is prefilled by itself and its keys are stored without
  positions) and the ordinary prefill it stands in for.  A prefill of T tokens is Stage II
  of the carried-rows model with every row selected.
* ``query_attention_score``: the fused user-query attention to the context (Algorithm 1,
  first stage) over given caches - ProphetKV's criterion on the chunk caches, the ground
  truth G of Sec. 3.1 (Fig. 2) on the full-prefill ones.
* ``column_sum_score``: the attention every context token receives from ALL rows of the
  prompt at one layer (Appendix B, Tab. 3, first factor of the KVShare row), the
  criterion whose budget the globally salient tokens crowd (Sec. 3.1).
* ``overlap_ratio``: |S n G| / |G|.
"""

from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import api
from .model import BLOCK_WEIGHTS, VARIANT_WEIGHTS, CarriedRows
from .pipeline import layer_cfg
from .synth import Config, select_count

Block = Dict[str, torch.Tensor]


def overlap_ratio(selected: torch.Tensor, ground_truth: torch.Tensor) -> float:
    """|S n G| / |G| of two index tensors (Sec. 3.1)."""
    s = np.unique(selected.detach().cpu().numpy())
    g = np.unique(ground_truth.detach().cpu().numpy())
    if g.size == 0:
        raise ValueError("empty ground-truth set")
    return float(np.intersect1d(s, g).size) / float(g.size)


def top_indices(score: torch.Tensor, k: int) -> torch.Tensor:
    idx = torch.empty(k, dtype=torch.int32, device=score.device)
    api.pkv_topk_select(score, k, idx)
    return idx


class Diagnostics:
    """Work buffers for one model geometry (``cfg``: context, query and head sizes; the
    block weights are passed to the methods as lists of device tensors)."""

    def __init__(self, cfg: Config, inter: int, eps: float, device: torch.device):
        self.cfg, self.inter, self.eps, self.device = cfg, int(inter), float(eps), device
        self.lc = layer_cfg(cfg)
        self.dt = self.lc.torch_dtype
        self._prefill: Dict[int, CarriedRows] = {}
        self._stage1: Optional[CarriedRows] = None

    def _cache_pair(self, rows: int) -> Tuple[torch.Tensor, torch.Tensor]:
        shape = (rows, self.cfg.n_kv_heads, self.cfg.head_dim)
        return (torch.zeros(shape, dtype=self.dt, device=self.device),
                torch.zeros(shape, dtype=self.dt, device=self.device))

    # ---- producers -------------------------------------------------------------------
    def prefill_cache(self, embed_rows: torch.Tensor,
                      blocks: Sequence[Block]) -> Tuple[List[torch.Tensor], List[torch.Tensor]]:
        """Ordinary causal prefill of ``embed_rows [T, hid]`` at positions 0..T-1; returns
        per layer the keys in their stored, position-free form and the values."""
        t = embed_rows.shape[0]
        if t < 2:
            raise ValueError("a chunk needs at least two tokens")
        cr = self._prefill.get(t)
        if cr is None:   # every row recomputed: T - 1 "selected" rows and one closing row
            sub = self.cfg.with_(n_chunks=1, chunk_len=t - 1, n_query=1)
            cr = CarriedRows(sub, self.inter, self.eps, self.device, k=t - 1)
            cr.rows[:t - 1] = torch.arange(t - 1, dtype=torch.int32, device=self.device)
            cr.neg_pos = -torch.arange(t, dtype=torch.int32, device=self.device)
            self._prefill[t] = cr
        layers = []
        for b in blocks:
            L = {name: b[name] for name in BLOCK_WEIGHTS + VARIANT_WEIGHTS if name in b}
            L["k_cache"], L["v_cache"] = self._cache_pair(t)
            layers.append(L)
        cr.stage2(embed_rows.contiguous(), layers)
        k_nope = []
        for L in layers:
            out = torch.empty_like(L["k_cache"])
            api.pkv_rope_restore(self.lc, L["k_cache"], out, cr.neg_pos)   # inverse rotation
            k_nope.append(out)
        return k_nope, [L["v_cache"] for L in layers]

    def chunk_isolated_cache(self, embed: torch.Tensor, blocks: Sequence[Block],
                             chunk_len: int):
        """Per-layer ``(k_nope, v) [n_ctx, Hkv, D]`` with every chunk prefilled alone."""
        n = self.cfg.n_ctx
        ks = [[] for _ in blocks]
        vs = [[] for _ in blocks]
        for a in range(0, n, chunk_len):
            k, v = self.prefill_cache(embed[a:min(a + chunk_len, n)], blocks)
            for li in range(len(blocks)):
                ks[li].append(k[li])
                vs[li].append(v[li])
        return [torch.cat(x) for x in ks], [torch.cat(x) for x in vs]

    def full_prefill_cache(self, embed: torch.Tensor, blocks: Sequence[Block]):
        return self.chunk_isolated_cache(embed, blocks, self.cfg.n_ctx)

    # ---- criteria --------------------------------------------------------------------
    def _layers_with_cache(self, blocks, k_nope, v):
        n, qn = self.cfg.n_ctx, self.cfg.n_query
        layers = []
        for li, b in enumerate(blocks):
            L = {name: b[name] for name in BLOCK_WEIGHTS + VARIANT_WEIGHTS if name in b}
            L["k_nope"] = k_nope[li]
            L["k_cache"], L["v_cache"] = self._cache_pair(n + qn)
            L["v_cache"][:n] = v[li]
            layers.append(L)
        return layers

    def query_attention_score(self, embed: torch.Tensor, blocks: Sequence[Block],
                              k_nope, v, n_score_layers: int) -> torch.Tensor:
        """Fused Stage I score of the user-query rows over the given per-layer caches."""
        if self._stage1 is None:
            self._stage1 = CarriedRows(self.cfg, self.inter, self.eps, self.device, k=0)
        cr = self._stage1
        layers = self._layers_with_cache(blocks[:n_score_layers], k_nope, v)
        cr.stage1(embed, layers, n_score_layers)
        return cr.score.clone()

    def column_sum_score(self, embed: torch.Tensor, block: Block, k_nope: torch.Tensor,
                         v: torch.Tensor) -> torch.Tensor:
        """Attention received by every context token from all prompt rows at the layer
        ``block`` whose (normalised) input rows are RMSNorm(embed) - the first layer."""
        n, qn = self.cfg.n_ctx, self.cfg.n_query
        x = torch.empty_like(embed)
        api.pkv_rmsnorm_rows(embed, None, block["w_in"], self.eps, x)
        return self.column_sum_from_hidden(x, block, k_nope, v)

    def column_sum_from_hidden(self, hidden: torch.Tensor, w: Block, k_nope: torch.Tensor,
                               v: torch.Tensor) -> torch.Tensor:
        """The same with the layer's input rows ``hidden [n_ctx + n_query, hid]`` supplied
        (``w`` holds ``wq, wk, wv``): context keys are the restored chunk keys, the query
        rows' keys are projected; every row attends causally over that cache."""
        cfg, lc = self.cfg, self.lc
        n, qn = cfg.n_ctx, cfg.n_query
        t = n + qn
        dev = self.device
        pos = torch.arange(t, dtype=torch.int32, device=dev)
        k_cache, v_cache = self._cache_pair(t)
        v_cache[:n] = v
        api.pkv_rope_restore(lc, k_nope, k_cache[:n], None, 0)
        q = torch.empty((t, cfg.n_q_heads, cfg.head_dim), dtype=self.dt, device=dev)
        ws = torch.empty(max(api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, lc, 0, t),
                             api.pkv_workspace_bytes(api.CALL_SPARSE_ROW_ATTN, lc, t, t),
                             api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, lc, t, t), 256),
                         dtype=torch.uint8, device=dev)
        variant = {name: w[name] for name in VARIANT_WEIGHTS if name in w}
        api.pkv_gather_qkv_proj_ex(lc, hidden, None, pos, w["wq"], None, None, q, None, None,
                                   ws=ws, norm_eps=self.eps, **variant)
        q_tail = torch.empty((qn, cfg.n_q_heads, cfg.head_dim), dtype=self.dt, device=dev)
        api.pkv_gather_qkv_proj_scatter(lc, hidden, pos[n:], pos[n:], w["wq"], w["wk"], w["wv"],
                                        q_tail, k_cache, v_cache, pos[n:], ws=ws,
                                        norm_eps=self.eps, **variant)
        out = torch.empty_like(q)
        lse = torch.empty((t, cfg.n_q_heads), dtype=torch.float32, device=dev)
        api.pkv_sparse_row_attn(lc, q, k_cache, v_cache, pos, out, lse, ws=ws)
        beta = torch.empty(t, dtype=torch.float32, device=dev)
        api.pkv_query_score_lse(lc, q, k_cache, lse, pos, beta, accumulate=False, ws=ws)
        return beta[:n].clone()

    # ---- the tables ------------------------------------------------------------------
    def selection_diagnostics(self, embed: torch.Tensor, blocks: Sequence[Block],
                              chunk_len: int, ratios: Sequence[float]):
        """Overlap with the full-prefill ground truth (Sec. 3.1) of the fused
        query-attention criterion, its first-layer-only form (Sec. 4.3) and the global
        column sum of the first layer (Appendix B), at each selection ratio."""
        n = self.cfg.n_ctx
        n_layers = len(blocks)
        kc, vc = self.chunk_isolated_cache(embed, blocks, chunk_len)
        kf, vf = self.full_prefill_cache(embed, blocks)
        scores = dict(
            truth=self.query_attention_score(embed, blocks, kf, vf, n_layers),
            fused=self.query_attention_score(embed, blocks, kc, vc, n_layers),
            first_layer=self.query_attention_score(embed, blocks, kc, vc, 1),
            column_sum=self.column_sum_score(embed, blocks[0], kc[0], vc[0]))
        out = dict(fused=[], first_layer=[], column_sum=[], scores=scores)
        for r in ratios:
            k = select_count(r, n)
            g = top_indices(scores["truth"], k)
            for name in ("fused", "first_layer", "column_sum"):
                out[name].append(overlap_ratio(top_indices(scores[name], k), g))
        return out
