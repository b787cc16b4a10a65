"""Call sequence of the hot path over preallocated device buffers.

Orchestration only: this module allocates torch tensors once, then issues the
six C-ABI calls in the order of Algorithm 1 (Stage I scoring over the first
``n_score_layers`` layers, one top-p selection, Stage II recomputation in every
layer).  All arithmetic runs inside ``libpkv.so``.
"""

from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import api
from .synth import Config, select_count


def layer_cfg(cfg: Config) -> api.LayerCfg:
    return api.LayerCfg(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.hidden,
                        cfg.theta, cfg.dtype)


def upload_layer(cfg: Config, layer: Dict[str, np.ndarray],
                 device: torch.device) -> Dict[str, torch.Tensor]:
    """Host fp32 arrays (storage-exact values) -> device tensors in storage dtype.

    ``v_cache`` is the assembled value cache with room for the query rows
    appended after the context; ``k_nope`` stays position-free."""
    dt = layer_cfg(cfg).torch_dtype
    out = {name: torch.from_numpy(np.ascontiguousarray(layer[name])).to(dt).to(device)
           for name in ("k_nope", "hidden", "wq", "wk", "wv")}
    n, qn = cfg.n_ctx, cfg.n_query
    v_cache = torch.zeros((n + qn, cfg.n_kv_heads, cfg.head_dim), dtype=dt, device=device)
    v_cache[:n] = torch.from_numpy(np.ascontiguousarray(layer["v"])).to(dt).to(device)
    out["v_cache"] = v_cache
    out["k_cache"] = torch.zeros_like(v_cache)
    return out


class SelectiveRecompute:
    """Work buffers and the per-layer call sequence for one configuration."""

    def __init__(self, cfg: Config, device: torch.device, k: Optional[int] = None,
                 fused_scatter: bool = False):
        self.cfg = cfg
        # True: steps 4a and 4b in one call (K/V go straight to their cache rows)
        self.fused_scatter = fused_scatter
        self.lc = layer_cfg(cfg)
        self.device = device
        n, qn = cfg.n_ctx, cfg.n_query
        self.n, self.qn = n, qn
        self.k = select_count(cfg.ratio, n) if k is None else int(k)
        self.m = self.k + qn
        dt = self.lc.torch_dtype
        hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        i32 = dict(dtype=torch.int32, device=device)
        self.ctx_pos = None  # rope_restore uses pos_base + t
        self.q_rows = torch.arange(n, n + qn, **i32)
        self.rows = torch.empty(self.m, **i32)       # T_p ++ query rows
        self.rows[self.k:] = self.q_rows
        self.score = torch.zeros(n, dtype=torch.float32, device=device)
        self.q_s = torch.empty((qn, hq, d), dtype=dt, device=device)
        self.q = torch.empty((self.m, hq, d), dtype=dt, device=device)
        self.k_new = torch.empty((self.m, hkv, d), dtype=dt, device=device)
        self.v_new = torch.empty((self.m, hkv, d), dtype=dt, device=device)
        self.out = torch.empty((self.m, hq, d), dtype=dt, device=device)
        self.lse = torch.empty((self.m, hq), dtype=torch.float32, device=device)
        ws_bytes = max(
            api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, self.lc, n, qn),
            api.pkv_workspace_bytes(api.CALL_SPARSE_ROW_ATTN, self.lc, n + qn, self.m),
            api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, self.lc, 0, self.m),
            api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, self.lc, 0, qn),
            api.pkv_workspace_bytes(api.CALL_TOPK_SELECT, self.lc, n, 0),
            256)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=device)

    # ---- Stage I ---------------------------------------------------------
    def restore(self, L: Dict[str, torch.Tensor]) -> None:
        api.pkv_rope_restore(self.lc, L["k_nope"], L["k_cache"][:self.n], None, 0)

    def score_layer(self, L: Dict[str, torch.Tensor], accumulate: bool) -> None:
        api.pkv_gather_qkv_proj(self.lc, L["hidden"], self.q_rows, self.q_rows,
                                L["wq"], None, None, self.q_s, None, None, ws=self.ws)
        api.pkv_query_score(self.lc, self.q_s, L["k_cache"][:self.n], self.score,
                            accumulate=accumulate, ws=self.ws)

    def select(self) -> None:
        api.pkv_topk_select(self.score, self.k, self.rows, ws=self.ws)

    # ---- Stage II --------------------------------------------------------
    def recompute_layer(self, L: Dict[str, torch.Tensor]) -> None:
        if self.fused_scatter:
            api.pkv_gather_qkv_proj_scatter(self.lc, L["hidden"], self.rows, self.rows, L["wq"],
                                            L["wk"], L["wv"], self.q, L["k_cache"],
                                            L["v_cache"], self.rows, ws=self.ws)
        else:
            api.pkv_gather_qkv_proj(self.lc, L["hidden"], self.rows, self.rows, L["wq"],
                                    L["wk"], L["wv"], self.q, self.k_new, self.v_new,
                                    ws=self.ws)
            api.pkv_scatter_kv(self.lc, self.k_new, self.v_new, self.rows, L["k_cache"],
                               L["v_cache"])
        api.pkv_sparse_row_attn(self.lc, self.q, L["k_cache"], L["v_cache"], self.rows,
                                self.out, self.lse, ws=self.ws)

    # ---- whole path --------------------------------------------------------
    def run(self, layers: List[Dict[str, torch.Tensor]],
            n_score_layers: Optional[int] = None) -> None:
        """One pass of the whole hot path over ``layers`` (outputs of the last
        layer stay in ``self.out`` / ``self.lse``; caches are updated in place)."""
        ls = self.cfg.n_score_layers if n_score_layers is None else n_score_layers
        for li, L in enumerate(layers):
            self.restore(L)
            if li < ls:
                self.score_layer(L, accumulate=li > 0)
        self.select()
        for L in layers:
            self.recompute_layer(L)
