"""Both stages of ProphetKV with the hidden states carried through the layers.

Orchestration only, like ``pipeline``: preallocated torch buffers and the sequence
of C-ABI calls.  Stage I (Sec. 4.2) runs the user-query rows alone through the
first ``n_score_layers`` layers against the imprecise cache and accumulates their
attention to the context; Stage II (Sec. 4.3, Appendix E) runs the selected and the
query rows through every layer, replacing their cache rows before they attend.
Between the hot-path calls the rows pass through the rest of a pre-norm decoder
block (RMSNorm, output projection + residual, gated MLP + residual) - the public
Llama block of the models the paper evaluates (Sec. 5.1).
"""

from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import api
from .pipeline import layer_cfg
from .synth import Config, select_count

BLOCK_WEIGHTS = ("w_in", "wq", "wk", "wv", "wo", "w_post", "w_gate", "w_up", "w_down")
# block variants of the other public model families the paper evaluates (Sec. 5.1):
# projection biases (Qwen2.5) and per-head RMS-norm gains of Q and K (Qwen3)
VARIANT_WEIGHTS = ("bq", "bk", "bv", "q_norm", "k_norm")


def upload_block(cfg: Config, layer: Dict[str, np.ndarray],
                 device: torch.device) -> Dict[str, torch.Tensor]:
    """Host arrays of one layer (``k_nope, v`` and the block weights) -> device tensors;
    ``k_cache``/``v_cache`` get room for the query rows after the context."""
    dt = layer_cfg(cfg).torch_dtype
    names = ("k_nope",) + BLOCK_WEIGHTS + tuple(v for v in VARIANT_WEIGHTS if v in layer)
    out = {name: torch.from_numpy(np.ascontiguousarray(layer[name])).to(dt).to(device)
           for name in names}
    n, qn = cfg.n_ctx, cfg.n_query
    v_cache = torch.zeros((n + qn, cfg.n_kv_heads, cfg.head_dim), dtype=dt, device=device)
    v_cache[:n] = torch.from_numpy(np.ascontiguousarray(layer["v"])).to(dt).to(device)
    out["v_cache"] = v_cache
    out["k_cache"] = torch.zeros_like(v_cache)
    return out


class CarriedRows:
    """Work buffers and call sequence for one configuration and MLP width."""

    def __init__(self, cfg: Config, inter: int, eps: float, device: torch.device,
                 k: Optional[int] = None, fuse_stage1: Optional[bool] = None):
        self.cfg, self.inter, self.eps, self.device = cfg, int(inter), float(eps), device
        self.lc = layer_cfg(cfg)
        n, qn = cfg.n_ctx, cfg.n_query
        # Stage I with one key stream less: the query rows' attention emits the
        # normaliser over the context keys and the score only sums the columns
        # (None = whenever the library has it for this geometry)
        ctx_ws = api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(self.lc, n + qn, n, qn)
        self.fuse_stage1 = ctx_ws > 0 if fuse_stage1 is None else bool(fuse_stage1)
        if self.fuse_stage1 and ctx_ws == 0:
            raise ValueError("fused Stage I is not available for this geometry")
        self.n, self.qn = n, qn
        self.k = select_count(cfg.ratio, n) if k is None else int(k)
        self.m = self.k + qn
        dt = self.lc.torch_dtype
        hq, hkv, d, hid = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.hidden
        i32 = dict(dtype=torch.int32, device=device)
        new = lambda *shape: torch.empty(shape, dtype=dt, device=device)  # noqa: E731
        self.q_rows = torch.arange(n, n + qn, **i32)
        self.rows = torch.empty(self.m, **i32)          # T_p ++ query rows
        self.rows[self.k:] = self.q_rows
        self.score = torch.zeros(n, dtype=torch.float32, device=device)
        self.lse_ctx = torch.empty((qn, hq), dtype=torch.float32, device=device)
        rows_max = max(self.m, qn)
        self.h = new(rows_max, hid)                     # carried hidden states
        self.x = new(rows_max, hid)                     # normalised rows
        self.q = new(rows_max, hq, d)
        self.attn = new(rows_max, hq, d)
        self.g = new(rows_max, self.inter)
        tdt = dt
        ws_bytes = 256
        for rows in (self.m, qn):
            ws_bytes = max(
                ws_bytes,
                api.pkv_workspace_bytes(api.CALL_SPARSE_ROW_ATTN, self.lc, n + qn, rows),
                api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, self.lc, 0, rows),
                api.pkv_glue_workspace_bytes(tdt, rows, hq * d, hid),
                api.pkv_glue_workspace_bytes(tdt, rows, hid, self.inter),
                api.pkv_glue_workspace_bytes(tdt, rows, self.inter, hid))
        ws_bytes = max(ws_bytes, api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, self.lc, n, qn),
                       api.pkv_workspace_bytes(api.CALL_TOPK_SELECT, self.lc, n, 0), ctx_ws)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=device)

    # one decoder layer for the first ``cnt`` rows of the buffers, at positions ``rows``
    def _layer(self, L: Dict[str, torch.Tensor], rows: torch.Tensor, cnt: int,
               score: Optional[bool]) -> None:
        lc, ws = self.lc, self.ws
        h, x = self.h[:cnt], self.x[:cnt]
        q = self.q[:cnt]
        attn, g = self.attn[:cnt], self.g[:cnt]
        api.pkv_rmsnorm_rows(h, None, L["w_in"], self.eps, x)
        # Q/K/V of the rows; K and V go straight to their cache rows (steps 4a + 4b).  The
        # score of Stage I reads only the context rows of the key cache, which the query
        # rows' own keys (stored behind the context) do not touch.
        api.pkv_gather_qkv_proj_scatter(lc, x, None, rows, L["wq"], L["wk"], L["wv"], q,
                                        L["k_cache"], L["v_cache"], rows, ws=ws,
                                        norm_eps=self.eps,
                                        **{v: L[v] for v in VARIANT_WEIGHTS if v in L})
        if score is not None and self.fuse_stage1:
            api.pkv_sparse_row_attn_ctx_lse(lc, q, L["k_cache"], L["v_cache"], rows, attn, None,
                                            self.lse_ctx[:cnt], self.n, ws=ws)
            api.pkv_query_score_lse(lc, q, L["k_cache"][:self.n], self.lse_ctx[:cnt], None,
                                    self.score, accumulate=score, ws=ws)
        else:
            if score is not None:
                api.pkv_query_score(lc, q, L["k_cache"][:self.n], self.score,
                                    accumulate=score, ws=ws)
            api.pkv_sparse_row_attn(lc, q, L["k_cache"], L["v_cache"], rows, attn, None,
                                    ws=ws)
        api.pkv_linear_rows(attn.view(cnt, -1), L["wo"], h, h, ws=ws)
        api.pkv_rmsnorm_rows(h, None, L["w_post"], self.eps, x)
        api.pkv_swiglu_rows(x, L["w_gate"], L["w_up"], g, ws=ws)
        api.pkv_linear_rows(g, L["w_down"], h, h, ws=ws)

    def stage1(self, embed: torch.Tensor, layers: List[Dict[str, torch.Tensor]],
               n_score_layers: Optional[int] = None) -> None:
        """Restores every layer's context keys, scores with the query rows over the first
        ``n_score_layers`` layers and writes the selection into ``self.rows[:k]``."""
        ls = self.cfg.n_score_layers if n_score_layers is None else n_score_layers
        api.pkv_gather_rows(embed, self.q_rows, self.h[:self.qn])
        for li, L in enumerate(layers):
            api.pkv_rope_restore(self.lc, L["k_nope"], L["k_cache"][:self.n], None, 0)
            if li < ls:
                self._layer(L, self.q_rows, self.qn, score=li > 0)
        api.pkv_topk_select(self.score, self.k, self.rows, ws=self.ws)

    def stage2(self, embed: torch.Tensor, layers: List[Dict[str, torch.Tensor]]) -> torch.Tensor:
        """The rows ``self.rows`` through every layer; returns their final hidden states
        (a view of the work buffer).  Caches are updated in place."""
        api.pkv_gather_rows(embed, self.rows, self.h[:self.m])
        for L in layers:
            self._layer(L, self.rows, self.m, score=None)
        return self.h[:self.m]

    def run(self, embed, layers, n_score_layers: Optional[int] = None) -> torch.Tensor:
        self.stage1(embed, layers, n_score_layers)
        return self.stage2(embed, layers)
