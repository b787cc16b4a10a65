"""Python binding of the pkv C ABI (``include/pkv.h``).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, checks shapes/dtypes/contiguity on the host, passes raw
device pointers and the current HIP stream to ``libpkv.so`` and raises
``PkvError`` on a non-zero status.  No arithmetic happens here and there is
no fallback: if the compiled library is missing, loading fails loudly.
"""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

__all__ = ["LayerCfg", "PkvError", "load_library", "library_path",
           "pkv_rope_restore", "pkv_query_score", "pkv_query_score_static",
           "pkv_query_score_lse", "pkv_sparse_row_attn_ctx_lse",
           "pkv_sparse_row_attn_ctx_lse_workspace_bytes",
           "pkv_topk_select", "pkv_gather_qkv_proj", "pkv_gather_qkv_proj_ex",
           "pkv_gather_qkv_proj_scatter", "pkv_scatter_kv",
           "pkv_sparse_row_attn", "pkv_rmsnorm_rows", "pkv_gather_rows", "pkv_linear_rows", "pkv_swiglu_rows",
           "pkv_glue_workspace_bytes",
           "pkv_workspace_bytes", "pkv_status_string", "pkv_version",
           "EXPORTED_SYMBOLS"]

PKV_F32, PKV_BF16 = 0, 1
CALL_ROPE_RESTORE, CALL_QUERY_SCORE, CALL_TOPK_SELECT = 1, 2, 3
CALL_GATHER_QKV_PROJ, CALL_SCATTER_KV, CALL_SPARSE_ROW_ATTN = 4, 5, 6

STATIC_SCRATCH_BYTES = 16 << 20   # PKV_STATIC_SCRATCH_BYTES of the header

EXPORTED_SYMBOLS = [
    "pkv_rope_restore", "pkv_query_score", "pkv_query_score_static", "pkv_topk_select",
    "pkv_gather_qkv_proj", "pkv_gather_qkv_proj_ex", "pkv_gather_qkv_proj_scatter",
    "pkv_scatter_kv", "pkv_sparse_row_attn", "pkv_rmsnorm_rows", "pkv_gather_rows", "pkv_linear_rows", "pkv_swiglu_rows",
    "pkv_glue_workspace_bytes", "pkv_query_score_lse", "pkv_sparse_row_attn_ctx_lse",
    "pkv_sparse_row_attn_ctx_lse_workspace_bytes",
    "pkv_workspace_bytes", "pkv_status_string", "pkv_version",
]


class PkvError(RuntimeError):
    def __init__(self, call: str, status: int, text: str):
        super().__init__(f"{call} failed: status {status} ({text})")
        self.status = status


class _CVariant(ctypes.Structure):
    _fields_ = [("bq", ctypes.c_void_p), ("bk", ctypes.c_void_p), ("bv", ctypes.c_void_p),
                ("q_norm", ctypes.c_void_p), ("k_norm", ctypes.c_void_p),
                ("norm_eps", ctypes.c_float)]


class _CCfg(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("rope_theta", ctypes.c_float), ("dtype", ctypes.c_int32)]


@dataclass(frozen=True)
class LayerCfg:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int
    rope_theta: float
    dtype: str  # "f32" or "bf16"

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    def _c(self) -> _CCfg:
        return _CCfg(self.n_q_heads, self.n_kv_heads, self.head_dim, self.hidden,
                     float(self.rope_theta), {"f32": PKV_F32, "bf16": PKV_BF16}[self.dtype])


_LIB: Optional[ctypes.CDLL] = None


def library_path() -> str:
    """Path of the compiled library; PKV_LIBRARY overrides it (for developers who
    compare builds), there is still no fallback if the file is missing."""
    override = os.environ.get("PKV_LIBRARY")
    if override:
        return override
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpkv.so")


def load_library() -> ctypes.CDLL:
    """Load ``libpkv.so`` (once).  Raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2602_02579_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i64, i32p, f32p = (ctypes.c_void_p, ctypes.c_int64,
                           ctypes.c_void_p, ctypes.c_void_p)
    cfgp = ctypes.POINTER(_CCfg)
    lib.pkv_rope_restore.argtypes = [cfgp, vp, vp, i32p, i64, i64, vp]
    lib.pkv_query_score.argtypes = [cfgp, vp, vp, f32p, i64, i64, ctypes.c_float,
                                    ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.pkv_query_score_static.argtypes = [cfgp, vp, vp, f32p, i64, i64, ctypes.c_float,
                                           ctypes.c_int, vp]
    lib.pkv_topk_select.argtypes = [f32p, i64, i64, i32p, vp, ctypes.c_size_t, vp]
    lib.pkv_query_score_lse.argtypes = [cfgp, vp, vp, f32p, i32p, f32p, i64, i64,
                                        ctypes.c_float, ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.pkv_sparse_row_attn_ctx_lse.argtypes = [cfgp, vp, vp, vp, i32p, vp, f32p, f32p, i64,
                                                i64, i64, ctypes.c_float, vp,
                                                ctypes.c_size_t, vp]
    lib.pkv_sparse_row_attn_ctx_lse_workspace_bytes.argtypes = [cfgp, i64, i64, i64]
    lib.pkv_sparse_row_attn_ctx_lse_workspace_bytes.restype = ctypes.c_size_t
    lib.pkv_gather_qkv_proj.argtypes = [cfgp, vp, i32p, i32p, vp, vp, vp, vp, vp, vp,
                                        i64, vp, ctypes.c_size_t, vp]
    lib.pkv_gather_qkv_proj_ex.argtypes = [cfgp, vp, i32p, i32p, vp, vp, vp,
                                           ctypes.POINTER(_CVariant), vp, vp, vp,
                                           i64, vp, ctypes.c_size_t, vp]
    lib.pkv_gather_qkv_proj_scatter.argtypes = [cfgp, vp, i32p, i32p, vp, vp, vp,
                                                ctypes.POINTER(_CVariant), vp, vp, vp, i32p,
                                                i64, i64, vp, ctypes.c_size_t, vp]
    lib.pkv_scatter_kv.argtypes = [cfgp, vp, vp, i32p, vp, vp, i64, i64, vp]
    lib.pkv_sparse_row_attn.argtypes = [cfgp, vp, vp, vp, i32p, vp, f32p, i64, i64,
                                        ctypes.c_float, vp, ctypes.c_size_t, vp]
    i32 = ctypes.c_int32
    lib.pkv_rmsnorm_rows.argtypes = [i32, vp, i32p, vp, ctypes.c_float, vp, i64, i64, vp]
    lib.pkv_gather_rows.argtypes = [i32, vp, i32p, vp, i64, i64, vp]
    lib.pkv_linear_rows.argtypes = [i32, vp, vp, vp, vp, i64, i64, i64, vp,
                                    ctypes.c_size_t, vp]
    lib.pkv_swiglu_rows.argtypes = [i32, vp, vp, vp, vp, i64, i64, i64, vp,
                                    ctypes.c_size_t, vp]
    lib.pkv_glue_workspace_bytes.argtypes = [i32, i64, i64, i64]
    lib.pkv_glue_workspace_bytes.restype = ctypes.c_size_t
    for name in ("pkv_rope_restore", "pkv_query_score", "pkv_query_score_static",
                 "pkv_topk_select", "pkv_query_score_lse", "pkv_sparse_row_attn_ctx_lse",
                 "pkv_gather_qkv_proj", "pkv_gather_qkv_proj_ex",
                 "pkv_gather_qkv_proj_scatter", "pkv_scatter_kv",
                 "pkv_sparse_row_attn", "pkv_rmsnorm_rows", "pkv_gather_rows", "pkv_linear_rows",
                 "pkv_swiglu_rows"):
        getattr(lib, name).restype = ctypes.c_int
    lib.pkv_workspace_bytes.argtypes = [ctypes.c_int, cfgp, i64, i64]
    lib.pkv_workspace_bytes.restype = ctypes.c_size_t
    lib.pkv_status_string.argtypes = [ctypes.c_int]
    lib.pkv_status_string.restype = ctypes.c_char_p
    lib.pkv_version.argtypes = []
    lib.pkv_version.restype = ctypes.c_int
    _LIB = lib
    return lib


def pkv_status_string(status: int) -> str:
    return load_library().pkv_status_string(int(status)).decode()


def pkv_version() -> int:
    return load_library().pkv_version()


def _check(call: str, status: int) -> None:
    if status != 0:
        raise PkvError(call, status, pkv_status_string(status))


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype], name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    if not ws.is_cuda or not ws.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def pkv_workspace_bytes(which_call: int, cfg: LayerCfg, n: int, m: int) -> int:
    c = cfg._c()
    return int(load_library().pkv_workspace_bytes(which_call, ctypes.byref(c), n, m))


def pkv_rope_restore(cfg: LayerCfg, k_in: torch.Tensor, k_out: torch.Tensor,
                     pos: Optional[torch.Tensor] = None, pos_base: int = 0) -> None:
    n = k_in.shape[0]
    if tuple(k_in.shape) != (n, cfg.n_kv_heads, cfg.head_dim) or k_out.shape != k_in.shape:
        raise ValueError("k_in/k_out must be [n, Hkv, D]")
    if pos is not None and tuple(pos.shape) != (n,):
        raise ValueError("pos must be [n]")
    c = cfg._c()
    _check("pkv_rope_restore", load_library().pkv_rope_restore(
        ctypes.byref(c), _ptr(k_in, cfg.torch_dtype, "k_in"),
        _ptr(k_out, cfg.torch_dtype, "k_out"), _ptr(pos, torch.int32, "pos"),
        int(pos_base), n, _stream()))


def pkv_query_score(cfg: LayerCfg, q: torch.Tensor, k: torch.Tensor,
                    score: torch.Tensor, accumulate: bool = False,
                    softmax_scale: float = 0.0,
                    ws: Optional[torch.Tensor] = None) -> None:
    nq, n_ctx = q.shape[0], k.shape[0]
    if tuple(q.shape) != (nq, cfg.n_q_heads, cfg.head_dim):
        raise ValueError("q must be [nq, Hq, D]")
    if tuple(k.shape) != (n_ctx, cfg.n_kv_heads, cfg.head_dim):
        raise ValueError("k must be [n_ctx, Hkv, D]")
    if tuple(score.shape) != (n_ctx,):
        raise ValueError("score must be [n_ctx]")
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_query_score", load_library().pkv_query_score(
        ctypes.byref(c), _ptr(q, cfg.torch_dtype, "q"), _ptr(k, cfg.torch_dtype, "k"),
        _ptr(score, torch.float32, "score"), nq, n_ctx, float(softmax_scale),
        int(bool(accumulate)), wp, wb, _stream()))


def pkv_query_score_static(cfg: LayerCfg, q: torch.Tensor, k: torch.Tensor,
                           score: torch.Tensor, accumulate: bool = False,
                           softmax_scale: float = 0.0) -> None:
    """pkv_query_score without a workspace (scratch inside the library)."""
    nq, n_ctx = q.shape[0], k.shape[0]
    if tuple(q.shape) != (nq, cfg.n_q_heads, cfg.head_dim):
        raise ValueError("q must be [nq, Hq, D]")
    if tuple(k.shape) != (n_ctx, cfg.n_kv_heads, cfg.head_dim):
        raise ValueError("k must be [n_ctx, Hkv, D]")
    if tuple(score.shape) != (n_ctx,):
        raise ValueError("score must be [n_ctx]")
    c = cfg._c()
    _check("pkv_query_score_static", load_library().pkv_query_score_static(
        ctypes.byref(c), _ptr(q, cfg.torch_dtype, "q"), _ptr(k, cfg.torch_dtype, "k"),
        _ptr(score, torch.float32, "score"), nq, n_ctx, float(softmax_scale),
        int(bool(accumulate)), _stream()))


def pkv_topk_select(score: torch.Tensor, k: int, idx_out: torch.Tensor,
                    ws: Optional[torch.Tensor] = None) -> None:
    n = score.shape[0]
    if score.dim() != 1 or idx_out.dim() != 1 or idx_out.shape[0] < k:
        raise ValueError("score must be [n] and idx_out at least [k]")
    wp, wb = _ws(ws)
    _check("pkv_topk_select", load_library().pkv_topk_select(
        _ptr(score, torch.float32, "score"), n, int(k),
        _ptr(idx_out, torch.int32, "idx_out"), wp, wb, _stream()))


def _check_proj_args(cfg, hidden, row_idx, row_pos, wq, wk, wv, q_out, k_out, v_out):
    m = row_pos.shape[0]
    if hidden.dim() != 2 or hidden.shape[1] != cfg.hidden:
        raise ValueError("hidden must be [rows, hidden]")
    if row_idx is not None and tuple(row_idx.shape) != (m,):
        raise ValueError("row_idx must be [m]")
    if row_idx is None and hidden.shape[0] < m:
        raise ValueError("hidden has fewer than m rows")
    for t, heads, name in ((q_out, cfg.n_q_heads, "q_out"), (k_out, cfg.n_kv_heads, "k_out"),
                           (v_out, cfg.n_kv_heads, "v_out")):
        if t is not None and tuple(t.shape) != (m, heads, cfg.head_dim):
            raise ValueError(f"{name} must be [m, heads, D]")
    for t, heads, name in ((wq, cfg.n_q_heads, "wq"), (wk, cfg.n_kv_heads, "wk"),
                           (wv, cfg.n_kv_heads, "wv")):
        if t is not None and tuple(t.shape) != (heads * cfg.head_dim, cfg.hidden):
            raise ValueError(f"{name} must be [heads*D, hidden]")
    return m


def pkv_gather_qkv_proj(cfg: LayerCfg, hidden: torch.Tensor,
                        row_idx: Optional[torch.Tensor], row_pos: torch.Tensor,
                        wq: Optional[torch.Tensor], wk: Optional[torch.Tensor],
                        wv: Optional[torch.Tensor], q_out: Optional[torch.Tensor],
                        k_out: Optional[torch.Tensor],
                        v_out: Optional[torch.Tensor],
                        ws: Optional[torch.Tensor] = None) -> None:
    m = _check_proj_args(cfg, hidden, row_idx, row_pos, wq, wk, wv, q_out, k_out, v_out)
    dt = cfg.torch_dtype
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_gather_qkv_proj", load_library().pkv_gather_qkv_proj(
        ctypes.byref(c), _ptr(hidden, dt, "hidden"), _ptr(row_idx, torch.int32, "row_idx"),
        _ptr(row_pos, torch.int32, "row_pos"), _ptr(wq, dt, "wq"), _ptr(wk, dt, "wk"),
        _ptr(wv, dt, "wv"), _ptr(q_out, dt, "q_out"), _ptr(k_out, dt, "k_out"),
        _ptr(v_out, dt, "v_out"), m, wp, wb, _stream()))


def pkv_gather_qkv_proj_ex(cfg: LayerCfg, hidden: torch.Tensor,
                           row_idx: Optional[torch.Tensor], row_pos: torch.Tensor,
                           wq: Optional[torch.Tensor], wk: Optional[torch.Tensor],
                           wv: Optional[torch.Tensor], q_out: Optional[torch.Tensor],
                           k_out: Optional[torch.Tensor], v_out: Optional[torch.Tensor],
                           ws: Optional[torch.Tensor] = None, *,
                           bq: Optional[torch.Tensor] = None,
                           bk: Optional[torch.Tensor] = None,
                           bv: Optional[torch.Tensor] = None,
                           q_norm: Optional[torch.Tensor] = None,
                           k_norm: Optional[torch.Tensor] = None,
                           norm_eps: float = 1e-6) -> None:
    m = _check_proj_args(cfg, hidden, row_idx, row_pos, wq, wk, wv, q_out, k_out, v_out)
    dt = cfg.torch_dtype
    for t, n, name in ((bq, cfg.n_q_heads, "bq"), (bk, cfg.n_kv_heads, "bk"),
                       (bv, cfg.n_kv_heads, "bv")):
        if t is not None and tuple(t.shape) != (n * cfg.head_dim,):
            raise ValueError(f"{name} must be [heads*D]")
    for t, name in ((q_norm, "q_norm"), (k_norm, "k_norm")):
        if t is not None and tuple(t.shape) != (cfg.head_dim,):
            raise ValueError(f"{name} must be [D]")

    def raw(t, name):
        p = _ptr(t, dt, name)
        return None if p is None else p.value
    var = _CVariant(raw(bq, "bq"), raw(bk, "bk"), raw(bv, "bv"), raw(q_norm, "q_norm"),
                    raw(k_norm, "k_norm"), float(norm_eps))
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_gather_qkv_proj_ex", load_library().pkv_gather_qkv_proj_ex(
        ctypes.byref(c), _ptr(hidden, dt, "hidden"), _ptr(row_idx, torch.int32, "row_idx"),
        _ptr(row_pos, torch.int32, "row_pos"), _ptr(wq, dt, "wq"), _ptr(wk, dt, "wk"),
        _ptr(wv, dt, "wv"), ctypes.byref(var), _ptr(q_out, dt, "q_out"),
        _ptr(k_out, dt, "k_out"), _ptr(v_out, dt, "v_out"), m, wp, wb, _stream()))


def pkv_gather_qkv_proj_scatter(cfg: LayerCfg, hidden: torch.Tensor,
                                row_idx: Optional[torch.Tensor], row_pos: torch.Tensor,
                                wq: Optional[torch.Tensor], wk: torch.Tensor, wv: torch.Tensor,
                                q_out: Optional[torch.Tensor], k_cache: torch.Tensor,
                                v_cache: torch.Tensor, dst_row: torch.Tensor,
                                ws: Optional[torch.Tensor] = None, *,
                                bq: Optional[torch.Tensor] = None,
                                bk: Optional[torch.Tensor] = None,
                                bv: Optional[torch.Tensor] = None,
                                q_norm: Optional[torch.Tensor] = None,
                                k_norm: Optional[torch.Tensor] = None,
                                norm_eps: float = 1e-6) -> None:
    m = _check_proj_args(cfg, hidden, row_idx, row_pos, wq, wk, wv, q_out, None, None)
    dt = cfg.torch_dtype
    n_cache = k_cache.shape[0]
    if tuple(k_cache.shape) != (n_cache, cfg.n_kv_heads, cfg.head_dim) or \
            v_cache.shape != k_cache.shape:
        raise ValueError("caches must be [n_cache, Hkv, D]")
    if tuple(dst_row.shape) != (m,):
        raise ValueError("dst_row must be [m]")

    def raw(t, name):
        p = _ptr(t, dt, name)
        return None if p is None else p.value
    var = _CVariant(raw(bq, "bq"), raw(bk, "bk"), raw(bv, "bv"), raw(q_norm, "q_norm"),
                    raw(k_norm, "k_norm"), float(norm_eps))
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_gather_qkv_proj_scatter", load_library().pkv_gather_qkv_proj_scatter(
        ctypes.byref(c), _ptr(hidden, dt, "hidden"), _ptr(row_idx, torch.int32, "row_idx"),
        _ptr(row_pos, torch.int32, "row_pos"), _ptr(wq, dt, "wq"), _ptr(wk, dt, "wk"),
        _ptr(wv, dt, "wv"), ctypes.byref(var), _ptr(q_out, dt, "q_out"),
        _ptr(k_cache, dt, "k_cache"), _ptr(v_cache, dt, "v_cache"),
        _ptr(dst_row, torch.int32, "dst_row"), m, n_cache, wp, wb, _stream()))


def pkv_scatter_kv(cfg: LayerCfg, k_new: torch.Tensor, v_new: torch.Tensor,
                   dst_row: torch.Tensor, k_cache: torch.Tensor,
                   v_cache: torch.Tensor) -> None:
    m, n_cache = dst_row.shape[0], k_cache.shape[0]
    dt = cfg.torch_dtype
    row = (cfg.n_kv_heads, cfg.head_dim)
    if tuple(k_new.shape) != (m, *row) or tuple(v_new.shape) != (m, *row):
        raise ValueError("k_new/v_new must be [m, Hkv, D]")
    if tuple(k_cache.shape) != (n_cache, *row) or v_cache.shape != k_cache.shape:
        raise ValueError("caches must be [n_cache, Hkv, D]")
    c = cfg._c()
    _check("pkv_scatter_kv", load_library().pkv_scatter_kv(
        ctypes.byref(c), _ptr(k_new, dt, "k_new"), _ptr(v_new, dt, "v_new"),
        _ptr(dst_row, torch.int32, "dst_row"), _ptr(k_cache, dt, "k_cache"),
        _ptr(v_cache, dt, "v_cache"), m, n_cache, _stream()))


def pkv_sparse_row_attn(cfg: LayerCfg, q: torch.Tensor, k_cache: torch.Tensor,
                        v_cache: torch.Tensor, row_pos: torch.Tensor,
                        out: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                        softmax_scale: float = 0.0,
                        ws: Optional[torch.Tensor] = None) -> None:
    m, n_keys = row_pos.shape[0], k_cache.shape[0]
    dt = cfg.torch_dtype
    if tuple(q.shape) != (m, cfg.n_q_heads, cfg.head_dim) or out.shape != q.shape:
        raise ValueError("q/out must be [m, Hq, D]")
    if tuple(k_cache.shape) != (n_keys, cfg.n_kv_heads, cfg.head_dim) or \
            v_cache.shape != k_cache.shape:
        raise ValueError("caches must be [n_keys, Hkv, D]")
    if lse_out is not None and tuple(lse_out.shape) != (m, cfg.n_q_heads):
        raise ValueError("lse_out must be [m, Hq]")
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_sparse_row_attn", load_library().pkv_sparse_row_attn(
        ctypes.byref(c), _ptr(q, dt, "q"), _ptr(k_cache, dt, "k_cache"),
        _ptr(v_cache, dt, "v_cache"), _ptr(row_pos, torch.int32, "row_pos"),
        _ptr(out, dt, "out"), _ptr(lse_out, torch.float32, "lse_out"), m, n_keys,
        float(softmax_scale), wp, wb, _stream()))


def pkv_sparse_row_attn_ctx_lse_workspace_bytes(cfg: LayerCfg, n_keys: int, n_ctx: int,
                                                m: int) -> int:
    """Scratch of pkv_sparse_row_attn_ctx_lse; 0 when the geometry is not supported."""
    c = cfg._c()
    return int(load_library().pkv_sparse_row_attn_ctx_lse_workspace_bytes(
        ctypes.byref(c), int(n_keys), int(n_ctx), int(m)))


def pkv_sparse_row_attn_ctx_lse(cfg: LayerCfg, q: torch.Tensor, k_cache: torch.Tensor,
                                v_cache: torch.Tensor, row_pos: torch.Tensor,
                                out: torch.Tensor, lse_out: Optional[torch.Tensor],
                                lse_ctx_out: torch.Tensor, n_ctx: int,
                                softmax_scale: float = 0.0,
                                ws: Optional[torch.Tensor] = None) -> None:
    m, n_keys = row_pos.shape[0], k_cache.shape[0]
    dt = cfg.torch_dtype
    if tuple(q.shape) != (m, cfg.n_q_heads, cfg.head_dim) or out.shape != q.shape:
        raise ValueError("q/out must be [m, Hq, D]")
    if tuple(k_cache.shape) != (n_keys, cfg.n_kv_heads, cfg.head_dim) or \
            v_cache.shape != k_cache.shape:
        raise ValueError("caches must be [n_keys, Hkv, D]")
    for name, t in (("lse_out", lse_out), ("lse_ctx_out", lse_ctx_out)):
        if t is not None and tuple(t.shape) != (m, cfg.n_q_heads):
            raise ValueError(f"{name} must be [m, Hq]")
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_sparse_row_attn_ctx_lse", load_library().pkv_sparse_row_attn_ctx_lse(
        ctypes.byref(c), _ptr(q, dt, "q"), _ptr(k_cache, dt, "k_cache"),
        _ptr(v_cache, dt, "v_cache"), _ptr(row_pos, torch.int32, "row_pos"),
        _ptr(out, dt, "out"), _ptr(lse_out, torch.float32, "lse_out"),
        _ptr(lse_ctx_out, torch.float32, "lse_ctx_out"), m, n_keys, int(n_ctx),
        float(softmax_scale), wp, wb, _stream()))


def pkv_query_score_lse(cfg: LayerCfg, q: torch.Tensor, k: torch.Tensor, lse: torch.Tensor,
                        row_pos: Optional[torch.Tensor], score: torch.Tensor,
                        accumulate: bool = False, softmax_scale: float = 0.0,
                        ws: Optional[torch.Tensor] = None) -> None:
    nq, n_ctx = q.shape[0], k.shape[0]
    if tuple(q.shape) != (nq, cfg.n_q_heads, cfg.head_dim):
        raise ValueError("q must be [nq, Hq, D]")
    if tuple(k.shape) != (n_ctx, cfg.n_kv_heads, cfg.head_dim):
        raise ValueError("k must be [n_ctx, Hkv, D]")
    if tuple(lse.shape) != (nq, cfg.n_q_heads):
        raise ValueError("lse must be [nq, Hq]")
    if row_pos is not None and tuple(row_pos.shape) != (nq,):
        raise ValueError("row_pos must be [nq]")
    if tuple(score.shape) != (n_ctx,):
        raise ValueError("score must be [n_ctx]")
    wp, wb = _ws(ws)
    c = cfg._c()
    _check("pkv_query_score_lse", load_library().pkv_query_score_lse(
        ctypes.byref(c), _ptr(q, cfg.torch_dtype, "q"), _ptr(k, cfg.torch_dtype, "k"),
        _ptr(lse, torch.float32, "lse"), _ptr(row_pos, torch.int32, "row_pos"),
        _ptr(score, torch.float32, "score"), nq, n_ctx, float(softmax_scale),
        int(bool(accumulate)), wp, wb, _stream()))


# ---- layer glue -------------------------------------------------------------------

def _dtype_code(t: torch.Tensor) -> int:
    try:
        return {torch.float32: PKV_F32, torch.bfloat16: PKV_BF16}[t.dtype]
    except KeyError:
        raise ValueError(f"dtype {t.dtype} is not supported (fp32 or bf16)") from None


def pkv_glue_workspace_bytes(dtype: torch.dtype, m: int, k_in: int, n_out: int) -> int:
    code = {torch.float32: PKV_F32, torch.bfloat16: PKV_BF16}[dtype]
    return int(load_library().pkv_glue_workspace_bytes(code, m, k_in, n_out))


def pkv_rmsnorm_rows(h: torch.Tensor, row_idx: Optional[torch.Tensor],
                     weight: torch.Tensor, eps: float, y: torch.Tensor) -> None:
    m, hidden = y.shape
    dt = h.dtype
    if h.dim() != 2 or h.shape[1] != hidden or tuple(weight.shape) != (hidden,):
        raise ValueError("h must be [rows, hidden], weight [hidden], y [m, hidden]")
    if row_idx is not None and tuple(row_idx.shape) != (m,):
        raise ValueError("row_idx must be [m]")
    if row_idx is None and h.shape[0] < m:
        raise ValueError("h has fewer than m rows")
    _check("pkv_rmsnorm_rows", load_library().pkv_rmsnorm_rows(
        _dtype_code(h), _ptr(h, dt, "h"), _ptr(row_idx, torch.int32, "row_idx"),
        _ptr(weight, dt, "weight"), float(eps), _ptr(y, dt, "y"), m, hidden, _stream()))


def pkv_gather_rows(src: torch.Tensor, row_idx: torch.Tensor, dst: torch.Tensor) -> None:
    m, width = dst.shape
    if src.dim() != 2 or src.shape[1] != width or tuple(row_idx.shape) != (m,):
        raise ValueError("src must be [rows, width], row_idx [m], dst [m, width]")
    _check("pkv_gather_rows", load_library().pkv_gather_rows(
        _dtype_code(src), _ptr(src, src.dtype, "src"), _ptr(row_idx, torch.int32, "row_idx"),
        _ptr(dst, src.dtype, "dst"), m, width, _stream()))


def pkv_linear_rows(x: torch.Tensor, w: torch.Tensor, residual: Optional[torch.Tensor],
                    y: torch.Tensor, ws: Optional[torch.Tensor] = None) -> None:
    m, k_in = x.shape
    n_out = w.shape[0]
    dt = x.dtype
    if tuple(w.shape) != (n_out, k_in) or tuple(y.shape) != (m, n_out):
        raise ValueError("w must be [n_out, k_in] and y [m, n_out]")
    if residual is not None and tuple(residual.shape) != (m, n_out):
        raise ValueError("residual must be [m, n_out]")
    wp, wb = _ws(ws)
    _check("pkv_linear_rows", load_library().pkv_linear_rows(
        _dtype_code(x), _ptr(x, dt, "x"), _ptr(w, dt, "w"), _ptr(residual, dt, "residual"),
        _ptr(y, dt, "y"), m, k_in, n_out, wp, wb, _stream()))


def pkv_swiglu_rows(x: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor,
                    y: torch.Tensor, ws: Optional[torch.Tensor] = None) -> None:
    m, k_in = x.shape
    n_out = w_gate.shape[0]
    dt = x.dtype
    if tuple(w_gate.shape) != (n_out, k_in) or w_up.shape != w_gate.shape or \
            tuple(y.shape) != (m, n_out):
        raise ValueError("w_gate/w_up must be [n_out, k_in] and y [m, n_out]")
    wp, wb = _ws(ws)
    _check("pkv_swiglu_rows", load_library().pkv_swiglu_rows(
        _dtype_code(x), _ptr(x, dt, "x"), _ptr(w_gate, dt, "w_gate"), _ptr(w_up, dt, "w_up"),
        _ptr(y, dt, "y"), m, k_in, n_out, wp, wb, _stream()))
