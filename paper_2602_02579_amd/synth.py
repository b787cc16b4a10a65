"""Seeded synthetic inputs shaped like the paper's long-context RAG prefill.

The paper evaluates on retrieval benchmarks cut into 512-token chunks with
the user query closing the prompt, a 20 % recomputation ratio and
Llama-3-8B geometry (Sec. 5.1).  Neither those datasets nor trained weights
are available here, so every tensor is drawn from a seeded generator with
the same shapes and a planted structure that makes the selection meaningful:
a few context tokens whose keys line up with the user-query queries
("query-relevant") and, optionally, tokens that attract attention from
context rows but not from the user query ("globally salient", the tokens a
global column-sum criterion would over-select, Sec. 1).

This module serves both the GPU library's callers and the CPU oracle's
callers, and therefore contains none of the method's arithmetic: no rotary
embedding, no projection, no softmax.  Where planting needs a rotated query
block or an inverse rotation, the caller passes them in as callables
(``project_q``, ``rotate``) built from whichever implementation it is
driving.

All arrays are ``numpy.float32`` holding values that are exactly
representable in the configuration's storage dtype.
"""

from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Callable, Dict, Optional

import numpy as np
import torch

__all__ = ["Config", "CONFIGS", "make_layer", "plant", "nudge_keys",
           "to_storage", "select_count", "make_embed", "make_block_weights"]


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str            # storage dtype: "f32" or "bf16"
    n_chunks: int
    chunk_len: int
    n_query: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int
    theta: float
    ratio: float = 0.2
    seed: int = 0
    n_relevant: int = 0   # planted query-relevant context tokens
    n_salient: int = 0    # planted globally-salient context tokens
    n_layers: int = 1
    n_score_layers: int = 1

    @property
    def n_ctx(self) -> int:
        return self.n_chunks * self.chunk_len

    @property
    def n_tokens(self) -> int:
        return self.n_ctx + self.n_query

    def with_(self, **kw) -> "Config":
        return replace(self, **kw)


def select_count(ratio: float, n_ctx: int) -> int:
    """k = floor(ratio * N) over context tokens only (Eq. 4, top-p fraction)."""
    return int(np.floor(ratio * n_ctx + 1e-9))


_LLAMA = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, hidden=4096,
              theta=500000.0, dtype="bf16", chunk_len=512)

CONFIGS: Dict[int, Config] = {
    1: Config("cfg1-f32-1k", "f32", 4, 256, 16, 4, 4, 64, 256, 10000.0,
              seed=0, n_relevant=10),
    2: Config("cfg2-llama8b-8k", n_chunks=16, n_query=64, seed=2,
              n_relevant=82, **_LLAMA),
    3: Config("cfg3-llama8b-32k", n_chunks=64, n_query=128, seed=3,
              n_relevant=328, n_salient=655, **_LLAMA),
    4: Config("cfg4-llama8b-32k-32layers", n_chunks=64, n_query=128, seed=4,
              n_relevant=328, n_salient=655, n_layers=32, n_score_layers=2,
              **_LLAMA),
    5: Config("cfg5-llama8b-128k", n_chunks=256, n_query=256, seed=5,
              n_relevant=1311, **_LLAMA),
    # layer geometry of the 14B Qwen models the paper also evaluates (Sec. 5.1): 40 query
    # heads over 8 kv heads (groups of 5), hidden 5120 - public model configurations
    6: Config("cfg6-qwen14b-4k", "bf16", 8, 512, 64, 40, 8, 128, 5120, 1000000.0,
              seed=6, n_relevant=41),
    7: Config("cfg7-qwen14b-32k", "bf16", 64, 512, 128, 40, 8, 128, 5120, 1000000.0,
              seed=7, n_relevant=328, n_salient=655),
}


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to the storage dtype (library conversion), keep fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(dtype)


def _rng(cfg: Config, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(
        np.random.SeedSequence([cfg.seed, layer, stream])))


def make_layer(cfg: Config, layer: int = 0) -> Dict[str, np.ndarray]:
    """Raw draws for one layer (nothing planted yet).

    Returns ``k_nope, v [N, Hkv, D]`` ~ N(0,1) (the chunk-wise precomputed
    cache in assembled order, keys without positions), ``hidden
    [N + Qn, hid]`` (stands for the layer's normalised input: context rows
    N(0,1) plus half of a common component, query rows a strong common
    component plus 0.3 noise), ``wq [Hq*D, hid]``, ``wk, wv [Hkv*D, hid]`` ~
    N(0, 0.02).
    """
    n, qn = cfg.n_ctx, cfg.n_query
    hkv, hq, d, hid = cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.hidden
    f32 = np.float32
    out = {}
    out["k_nope"] = _rng(cfg, layer, 0).standard_normal((n, hkv, d), dtype=f32)
    out["v"] = _rng(cfg, layer, 1).standard_normal((n, hkv, d), dtype=f32)
    g = _rng(cfg, layer, 2)
    hidden = g.standard_normal((n + qn, hid), dtype=f32)
    ctx_common = g.standard_normal(hid, dtype=f32)
    qry_common = g.standard_normal(hid, dtype=f32)
    hidden[:n] += f32(0.5) * ctx_common
    hidden[n:] = qry_common + f32(0.3) * hidden[n:]
    out["hidden"] = hidden
    gw = _rng(cfg, layer, 3)
    out["wq"] = f32(0.02) * gw.standard_normal((hq * d, hid), dtype=f32)
    out["wk"] = f32(0.02) * gw.standard_normal((hkv * d, hid), dtype=f32)
    out["wv"] = f32(0.02) * gw.standard_normal((hkv * d, hid), dtype=f32)
    for name in out:
        out[name] = to_storage(out[name], cfg.dtype)
    return out


def _group_direction(q: np.ndarray, n_kv_heads: int):
    """Per kv-head unit mean direction of a query block, and two norms.

    ``q [rows, Hq, D]``.  Returns ``u [Hkv, D]`` (unit mean over rows and the
    heads of the group), ``mu [Hkv]`` (norm of that mean) and ``sigma [Hkv]``
    (rms query norm: the std of ``q . k`` for a unit-variance random key).
    """
    rows, hq, d = q.shape
    qg = q.astype(np.float64).reshape(rows, n_kv_heads, hq // n_kv_heads, d)
    mean = qg.mean(axis=(0, 2))                                  # [Hkv, D]
    mu = np.linalg.norm(mean, axis=1)
    sigma = np.sqrt((qg ** 2).sum(axis=3).mean(axis=(0, 2)))
    return mean / mu[:, None], mu, sigma


def plant(cfg: Config, layer: Dict[str, np.ndarray], layer_index: int,
          project_q: Callable[[np.ndarray], np.ndarray],
          rotate: Callable[[np.ndarray, np.ndarray], np.ndarray],
          boost_sigma: float = 4.0) -> Dict[str, np.ndarray]:
    """Plant query-relevant (and globally salient) keys into ``layer['k_nope']``.

    ``project_q(rows) -> [len(rows), Hq, D]`` must return the rotated queries
    of the given hidden rows at positions equal to the row indices;
    ``rotate(x [n, Hkv, D], pos [n]) -> same shape`` must apply the rotary
    rotation for ``pos`` (negative ``pos`` = inverse).  Both come from the
    caller, so that this module stays free of the method's arithmetic.

    For a relevant token ``t`` the *rotated* key gains ``c_g * u_g`` per kv
    head ``g``: ``u_g`` is the unit mean of the user-query queries of the
    group and ``c_g`` is chosen so that the mean logit rises by
    ``boost_sigma`` standard deviations of a random-key logit.  A salient
    token gains a component (three such standard deviations) along the mean
    direction of a sample of context-row queries, taken orthogonal to
    ``u_g``, with its component along ``u_g`` then set to
    ``-3 sigma / mu`` (low user-query affinity).  The stored, position-free
    key is the inverse rotation of the result, re-rounded to storage.
    Returns the index sets and ``u``.
    """
    n, qn, hkv = cfg.n_ctx, cfg.n_query, cfg.n_kv_heads
    g = _rng(cfg, layer_index, 7)
    picks = g.choice(n, size=cfg.n_relevant + cfg.n_salient, replace=False)
    relevant = np.sort(picks[:cfg.n_relevant])
    salient = np.sort(picks[cfg.n_relevant:])

    q_user = project_q(np.arange(n, n + qn))
    u, mu, sigma = _group_direction(np.asarray(q_user), hkv)
    info = dict(relevant=relevant, salient=salient, u=u, mu=mu, sigma=sigma)

    def rewrite(idx, fn):
        if idx.size == 0:
            return
        pos = idx.astype(np.int64)
        kr = np.asarray(rotate(layer["k_nope"][idx], pos), dtype=np.float64)
        kr = fn(kr)
        back = np.asarray(rotate(kr, -pos), dtype=np.float64)
        layer["k_nope"][idx] = to_storage(back.astype(np.float32), cfg.dtype)

    c_rel = boost_sigma * sigma / mu                              # [Hkv]
    rewrite(relevant, lambda kr: kr + c_rel[None, :, None] * u[None])

    if salient.size:
        sample = np.sort(g.choice(n, size=min(256, n), replace=False))
        q_ctx = project_q(sample)
        w, mu_c, sigma_c = _group_direction(np.asarray(q_ctx), hkv)
        mu_c = mu_c * np.sqrt(1.0 - (w * u).sum(axis=1) ** 2)   # part of the
        w = w - (w * u).sum(axis=1, keepdims=True) * u           # mean left
        w = w / np.linalg.norm(w, axis=1, keepdims=True)         # after this
        c_sal = 3.0 * sigma_c / mu_c

        def make_salient(kr):
            kr = kr + c_sal[None, :, None] * w[None]
            along = (kr * u[None]).sum(axis=2, keepdims=True)
            target = (-3.0 * sigma / mu)[None, :, None]
            return kr + (target - along) * u[None]
        rewrite(salient, make_salient)
        info["w"] = w
    return info


def nudge_keys(cfg: Config, layer: Dict[str, np.ndarray], idx: np.ndarray,
               coeff: np.ndarray, u: np.ndarray,
               rotate: Callable[[np.ndarray, np.ndarray], np.ndarray]) -> None:
    """Add ``coeff[j] * u[g]`` to the rotated key of token ``idx[j]``, every kv
    head ``g``, and store the inverse-rotated, re-rounded result.  Used to
    clear a guard band around the selection threshold."""
    if len(idx) == 0:
        return
    pos = np.asarray(idx, dtype=np.int64)
    kr = np.asarray(rotate(layer["k_nope"][pos], pos), dtype=np.float64)
    kr = kr + np.asarray(coeff, np.float64)[:, None, None] * u[None]
    back = np.asarray(rotate(kr, -pos), dtype=np.float64)
    layer["k_nope"][pos] = to_storage(back.astype(np.float32), cfg.dtype)


def make_embed(cfg: Config) -> np.ndarray:
    """Layer-0 hidden state of every prompt token, ``[N + Qn, hid]`` ~ N(0, 1): stands
    for the embedding lookup of a model whose hidden states are carried through the
    layers (the rows of the user query share a common component, as in ``make_layer``)."""
    g = _rng(cfg, 0, 11)
    e = g.standard_normal((cfg.n_tokens, cfg.hidden), dtype=np.float32)
    common = g.standard_normal(cfg.hidden, dtype=np.float32)
    e[cfg.n_ctx:] = np.float32(0.7) * common + np.float32(0.7) * e[cfg.n_ctx:]
    return to_storage(e, cfg.dtype)


def make_block_weights(cfg: Config, layer: int, inter: int) -> Dict[str, np.ndarray]:
    """Weights of one pre-norm decoder block with a gated MLP of width ``inter``:
    norm gains ``w_in, w_post [hid]`` ~ 1 + 0.1 N(0,1); ``wq [Hq*D, hid]``,
    ``wk, wv [Hkv*D, hid]``, ``wo [hid, Hq*D]``, ``w_gate, w_up [inter, hid]``,
    ``w_down [hid, inter]`` ~ N(0, 1/fan_in) (outputs of unit scale for unit-scale
    inputs, so that hidden states neither vanish nor blow up over a few layers)."""
    hq, hkv, d, hid = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.hidden
    g = _rng(cfg, layer, 12)
    f32 = np.float32

    def mat(rows, cols, gain=1.0):
        return f32(gain / np.sqrt(cols)) * g.standard_normal((rows, cols), dtype=f32)

    out = dict(
        w_in=f32(1.0) + f32(0.1) * g.standard_normal(hid, dtype=f32),
        w_post=f32(1.0) + f32(0.1) * g.standard_normal(hid, dtype=f32),
        wq=mat(hq * d, hid, 1.5), wk=mat(hkv * d, hid, 1.5), wv=mat(hkv * d, hid),
        wo=mat(hid, hq * d), w_gate=mat(inter, hid, 1.5), w_up=mat(inter, hid),
        w_down=mat(hid, inter))
    return {k: to_storage(v, cfg.dtype) for k, v in out.items()}
