"""Test-side workload builder: synthetic draws + planting + margin repair.

The seeded generator holds none of the method's arithmetic, so planting gets
its rotated-query block and its rotation from the CPU oracle here, and the
guard band around the top-k threshold is cleared with the oracle's fp64
score.  Everything runs on the CPU; no value comes from the GPU library.
"""

from __future__ import annotations

import numpy as np

from oracle import pkv_oracle as O
from paper_2602_02579_amd import synth


def geometry(cfg):
    return dict(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                head_dim=cfg.head_dim, theta=cfg.theta)


def oracle_callables(cfg, layer):
    def project_q(rows):
        rows = np.asarray(rows)
        q, _, _ = O.project_qkv_rows(layer["hidden"], rows, rows, layer["wq"],
                                     layer["wk"], layer["wv"], cfg.n_q_heads,
                                     cfg.n_kv_heads, cfg.head_dim, cfg.theta,
                                     cfg.dtype)
        return q

    def rotate(x, pos):
        return O.rope_rotate(x, pos, cfg.theta)
    return project_q, rotate


class ScoreState:
    """Oracle inputs of the fused score, kept between margin-repair rounds: the rotated
    user-query queries and the restored keys of every scoring layer.  A nudge touches a
    few key rows of one layer; `refresh_rows` restores just those rows again (the
    restore acts on every token by itself), so a round costs one oracle score per
    scoring layer instead of a restore of the whole cache as well."""

    def __init__(self, cfg, layers):
        self.cfg, self.layers = cfg, layers
        n, qn = cfg.n_ctx, cfg.n_query
        q_rows = np.arange(n, n + qn)
        self.q_s, self.k_rope = [], []
        for li in range(cfg.n_score_layers):
            l = layers[li]
            q_s, _, _ = O.project_qkv_rows(l["hidden"], q_rows, q_rows, l["wq"], l["wk"],
                                           l["wv"], cfg.n_q_heads, cfg.n_kv_heads,
                                           cfg.head_dim, cfg.theta, cfg.dtype)
            self.q_s.append(q_s)
            self.k_rope.append(O.rope_restore(l["k_nope"], np.arange(n), cfg.theta,
                                              cfg.dtype))

    def refresh_rows(self, li, idx):
        idx = np.asarray(idx, dtype=np.int64)
        self.k_rope[li][idx] = O.rope_restore(self.layers[li]["k_nope"][idx], idx,
                                              self.cfg.theta, self.cfg.dtype)

    def score(self):
        """fp64 per-layer scores fused in fp32 storage, as the oracle defines."""
        score = np.zeros(self.cfg.n_ctx)
        for q_s, k_rope in zip(self.q_s, self.k_rope):
            score = O.fuse_score(score, O.query_score(q_s, k_rope))
        return score


def fused_score(cfg, layers):
    """The oracle's fused score of the layers as they stand (everything recomputed)."""
    return ScoreState(cfg, layers).score()


def guard_band(score, k, margin):
    """Threshold between ranks k and k+1 and the tokens closer than margin*tau."""
    n = score.shape[0]
    if k <= 0 or k >= n:
        return None, np.zeros(0, np.int64)
    srt = np.sort(score)[::-1]
    tau = 0.5 * (srt[k - 1] + srt[k])
    inside = np.nonzero(np.abs(score - tau) < margin * tau)[0]
    return tau, inside


def plant_layers(cfg):
    """Seeded draws with the query-relevant / salient plants of every scoring layer."""
    layers = [synth.make_layer(cfg, li) for li in range(cfg.n_layers)]
    infos = []
    for li in range(cfg.n_score_layers):
        pq, rot = oracle_callables(cfg, layers[li])
        infos.append(synth.plant(cfg, layers[li], li, pq, rot))
    return layers, infos


def repair_margin(cfg, layers, infos, k, margin=None, max_iter=12, verbose=False):
    """Empties the guard band around the top-k threshold of the fused oracle score by
    nudging keys of the first scoring layer along the user-query direction (in place).
    Returns the final score and the threshold."""
    if margin is None:
        margin = 1e-3 if cfg.dtype == "f32" else 5e-2
    _, rot = oracle_callables(cfg, layers[0])
    u = infos[0]["u"]
    # a coefficient of `unit` along u raises the mean scaled logit by one
    unit = np.sqrt(cfg.head_dim) / float(np.mean(infos[0]["mu"]))
    step = 2.0 * margin * unit
    state = ScoreState(cfg, layers)
    for it in range(max_iter):
        score = state.score()
        tau, inside = guard_band(score, k, margin)
        if verbose:
            print(f"margin repair iter {it}: {inside.size} tokens in band")
        if inside.size == 0:
            return score, tau
        sign = np.where(score[inside] >= tau, 1.0, -1.0)
        synth.nudge_keys(cfg, layers[0], inside, sign * step * (1 + it), u, rot)
        state.refresh_rows(0, inside)
    raise RuntimeError("guard band not cleared")


def build(cfg, margin=None, max_iter=12, verbose=False, k=None):
    """Layers with plants and an empty guard band around the top-k threshold.

    Returns ``(layers, info)``; ``info`` has the planted index sets, ``k``,
    the final fused oracle score and the margin reached.
    """
    if margin is None:
        margin = 1e-3 if cfg.dtype == "f32" else 5e-2
    layers, infos = plant_layers(cfg)
    if k is None:
        k = synth.select_count(cfg.ratio, cfg.n_ctx)
    score, tau = repair_margin(cfg, layers, infos, k, margin, max_iter, verbose)
    info = dict(k=k, score=score, relevant=infos[0]["relevant"],
                salient=infos[0]["salient"], margin=margin, tau=tau)
    return layers, info
