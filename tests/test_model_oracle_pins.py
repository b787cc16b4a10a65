"""Pins of the layer-glue oracle (oracle/pkv_model_oracle.py) against things that
are not the oracle: torch's CPU rms_norm / linear / silu / scaled_dot_product_attention
on fp64 inputs, closed forms, and an independent full-model forward written here with
torch.  The strongest pin: with ONE chunk, the precomputed chunk cache IS the true
prefill cache, so both stages of the carried-hidden-state algorithm must reproduce
the hidden states of an ordinary causal forward over context + query, for any
selection."""

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pkv_model_oracle as M
from oracle import pkv_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


def test_rmsnorm_matches_torch_and_closed_forms():
    g = rng(1)
    h = g.standard_normal((37, 64))
    w = 1.0 + 0.1 * g.standard_normal(64)
    rows = np.array([5, 0, 36, 5])
    got = M.rmsnorm_rows(h, rows, w, 1e-5, "f64")
    want = F.rms_norm(torch.from_numpy(h[rows]), (64,), torch.from_numpy(w), 1e-5).numpy()
    assert np.abs(got - want).max() < 1e-12
    # a constant row c normalises to sign(c) * w (up to eps); scaling a row changes nothing
    c = np.full((1, 64), -3.0)
    assert np.abs(M.rmsnorm_rows(c, None, w, 0.0, "f64") + w).max() < 1e-12
    assert np.abs(M.rmsnorm_rows(7.0 * h, None, w, 0.0, "f64") -
                  M.rmsnorm_rows(h, None, w, 0.0, "f64")).max() < 1e-12
    # storage rounding happens once, at the end
    assert np.array_equal(M.rmsnorm_rows(h, None, w, 1e-5, "bf16"),
                          O.round_to_storage(M.rmsnorm_rows(h, None, w, 1e-5, "f64"), "bf16"))


def test_linear_and_swiglu_match_torch():
    g = rng(2)
    x, w, r = g.standard_normal((9, 32)), g.standard_normal((20, 32)), g.standard_normal((9, 20))
    tx, tw = torch.from_numpy(x), torch.from_numpy(w)
    assert np.abs(M.linear_rows(x, w, None, "f64") - F.linear(tx, tw).numpy()).max() < 1e-12
    assert np.abs(M.linear_rows(x, w, r, "f64") - (F.linear(tx, tw).numpy() + r)).max() < 1e-12
    # zero weight: the residual comes back (rounded once)
    assert np.array_equal(M.linear_rows(x, 0 * w, r, "bf16"), O.round_to_storage(r, "bf16"))
    wg, wu = g.standard_normal((24, 32)), g.standard_normal((24, 32))
    want = (F.silu(F.linear(tx, torch.from_numpy(wg))) * F.linear(tx, torch.from_numpy(wu))).numpy()
    assert np.abs(M.swiglu_up(x, wg, wu, "f64") - want).max() < 1e-12
    # silu(0) = 0: a zero gate silences the unit; a huge gate passes the up value times the gate
    assert np.abs(M.swiglu_up(x, 0 * wg, wu, "f64")).max() == 0.0
    # bf16: every intermediate is a bf16 value
    y = M.swiglu_up(x, wg, wu, "bf16")
    assert np.array_equal(y, O.round_to_storage(y, "bf16"))


# ---- an independent full-model forward in torch (fp64) ---------------------------------

def torch_rope(x, pos, theta):
    """x [n, heads, D] rotated with the half-split pairing, via complex multiplication."""
    d = x.shape[-1]
    inv = theta ** (-torch.arange(0, d // 2, dtype=torch.float64) * 2.0 / d)
    ang = pos.to(torch.float64)[:, None] * inv[None, :]
    z = torch.complex(x[..., : d // 2], x[..., d // 2:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def torch_forward(embed, layers, hq, hkv, d, theta, eps):
    """Ordinary causal decoder forward over all tokens.  Returns the hidden state after
    every layer and, per layer, the UN-rotated keys and the values of every token."""
    n = embed.shape[0]
    h = torch.from_numpy(embed)
    pos = torch.arange(n)
    hs, ks, vs = [], [], []
    for l in layers:
        t = {k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in l.items()
             if k[0] in "wbqk" and k not in ("k_nope",)}
        x = F.rms_norm(h, (h.shape[1],), t["w_in"], eps)
        q = F.linear(x, t["wq"], t.get("bq")).view(n, hq, d)
        k = F.linear(x, t["wk"], t.get("bk")).view(n, hkv, d)
        v = F.linear(x, t["wv"], t.get("bv")).view(n, hkv, d)
        if "q_norm" in t:       # per-head RMS norm before the rotation
            q = F.rms_norm(q, (d,), t["q_norm"], eps)
            k = F.rms_norm(k, (d,), t["k_norm"], eps)
        ks.append(k.numpy().copy())
        vs.append(v.numpy().copy())
        qr, kr = torch_rope(q, pos, theta), torch_rope(k, pos, theta)
        rep = hq // hkv
        a = F.scaled_dot_product_attention(
            qr.transpose(0, 1)[None], kr.repeat_interleave(rep, 1).transpose(0, 1)[None],
            v.repeat_interleave(rep, 1).transpose(0, 1)[None], is_causal=True)[0]
        a = a.transpose(0, 1).reshape(n, hq * d)
        h = h + F.linear(a, t["wo"])
        y = F.rms_norm(h, (h.shape[1],), t["w_post"], eps)
        h = h + F.linear(F.silu(F.linear(y, t["w_gate"])) * F.linear(y, t["w_up"]), t["w_down"])
        hs.append(h.numpy().copy())
    return hs, ks, vs


def tiny_model(seed, n_ctx, n_query, hid, inter, hq, hkv, d, n_layers, variant="llama"):
    g = rng(seed)
    embed = g.standard_normal((n_ctx + n_query, hid))
    layers = []
    for _ in range(n_layers):
        layers.append(dict(
            w_in=1 + 0.1 * g.standard_normal(hid), w_post=1 + 0.1 * g.standard_normal(hid),
            wq=g.standard_normal((hq * d, hid)) * 0.2, wk=g.standard_normal((hkv * d, hid)) * 0.2,
            wv=g.standard_normal((hkv * d, hid)) * 0.2, wo=g.standard_normal((hid, hq * d)) * 0.2,
            w_gate=g.standard_normal((inter, hid)) * 0.2, w_up=g.standard_normal((inter, hid)) * 0.2,
            w_down=g.standard_normal((hid, inter)) * 0.2))
        if variant == "qkv-bias":
            layers[-1].update(bq=g.standard_normal(hq * d), bk=g.standard_normal(hkv * d),
                              bv=g.standard_normal(hkv * d))
        elif variant == "qk-norm":
            layers[-1].update(q_norm=1 + 0.3 * g.standard_normal(d),
                              k_norm=1 + 0.3 * g.standard_normal(d))
    return embed, layers


@pytest.mark.parametrize("variant", ["llama", "qkv-bias", "qk-norm"])
@pytest.mark.parametrize("k_sel", [0, 7, 40])
def test_exact_cache_reproduces_the_ordinary_forward_for_any_selection(k_sel, variant):
    n_ctx, n_query, hid, inter, hq, hkv, d, L = 40, 5, 32, 48, 4, 2, 8, 3
    theta, eps = 10000.0, 1e-6
    embed, layers = tiny_model(3, n_ctx, n_query, hid, inter, hq, hkv, d, L, variant)
    hs, ks, vs = torch_forward(embed, layers, hq, hkv, d, theta, eps)
    for l, k, v in zip(layers, ks, vs):      # one chunk: its cache is the true one
        l["k_nope"], l["v"] = k[:n_ctx], v[:n_ctx]
    sel, score, out = M.prophetkv_model(embed, layers, n_query, k_sel, L, hq, hkv, d,
                                        theta, eps, "f64")
    assert len(sel) == k_sel and abs(score.sum() - L) < 1e-5     # each layer's alpha sums to 1
    q_rows = np.arange(n_ctx, n_ctx + n_query)
    for li in range(L):
        # Stage I: the query rows alone, against the (here exact) cache
        assert np.abs(out["stage1_h"][li] - hs[li][q_rows]).max() < 1e-9
        # Stage II: the carried rows, whatever was selected
        assert np.abs(out["h"][li] - hs[li][out["rows"]]).max() < 1e-9
        # recomputed K/V rows land where they belong and equal the true ones
        kr = torch_rope(torch.from_numpy(ks[li]), torch.arange(n_ctx + n_query), theta).numpy()
        assert np.abs(out["k_cache"][li] - kr).max() < 1e-9
        assert np.abs(out["v_cache"][li] - vs[li]).max() < 1e-9


def test_imprecise_cache_changes_only_what_it_should():
    """Chunk caches that are NOT the true cache: rows that are not selected keep the
    given cache bit for bit, and the selection passed in is the one used."""
    n_ctx, n_query, hid, inter, hq, hkv, d, L = 32, 4, 32, 48, 4, 2, 8, 2
    embed, layers = tiny_model(4, n_ctx, n_query, hid, inter, hq, hkv, d, L)
    g = rng(5)
    for l in layers:
        l["k_nope"], l["v"] = g.standard_normal((n_ctx, hkv, d)), g.standard_normal((n_ctx, hkv, d))
    forced = np.array([1, 9, 30])
    sel, score, out = M.prophetkv_model(embed, layers, n_query, 3, 1, hq, hkv, d, 10000.0,
                                        1e-6, "bf16", sel=forced)
    assert np.array_equal(sel, forced) and len(out["selection_found"]) == 3
    rest = np.setdiff1d(np.arange(n_ctx), forced)
    for li in range(L):
        want_k = O.rope_restore(layers[li]["k_nope"], np.arange(n_ctx), 10000.0, "bf16")
        assert np.array_equal(out["k_cache"][li][rest], want_k[rest])
        assert np.array_equal(out["v_cache"][li][rest],
                              O.round_to_storage(layers[li]["v"], "bf16")[rest])
    assert abs(score.sum() - 1.0) < 1e-5          # one scoring layer (fp32 score)
