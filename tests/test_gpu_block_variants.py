"""GPU parity of the projection with the block variants of the other public model
families the paper evaluates (projection biases; per-head RMS norm of Q and K before
the rotation), per call on every kernel path and through a small carried-rows model.

Tolerance as everywhere: max|a - b| / max|b| <= 1e-4 (fp32) or 2e-2 (bf16)."""

import numpy as np
import pytest
import torch

from oracle import pkv_model_oracle as MO
from oracle import pkv_oracle as O
from paper_2602_02579_amd import api, model, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def dev(x, dtype, device):
    return torch.from_numpy(np.ascontiguousarray(x)).to(TDT[dtype]).to(device)


def host(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(got, want):
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


def rnd(seed, shape, dtype, scale=1.0, shift=0.0):
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * np.float32(scale)
    return synth.to_storage(x + np.float32(shift), dtype)


# dtype, m, hq, hkv, d, hid, n_hidden_rows -> which kernel
SHAPES = [
    ("bf16", 300, 4, 2, 128, 256, 400),    # 256 x 256 tile kernel, contraction not split
    ("bf16", 64, 4, 2, 128, 2048, 64),     # tile kernel, split contraction + finishing kernel
    ("bf16", 515, 2, 2, 128, 160, 600),    # tile kernel, ragged rows, shortest contraction
    ("bf16", 77, 4, 2, 64, 128, 100),      # head_dim 64: plain kernel
    ("f32", 45, 4, 4, 64, 64, 45),         # fp32: plain kernel
    ("f32", 20, 6, 2, 32, 40, 33),         # two rows of a block share a wave
]
VARIANTS = ["bias", "norm", "bias+norm", "bias-q-only"]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype,m,hq,hkv,d,hid,n_rows", SHAPES)
def test_gather_qkv_proj_variants_match_oracle(gpu_device, dtype, m, hq, hkv, d, hid, n_rows,
                                                variant):
    cfg = api.LayerCfg(hq, hkv, d, hid, 500000.0, dtype)
    hidden = rnd(61, (n_rows, hid), dtype)
    w = [rnd(62, (hq * d, hid), dtype, 1.0 / np.sqrt(hid)),
         rnd(63, (hkv * d, hid), dtype, 1.0 / np.sqrt(hid)),
         rnd(64, (hkv * d, hid), dtype, 1.0 / np.sqrt(hid))]
    g = np.random.default_rng(65)
    rows = (np.arange(m) if n_rows == m else
            np.sort(g.choice(n_rows, m, replace=False))).astype(np.int32)
    pos = np.sort(g.choice(40000, m, replace=False)).astype(np.int32)
    kw = {}
    if "bias" in variant:
        kw["bq"] = rnd(66, (hq * d,), dtype, 0.7)
        if variant != "bias-q-only":
            kw["bk"] = rnd(67, (hkv * d,), dtype, 0.7)
            kw["bv"] = rnd(68, (hkv * d,), dtype, 0.7)
    if "norm" in variant:
        kw["q_norm"] = rnd(69, (d,), dtype, 0.3, 1.0)
        kw["k_norm"] = rnd(70, (d,), dtype, 0.3, 1.0)
        kw["norm_eps"] = 1e-6
    want = O.project_qkv_rows(hidden, rows, pos, *w, hq, hkv, d, cfg.rope_theta, dtype, **kw)
    tk = {k: (v if k == "norm_eps" else dev(v, dtype, gpu_device)) for k, v in kw.items()}
    outs = [torch.full((m, h, d), float("nan"), dtype=TDT[dtype], device=gpu_device)
            for h in (hq, hkv, hkv)]
    nbytes = api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, cfg, 0, m)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=gpu_device)
    api.pkv_gather_qkv_proj_ex(cfg, dev(hidden, dtype, gpu_device),
                               torch.from_numpy(rows).to(gpu_device),
                               torch.from_numpy(pos).to(gpu_device),
                               *[dev(x, dtype, gpu_device) for x in w], *outs, ws=ws, **tk)
    for got, exp, name in zip(outs, want, "qkv"):
        got = host(got)
        assert np.isfinite(got).all(), name
        assert rel_err(got, exp) <= TOL[dtype], name


def test_variant_struct_is_optional_and_checked(gpu_device):
    """NULL variant = the plain call, bit for bit; q_norm without k_norm is refused."""
    dtype, m, hq, hkv, d, hid = "bf16", 130, 2, 2, 128, 256
    cfg = api.LayerCfg(hq, hkv, d, hid, 500000.0, dtype)
    hidden = dev(rnd(71, (m, hid), dtype), dtype, gpu_device)
    w = [dev(rnd(72 + i, (h * d, hid), dtype, 0.06), dtype, gpu_device)
         for i, h in enumerate((hq, hkv, hkv))]
    pos = torch.arange(m, dtype=torch.int32, device=gpu_device)
    ws = torch.empty(max(api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, cfg, 0, m), 256),
                     dtype=torch.uint8, device=gpu_device)
    a = [torch.empty((m, h, d), dtype=torch.bfloat16, device=gpu_device) for h in (hq, hkv, hkv)]
    b = [torch.empty_like(t) for t in a]
    api.pkv_gather_qkv_proj(cfg, hidden, None, pos, *w, *a, ws=ws)
    api.pkv_gather_qkv_proj_ex(cfg, hidden, None, pos, *w, *b, ws=ws)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    gain = torch.ones(d, dtype=torch.bfloat16, device=gpu_device)
    with pytest.raises(api.PkvError) as e:
        api.pkv_gather_qkv_proj_ex(cfg, hidden, None, pos, *w, *b, ws=ws, q_norm=gain)
    assert e.value.status == 1
    with pytest.raises(api.PkvError) as e:
        api.pkv_gather_qkv_proj_ex(cfg, hidden, None, pos, *w, *b, ws=ws, q_norm=gain,
                                   k_norm=gain, norm_eps=-1.0)
    assert e.value.status == 2
    torch.cuda.synchronize()


@pytest.mark.parametrize("variant", ["qkv-bias", "qk-norm"])
@pytest.mark.parametrize("case", ["f32-small", "bf16-tiles"])
def test_model_with_block_variant_matches_oracle(gpu_device, case, variant):
    from tests.test_gpu_model import CASES, EPS, build
    cfg, inter = CASES[case]
    tol = TOL[cfg.dtype]
    embed, layers = build(cfg, inter, margin=False)   # Stage II runs on the oracle's set
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    for li, l in enumerate(layers):
        if variant == "qkv-bias":
            l.update(bq=rnd(80 + li, (hq * d,), cfg.dtype, 0.5),
                     bk=rnd(90 + li, (hkv * d,), cfg.dtype, 0.5),
                     bv=rnd(100 + li, (hkv * d,), cfg.dtype, 0.5))
        else:
            l.update(q_norm=rnd(110 + li, (d,), cfg.dtype, 0.2, 1.0),
                     k_norm=rnd(120 + li, (d,), cfg.dtype, 0.2, 1.0))
    n, qn = cfg.n_ctx, cfg.n_query
    k = synth.select_count(cfg.ratio, n)
    sel, score, want = MO.prophetkv_model(
        embed, [{a: b.astype(np.float64) for a, b in l.items()} for l in layers], qn, k,
        cfg.n_score_layers, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, theta=cfg.theta,
        eps=EPS, dtype=cfg.dtype)
    dev_layers = [model.upload_block(cfg, l, gpu_device) for l in layers]
    dev_embed = torch.from_numpy(embed).to(TDT[cfg.dtype]).to(gpu_device)
    cr = model.CarriedRows(cfg, inter, EPS, gpu_device)
    cr.stage1(dev_embed, dev_layers)
    torch.cuda.synchronize()
    assert rel_err(host(cr.score), score) <= (2e-2 if cfg.dtype == "bf16" else 1e-4)
    assert rel_err(host(cr.h[:qn]), want["stage1_h"][-1]) <= tol
    cr.rows[:k] = torch.from_numpy(sel.astype(np.int32)).to(gpu_device)
    h_final = cr.stage2(dev_embed, dev_layers)
    torch.cuda.synchronize()
    rows = want["rows"]
    for li, L in enumerate(dev_layers):
        assert rel_err(host(L["k_cache"])[rows], want["k_cache"][li][rows]) <= tol
        assert rel_err(host(L["v_cache"])[rows], want["v_cache"][li][rows]) <= tol
    assert rel_err(host(h_final), want["h_final"]) <= tol


@pytest.mark.parametrize("dtype,m,hq,hkv,d,hid,n_rows", SHAPES + [("bf16", 200, 4, 2, 64, 128, 300)])
@pytest.mark.parametrize("with_q", [True, False])
def test_fused_projection_and_cache_update(gpu_device, dtype, m, hq, hkv, d, hid, n_rows, with_q):
    """pkv_gather_qkv_proj_scatter against the oracle's projection followed by its cache
    update, and bit for bit against the two separate GPU calls."""
    cfg = api.LayerCfg(hq, hkv, d, hid, 500000.0, dtype)
    g = np.random.default_rng(75)
    n_cache = n_rows + 37
    hidden = rnd(76, (n_rows, hid), dtype)
    w = [rnd(77 + i, (h * d, hid), dtype, 1.0 / np.sqrt(hid)) for i, h in enumerate((hq, hkv, hkv))]
    rows = np.sort(g.choice(n_rows, m, replace=False)).astype(np.int32) if n_rows > m else \
        np.arange(m, dtype=np.int32)
    dst = g.permutation(n_cache)[:m].astype(np.int32)          # distinct, unsorted targets
    kc0 = rnd(80, (n_cache, hkv, d), dtype)
    vc0 = rnd(81, (n_cache, hkv, d), dtype)
    q_w, k_w, v_w = O.project_qkv_rows(hidden, rows, dst, *w, hq, hkv, d, cfg.rope_theta, dtype)
    kc_w, vc_w = O.scatter_kv(kc0.astype(np.float64), vc0.astype(np.float64), k_w, v_w, dst)

    d_hidden = dev(hidden, dtype, gpu_device)
    d_w = [dev(x, dtype, gpu_device) for x in w]
    d_rows = torch.from_numpy(rows).to(gpu_device)
    d_dst = torch.from_numpy(dst).to(gpu_device)
    ws = torch.empty(max(api.pkv_workspace_bytes(api.CALL_GATHER_QKV_PROJ, cfg, 0, m), 256),
                     dtype=torch.uint8, device=gpu_device)
    kc, vc = dev(kc0, dtype, gpu_device), dev(vc0, dtype, gpu_device)
    q = torch.full((m, hq, d), float("nan"), dtype=TDT[dtype], device=gpu_device) if with_q else None
    api.pkv_gather_qkv_proj_scatter(cfg, d_hidden, d_rows, d_dst, d_w[0] if with_q else None,
                                    d_w[1], d_w[2], q, kc, vc, d_dst, ws=ws)
    # the two-call path on the same inputs
    kc2, vc2 = dev(kc0, dtype, gpu_device), dev(vc0, dtype, gpu_device)
    q2 = torch.empty((m, hq, d), dtype=TDT[dtype], device=gpu_device)
    k_new = torch.empty((m, hkv, d), dtype=TDT[dtype], device=gpu_device)
    v_new = torch.empty_like(k_new)
    api.pkv_gather_qkv_proj(cfg, d_hidden, d_rows, d_dst, *d_w, q2, k_new, v_new, ws=ws)
    api.pkv_scatter_kv(cfg, k_new, v_new, d_dst, kc2, vc2)
    assert torch.equal(kc, kc2) and torch.equal(vc, vc2)
    if with_q:
        assert torch.equal(q, q2)
        assert rel_err(host(q), q_w) <= TOL[dtype]
    assert rel_err(host(kc), kc_w) <= TOL[dtype]
    assert rel_err(host(vc), vc_w) <= TOL[dtype]
    rest = np.setdiff1d(np.arange(n_cache), dst)
    assert np.array_equal(host(kc)[rest], kc0[rest].astype(np.float64))
    assert np.array_equal(host(vc)[rest], vc0[rest].astype(np.float64))
