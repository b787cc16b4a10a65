"""GPU parity of the layer-glue calls (RMSNorm of gathered rows, linear + residual,
gated up-projection) against the CPU oracle, through the C ABI.

Sizes cover the matrix-core tile path (bf16, multiples of the 256 x 256 tile, with
ragged row counts, split and unsplit contractions) and the simple path (fp32, odd
sizes).  Tolerance: max|a - b| / max|b| <= 1e-4 (fp32) or 2e-2 (bf16); for bf16 the
result must also be the oracle's bf16 value or a neighbouring one almost everywhere."""

import numpy as np
import pytest
import torch

from oracle import pkv_model_oracle as MO
from paper_2602_02579_amd import api, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def dev(x, dtype, device):
    return torch.from_numpy(np.ascontiguousarray(x)).to(TDT[dtype]).to(device)


def host(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(got, want):
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


def rnd(seed, shape, dtype, scale=1.0):
    x = np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * np.float32(scale)
    return synth.to_storage(x, dtype)


def ws_for(dtype, m, k_in, n_out, device):
    nbytes = api.pkv_glue_workspace_bytes(TDT[dtype], m, k_in, n_out)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def check_bf16_neighbours(got, want, frac=0.02):
    # two bf16 values one step apart differ by at most 2^-7 of the larger one; a sum
    # that lands near a rounding boundary may take either
    diff = np.abs(got - want)
    assert (diff <= np.abs(want) * 2.0 ** -6 + 1e-3 * np.abs(want).max()).all()
    assert (diff > 0).mean() < frac


@pytest.mark.parametrize("dtype,n_rows,m,hidden,gather", [
    ("bf16", 700, 333, 4096, True), ("bf16", 64, 64, 4096, False),
    ("bf16", 50, 7, 8192, True), ("bf16", 40, 40, 16384, False),
    ("f32", 300, 129, 256, True), ("f32", 5, 5, 4096, False), ("bf16", 9, 9, 8, False)])
def test_rmsnorm_rows_matches_oracle(gpu_device, dtype, n_rows, m, hidden, gather):
    h = rnd(11, (n_rows, hidden), dtype, 3.0)
    h[1] *= 2.0 ** -10                 # a row whose mean square is near eps
    w = rnd(12, (hidden,), dtype, 0.5) + synth.to_storage(np.ones(hidden, np.float32), dtype)
    w = synth.to_storage(w, dtype)
    eps = 1e-5
    idx = np.random.default_rng(13).permutation(n_rows)[:m].astype(np.int32) if gather else None
    if gather:
        idx[0] = 1
    want = MO.rmsnorm_rows(h, idx, w, eps, dtype)[:m]
    y = torch.empty((m, hidden), dtype=TDT[dtype], device=gpu_device)
    api.pkv_rmsnorm_rows(dev(h, dtype, gpu_device),
                         None if idx is None else torch.from_numpy(idx).to(gpu_device),
                         dev(w, dtype, gpu_device), eps, y)
    got = host(y)
    assert rel_err(got, want) <= TOL[dtype]
    if dtype == "bf16":
        check_bf16_neighbours(got, want)


@pytest.mark.parametrize("dtype,n_rows,m,width", [("bf16", 500, 333, 4096), ("f32", 40, 64, 8),
                                                   ("bf16", 3, 1000, 136)])
def test_gather_rows_is_a_bit_exact_copy(gpu_device, dtype, n_rows, m, width):
    src = rnd(51, (n_rows, width), dtype)
    idx = np.random.default_rng(52).integers(0, n_rows, size=m).astype(np.int32)
    dst = torch.empty((m, width), dtype=TDT[dtype], device=gpu_device)
    api.pkv_gather_rows(dev(src, dtype, gpu_device), torch.from_numpy(idx).to(gpu_device), dst)
    assert np.array_equal(host(dst), src[idx].astype(np.float64))


LINEAR_CASES = [
    # dtype, m, k_in, n_out: tile path unsplit, split (few rows), ragged rows; simple path
    ("bf16", 300, 512, 512), ("bf16", 128, 2048, 256), ("bf16", 1, 4096, 256),
    ("bf16", 515, 160, 768), ("bf16", 257, 4096, 512),
    ("bf16", 37, 136, 72), ("f32", 65, 200, 136), ("f32", 3, 8, 8),
]


@pytest.mark.parametrize("dtype,m,k_in,n_out", LINEAR_CASES)
@pytest.mark.parametrize("with_residual", [False, True])
def test_linear_rows_matches_oracle(gpu_device, dtype, m, k_in, n_out, with_residual):
    x = rnd(21, (m, k_in), dtype)
    w = rnd(22, (n_out, k_in), dtype, 1.0 / np.sqrt(k_in))
    res = rnd(23, (m, n_out), dtype, 2.0) if with_residual else None
    want = MO.linear_rows(x, w, res, dtype)
    y = torch.full((m, n_out), float("nan"), dtype=TDT[dtype], device=gpu_device)
    api.pkv_linear_rows(dev(x, dtype, gpu_device), dev(w, dtype, gpu_device),
                        None if res is None else dev(res, dtype, gpu_device), y,
                        ws_for(dtype, m, k_in, n_out, gpu_device))
    got = host(y)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL[dtype]
    if dtype == "bf16":
        check_bf16_neighbours(got, want)


@pytest.mark.parametrize("dtype,m,k_in,n_out", [("bf16", 300, 512, 512), ("f32", 65, 200, 136)])
def test_linear_rows_residual_in_place(gpu_device, dtype, m, k_in, n_out):
    x = rnd(31, (m, k_in), dtype)
    w = rnd(32, (n_out, k_in), dtype, 1.0 / np.sqrt(k_in))
    res = rnd(33, (m, n_out), dtype, 2.0)
    want = MO.linear_rows(x, w, res, dtype)
    buf = dev(res, dtype, gpu_device)
    api.pkv_linear_rows(dev(x, dtype, gpu_device), dev(w, dtype, gpu_device), buf, buf,
                        ws_for(dtype, m, k_in, n_out, gpu_device))
    assert rel_err(host(buf), want) <= TOL[dtype]


@pytest.mark.parametrize("dtype,m,k_in,n_out", [
    ("bf16", 300, 512, 384), ("bf16", 128, 2048, 128), ("bf16", 515, 160, 640),
    ("bf16", 1, 4096, 256), ("bf16", 37, 136, 72), ("f32", 65, 200, 136)])
def test_swiglu_rows_matches_oracle(gpu_device, dtype, m, k_in, n_out):
    x = rnd(41, (m, k_in), dtype)
    # gate values spread over [-6, 6] so that silu's curved part and both tails are hit
    wg = rnd(42, (n_out, k_in), dtype, 2.0 / np.sqrt(k_in))
    wu = rnd(43, (n_out, k_in), dtype, 1.0 / np.sqrt(k_in))
    want = MO.swiglu_up(x, wg, wu, dtype)
    y = torch.full((m, n_out), float("nan"), dtype=TDT[dtype], device=gpu_device)
    api.pkv_swiglu_rows(dev(x, dtype, gpu_device), dev(wg, dtype, gpu_device),
                        dev(wu, dtype, gpu_device), y, ws_for(dtype, m, k_in, n_out, gpu_device))
    got = host(y)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL[dtype]
    if dtype == "bf16":
        # three roundings in a row: a flipped first one can move the result by a few steps
        diff = np.abs(got - want)
        assert (diff > np.abs(want) * 2.0 ** -7 + 1e-3 * np.abs(want).max()).mean() < 0.01


def test_glue_rejects_bad_arguments(gpu_device):
    x = torch.zeros((4, 16), dtype=torch.bfloat16, device=gpu_device)
    w = torch.zeros((8, 16), dtype=torch.bfloat16, device=gpu_device)
    y = torch.zeros((4, 8), dtype=torch.bfloat16, device=gpu_device)
    lib = api.load_library()
    st = torch.cuda.current_stream().cuda_stream
    # null pointers, bad dtype, sizes that are not multiples of 8, missing workspace
    assert lib.pkv_linear_rows(1, None, w.data_ptr(), None, y.data_ptr(), 4, 16, 8, None, 0, st) == 1
    assert lib.pkv_linear_rows(7, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), 4, 16, 8,
                               None, 0, st) == 3
    assert lib.pkv_linear_rows(1, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), 4, 12, 8,
                               None, 0, st) == 3
    assert lib.pkv_linear_rows(1, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), -1, 16, 8,
                               None, 0, st) == 2
    assert lib.pkv_swiglu_rows(1, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), 4, 16, 8,
                               None, 0, st) == 1
    assert lib.pkv_rmsnorm_rows(1, x.data_ptr(), None, None, 1e-5, y.data_ptr(), 4, 16, st) == 1
    assert lib.pkv_rmsnorm_rows(1, x.data_ptr(), None, w.data_ptr(), 1e-5, y.data_ptr(), 4,
                                32768, st) == 3
    # a split contraction needs its workspace
    need = api.pkv_glue_workspace_bytes(torch.bfloat16, 128, 2048, 256)
    assert need > 0
    assert lib.pkv_linear_rows(1, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), 128, 2048, 256,
                               None, 0, st) == 4
    # m == 0 is a no-op whatever the pointers
    assert lib.pkv_linear_rows(1, None, None, None, None, 0, 16, 8, None, 0, st) == 0
    assert lib.pkv_rmsnorm_rows(1, None, None, None, 1e-5, None, 0, 16, st) == 0
    torch.cuda.synchronize()


def test_glue_at_the_benchmark_widths_on_sampled_rows(gpu_device):
    """The launch configuration bench.py times (6681 rows, hidden 4096, MLP 14336: 12 rounds of
    256 x 256 tiles with a ragged last row tile), checked on a seeded sample of rows that the
    oracle computes one by one; plus the 128-row launches of the scoring stage, whose
    contraction is split."""
    dtype, hid, inter = "bf16", 4096, 14336
    g = np.random.default_rng(91)
    wo = rnd(92, (hid, hid), dtype, 1.0 / np.sqrt(hid))
    wg = rnd(93, (inter, hid), dtype, 2.0 / np.sqrt(hid))
    wu = rnd(94, (inter, hid), dtype, 1.0 / np.sqrt(hid))
    wd = rnd(95, (hid, inter), dtype, 1.0 / np.sqrt(inter))
    gain = rnd(96, (hid,), dtype, 0.1, ) + 1.0
    gain = synth.to_storage(gain, dtype)
    d_wo, d_wg, d_wu, d_wd, d_gain = (dev(t, dtype, gpu_device) for t in (wo, wg, wu, wd, gain))
    for m in (6681, 128):
        x = rnd(97, (m, hid), dtype)
        res = rnd(98, (m, hid), dtype, 2.0)
        act = rnd(99, (m, inter), dtype, 0.5)
        pick = np.unique(np.concatenate([[0, m - 1, min(m - 1, 255), min(m - 1, 256)],
                                         g.choice(m, 12, replace=False)]))
        d_x, d_res, d_act = (dev(t, dtype, gpu_device) for t in (x, res, act))
        ws = torch.empty(max(api.pkv_glue_workspace_bytes(TDT[dtype], m, hid, inter),
                             api.pkv_glue_workspace_bytes(TDT[dtype], m, inter, hid),
                             api.pkv_glue_workspace_bytes(TDT[dtype], m, hid, hid), 256),
                         dtype=torch.uint8, device=gpu_device)
        y = torch.empty((m, hid), dtype=TDT[dtype], device=gpu_device)
        api.pkv_rmsnorm_rows(d_res, None, d_gain, 1e-5, y)
        assert rel_err(host(y)[pick], MO.rmsnorm_rows(res[pick], None, gain, 1e-5, dtype)) <= TOL[dtype]
        api.pkv_linear_rows(d_x, d_wo, d_res, y, ws)
        assert rel_err(host(y)[pick], MO.linear_rows(x[pick], wo, res[pick], dtype)) <= TOL[dtype]
        gbuf = torch.empty((m, inter), dtype=TDT[dtype], device=gpu_device)
        api.pkv_swiglu_rows(d_x, d_wg, d_wu, gbuf, ws)
        got = host(gbuf)
        assert np.isfinite(got).all()
        assert rel_err(got[pick], MO.swiglu_up(x[pick], wg, wu, dtype)) <= TOL[dtype]
        api.pkv_linear_rows(d_act, d_wd, d_res, y, ws)
        got = host(y)
        assert np.isfinite(got).all()
        assert rel_err(got[pick], MO.linear_rows(act[pick], wd, res[pick], dtype)) <= TOL[dtype]


def test_unaligned_pointers_take_the_plain_kernels(gpu_device):
    """Tensors whose storage is only 2-byte aligned: the tile kernel (16-byte loads) must not be
    used; the results still match the oracle.  RMSNorm and the row gather need 16-byte alignment
    and refuse instead."""
    dtype, m, k_in, n_out = "bf16", 70, 512, 256
    x = rnd(101, (m, k_in), dtype)
    w = rnd(102, (n_out, k_in), dtype, 1.0 / np.sqrt(k_in))
    wu = rnd(103, (n_out, k_in), dtype, 1.0 / np.sqrt(k_in))
    res = rnd(104, (m, n_out), dtype)

    def shifted(a):
        flat = torch.zeros(a.size + 1, dtype=torch.bfloat16, device=gpu_device)
        view = flat[1:].view(a.shape)
        view.copy_(dev(a, dtype, gpu_device))
        assert view.data_ptr() % 16 == 2 and view.is_contiguous()
        return view
    ws = ws_for(dtype, m, k_in, n_out, gpu_device)
    y = shifted(np.zeros((m, n_out), np.float32))
    api.pkv_linear_rows(shifted(x), shifted(w), shifted(res), y, ws)
    assert rel_err(host(y), MO.linear_rows(x, w, res, dtype)) <= TOL[dtype]
    api.pkv_swiglu_rows(shifted(x), shifted(w), shifted(wu), y, ws)
    assert rel_err(host(y), MO.swiglu_up(x, w, wu, dtype)) <= TOL[dtype]
    # one unaligned operand is enough to leave the tile kernel
    y2 = torch.empty((m, n_out), dtype=torch.bfloat16, device=gpu_device)
    api.pkv_linear_rows(dev(x, dtype, gpu_device), shifted(w), None, y2, ws)
    assert rel_err(host(y2), MO.linear_rows(x, w, None, dtype)) <= TOL[dtype]
    gain = dev(np.ones(k_in, np.float32), dtype, gpu_device)
    out = torch.empty((m, k_in), dtype=torch.bfloat16, device=gpu_device)
    with pytest.raises(api.PkvError) as e:
        api.pkv_rmsnorm_rows(shifted(x), None, gain, 1e-5, out)
    assert e.value.status == 3
    idx = torch.arange(m, dtype=torch.int32, device=gpu_device)
    with pytest.raises(api.PkvError) as e:
        api.pkv_gather_rows(shifted(x), idx, out)
    assert e.value.status == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rmsnorm_degenerate_rows(gpu_device, dtype):
    """An all-zero row stays zero (no 0/0), a huge row and a tiny row normalise like any other."""
    hidden = 4096
    h = rnd(111, (6, hidden), dtype)
    h[0] = 0.0
    h[1] = synth.to_storage(h[1] * np.float32(2.0 ** 40), dtype)      # squares near 2^80
    h[2] = synth.to_storage(h[2] * np.float32(2.0 ** -40), dtype)     # far below eps
    h[3] = 0.0
    h[3, 17] = 1.0                                                     # a single spike
    w = synth.to_storage(np.linspace(0.5, 1.5, hidden).astype(np.float32), dtype)
    want = MO.rmsnorm_rows(h, None, w, 1e-6, dtype)
    y = torch.full((6, hidden), float("nan"), dtype=TDT[dtype], device=gpu_device)
    api.pkv_rmsnorm_rows(dev(h, dtype, gpu_device), None, dev(w, dtype, gpu_device), 1e-6, y)
    got = host(y)
    assert np.isfinite(got).all()
    assert np.all(got[0] == 0.0)
    for r in range(6):
        assert rel_err(got[r], want[r]) <= TOL[dtype] or np.abs(want[r]).max() < 1e-30, r
