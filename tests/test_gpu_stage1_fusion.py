"""GPU parity of the two fused first-stage calls against the CPU oracle:

* pkv_sparse_row_attn_ctx_lse - attention that also emits the log-sum-exp over the
  context keys alone; oracle: O.sparse_row_attn over the first n_ctx cache rows.
* pkv_query_score_lse - column sums with given normalisers; without row limits the
  oracle is O.query_score (Algorithm 1's value function, softmax over the context
  keys), with row limits it is the global column sum of the diagnostics oracle.
"""

import numpy as np
import pytest
import torch

from oracle import pkv_diag_oracle as DG
from oracle import pkv_oracle as O
from paper_2602_02579_amd import api, synth

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def rnd(seed, shape, dtype="bf16", scale=1.0):
    g = np.random.default_rng(seed)
    return synth.to_storage(g.standard_normal(shape, dtype=np.float32) * np.float32(scale),
                            dtype)


def dev(x, dtype, device):
    return torch.from_numpy(np.ascontiguousarray(x)).to(TDT[dtype]).to(device)


def host(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def ctx_lse_case(gpu_device, n_ctx, n_tail, pos, seed, q_scale=1.2, spike=None):
    cfg = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    n_keys = n_ctx + n_tail
    pos = np.asarray(pos, np.int32)
    m = len(pos)
    q = rnd(seed, (m, 32, 128), scale=q_scale)
    kc, vc = rnd(seed + 1, (n_keys, 8, 128)), rnd(seed + 2, (n_keys, 8, 128))
    if spike is not None:            # a key far above the softmax reference of its tile
        kc[spike] = synth.to_storage(6.0 * q[-1, ::4].astype(np.float32), "bf16")
    need = api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(cfg, n_keys, n_ctx, m)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=gpu_device)
    out = torch.empty((m, 32, 128), dtype=torch.bfloat16, device=gpu_device)
    lse = torch.empty((m, 32), dtype=torch.float32, device=gpu_device)
    lse_ctx = torch.full((m, 32), float("nan"), dtype=torch.float32, device=gpu_device)
    api.pkv_sparse_row_attn_ctx_lse(cfg, dev(q, "bf16", gpu_device), dev(kc, "bf16", gpu_device),
                                    dev(vc, "bf16", gpu_device),
                                    torch.from_numpy(pos).to(gpu_device), out, lse, lse_ctx,
                                    n_ctx, ws=ws)
    torch.cuda.synchronize()
    q64, k64, v64 = q.astype(np.float64), kc.astype(np.float64), vc.astype(np.float64)
    want, want_lse = O.sparse_row_attn(q64, k64, v64, pos, dtype="bf16")
    _, want_ctx = O.sparse_row_attn(q64, k64[:n_ctx], v64[:n_ctx], np.minimum(pos, n_ctx - 1),
                                    dtype="bf16")
    assert np.abs(host(out) - want).max() / np.abs(want).max() <= 2e-2
    assert np.abs(host(lse) - want_lse).max() <= 4e-3
    assert np.abs(host(lse_ctx) - want_ctx).max() <= 4e-3
    return q, kc, host(lse_ctx), want_ctx


def test_context_lse_of_the_query_rows(gpu_device, v_source):
    """The first stage's shape: the query rows behind a 4096-key context."""
    n_ctx, qn = 4096, 128
    ctx_lse_case(gpu_device, n_ctx, qn, np.arange(n_ctx, n_ctx + qn), 700)


def test_context_lse_with_rows_inside_the_context_and_a_ragged_tail(gpu_device, v_source):
    n_ctx, tail = 1536, 37
    g = np.random.default_rng(5)
    pos = np.sort(np.concatenate([g.choice(n_ctx, 90, replace=False),
                                  [0, 63, 64, n_ctx - 1, n_ctx],
                                  n_ctx + g.choice(tail, 20, replace=False)]))
    ctx_lse_case(gpu_device, n_ctx, tail, pos, 710)


def test_context_lse_when_every_key_is_a_context_key(gpu_device, v_source):
    ctx_lse_case(gpu_device, 2048, 0, np.arange(2048 - 70, 2048), 720)


def test_context_lse_through_the_exact_kernel(gpu_device, v_source):
    """A key far above the reference of its column marks the tile; the exact kernel
    redoes it and must cut its running sums at the context boundary too."""
    n_ctx, qn = 2048, 64
    ctx_lse_case(gpu_device, n_ctx, qn, np.arange(n_ctx, n_ctx + qn), 730, q_scale=3.0,
                 spike=1500)
    ctx_lse_case(gpu_device, n_ctx, qn, np.arange(n_ctx, n_ctx + qn), 731, q_scale=3.0,
                 spike=n_ctx + 5)


def test_context_lse_at_the_benchmark_shape_feeds_the_score(gpu_device):
    """32k context, 128 query rows: lse_ctx, then the one-pass score from it, against
    the oracle's value function."""
    n_ctx, qn = 32768, 128
    q, kc, got_ctx, _ = ctx_lse_case(gpu_device, n_ctx, qn, np.arange(n_ctx, n_ctx + qn), 740)
    cfg = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    ws = torch.empty(api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, n_ctx, qn),
                     dtype=torch.uint8, device=gpu_device)
    score = torch.empty(n_ctx, dtype=torch.float32, device=gpu_device)
    api.pkv_query_score_lse(cfg, dev(q, "bf16", gpu_device), dev(kc[:n_ctx], "bf16", gpu_device),
                            torch.from_numpy(got_ctx.astype(np.float32)).to(gpu_device), None,
                            score, ws=ws)
    two_pass = torch.empty_like(score)
    api.pkv_query_score(cfg, dev(q, "bf16", gpu_device), dev(kc[:n_ctx], "bf16", gpu_device),
                        two_pass, ws=ws)
    torch.cuda.synchronize()
    want = O.query_score(q.astype(np.float64), kc[:n_ctx].astype(np.float64))
    got = host(score)
    assert abs(got.sum() - 1.0) < 1e-3
    assert np.abs(got - want).max() / want.max() <= 1e-2
    assert (np.abs(got - want) / want).max() <= 2e-2
    assert np.abs(host(two_pass) - want).max() / want.max() <= 1e-2


def oracle_lse(q, k, pos):
    _, lse = O.sparse_row_attn(q, k, k, pos)
    return lse


@pytest.mark.parametrize("dtype,nq,n_ctx,hq,hkv,d", [
    ("bf16", 128, 4096, 32, 8, 128),    # streaming kernels
    ("bf16", 37, 1000, 8, 2, 128),      # ragged
    ("bf16", 20, 700, 6, 2, 64),        # key-blocked matrix-core kernel
    ("f32", 16, 1024, 4, 4, 64),        # plain kernels
    ("f32", 5, 333, 6, 3, 32),
])
@pytest.mark.parametrize("causal", [False, True])
def test_score_from_given_normalisers(gpu_device, dtype, nq, n_ctx, hq, hkv, d, causal):
    cfg = api.LayerCfg(hq, hkv, d, 256, 1e4, dtype)
    q, k = rnd(800, (nq, hq, d), dtype, 1.2), rnd(801, (n_ctx, hkv, d), dtype)
    q64, k64 = q.astype(np.float64), k.astype(np.float64)
    g = np.random.default_rng(9)
    if causal:
        pos = np.sort(g.choice(n_ctx, nq, replace=False)).astype(np.int32)
        pos[-1] = n_ctx - 1
        want = DG.column_sum_score(q64, k64, pos)
    else:
        pos = np.full(nq, n_ctx - 1, np.int32)
        want = O.query_score(q64, k64)
    lse = oracle_lse(q64, k64, pos).astype(np.float32)
    ws = torch.empty(max(api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, n_ctx, nq), 256),
                     dtype=torch.uint8, device=gpu_device)
    prior = torch.rand(n_ctx, dtype=torch.float32, device=gpu_device)
    for accumulate in (False, True):
        score = prior.clone()
        api.pkv_query_score_lse(cfg, dev(q, dtype, gpu_device), dev(k, dtype, gpu_device),
                                torch.from_numpy(lse).to(gpu_device),
                                torch.from_numpy(pos).to(gpu_device) if causal else None,
                                score, accumulate=accumulate, ws=ws)
        torch.cuda.synchronize()
        got = host(score) - (host(prior) if accumulate else 0.0)
        tol = 1e-2 if dtype == "bf16" else 1e-4
        assert np.abs(got - want).max() / want.max() <= tol
        assert abs(got.sum() - 1.0) < 1e-3


def test_unsupported_geometries_are_refused(gpu_device):
    f32 = api.LayerCfg(4, 4, 64, 256, 1e4, "f32")
    d64 = api.LayerCfg(8, 2, 64, 256, 1e4, "bf16")
    ok = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    assert api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(f32, 1040, 1024, 16) == 0
    assert api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(d64, 1040, 1024, 16) == 0
    assert api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(ok, 1040, 1000, 16) == 0   # not /64
    assert api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(ok, 64 * 40, 64, 16) == 0  # too many ranges
    assert api.pkv_sparse_row_attn_ctx_lse_workspace_bytes(ok, 1040, 1024, 16) > 0
    t = torch.zeros((16, 32, 128), dtype=torch.bfloat16, device=gpu_device)
    kc = torch.zeros((1040, 8, 128), dtype=torch.bfloat16, device=gpu_device)
    pos = torch.arange(1024, 1040, dtype=torch.int32, device=gpu_device)
    lse = torch.zeros((16, 32), dtype=torch.float32, device=gpu_device)
    with pytest.raises(api.PkvError) as e:
        api.pkv_sparse_row_attn_ctx_lse(ok, t, kc, kc, pos, t.clone(), None, lse, 1000, ws=kc)
    assert e.value.status == 3
