"""pkv_query_score_static (scratch inside the library, nothing allocated) against
pkv_query_score (caller's workspace) through the C ABI: the same kernels, so the same
bits, on two calls in a row of which the second is smaller (the array keeps the first
call's contents), with and without layer accumulation, plus the oracle's bar and the
refusal of a problem whose scratch exceeds the array."""

import numpy as np
import pytest
import torch

from oracle import pkv_oracle as O
from paper_2602_02579_amd import api, synth

pytestmark = pytest.mark.gpu


def rnd(seed, shape, scale=1.0):
    g = np.random.default_rng(seed)
    return synth.to_storage(g.standard_normal(shape, dtype=np.float32) * np.float32(scale),
                            "bf16")


def dev(x, device):
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(device)


def test_static_scratch_entry_point_matches_the_workspace_one(gpu_device):
    cfg = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    # the benchmark's scoring shape first, then a smaller, ragged one
    for seed, (n_ctx, nq) in enumerate([(32768, 128), (5000, 37)]):
        q_h, k_h = rnd(900 + seed, (nq, 32, 128), 1.3), rnd(910 + seed, (n_ctx, 8, 128))
        q, k = dev(q_h, gpu_device), dev(k_h, gpu_device)
        need = api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, n_ctx, nq)
        assert 0 < need <= api.STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device=gpu_device)
        prior = torch.rand(n_ctx, dtype=torch.float32, device=gpu_device)
        warm = prior.clone()
        api.pkv_query_score_static(cfg, q, k, warm)     # first call on the device: address lookup
        torch.cuda.synchronize()
        for accumulate in (False, True):
            a, b = prior.clone(), prior.clone()
            api.pkv_query_score(cfg, q, k, a, accumulate=accumulate, ws=ws)
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info(gpu_device)[0]   # device-wide, not torch's pool
            api.pkv_query_score_static(cfg, q, k, b, accumulate=accumulate)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info(gpu_device)[0] == free_before
            assert torch.equal(a, b)
        want = O.query_score(q_h.astype(np.float64), k_h.astype(np.float64))
        got = b.double().cpu().numpy() - prior.double().cpu().numpy()
        assert np.abs(got - want).max() / want.max() <= 1e-2


def test_static_scratch_entry_point_refuses_what_does_not_fit(gpu_device):
    cfg = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    n_ctx, nq = 131072, 256
    assert api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, n_ctx, nq) > api.STATIC_SCRATCH_BYTES
    q = torch.zeros((nq, 32, 128), dtype=torch.bfloat16, device=gpu_device)
    k = torch.zeros((n_ctx, 8, 128), dtype=torch.bfloat16, device=gpu_device)
    score = torch.full((n_ctx,), 7.0, dtype=torch.float32, device=gpu_device)
    with pytest.raises(api.PkvError) as e:
        api.pkv_query_score_static(cfg, q, k, score)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert bool((score == 7.0).all())          # nothing was enqueued
