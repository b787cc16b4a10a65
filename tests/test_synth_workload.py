"""The synthetic recipe: deterministic, storage-exact, planted tokens selected,
guard band around the top-k threshold empty (CPU only, oracle-backed)."""

import numpy as np
import torch

from oracle import pkv_oracle as O
from paper_2602_02579_amd import synth
from tests import workload


def test_draws_are_deterministic_and_storage_exact():
    cfg = synth.CONFIGS[2].with_(n_chunks=1, chunk_len=64, n_query=4)
    a = synth.make_layer(cfg, 0)
    b = synth.make_layer(cfg, 0)
    c = synth.make_layer(cfg, 1)
    for name in a:
        assert np.array_equal(a[name], b[name])
        assert a[name].dtype == np.float32
        back = torch.from_numpy(a[name]).to(torch.bfloat16).float().numpy()
        assert np.array_equal(back, a[name])
    assert not np.array_equal(a["k_nope"], c["k_nope"])
    assert a["k_nope"].shape == (64, 8, 128) and a["hidden"].shape == (68, 4096)
    assert abs(float(a["wq"].std()) - 0.02) < 1e-3


def test_select_count_is_floor_of_ratio_times_context():
    assert synth.select_count(0.2, 1024) == 204
    assert synth.select_count(0.2, 32768) == 6553
    assert synth.select_count(0.4, 32768) == 13107
    assert synth.select_count(0.0, 10) == 0 and synth.select_count(1.0, 10) == 10


def test_config1_plants_are_selected_and_band_is_empty():
    cfg = synth.CONFIGS[1]
    layers, info = workload.build(cfg)
    assert info["k"] == 204
    sel = O.topk_select(info["score"], info["k"])
    assert np.isin(info["relevant"], sel).all() and len(info["relevant"]) == 10
    tau, inside = workload.guard_band(info["score"], info["k"], info["margin"])
    assert inside.size == 0
    # building twice gives the same bits
    layers2, _ = workload.build(cfg)
    assert np.array_equal(layers[0]["k_nope"], layers2[0]["k_nope"])


def test_salient_plants_are_not_query_relevant():
    cfg = synth.CONFIGS[3].with_(n_chunks=4, chunk_len=256, n_query=16,
                                 n_relevant=10, n_salient=20, hidden=512)
    layers, info = workload.build(cfg)
    sel = O.topk_select(info["score"], info["k"])
    assert np.isin(info["relevant"], sel).all()
    assert np.isin(info["salient"], sel).mean() < 0.2
