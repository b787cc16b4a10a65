"""Pins of the diagnostics oracle (oracle/pkv_diag_oracle.py) against things that are
not it: brute force on tiny inputs, closed forms, the independent torch forward of
tests/test_model_oracle_pins.py, and the hot-path oracle's functions."""

import numpy as np
import pytest

from oracle import pkv_diag_oracle as DG
from oracle import pkv_oracle as O
from tests.test_model_oracle_pins import tiny_model, torch_forward, torch_rope

GEO = dict(n_q_heads=4, n_kv_heads=2, head_dim=8, theta=10000.0, eps=1e-6, dtype="f64")


def test_overlap_ratio_closed_forms():
    assert DG.overlap_ratio([1, 2, 3], [1, 2, 3]) == 1.0
    assert DG.overlap_ratio([4, 5], [1, 2, 3]) == 0.0
    assert DG.overlap_ratio([3, 9, 1, 7], [1, 2, 3, 4]) == 0.5      # |{1,3}| / |G|
    assert DG.overlap_ratio([1, 1, 2], [2, 2, 5, 6]) == pytest.approx(1 / 3)   # sets
    assert DG.overlap_ratio([], [1]) == 0.0
    with pytest.raises(ValueError):
        DG.overlap_ratio([1], [])


def test_column_sum_brute_force_and_invariants():
    g = np.random.default_rng(1)
    m, n_keys, hq, hkv, d = 7, 9, 4, 2, 6
    q, k = g.standard_normal((m, hq, d)), g.standard_normal((n_keys, hkv, d))
    pos = np.array([0, 2, 2, 5, 6, 8, 8])
    got = DG.column_sum_score(q, k, pos)
    want = np.zeros(n_keys)
    for i in range(m):
        for h in range(hq):
            s = [float(q[i, h] @ k[t, h // 2]) / np.sqrt(d) for t in range(pos[i] + 1)]
            z = sum(np.exp(x) for x in s)
            for t, x in enumerate(s):
                want[t] += np.exp(x) / z / (m * hq)
    assert np.abs(got - want).max() < 1e-14
    assert abs(got.sum() - 1.0) < 1e-14            # every row's softmax sums to one
    assert got[7] > 0 and np.all(got[:1] > 0)
    # a key nobody sees receives nothing; the first key receives all of row 0
    got2 = DG.column_sum_score(q, k, np.minimum(pos, 6))
    assert got2[7] == 0.0 and got2[8] == 0.0
    # when every row sees every key it is the query-attention score of the hot-path oracle
    full = DG.column_sum_score(q, k, np.full(m, n_keys - 1))
    assert np.abs(full - O.query_score(q, k)).max() < 1e-15


def test_prefill_rows_is_the_ordinary_causal_forward():
    n, hid, inter, L = 23, 32, 48, 3
    embed, layers = tiny_model(7, n, 0, hid, inter, 4, 2, 8, L)
    hs, ks, vs = torch_forward(embed, layers, 4, 2, 8, 10000.0, 1e-6)
    import torch
    got_k, got_v, got_h = DG.prefill_rows(embed, layers, np.arange(n), **GEO)
    for li in range(L):
        kr = torch_rope(torch.from_numpy(ks[li]), torch.arange(n), 10000.0).numpy()
        assert np.abs(got_k[li] - kr).max() < 1e-9
        assert np.abs(got_v[li] - vs[li]).max() < 1e-9
    assert np.abs(got_h - hs[-1]).max() < 1e-9


def test_chunk_isolated_cache_closed_forms():
    n_ctx, n_query, hid, inter, L = 24, 4, 32, 48, 3
    embed, layers = tiny_model(8, n_ctx, n_query, hid, inter, 4, 2, 8, L)
    hs, ks, vs = torch_forward(embed[:n_ctx], layers, 4, 2, 8, 10000.0, 1e-6)
    # one chunk: the stored (position-free) keys and the values of an ordinary prefill
    k1, v1 = DG.chunk_isolated_cache(embed, layers, n_ctx, n_ctx, **GEO)
    for li in range(L):
        assert np.abs(k1[li] - ks[li]).max() < 1e-9
        assert np.abs(v1[li] - vs[li]).max() < 1e-9
    kf, vf = DG.full_prefill_cache(embed, layers, n_ctx, **GEO)
    assert all(np.array_equal(a, b) for a, b in zip(k1 + v1, kf + vf))
    # several chunks: the first layer sees only embeddings, so its K/V are still exact;
    # the first chunk is exact in every layer; later chunks differ from the second layer on
    k4, v4 = DG.chunk_isolated_cache(embed, layers, n_ctx, 6, **GEO)
    assert np.abs(k4[0] - ks[0]).max() < 1e-9 and np.abs(v4[0] - vs[0]).max() < 1e-9
    for li in range(1, L):
        assert np.abs(v4[li][:6] - vs[li][:6]).max() < 1e-9
        assert np.abs(v4[li][6:] - vs[li][6:]).max() > 1e-3
    # a chunk is prefilled at positions 0..len-1 whatever its place in the prompt: chunk 2
    # alone gives the same stored cache
    hs2, ks2, vs2 = torch_forward(embed[12:18], layers, 4, 2, 8, 10000.0, 1e-6)
    for li in range(L):
        assert np.abs(k4[li][12:18] - ks2[li]).max() < 1e-9
        assert np.abs(v4[li][12:18] - vs2[li]).max() < 1e-9
    # ragged last chunk
    k5, v5 = DG.chunk_isolated_cache(embed, layers, n_ctx, 10, **GEO)
    assert k5[0].shape == (n_ctx, 2, 8) and np.abs(v5[0] - vs[0]).max() < 1e-9


def test_full_prefill_query_attention_is_what_the_forward_computes():
    """G of Sec. 3.1: with the true cache, the fused score is the mean over layers'
    query-to-context attention of an ordinary forward (softmax over the context keys)."""
    n_ctx, n_query, hid, inter, L = 20, 3, 32, 48, 2
    embed, layers = tiny_model(9, n_ctx, n_query, hid, inter, 4, 2, 8, L)
    kf, vf = DG.full_prefill_cache(embed, layers, n_ctx, **GEO)
    got = DG.query_attention_score(embed, layers, kf, vf, n_query, L, **GEO)
    # independent: queries of the query rows from the torch forward of the whole prompt
    import torch
    import torch.nn.functional as F
    hs, ks, vs = torch_forward(embed, layers, 4, 2, 8, 10000.0, 1e-6)
    want = np.zeros(n_ctx)
    h_in = [embed] + hs[:-1]
    for li, l in enumerate(layers):
        h = torch.from_numpy(h_in[li])
        x = F.rms_norm(h, (hid,), torch.from_numpy(l["w_in"]), 1e-6)
        q = F.linear(x, torch.from_numpy(l["wq"])).view(-1, 4, 8)
        pos = torch.arange(n_ctx + n_query)
        qr = torch_rope(q, pos, 10000.0)[n_ctx:]
        kr = torch_rope(torch.from_numpy(ks[li]), pos, 10000.0)[:n_ctx]
        for hh in range(4):
            s = (qr[:, hh] @ kr[:, hh // 2].T) / np.sqrt(8)
            want += torch.softmax(s, dim=1).sum(0).numpy() / (4 * n_query)
    assert np.abs(got - want).max() < 1e-6          # the fused score is stored in fp32


def test_selection_diagnostics_end_points():
    n_ctx, n_query, hid, inter, L = 32, 4, 32, 48, 2
    embed, layers = tiny_model(10, n_ctx, n_query, hid, inter, 4, 2, 8, L)
    # one chunk = the cache is exact: the fused criterion IS the ground truth
    one = DG.selection_diagnostics(embed, layers, n_ctx, n_query, n_ctx, [0.25, 0.5], **GEO)
    assert one["fused"] == [1.0, 1.0]
    assert np.array_equal(one["scores"]["fused"], one["scores"]["truth"])
    # ratio 1 selects everything whatever the criterion
    many = DG.selection_diagnostics(embed, layers, n_ctx, n_query, 8, [0.25, 1.0], **GEO)
    assert many["fused"][1] == many["first_layer"][1] == many["column_sum"][1] == 1.0
    assert all(0.0 <= x <= 1.0 for name in ("fused", "first_layer", "column_sum")
               for x in many[name])
    assert abs(many["scores"]["column_sum"].sum() - 1.0) < 0.2   # most mass sits on the context
