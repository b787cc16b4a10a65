"""Pins for the CPU oracle: closed forms, library routines and brute force.

None of these tests re-types an oracle formula or re-calls the routine the
oracle itself uses; each checks the oracle against something fixed by the
paper's definitions or by mathematics:

* ratio 1.0 must equal full causal prefill attention (recomputation restores
  ground truth, Sec. 4.2; full recompute is the accuracy ceiling, Tab. 1);
* ratio 0 must equal plain concatenation of the chunk caches (naive reuse,
  Sec. 2.2 / Sec. 5.1 baselines);
* rows outside T_p are reused verbatim (Algorithm 1, cache update);
* rotary restore is a rotation: invertible, norm preserving, relative;
* attention weights are normalised inside a layer (Sec. 4.3), so the score
  of one layer sums to one;
* top-p is the p-fraction with the largest value function (Eq. 4).
"""

import cmath
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import pkv_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- rounding

def test_bf16_rounding_matches_library_on_fp32_values():
    x32 = rng(0).standard_normal(20000).astype(np.float32) * np.float32(37.0)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to_storage(x32.astype(np.float64), "bf16")
    assert np.array_equal(got, want)


def test_bf16_rounding_closed_forms():
    one = 1.0
    ulp = 2.0 ** -7                      # spacing of bfloat16 in [1, 2)
    cases = {
        one + ulp / 2: one,              # tie -> even mantissa (1.0)
        one + 3 * ulp / 2: one + 2 * ulp,  # tie -> even mantissa
        one + ulp / 2 + 2.0 ** -40: one + ulp,  # just above a tie: a trip
                                         # through fp32 would lose the 2**-40
        -(one + ulp / 2 + 2.0 ** -40): -(one + ulp),
        0.0: 0.0,
        (2.0 - 2.0 ** -8) : 2.0,         # mantissa carry into the exponent
        (2.0 - 2.0 ** -7) * 2.0 ** 127: (2.0 - 2.0 ** -7) * 2.0 ** 127,  # max
        1e39: math.inf,
        2.0 ** -133: 2.0 ** -133,        # smallest subnormal survives
        2.0 ** -135: 0.0,
    }
    for x, want in cases.items():
        got = float(O.round_to_storage(np.array([x]), "bf16")[0])
        assert got == want, (x, got, want)


def test_f32_rounding_closed_forms():
    """binary32 has 24 significant bits: ties go to the even neighbour, the slightest
    excess over a tie rounds up, overflow gives inf, the subnormal quantum is 2**-149."""
    r = lambda v: float(O.round_to_storage(np.array([v]), "f32")[0])  # noqa: E731
    assert r(1.0 + 2.0 ** -24) == 1.0                          # tie, even mantissa below
    assert r(1.0 + 2.0 ** -24 + 2.0 ** -40) == 1.0 + 2.0 ** -23
    assert r(1.0 + 3 * 2.0 ** -24) == 1.0 + 2.0 ** -22         # tie, even mantissa above
    assert r(1.0 + 2.0 ** -23) == 1.0 + 2.0 ** -23             # representable: unchanged
    assert r(-(1.0 + 2.0 ** -24 + 2.0 ** -40)) == -(1.0 + 2.0 ** -23)
    big = (2.0 - 2.0 ** -24) * 2.0 ** 127                      # halfway to 2**128
    assert r(big) == np.inf and r(-big) == -np.inf
    assert r((2.0 - 2.0 ** -23) * 2.0 ** 127) == (2.0 - 2.0 ** -23) * 2.0 ** 127
    assert r(2.0 ** -150) == 0.0                               # tie between 0 and 2**-149
    assert r(2.0 ** -150 + 2.0 ** -170) == 2.0 ** -149
    assert r(3 * 2.0 ** -150) == 2.0 ** -148                   # tie, even multiple
    # every result is a binary32 value: it survives a trip through 4-byte packing
    import struct
    x = rng(1).standard_normal(1000) * 1e3
    y = O.round_to_storage(x, "f32")
    back = np.array([struct.unpack("<f", struct.pack("<f", v))[0] for v in y])
    assert np.array_equal(back, y)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -24)


# ---------------------------------------------------------------- RoPE

def complex_rope(x, pos, theta):
    """Independent statement of the rotary embedding: the pair (i, i + D/2)
    is a complex number multiplied by exp(i * pos * theta**(-2i/D))."""
    n, h, d = x.shape
    out = np.empty_like(x)
    for t in range(n):
        for hh in range(h):
            for i in range(d // 2):
                z = complex(x[t, hh, i], x[t, hh, i + d // 2])
                z *= cmath.exp(1j * pos[t] * theta ** (-2.0 * i / d))
                out[t, hh, i] = z.real
                out[t, hh, i + d // 2] = z.imag
    return out


def test_rope_quarter_turn_fixes_the_sign_convention():
    # D = 2: a single pair with inv_freq = 1.  A rotation by +pi/2 carries
    # (1, 0) to (0, 1); the opposite sign convention would give (0, -1).
    x = np.array([[[1.0, 0.0]]])
    y = O.rope_rotate(x, np.array([math.pi / 2]), 10000.0)
    assert np.allclose(y, [[[0.0, 1.0]]], atol=1e-15)


def test_rope_closed_form_d4():
    # D = 4, theta = 10000: inv_freq = (1, 0.01); pairs are (x0,x2), (x1,x3)
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    y = O.rope_rotate(x, np.array([3.0]), 10000.0)[0, 0]
    c0, s0, c1, s1 = math.cos(3.0), math.sin(3.0), math.cos(0.03), math.sin(0.03)
    want = [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 3 * c0 + 1 * s0, 4 * c1 + 2 * s1]
    assert np.allclose(y, want, rtol=0, atol=1e-14)


def test_rope_matches_complex_formulation():
    g = rng(2)
    x = g.standard_normal((9, 3, 16))
    pos = g.integers(0, 5000, size=9).astype(np.float64)
    assert np.allclose(O.rope_rotate(x, pos, 500000.0),
                       complex_rope(x, pos, 500000.0), rtol=0, atol=1e-12)


def test_rope_identity_inverse_norm_relative():
    g = rng(3)
    d = 32
    x = g.standard_normal((7, 2, d))
    pos = np.array([0, 1, 17, 1023, 32767, 131071, 5], dtype=np.float64)
    y = O.rope_rotate(x, pos, 500000.0)
    assert np.array_equal(y[0], x[0])                       # position 0
    back = O.rope_rotate(y, -pos, 500000.0)                 # invertible
    assert np.allclose(back, x, rtol=0, atol=1e-11)
    assert np.allclose(np.linalg.norm(y, axis=2), np.linalg.norm(x, axis=2))
    # <R_m q, R_n k> depends on m - n only
    q = g.standard_normal((1, 1, d))
    k = g.standard_normal((1, 1, d))
    for m, n in [(100, 40), (5000, 4940), (60, 0)]:
        a = (O.rope_rotate(q, [m], 1e4) * O.rope_rotate(k, [n], 1e4)).sum()
        b = (O.rope_rotate(q, [m - n], 1e4) * k).sum()
        assert abs(a - b) < 1e-10


def test_rope_restore_rounds_to_storage():
    x = rng(4).standard_normal((5, 2, 8))
    y = O.rope_restore(x, np.arange(5), 1e4, "bf16")
    y32 = y.astype(np.float32)
    assert np.array_equal(y32.astype(np.float64), y)
    assert np.array_equal(
        torch.from_numpy(y32).to(torch.bfloat16).double().numpy(), y)
    assert np.abs(y - O.rope_rotate(x, np.arange(5), 1e4)).max() < 2.0 ** -7


# ---------------------------------------------------------------- score

def brute_score(q, k, hq, hkv):
    """Pure-Python triple loop of the Stage-I value function."""
    qn, _, d = q.shape
    n = k.shape[0]
    alpha = [0.0] * n
    for h in range(hq):
        g = h // (hq // hkv)
        for i in range(qn):
            logits = [sum(q[i, h, c] * k[t, g, c] for c in range(d)) / math.sqrt(d)
                      for t in range(n)]
            mx = max(logits)
            e = [math.exp(v - mx) for v in logits]
            z = sum(e)
            for t in range(n):
                alpha[t] += e[t] / z
    return np.array(alpha) / (hq * qn)


def test_score_brute_force_tiny():
    g = rng(5)
    q = g.standard_normal((3, 4, 6))
    k = g.standard_normal((11, 2, 6))
    assert np.allclose(O.query_score(q, k), brute_score(q, k, 4, 2),
                       rtol=1e-12, atol=0)


def test_score_is_normalised_and_uniform_cases():
    g = rng(6)
    q = g.standard_normal((5, 8, 16)) * 3
    k = g.standard_normal((200, 2, 16))
    a = O.query_score(q, k)
    assert abs(a.sum() - 1.0) < 1e-12 and (a > 0).all()
    same = np.broadcast_to(k[:1], k.shape)
    assert np.allclose(O.query_score(q, same), 1.0 / 200, rtol=1e-12)
    assert np.allclose(O.query_score(np.zeros_like(q), k), 1.0 / 200, rtol=1e-12)


def test_score_single_row_is_library_softmax():
    g = rng(7)
    q = g.standard_normal((1, 1, 10))
    k = g.standard_normal((50, 1, 10))
    want = scipy.special.softmax(k[:, 0, :] @ q[0, 0] / math.sqrt(10))
    assert np.allclose(O.query_score(q, k), want, rtol=1e-12)


def test_score_gqa_equals_mha_with_repeated_kv():
    g = rng(8)
    q = g.standard_normal((4, 6, 8))
    k = g.standard_normal((30, 2, 8))
    k_rep = np.repeat(k, 3, axis=1)
    assert np.allclose(O.query_score(q, k), O.query_score(q, k_rep), rtol=1e-13)


def test_score_scale_argument():
    g = rng(9)
    q = g.standard_normal((2, 2, 4))
    k = g.standard_normal((9, 2, 4))
    assert np.allclose(O.query_score(q, k, scale=0.5), O.query_score(q, k))
    assert not np.allclose(O.query_score(q, k, scale=1.0), O.query_score(q, k))


def test_fuse_score_is_a_running_fp32_sum():
    """The fused score is rounded to binary32 after every layer: closed forms that an
    unrounded (or once-rounded) sum would not give."""
    one = np.array([1.0])
    half_ulp = np.array([2.0 ** -24])
    assert O.fuse_score(one, half_ulp)[0] == 1.0                       # tie to even
    assert O.fuse_score(one, half_ulp + 2.0 ** -40)[0] == 1.0 + 2.0 ** -23
    s = one
    for _ in range(4):                       # four layers of half an ulp each
        s = O.fuse_score(s, half_ulp)
    assert s[0] == 1.0                       # the exact sum would be 1 + 2**-22
    assert O.fuse_score(np.zeros(1), np.array([0.1]))[0] == 13421773 * 2.0 ** -27
    # order matters as stated (layer order): small terms first survive
    s = np.zeros(1)
    for v in (2.0 ** -24, 2.0 ** -24, 1.0):
        s = O.fuse_score(s, np.array([v]))
    assert s[0] == 1.0 + 2.0 ** -23


# ---------------------------------------------------------------- top-k

def brute_topk(score, k):
    order = sorted(range(len(score)), key=lambda t: (-score[t], t))
    return sorted(order[:k])


@pytest.mark.parametrize("n,k", [(1, 0), (1, 1), (17, 5), (64, 64), (100, 0),
                                 (257, 100)])
def test_topk_brute_force(n, k):
    s = rng(n * 1000 + k).random(n)
    assert list(O.topk_select(s, k)) == brute_topk(list(s), k)


def test_topk_ties_go_to_the_lower_index():
    assert list(O.topk_select(np.ones(10), 4)) == [0, 1, 2, 3]
    s = np.array([0.5, 0.9, 0.5, 0.9, 0.5, 0.1, 0.5])
    assert list(O.topk_select(s, 2)) == [1, 3]
    assert list(O.topk_select(s, 4)) == [0, 1, 2, 3]
    assert list(O.topk_select(s, 5)) == [0, 1, 2, 3, 4]
    g = rng(11)
    s = g.integers(0, 5, size=300).astype(np.float64)       # heavy ties
    for k in (1, 50, 150, 299, 300):
        assert list(O.topk_select(s, k)) == brute_topk(list(s), k)


def test_topk_rejects_bad_k():
    with pytest.raises(ValueError):
        O.topk_select(np.ones(3), 4)


# ---------------------------------------------------------------- projection

def test_projection_identity_rows_is_a_linear_layer_plus_rotation():
    g = rng(12)
    hq, hkv, d, hid, m = 4, 2, 8, 24, 6
    x = g.standard_normal((m, hid))
    wq = g.standard_normal((hq * d, hid))
    wk = g.standard_normal((hkv * d, hid))
    wv = g.standard_normal((hkv * d, hid))
    pos = np.array([0, 3, 4, 100, 101, 7])
    q, k, v = O.project_qkv_rows(x, np.arange(m), pos, wq, wk, wv,
                                 hq, hkv, d, 1e4, "f64")
    lin = lambda w: torch.nn.functional.linear(
        torch.from_numpy(x), torch.from_numpy(w)).numpy()
    assert np.allclose(v, lin(wv).reshape(m, hkv, d), rtol=1e-13, atol=1e-13)
    assert np.allclose(q, complex_rope(lin(wq).reshape(m, hq, d), pos, 1e4),
                       rtol=1e-12, atol=1e-12)
    assert np.allclose(k, complex_rope(lin(wk).reshape(m, hkv, d), pos, 1e4),
                       rtol=1e-12, atol=1e-12)


def test_projection_gathers_the_named_rows():
    g = rng(13)
    hq, hkv, d, hid = 2, 1, 4, 8
    x = g.standard_normal((20, hid))
    w = [g.standard_normal((hq * d, hid)), g.standard_normal((d, hid)),
         g.standard_normal((d, hid))]
    rows = np.array([17, 2, 9])
    a = O.project_qkv_rows(x, rows, rows, *w, hq, hkv, d, 1e4, "f32")
    b = O.project_qkv_rows(x[rows], np.arange(3), rows, *w, hq, hkv, d, 1e4, "f32")
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def _proj_inputs(seed, hq=4, hkv=2, d=8, hid=24, m=6):
    g = rng(seed)
    x = g.standard_normal((m, hid))
    w = [g.standard_normal((hq * d, hid)), g.standard_normal((hkv * d, hid)),
         g.standard_normal((hkv * d, hid))]
    b = [g.standard_normal(hq * d), g.standard_normal(hkv * d), g.standard_normal(hkv * d)]
    pos = np.array([0, 3, 4, 100, 101, 7])[:m]
    return x, w, b, pos, (hq, hkv, d)


def test_projection_bias_equals_an_augmented_weight_column():
    """x W^T + b = [x, 1] [W, b]^T: the biased projection must equal the unbiased one
    on inputs with a constant 1 appended and the bias as one more weight column."""
    x, w, b, pos, (hq, hkv, d) = _proj_inputs(41)
    m = x.shape[0]
    got = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64",
                             bq=b[0], bk=b[1], bv=b[2])
    x1 = np.concatenate([x, np.ones((m, 1))], axis=1)
    w1 = [np.concatenate([wi, bi[:, None]], axis=1) for wi, bi in zip(w, b)]
    want = O.project_qkv_rows(x1, np.arange(m), pos, *w1, hq, hkv, d, 1e4, "f64")
    for u, v in zip(got, want):
        assert np.allclose(u, v, rtol=1e-12, atol=1e-12)
    # and against torch's biased linear layer for V (no rotation there)
    lin = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w[2]),
                                     torch.from_numpy(b[2])).numpy()
    assert np.allclose(got[2], lin.reshape(m, hkv, d), rtol=1e-13, atol=1e-13)
    # a bias on one projection leaves the other two alone
    only_q = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64", bq=b[0])
    plain = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64")
    assert np.array_equal(only_q[1], plain[1]) and np.array_equal(only_q[2], plain[2])
    assert not np.allclose(only_q[0], plain[0])


def test_projection_head_norm_against_torch_rms_norm_and_its_invariances():
    x, w, b, pos, (hq, hkv, d) = _proj_inputs(42)
    m = x.shape[0]
    g = rng(43)
    gq, gk = g.standard_normal(d), g.standard_normal(d)
    eps = 1e-6
    q, k, v = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64",
                                 q_norm=gq, k_norm=gk, norm_eps=eps)
    lin = lambda wi: torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(wi))
    nq = torch.nn.functional.rms_norm(lin(w[0]).reshape(m, hq, d), (d,),
                                      torch.from_numpy(gq), eps).numpy()
    nk = torch.nn.functional.rms_norm(lin(w[1]).reshape(m, hkv, d), (d,),
                                      torch.from_numpy(gk), eps).numpy()
    assert np.allclose(q, complex_rope(nq, pos, 1e4), rtol=1e-12, atol=1e-12)
    assert np.allclose(k, complex_rope(nk, pos, 1e4), rtol=1e-12, atol=1e-12)
    assert np.allclose(v, lin(w[2]).numpy().reshape(m, hkv, d), rtol=1e-13, atol=1e-13)
    # with eps = 0 and unit gains every head of q and k has norm sqrt(D) at any position,
    # and scaling the hidden rows changes nothing but v
    ones = np.ones(d)
    q1, k1, v1 = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64",
                                    q_norm=ones, k_norm=ones, norm_eps=0.0)
    assert np.allclose(np.linalg.norm(q1, axis=2), np.sqrt(d), rtol=1e-12)
    assert np.allclose(np.linalg.norm(k1, axis=2), np.sqrt(d), rtol=1e-12)
    q2, k2, v2 = O.project_qkv_rows(7.5 * x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64",
                                    q_norm=ones, k_norm=ones, norm_eps=0.0)
    assert np.allclose(q1, q2, rtol=1e-12, atol=1e-12)
    assert np.allclose(k1, k2, rtol=1e-12, atol=1e-12)
    assert np.allclose(7.5 * v1, v2, rtol=1e-12, atol=1e-12)
    # the norm comes BEFORE the rotation: norm then rotate != rotate then norm only through
    # the gain, so with a non-constant gain the two orders differ while with unit gain they agree
    plain = O.project_qkv_rows(x, np.arange(m), pos, *w, hq, hkv, d, 1e4, "f64")
    after = plain[0] / np.sqrt((plain[0] ** 2).mean(axis=2, keepdims=True))
    assert np.allclose(q1, after, rtol=1e-12, atol=1e-12)
    assert not np.allclose(q[3], after[3] * gq, rtol=1e-3, atol=1e-3)


# ---------------------------------------------------------------- scatter

def test_scatter_replaces_only_the_named_rows():
    g = rng(14)
    kc, vc = g.standard_normal((12, 2, 4)), g.standard_normal((12, 2, 4))
    kn, vn = g.standard_normal((3, 2, 4)), g.standard_normal((3, 2, 4))
    dst = np.array([7, 0, 11])
    k2, v2 = O.scatter_kv(kc, vc, kn, vn, dst)
    assert np.array_equal(k2[dst], kn) and np.array_equal(v2[dst], vn)
    rest = np.setdiff1d(np.arange(12), dst)
    assert np.array_equal(k2[rest], kc[rest]) and np.array_equal(v2[rest], vc[rest])
    with pytest.raises(ValueError):
        O.scatter_kv(kc, vc, kn, vn, np.array([1, 1, 2]))


# ---------------------------------------------------------------- attention

def brute_attn(q, kc, vc, row_pos, hq, hkv):
    m, _, d = q.shape
    out = np.zeros((m, hq, d))
    lse = np.zeros((m, hq))
    for i in range(m):
        for h in range(hq):
            g = h // (hq // hkv)
            logits = [sum(q[i, h, c] * kc[t, g, c] for c in range(d)) / math.sqrt(d)
                      for t in range(row_pos[i] + 1)]
            mx = max(logits)
            e = [math.exp(v - mx) for v in logits]
            z = sum(e)
            for c in range(d):
                out[i, h, c] = sum(e[t] * vc[t, g, c] for t in range(len(e))) / z
            lse[i, h] = mx + math.log(z)
    return out, lse


def test_attention_brute_force_tiny():
    g = rng(15)
    hq, hkv, d = 4, 2, 6
    q = g.standard_normal((5, hq, d))
    kc, vc = g.standard_normal((13, hkv, d)), g.standard_normal((13, hkv, d))
    pos = np.array([0, 3, 3, 9, 12])
    out, lse = O.sparse_row_attn(q, kc, vc, pos)
    bo, bl = brute_attn(q, kc, vc, pos, hq, hkv)
    assert np.allclose(out, bo, rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, bl, rtol=1e-12, atol=1e-14)


def test_attention_closed_forms():
    g = rng(16)
    hq, hkv, d, n = 4, 2, 8, 40
    q = g.standard_normal((6, hq, d))
    kc, vc = g.standard_normal((n, hkv, d)), g.standard_normal((n, hkv, d))
    pos = np.array([0, 5, 5, 17, 30, 39])
    out, lse = O.sparse_row_attn(q, kc, vc, pos)
    # a row that sees only key 0 returns value 0 of its kv head
    for h in range(hq):
        assert np.allclose(out[0, h], vc[0, h // 2], rtol=1e-14)
    # constant values come back unchanged
    const = np.broadcast_to(g.standard_normal((1, hkv, d)), vc.shape)
    oc, _ = O.sparse_row_attn(q, kc, const, pos)
    for h in range(hq):
        assert np.allclose(oc[:, h], const[0, h // 2], rtol=1e-13)
    # keys and values beyond a row's position cannot matter
    k2, v2 = kc.copy(), vc.copy()
    k2[18:] += 100.0
    v2[18:] -= 50.0
    o2, l2 = O.sparse_row_attn(q, k2, v2, pos)
    assert np.array_equal(o2[:4], out[:4]) and np.array_equal(l2[:4], lse[:4])
    assert not np.allclose(o2[4:], out[4:])
    # the normaliser is the library log-sum-exp of the visible logits
    for i, p in enumerate(pos):
        for h in range(hq):
            logits = kc[:p + 1, h // 2] @ q[i, h] / math.sqrt(d)
            assert abs(lse[i, h] - scipy.special.logsumexp(logits)) < 1e-12


def test_attention_matches_library_sdpa_with_explicit_mask():
    g = rng(17)
    hq, hkv, d, n, m = 6, 3, 16, 70, 9
    q = g.standard_normal((m, hq, d))
    kc, vc = g.standard_normal((n, hkv, d)), g.standard_normal((n, hkv, d))
    pos = np.sort(g.choice(n, m, replace=False))
    out, _ = O.sparse_row_attn(q, kc, vc, pos)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(kc, 2, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(vc, 2, axis=1)).permute(1, 0, 2)[None]
    mask = torch.from_numpy(np.arange(n)[None, :] <= pos[:, None])
    want = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.allclose(out, want, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- whole path

def small_problem(seed, n=48, qn=5, hq=4, hkv=2, d=8, hid=24, layers=1):
    g = rng(seed)
    ls = []
    for _ in range(layers):
        ls.append(dict(
            k_nope=g.standard_normal((n, hkv, d)),
            v=g.standard_normal((n, hkv, d)),
            hidden=g.standard_normal((n + qn, hid)),
            wq=g.standard_normal((hq * d, hid)) * 0.3,
            wk=g.standard_normal((hkv * d, hid)) * 0.3,
            wv=g.standard_normal((hkv * d, hid)) * 0.3))
    return ls, dict(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, theta=1e4)


def full_prefill_reference(layer, geo):
    """Textbook causal prefill of one layer through library routines only."""
    hq, hkv, d, theta = (geo["n_q_heads"], geo["n_kv_heads"], geo["head_dim"],
                         geo["theta"])
    x = torch.from_numpy(layer["hidden"])
    s = x.shape[0]
    lin = lambda w: torch.nn.functional.linear(x, torch.from_numpy(w)).numpy()
    pos = np.arange(s, dtype=np.float64)
    q = complex_rope(lin(layer["wq"]).reshape(s, hq, d), pos, theta)
    k = complex_rope(lin(layer["wk"]).reshape(s, hkv, d), pos, theta)
    v = lin(layer["wv"]).reshape(s, hkv, d)
    rep = hq // hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, rep, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, rep, axis=1)).permute(1, 0, 2)[None]
    out = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    return out, k, v


def test_ratio_one_equals_full_causal_prefill():
    layers, geo = small_problem(20, layers=2)
    n, qn = 48, 5
    sel, score, res = O.prophetkv_stack(layers, qn, n, 2, dtype="f64", **geo)
    assert list(sel) == list(range(n))
    for layer, r in zip(layers, res):
        want_out, want_k, want_v = full_prefill_reference(layer, geo)
        assert np.allclose(r["out"], want_out, rtol=1e-10, atol=1e-11)
        assert np.allclose(r["k_cache"], want_k, rtol=1e-11, atol=1e-12)
        assert np.allclose(r["v_cache"], want_v, rtol=1e-11, atol=1e-12)


def test_ratio_one_bf16_storage_stays_within_bf16_of_full_prefill():
    layers, geo = small_problem(21)
    for l in layers:
        for name in l:
            l[name] = O.round_to_storage(l[name], "bf16")
    sel, _, res = O.prophetkv_stack(layers, 5, 48, 1, dtype="bf16", **geo)
    want_out, _, _ = full_prefill_reference(layers[0], geo)
    err = np.abs(res[0]["out"] - want_out).max() / np.abs(want_out).max()
    assert err < 2e-2


def test_ratio_zero_equals_plain_concatenation():
    layers, geo = small_problem(22)
    n, qn = 48, 5
    l = layers[0]
    sel, _, res = O.prophetkv_stack(layers, qn, 0, 1, dtype="f32", **geo)
    r = res[0]
    assert sel.shape == (0,)
    roped = complex_rope(l["k_nope"], np.arange(n, dtype=np.float64), geo["theta"])
    # (fp32 storage of two fp64 evaluations of the same rotation may differ
    # in the last fp32 bit, hence a tolerance of a few fp32 ulps)
    assert np.abs(r["k_cache"][:n] - roped).max() < 1e-6
    assert np.array_equal(r["v_cache"][:n], O.round_to_storage(l["v"], "f32"))
    assert list(r["rows"]) == list(range(n, n + qn))
    # the query rows attend to the concatenated cache plus their own K/V
    out, _ = brute_attn(r["q"], r["k_cache"], r["v_cache"], r["rows"],
                        geo["n_q_heads"], geo["n_kv_heads"])
    assert np.allclose(r["out"], out, rtol=0, atol=1e-6)


def test_unselected_rows_are_reused_bit_for_bit_and_selection_is_shared():
    layers, geo = small_problem(23, layers=3)
    n, qn, k = 48, 5, 9
    sel, score, res = O.prophetkv_stack(layers, qn, k, 3, dtype="bf16", **geo)
    assert sel.shape == (k,) and np.all(np.diff(sel) > 0)
    # one layer's score sums to one, so the plain sum over 3 layers sums to 3
    assert abs(score.sum() - 3.0) < 1e-5
    rest = np.setdiff1d(np.arange(n), sel)
    for l, r in zip(layers, res):
        kr = O.rope_restore(l["k_nope"], np.arange(n), geo["theta"], "bf16")
        assert np.array_equal(r["k_cache"][rest], kr[rest])
        assert np.array_equal(r["v_cache"][rest],
                              O.round_to_storage(l["v"], "bf16")[rest])
        assert list(r["rows"][:k]) == list(sel)
        assert np.array_equal(r["k_cache"][r["rows"]], r["k_new"])
        assert np.array_equal(r["v_cache"][r["rows"]], r["v_new"])
        # selected rows hold recomputed, not reused, keys
        assert not np.array_equal(r["k_cache"][sel], kr[sel])


def test_layer1_variant_uses_only_the_first_layer_score():
    layers, geo = small_problem(24, layers=2)
    sel1, s1, _ = O.prophetkv_stack(layers, 5, 9, 1, dtype="f32", **geo)
    sel_first, s_first, _ = O.prophetkv_stack(layers[:1], 5, 9, 1, dtype="f32", **geo)
    assert np.array_equal(sel1, sel_first) and np.array_equal(s1, s_first)
