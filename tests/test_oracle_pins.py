"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test states which passage of the paper it comes from.  None of them re-types the
oracle's own formula to check it: they use closed forms, special cases that reduce to a
library routine (scipy softmax, numpy matmul), the paper's printed numbers, invariants,
or an independent pure-Python brute force on tiny inputs.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import brute_force as BF
from oracle import sparq_oracle as O
from util import BF16, F16, codes_from_floats, floats_from_codes

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, B=1, H=1, H_kv=1, S=48, d_h=16, dtype=F16, S_max=None, scale=1.0, v_shift=0.0):
    rng = np.random.default_rng(seed)
    S_max = S if S_max is None else S_max
    Kc, K = codes_from_floats(rng.normal(size=(B, H_kv, S_max, d_h)) * scale, dtype)
    Vc, V = codes_from_floats(rng.normal(size=(B, H_kv, S_max, d_h)) + v_shift, dtype)
    qc, q = codes_from_floats(rng.normal(size=(B, H, d_h)) * scale, dtype)
    return dict(Kc=Kc, K=K, Vc=Vc, V=V, qc=qc, q=q, seq=np.full(B, S, dtype=np.int32), dtype=dtype)


def np_dense(q, K, V):
    """Eq. (2) with library routines: q [d], K, V [S, d]."""
    return scipy_softmax(K @ q / math.sqrt(len(q))) @ V


# ---------------------------------------------------------------- number formats

@pytest.mark.parametrize("dtype", [F16, BF16])
def test_widening_of_every_code(dtype):
    codes = np.arange(65536, dtype=np.uint16)
    got = O.to_double(codes, dtype)
    want = floats_from_codes(codes, dtype)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- Section 4 schematic

def read_schematic():
    out = {}
    for line in open(os.path.join(GOLDEN, "schematic_query.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [float(v) for v in vals]
    return out


def test_schematic_query_selects_by_magnitude():
    g = read_schematic()
    q = np.array(g["q"]); r = int(g["r"][0])
    rng = np.random.default_rng(0)
    for dtype in (F16, BF16):
        qc, qr = codes_from_floats(q[None, None, :], dtype)
        Kc, _ = codes_from_floats(rng.normal(size=(1, 1, 8, 4)), dtype)
        res = O.sparq_decode(Kc, Kc, qc, [8], r=r, k=3, dtype=dtype)
        assert res.i1[0, 0].tolist() == [int(v) for v in g["i1"]]
        # tau from the printed numbers, up to the rounding of 0.8 / -1.3 / ... to 16 bits
        assert abs(res.tau[0, 0] - g["tau"][0]) < (2e-3 if dtype == F16 else 1e-2)
        # and exactly Eq. (9) on the rounded query
        a = np.abs(qr[0, 0])
        assert res.tau[0, 0] == pytest.approx(math.sqrt(4 * (a[0] + a[2]) / a.sum()), rel=1e-14)


def test_top_r_ties_go_to_lower_channel():
    qc, _ = codes_from_floats(np.array([[[1.0, -1.0, 0.5, 1.0, -1.0, 0.25]]]), F16)
    Kc, _ = codes_from_floats(np.random.default_rng(1).normal(size=(1, 1, 5, 6)), F16)
    for r, want in [(1, [0]), (2, [0, 1]), (3, [0, 1, 3]), (4, [0, 1, 3, 4]), (5, [0, 1, 2, 3, 4])]:
        assert O.sparq_decode(Kc, Kc, qc, [5], r=r, k=2, dtype=F16).i1[0, 0].tolist() == want


# ---------------------------------------------------------------- reductions to dense attention

@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_full_rank_full_k_is_dense_attention(seed, dtype):
    """r = d_h and k = S: Steps 1-3 collapse to Eq. (2) and alpha = 1."""
    c = rand_case(seed, B=2, H=4, H_kv=2, S=40, d_h=16, dtype=dtype, S_max=48)
    c["seq"] = np.array([40, 33], dtype=np.int32)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=16, k=48, dtype=dtype)
    dense = O.dense_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], dtype=dtype)
    for b in range(2):
        S = c["seq"][b]
        for h in range(4):
            want = np_dense(c["q"][b, h], c["K"][b, h // 2, :S], c["V"][b, h // 2, :S])
            assert np.abs(dense[b, h] - want).max() < 1e-12
            assert np.abs(res.y[b, h] - want).max() < 1e-12
            assert abs(res.alpha[b, h] - 1.0) < 1e-12
            assert res.tau[b, h] == pytest.approx(4.0, rel=1e-15)
            assert res.i2[b, h, :S].tolist() == list(range(S))
            assert (res.i2[b, h, S:] == -1).all()


@pytest.mark.parametrize("k", [1, 5, 17, 40])
def test_full_rank_any_k_is_mean_value_reallocation(k):
    """r = d_h: tau = sqrt(d_h) so s-hat = s, and alpha*y3 + (1-alpha)*v_bar equals Eq. (6)."""
    c = rand_case(7, S=40, d_h=16, v_shift=0.7)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=16, k=k, dtype=F16)
    q, K, V = c["q"][0, 0], c["K"][0, 0], c["V"][0, 0]
    s = scipy_softmax(K @ q / 4.0)
    keep = np.argsort(-s, kind="stable")[:k]
    m = np.zeros(40); m[keep] = 1.0
    want = (s * m) @ V + (1.0 - s @ m) * V.mean(axis=0)
    assert np.abs(res.y[0, 0] - want).max() < 1e-12
    assert sorted(keep.tolist()) == res.i2[0, 0, :k].tolist()
    assert res.alpha[0, 0] == pytest.approx(s @ m, abs=1e-13)
    # and the brute force's independent Eq. (6)
    bf = BF.sparse_v_reallocation(q.tolist(), K.tolist(), V.tolist(), k)
    assert np.abs(res.y[0, 0] - np.array(bf)).max() < 1e-12


# ---------------------------------------------------------------- temperature (Eq. 9)

def test_query_supported_on_r_channels_keeps_sqrt_dh_and_exact_scores():
    """Section 3: were the top-r components the only non-zero ones, tau stays sqrt(d_h);
    the approximate logits then equal the exact ones."""
    rng = np.random.default_rng(3)
    d_h, S, r = 32, 50, 6
    qv = np.zeros(d_h); chans = rng.choice(d_h, r, replace=False); qv[chans] = rng.normal(size=r) + 2.0
    qc, q = codes_from_floats(qv[None, None], F16)
    Kc, K = codes_from_floats(rng.normal(size=(1, 1, S, d_h)), F16)
    res = O.sparq_decode(Kc, Kc, qc, [S], r=r, k=9, dtype=F16, want_z=True)
    assert res.tau[0, 0] == pytest.approx(math.sqrt(d_h), rel=1e-15)
    assert res.i1[0, 0].tolist() == sorted(chans.tolist())
    exact = K[0, 0] @ q[0, 0] / math.sqrt(d_h)
    assert np.abs(res.z[0, 0, :S] - exact).max() < 1e-12


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_tau_lies_between_sqrt_r_and_sqrt_dh(dtype):
    """The top-r magnitudes hold at least r/d_h of the L1 mass: the two extremes Section 3 names."""
    for seed in range(20):
        c = rand_case(seed, H=3, H_kv=3, S=8, d_h=32, dtype=dtype, scale=3.0)
        for r in (1, 4, 31, 32):
            tau = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=2, dtype=dtype).tau
            assert (tau >= math.sqrt(r) - 1e-12).all() and (tau <= math.sqrt(32) + 1e-12).all()
            if r == 32:
                assert np.allclose(tau, math.sqrt(32), rtol=1e-15)


def test_uniform_magnitude_query_gives_sqrt_r():
    """|q_j| all equal: the L1 share of any r channels is r/d_h, so tau = sqrt(r)."""
    d_h, r = 16, 4
    qv = np.where(np.arange(d_h) % 3 == 0, -0.5, 0.5)
    qc, _ = codes_from_floats(qv[None, None], F16)
    Kc, _ = codes_from_floats(np.random.default_rng(0).normal(size=(1, 1, 6, d_h)), F16)
    res = O.sparq_decode(Kc, Kc, qc, [6], r=r, k=2, dtype=F16)
    assert res.tau[0, 0] == pytest.approx(2.0, rel=1e-15)
    assert res.i1[0, 0].tolist() == [0, 1, 2, 3]


def test_zero_query():
    """0/0 in Eq. (9) is read as tau = sqrt(d_h): all logits 0, uniform scores, first k positions."""
    S, d_h, k = 12, 8, 5
    qc = np.zeros((1, 1, d_h), dtype=np.uint16); qc[0, 0, 3] = 0x8000   # one negative zero
    rng = np.random.default_rng(5)
    Kc, _ = codes_from_floats(rng.normal(size=(1, 1, S, d_h)), F16)
    Vc, V = codes_from_floats(rng.normal(size=(1, 1, S, d_h)), F16)
    res = O.sparq_decode(Kc, Vc, qc, [S], r=2, k=k, dtype=F16)
    assert res.tau[0, 0] == pytest.approx(math.sqrt(d_h))
    assert res.i1[0, 0].tolist() == [0, 1]
    assert res.i2[0, 0].tolist() == list(range(k))
    assert res.alpha[0, 0] == pytest.approx(k / S, rel=1e-14)
    want = (k / S) * V[0, 0, :k].mean(axis=0) + (1 - k / S) * V[0, 0].mean(axis=0)
    assert np.abs(res.y[0, 0] - want).max() < 1e-14


# ---------------------------------------------------------------- alpha and the blend (Eq. 10)

def test_identical_keys_pin_tie_break_alpha_and_blend():
    """All keys equal: s-hat is uniform, so alpha = k/S exactly, the k lowest positions win the
    ties, y3 is the plain mean of their values and y = (k/S) mean(V[:k]) + (1 - k/S) v_bar."""
    rng = np.random.default_rng(11)
    S, d_h, r, k = 37, 16, 5, 10
    row = rng.normal(size=d_h)
    Kc, _ = codes_from_floats(np.broadcast_to(row, (1, 1, S, d_h)), BF16)
    Vc, V = codes_from_floats(rng.normal(size=(1, 1, S, d_h)) + 1.0, BF16)
    qc, _ = codes_from_floats(rng.normal(size=(1, 1, d_h)), BF16)
    res = O.sparq_decode(Kc, Vc, qc, [S], r=r, k=k, dtype=BF16)
    assert res.i2[0, 0].tolist() == list(range(k))
    assert res.alpha[0, 0] == pytest.approx(k / S, rel=1e-14)
    want = (k / S) * V[0, 0, :k].mean(axis=0) + (1 - k / S) * V[0, 0].mean(axis=0)
    assert np.abs(res.y[0, 0] - want).max() < 1e-13


def test_constant_values_give_that_constant():
    """The weights of Eq. (10) sum to one: if every value row is c, the output is c for any r, k."""
    rng = np.random.default_rng(12)
    S, d_h = 33, 16
    crow = rng.normal(size=d_h)
    Vc, V = codes_from_floats(np.broadcast_to(crow, (1, 1, S, d_h)), F16)
    Kc, _ = codes_from_floats(rng.normal(size=(1, 1, S, d_h)), F16)
    qc, _ = codes_from_floats(rng.normal(size=(1, 1, d_h)) * 2, F16)
    for r, k in [(1, 1), (4, 7), (16, 33), (3, 50)]:
        res = O.sparq_decode(Kc, Vc, qc, [S], r=r, k=k, dtype=F16)
        assert np.abs(res.y[0, 0] - V[0, 0, 0]).max() < 1e-14


def test_alpha_is_a_mass_in_unit_interval_and_monotone_in_k():
    c = rand_case(21, S=64, d_h=16, scale=1.5)
    prev = 0.0
    for k in range(1, 66):
        res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=4, k=k, dtype=F16)
        a = res.alpha[0, 0]
        assert 0.0 <= a <= 1.0 + 1e-15 and a >= prev - 1e-15
        prev = a
    assert abs(prev - 1.0) < 1e-12          # k >= S: everything selected (k clamps to S)
    assert res.i2[0, 0].tolist() == list(range(64))


def test_no_reallocation_flag_returns_y3():
    c = rand_case(22, S=30, d_h=8, v_shift=2.0)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=6, dtype=F16, flags=O.NO_REALLOC)
    bf = BF.sparq(c["q"][0, 0].tolist(), c["K"][0, 0].tolist(), c["V"][0, 0].tolist(), 3, 6, realloc=False)
    assert np.abs(res.y[0, 0] - np.array(bf["y"])).max() < 1e-13
    # y3 is a convex combination of the selected rows: with alpha < 1 the blended output differs
    res2 = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=6, dtype=F16)
    assert np.abs(res2.y - res.y).max() > 1e-3


# ---------------------------------------------------------------- brute force on tiny inputs

@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("seed", range(8))
def test_against_pure_python_brute_force(seed, dtype):
    rng = np.random.default_rng(100 + seed)
    S = int(rng.integers(1, 64)); d_h = int(rng.choice([4, 8, 16])); r = int(rng.integers(1, d_h + 1))
    k = int(rng.integers(1, S + 3))
    c = rand_case(200 + seed, S=S, d_h=d_h, dtype=dtype, v_shift=0.5)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=dtype, want_z=True)
    bf = BF.sparq(c["q"][0, 0].tolist(), c["K"][0, 0].tolist(), c["V"][0, 0].tolist(), r, k)
    ke = min(k, S)
    assert res.i1[0, 0].tolist() == bf["i1"]
    assert res.tau[0, 0] == pytest.approx(bf["tau"], rel=1e-14)
    assert np.abs(res.z[0, 0, :S] - np.array(bf["z"])).max() < 1e-12
    assert res.i2[0, 0, :ke].tolist() == bf["i2"]
    assert res.alpha[0, 0] == pytest.approx(bf["alpha"], abs=1e-13)
    assert np.abs(res.y[0, 0] - np.array(bf["y"])).max() < 1e-12


def test_duplicate_keys_at_the_threshold_go_to_lower_positions():
    """Equal rows have equal scores; which of them enter the top-k is decided by position."""
    rng = np.random.default_rng(31)
    S, d_h = 20, 8
    K = rng.normal(size=(S, d_h)); q = rng.normal(size=d_h)
    qc, qr = codes_from_floats(q[None, None], F16)
    Kc, Kr = codes_from_floats(K[None, None], F16)
    order = np.argsort(-(Kr[0, 0] @ qr[0, 0]))
    third = order[2]
    for p in (order[10], order[15], order[17]):          # three more copies of the 3rd best row
        Kc[0, 0, p] = Kc[0, 0, third]
    same = sorted([int(third), int(order[10]), int(order[15]), int(order[17])])
    for k in (3, 4, 5, 6):
        res = O.sparq_decode(Kc, Kc, qc, [S], r=d_h, k=k, dtype=F16)
        want = sorted([int(order[0]), int(order[1])] + same[:k - 2])
        assert res.i2[0, 0].tolist() == want


# ---------------------------------------------------------------- invariances

def test_row_and_channel_permutations():
    c = rand_case(41, S=50, d_h=16, v_shift=0.3)
    base = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=5, k=9, dtype=F16)
    rng = np.random.default_rng(0)
    # jointly permuting cache rows permutes i2 and leaves y unchanged
    p = rng.permutation(50)
    res = O.sparq_decode(c["Kc"][:, :, p], c["Vc"][:, :, p], c["qc"], c["seq"], r=5, k=9, dtype=F16)
    assert sorted(p[res.i2[0, 0]].tolist()) == base.i2[0, 0].tolist()
    assert np.abs(res.y - base.y).max() < 1e-13
    assert res.alpha[0, 0] == pytest.approx(base.alpha[0, 0], abs=1e-14)
    # jointly permuting the channels of q and K (and, separately, of V) changes nothing but labels
    pc = rng.permutation(16); pv = rng.permutation(16)
    res = O.sparq_decode(c["Kc"][..., pc], c["Vc"][..., pv], c["qc"][..., pc], c["seq"], r=5, k=9, dtype=F16)
    assert sorted(pc[res.i1[0, 0]].tolist()) == base.i1[0, 0].tolist()
    assert res.i2[0, 0].tolist() == base.i2[0, 0].tolist()
    assert np.abs(res.y[..., :] - base.y[..., pv]).max() < 1e-13
    assert res.tau[0, 0] == pytest.approx(base.tau[0, 0], rel=1e-14)


def test_rows_beyond_the_sequence_are_invisible():
    c = rand_case(42, B=2, H=2, H_kv=2, S=30, d_h=8, S_max=40)
    c["seq"] = np.array([30, 17], dtype=np.int32)
    base = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=8, dtype=F16)
    Kp, Vp = c["Kc"].copy(), c["Vc"].copy()
    Kp[0, :, 30:] = 0x7BFF; Vp[0, :, 30:] = 0x7BFF        # 65504.0 in binary16
    Kp[1, :, 17:] = 0x7E00; Vp[1, :, 17:] = 0xFBFF        # NaN / -65504
    res = O.sparq_decode(Kp, Vp, c["qc"], c["seq"], r=3, k=8, dtype=F16)
    assert np.array_equal(res.i2, base.i2) and np.array_equal(res.y, base.y)
    assert np.array_equal(O.dense_decode(Kp, Vp, c["qc"], c["seq"], dtype=F16),
                          O.dense_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], dtype=F16))


def test_single_row_and_k_larger_than_s():
    c = rand_case(43, S=1, d_h=8, S_max=4)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=2, k=16, dtype=F16)
    assert res.i2[0, 0].tolist() == [0] and abs(res.alpha[0, 0] - 1) < 1e-15
    assert np.abs(res.y[0, 0] - c["V"][0, 0, 0]).max() < 1e-15


def test_given_positions_reproduce_the_default_path_and_differ_otherwise():
    c = rand_case(44, B=1, H=2, H_kv=1, S=40, d_h=8, v_shift=1.0)
    base = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=6, dtype=F16)
    again = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=6, dtype=F16, given_i2=base.i2)
    assert np.array_equal(again.y, base.y) and np.array_equal(again.alpha, base.alpha)
    other = base.i2.copy(); other[0, 0, 0] = [p for p in range(40) if p not in base.i2[0, 0]][0]
    moved = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=6, dtype=F16, given_i2=other)
    assert moved.alpha[0, 0] < base.alpha[0, 0]           # any other set has less approximate mass
    assert np.array_equal(moved.y[0, 1], base.y[0, 1])


# ---------------------------------------------------------------- grouped-query attention

def test_independent_heads_over_a_shared_kv_head():
    """Default GQA reading: each query head runs the single-head algorithm on its KV head."""
    c = rand_case(51, B=2, H=6, H_kv=2, S=32, d_h=8, v_shift=0.4)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=3, k=5, dtype=F16)
    Kx = np.repeat(c["Kc"], 3, axis=1); Vx = np.repeat(c["Vc"], 3, axis=1)
    flat = O.sparq_decode(Kx, Vx, c["qc"], c["seq"], r=3, k=5, dtype=F16)
    for name in ("y", "alpha", "tau", "i1", "i2"):
        assert np.array_equal(getattr(res, name), getattr(flat, name)), name


def test_shared_rule_with_identical_heads_is_the_independent_rule():
    """Section 4 'Grouped query attention' sums |q| and s-hat over the g heads of a group before the two
    selections.  If the g heads carry the same query, both sums are g times one head's values: the order of
    the channels and of the positions is that of the single head, so everything must equal the independent
    rule's result for that head, bit for bit (tau and alpha never see the sums)."""
    c = rand_case(52, B=2, H=2, H_kv=2, S=36, d_h=8, v_shift=0.4)
    r, k, g = 3, 7, 4
    qg = np.repeat(c["qc"], g, axis=1)                       # [B, H_kv * g, d_h]: every group holds one query g times
    single = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16)
    shared = O.sparq_decode(c["Kc"], c["Vc"], qg, c["seq"], r=r, k=k, dtype=F16, flags=O.GQA_SHARED)
    indep = O.sparq_decode(c["Kc"], c["Vc"], qg, c["seq"], r=r, k=k, dtype=F16)
    for name in ("i1", "i2", "tau", "alpha", "y"):
        want = np.repeat(getattr(single, name), g, axis=1)
        assert np.array_equal(getattr(indep, name), want), name
        assert np.array_equal(getattr(shared, name), want), name


def test_shared_rule_against_brute_force_and_with_one_head_per_group():
    """The grouped rule against the list-and-fsum brute force on tiny random groups (heads that disagree
    about channels and positions), and H = H_kv, where it is the single-head rule."""
    for seed in range(6):
        c = rand_case(520 + seed, B=1, H=4, H_kv=1, S=30 + seed, d_h=8, v_shift=0.4)
        r, k = 2 + seed % 3, 5 + seed
        res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16, flags=O.GQA_SHARED)
        S = int(c["seq"][0])
        bf = BF.sparq_group([c["q"][0, h].tolist() for h in range(4)], c["K"][0, 0, :S].tolist(), c["V"][0, 0, :S].tolist(), r, k)
        for h in range(4):
            assert res.i1[0, h].tolist() == bf["i1"] and res.i2[0, h, :min(k, S)].tolist() == bf["i2"]
            assert abs(res.tau[0, h] - bf["tau"][h]) < 1e-13 and abs(res.alpha[0, h] - bf["alpha"][h]) < 1e-13
            assert np.abs(res.y[0, h] - np.array(bf["y"][h])).max() < 1e-12
        # the heads of these groups do not agree with each other: the shared sets are not what each head alone picks
        alone = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16)
        assert any(alone.i2[0, h].tolist() != res.i2[0, h].tolist() for h in range(4)) or seed > 0
    c1 = rand_case(53, B=1, H=2, H_kv=2, S=20, d_h=8)
    a = O.sparq_decode(c1["Kc"], c1["Vc"], c1["qc"], c1["seq"], r=2, k=4, dtype=F16)
    b = O.sparq_decode(c1["Kc"], c1["Vc"], c1["qc"], c1["seq"], r=2, k=4, dtype=F16, flags=O.GQA_SHARED)
    assert np.array_equal(a.i2, b.i2) and np.abs(a.y - b.y).max() < 1e-14


def test_shared_group_head_without_mass_on_the_groups_channels():
    """A head that is zero on every channel the group selects has all-zero approximate logits:
    uniform s-hat (1/S each) whatever tau is, so its alpha is k/S, and the group's positions are
    decided by the other heads alone."""
    c = rand_case(54, B=1, H=2, H_kv=1, S=24, d_h=8, v_shift=0.3)
    q = c["q"].copy()
    q[0, 1] = 0.0; q[0, 0, 6] = 0.0; q[0, 1, 6] = 1e-3       # channel 6 carries the smallest group sum
    qc, _ = codes_from_floats(q, F16)
    res = O.sparq_decode(c["Kc"], c["Vc"], qc, c["seq"], r=3, k=6, dtype=F16, flags=O.GQA_SHARED, want_z=True)
    assert 6 not in res.i1[0, 0].tolist()
    assert np.all(res.z[0, 1, :24] == 0.0) and np.isfinite(res.tau[0, 1])
    assert res.alpha[0, 1] == pytest.approx(6 / 24, rel=1e-14)
    assert res.i2[0, 1].tolist() == np.sort(np.argsort(-res.z[0, 0, :24], kind="stable")[:6]).tolist()


# ---------------------------------------------------------------- ablation switches

@pytest.mark.parametrize("flag,mode", [(O.TAU_SQRT_DH, "sqrt_dh"), (O.TAU_SQRT_R, "sqrt_r")])
def test_fixed_temperatures_of_the_ablation(flag, mode):
    """Section 5.3 'Approximate softmax temperature': tau = sqrt(d_h) and tau = sqrt(r).  The logits
    scale by tau_l1 / tau against the default run, the position set is the same (one head: a positive
    rescaling keeps the order), and the brute force agrees."""
    c = rand_case(71, S=40, d_h=16, v_shift=0.5)
    r, k = 4, 9
    base = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16, want_z=True)
    res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16, flags=flag, want_z=True)
    fixed = math.sqrt(16) if mode == "sqrt_dh" else math.sqrt(r)
    assert res.tau[0, 0] == pytest.approx(fixed, rel=1e-15)
    assert np.allclose(res.z[0, 0] * fixed, base.z[0, 0] * base.tau[0, 0], rtol=1e-13, atol=1e-13)
    assert np.array_equal(res.i2, base.i2) and np.array_equal(res.i1, base.i1)
    bf = BF.sparq(c["q"][0, 0].tolist(), c["K"][0, 0].tolist(), c["V"][0, 0].tolist(), r, k, tau_mode=mode)
    assert res.alpha[0, 0] == pytest.approx(bf["alpha"], rel=1e-12)
    assert np.abs(res.y[0, 0] - np.array(bf["y"])).max() < 1e-12
    # a hotter softmax (larger tau) spreads the mass: alpha of the same set shrinks with tau
    if mode == "sqrt_dh":
        assert res.alpha[0, 0] <= base.alpha[0, 0] + 1e-15
    with pytest.raises(ValueError):
        O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=r, k=k, dtype=F16, flags=O.TAU_SQRT_DH | O.TAU_SQRT_R)


def test_local_window_keeps_the_most_recent_positions():
    """Experimental-setup table, 'Local window l': the l most recent positions are always selected and
    the other k - l come from the scores of the older ones.  l = 0 is the plain rule, l >= k keeps the
    last k positions only, and r = d_h turns alpha into the exact mass of the kept set."""
    c = rand_case(72, S=30, d_h=8, v_shift=0.5)
    r, k = 3, 8
    q, K, V = c["q"][0, 0], c["K"][0, 0], c["V"][0, 0]
    args = dict(r=r, k=k, dtype=F16)
    plain = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], **args)
    assert np.array_equal(O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], local_window=0, **args).i2, plain.i2)
    for l in (1, 3, 8, 20):
        res = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], local_window=l, want_z=True, **args)
        n_local = min(l, k)
        i2 = res.i2[0, 0].tolist()
        assert i2[k - n_local:] == list(range(30 - n_local, 30)) and len(set(i2)) == k and i2 == sorted(i2)
        older = np.sort(np.argsort(-res.z[0, 0, :30 - n_local], kind="stable")[:k - n_local]).tolist()
        assert i2[:k - n_local] == older
        bf = BF.sparq(q.tolist(), K.tolist(), V.tolist(), r, k, local_window=l)
        assert i2 == bf["i2"] and res.alpha[0, 0] == pytest.approx(bf["alpha"], rel=1e-12)
        assert np.abs(res.y[0, 0] - np.array(bf["y"])).max() < 1e-12
    full = O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=8, k=k, dtype=F16, local_window=5)
    s = scipy_softmax(K @ q / math.sqrt(8))
    assert full.alpha[0, 0] == pytest.approx(s[full.i2[0, 0]].sum(), rel=1e-12)
    # grouped-query rule: the window is shared like the rest of the list
    cg = rand_case(73, H=2, H_kv=1, S=30, d_h=8)
    rg = O.sparq_decode(cg["Kc"], cg["Vc"], cg["qc"], cg["seq"], r=3, k=8, dtype=F16, flags=O.GQA_SHARED, local_window=3)
    assert np.array_equal(rg.i2[0, 0], rg.i2[0, 1]) and rg.i2[0, 0, -3:].tolist() == [27, 28, 29]


# ---------------------------------------------------------------- cache maintenance

def test_kv_append_definition():
    rng = np.random.default_rng(61)
    B, H_kv, S_max, d_h = 2, 2, 8, 4
    K = np.zeros((B, H_kv, S_max, d_h), dtype=np.uint16); Kt = np.zeros((B, H_kv, d_h, S_max), dtype=np.uint16)
    V = np.zeros_like(K); seq = np.array([0, 0], dtype=np.int32)
    rows_v = []
    for step in range(8):
        kc, _ = codes_from_floats(rng.normal(size=(B, H_kv, d_h)), F16)
        vc, vr = codes_from_floats(rng.normal(size=(B, H_kv, d_h)), F16)
        rows_v.append(vr)
        K, Kt, V, vbar, seq = O.kv_append(K, Kt, V, seq, kc, vc, dtype=F16)
        assert seq.tolist() == [step + 1] * 2
        assert np.array_equal(Kt, np.swapaxes(K, -1, -2))
        assert np.array_equal(K[:, :, step], kc) and np.array_equal(V[:, :, step], vc)
        assert np.abs(vbar - np.mean(rows_v, axis=0)).max() < 1e-15
    # a full sequence is left untouched
    K2, Kt2, V2, _, seq2 = O.kv_append(K, Kt, V, seq, kc, vc, dtype=F16)
    assert np.array_equal(K2, K) and seq2.tolist() == [8, 8]


def test_invalid_arguments_are_rejected():
    c = rand_case(71, S=8, d_h=4)
    with pytest.raises(ValueError):
        O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=5, k=2, dtype=F16)
    with pytest.raises(ValueError):
        O.sparq_decode(c["Kc"], c["Vc"], c["qc"], c["seq"], r=2, k=0, dtype=F16)
    with pytest.raises(ValueError):
        O.sparq_decode(c["Kc"], c["Vc"], c["qc"], [9], r=2, k=2, dtype=F16)
