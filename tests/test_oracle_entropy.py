"""Pins for oracle O1 (softmax entropy, top-k, renormalised entropy, confidence; Sec. 3.1, Eq. 7-9).

Each test checks the oracle against something that is not the oracle: a closed
form, a library sort, or a brute-force selection written separately.
"""
import math

import numpy as np
import pytest

import oracle
from paper_2602_00523_amd import workloads as wl


def test_uniform_logits_give_ln_v_and_zero_confidence():
    for V, k in ((1024, 8), (152064, 10)):
        x = np.full((1, V), 0.37, np.float32)
        o = oracle.entropy_topk(x, k)
        assert abs(o["entropy"][0] - math.log(V)) < 1e-9
        assert list(o["topk_idx"][0]) == list(range(k))          # ties resolve to the lowest indices
        np.testing.assert_allclose(o["topk_prob"][0], 1.0 / V, rtol=1e-12)
        np.testing.assert_allclose(o["topk_renorm"][0], 1.0 / k, rtol=1e-12)
        assert abs(o["topk_entropy"][0] - math.log(k)) < 1e-12
        assert o["alpha"][0] == pytest.approx(0.0, abs=1e-12)


def test_one_hot_gives_zero_entropy_and_full_confidence():
    V, k = 1000, 10
    x = np.full((2, V), -np.inf, np.float32)
    x[0, 123] = 1.5                       # a single finite logit
    x[1, :] = 0.0
    x[1, 77] = 800.0                      # a gap so large that exp underflows to 0 in fp64
    o = oracle.entropy_topk(x, k)
    for r, hot in ((0, 123), (1, 77)):
        assert o["entropy"][r] == 0.0
        assert o["topk_idx"][r, 0] == hot
        assert o["topk_prob"][r, 0] == 1.0
        assert o["topk_entropy"][r] == 0.0
        assert o["alpha"][r] == 1.0
    # the remaining top-k slots follow the (value desc, index asc) order over the tied rest
    assert list(o["topk_idx"][0, 1:]) == list(range(9))


def test_two_equal_maxima_give_ln2():
    V = 64
    x = np.full((1, V), -np.inf, np.float32)
    x[0, 5] = x[0, 40] = 3.0
    o = oracle.entropy_topk(x, 2)
    assert abs(o["entropy"][0] - math.log(2)) < 1e-15
    assert list(o["topk_idx"][0]) == [5, 40]
    assert abs(o["topk_entropy"][0] - math.log(2)) < 1e-15
    assert o["alpha"][0] == pytest.approx(0.0, abs=1e-15)


def test_known_distribution_closed_form():
    # logits = ln p for p = (1/2, 1/4, 1/8, 1/8): H = 1.75 ln 2; top-2 renormalised = (2/3, 1/3)
    p = np.array([0.125, 0.5, 0.125, 0.25])
    x = np.log(p).astype(np.float32)[None, :]      # exact: powers of two
    o = oracle.entropy_topk(x, 2)
    assert abs(o["entropy"][0] - 1.75 * math.log(2)) < 1e-7
    assert list(o["topk_idx"][0]) == [1, 3]
    np.testing.assert_allclose(o["topk_prob"][0], [0.5, 0.25], rtol=1e-7)
    np.testing.assert_allclose(o["topk_renorm"][0], [2 / 3, 1 / 3], rtol=1e-7)
    hk = math.log(3) - (2 / 3) * math.log(2)
    assert abs(o["topk_entropy"][0] - hk) < 1e-7
    assert abs(o["alpha"][0] - (1 - hk / math.log(2))) < 1e-7
    # k = 4 takes the whole distribution: renormalisation is the identity, entropy equals the full one
    o4 = oracle.entropy_topk(x, 4)
    assert list(o4["topk_idx"][0]) == [1, 3, 0, 2]
    assert abs(o4["topk_entropy"][0] - o4["entropy"][0]) < 1e-12
    assert abs(o4["alpha"][0] - (1 - 1.75 / 2)) < 1e-7


def test_shift_invariance_and_bounds():
    g = np.random.default_rng(1)
    x = (3.0 * g.standard_normal((4, 5000))).astype(np.float32)
    a = oracle.entropy_topk(x, 10)
    # a grid of quarter-integers shifts by 64 without any rounding
    x2 = np.round(x * 4) / 4
    a2 = oracle.entropy_topk(x2.astype(np.float32), 10)
    b2 = oracle.entropy_topk((x2 + 64.0).astype(np.float32), 10)
    np.testing.assert_allclose(a2["entropy"], b2["entropy"], rtol=1e-10)
    np.testing.assert_array_equal(a2["topk_idx"], b2["topk_idx"])
    np.testing.assert_allclose(a2["topk_renorm"], b2["topk_renorm"], rtol=1e-10)
    for o in (a, a2):
        assert (o["entropy"] >= 0).all() and (o["entropy"] <= math.log(5000) + 1e-12).all()
        assert (o["topk_entropy"] >= 0).all() and (o["topk_entropy"] <= math.log(10) + 1e-12).all()
        assert (o["alpha"] >= 0).all() and (o["alpha"] <= 1).all()
        assert (np.diff(o["topk_prob"], axis=1) <= 0).all()
        np.testing.assert_allclose(o["topk_renorm"].sum(1), 1.0, rtol=1e-12)


def test_gaussian_logits_entropy_estimate():
    V = 152064
    for sigma in (1.0, 2.0):
        x = wl.gaussian(11, (1, V), "f32", sigma)
        o = oracle.entropy_topk(x, 10)
        assert abs(o["entropy"][0] - (math.log(V) - sigma * sigma / 2)) < 0.1


def test_topk_equals_library_stable_sort_with_ties():
    g = np.random.default_rng(2)
    for V, k in ((257, 16), (4096, 10), (152064, 16)):
        bits = wl.gaussian(int(g.integers(1 << 30)), (3, V), "bf16", 12.0)   # coarse bf16 grid => many ties
        x = wl.bf16_bits_to_f32(bits)
        o = oracle.entropy_topk(bits, k)
        for r in range(3):
            ref = np.argsort(-x[r].astype(np.float64), kind="stable")[:k]
            np.testing.assert_array_equal(o["topk_idx"][r], ref)
        assert len(set(x[0, o["topk_idx"][0]].tolist())) < k or V == 257    # ties really occur at scale


def test_topk_brute_force_selection_small():
    g = np.random.default_rng(3)
    for _ in range(20):
        V = int(g.integers(5, 40))
        k = int(g.integers(1, V + 1))
        x = g.integers(-3, 4, size=(1, V)).astype(np.float32)     # small alphabet => ties everywhere
        o = oracle.entropy_topk(x, k)
        chosen = []
        for _ in range(k):                                       # repeated scan for the best unchosen entry
            best = None
            for i in range(V):
                if i in chosen:
                    continue
                if best is None or x[0, i] > x[0, best]:
                    best = i
            chosen.append(best)
        assert list(o["topk_idx"][0]) == chosen
        p = np.exp(x[0].astype(np.float64))
        p /= p.sum()
        np.testing.assert_allclose(o["topk_prob"][0], p[chosen], rtol=1e-12)
        assert abs(o["entropy"][0] + (p * np.log(p)).sum()) < 1e-12


def test_k_equals_one_and_row_groups():
    g = np.random.default_rng(4)
    x = g.standard_normal((8, 300)).astype(np.float32)
    o = oracle.entropy_topk(x, 1, n_valid=np.array([3, 0]), rows_per_group=4)
    assert (o["alpha"][:3] == 1.0).all()
    np.testing.assert_array_equal(o["topk_idx"][:3, 0], x[:3].argmax(1))
    assert np.isnan(o["entropy"][3:]).all() and (o["topk_idx"][3:] == -1).all()   # skipped rows untouched


def test_bf16_rows_are_widened_exactly():
    bits = wl.gaussian(5, (2, 999), "bf16", 4.0)
    a = oracle.entropy_topk(bits, 7)
    b = oracle.entropy_topk(wl.bf16_bits_to_f32(bits), 7)
    for key in a:
        np.testing.assert_array_equal(a[key], b[key])


def test_row_stride():
    g = np.random.default_rng(6)
    big = g.standard_normal((3, 700)).astype(np.float32)
    view = big[:, :500]
    a = oracle.entropy_topk(view, 5)
    b = oracle.entropy_topk(np.ascontiguousarray(view), 5)
    for key in a:
        np.testing.assert_array_equal(a[key], b[key])
