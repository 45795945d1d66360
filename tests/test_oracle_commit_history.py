"""Pins for oracle O5 (commit of the accepted path into the KV cache; Alg. 1 Phase 3, Sec. 2.2) and O6 (adaptive
history tracking; Sec. 3.3, window and thresholds of Sec. 5 "Implementation details").

O5 is pinned through O3, an independent function: after the commit, a lone root query over the extended cache must
see exactly what the deepest accepted node saw through the tree mask before the commit (cache + its ancestors + itself).
O6 is pinned by depth sequences worked out by hand for constant and step-change acceptance lengths, and by recomputing
the moving average from the full history instead of a ring.
"""
import json
import os

import numpy as np
import pytest

import oracle
from helpers import MAX_NODES, depth_by_walk, mask_by_walk, pad_tree, random_parents
from paper_2602_00523_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_hyperparameters.json")


def _path_of(par, node):
    p = []
    while node >= 0:
        p.append(int(node))
        node = par[node]
    return p[::-1]


def _setup(seed, B, Hq, Hkv, d, lens, cap, dtype):
    inp = wl.attention_inputs(wl.seed_for("toy", seed), B, Hq, Hkv, d, lens, dtype, pad_tokens=0)
    # give every sequence room for cap tokens: rebuild a cache with capacity slots per sequence
    ts, hs = inp["kv_token_stride"], inp["kv_head_stride"]
    Kc = np.zeros((B * cap, Hkv, d), inp["Kc"].dtype)
    Vc = np.zeros_like(Kc)
    start = np.arange(B, dtype=np.int64) * cap
    for b in range(B):
        s0 = int(inp["kv_start"][b])
        Kc[start[b]:start[b] + lens[b]] = inp["Kc"][s0:s0 + lens[b]]
        Vc[start[b]:start[b] + lens[b]] = inp["Vc"][s0:s0 + lens[b]]
    return inp, Kc, Vc, start, ts, hs


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-12), ("bf16", 1e-12)])
@pytest.mark.parametrize("seed", range(6))
def test_commit_then_plain_decode_equals_tree_attention_of_the_accepted_node(seed, dtype, tol):
    g = np.random.default_rng(100 + seed)
    B, Hq, Hkv, d, cap = 2, 4, 2, 16, 64
    lens = [int(g.integers(1, 20)), int(g.integers(1, 20))]
    inp, Kc, Vc, start, ts, hs = _setup(seed, B, Hq, Hkv, d, lens, cap, dtype)
    n = int(g.integers(2, 14))
    par = random_parents(g, n, chain_bias=0.4)
    parent, depth, mask, nn = pad_tree(par, B)
    best = [int(g.integers(0, n)) for _ in range(B)]          # any node can be the deepest accepted one
    path_cap = 16
    path_nodes = np.full((B, path_cap), -1, np.int32)
    accept_len = np.zeros(B, np.int32)
    for b in range(B):
        p = _path_of(par, best[b])
        path_nodes[b, :len(p)] = p
        accept_len[b] = len(p) - 1
    # what the accepted node saw before the commit
    O_tree = oracle.tree_attention(inp["Q"], Kc, Vc, inp["Kt"], inp["Vt"], start, lens, ts, hs, mask, nn, Hq, Hkv, d)
    Kc2, Vc2 = Kc.copy(), Vc.copy()
    oracle.commit_path(inp["Kt"], inp["Vt"], Kc2, Vc2, start, lens, cap, ts, hs, path_nodes, accept_len, Hkv, d)
    new_len = oracle.advance_kv_len(lens, accept_len, cap)
    assert list(new_len) == [lens[b] + accept_len[b] + 1 for b in range(B)]
    # a lone query (the accepted node's Q as node 0) over the extended cache.  Its own key is already in the cache
    # now, so the tree part must contribute nothing: give the lone node a key that can never win (score -> -inf is
    # not expressible; instead compare against the definition written out below).
    for b in range(B):
        q = wl.bf16_bits_to_f32(inp["Q"][b, best[b]]).astype(np.float64) if dtype == "bf16" else inp["Q"][b, best[b]].astype(np.float64)
        wide = (lambda a: wl.bf16_bits_to_f32(a).astype(np.float64)) if dtype == "bf16" else (lambda a: a.astype(np.float64))
        K = wide(Kc2[start[b]:start[b] + new_len[b]])          # [L', Hkv, d]
        V = wide(Vc2[start[b]:start[b] + new_len[b]])
        for h in range(Hq):
            gk = h // (Hq // Hkv)
            s = K[:, gk, :] @ q[h] / np.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            ref = p @ V[:, gk, :]
            np.testing.assert_allclose(O_tree[b, best[b], h], ref, rtol=1e-9, atol=tol)


def test_commit_places_rows_in_path_order_and_touches_nothing_else():
    g = np.random.default_rng(5)
    B, Hq, Hkv, d, cap = 3, 2, 2, 8, 40
    lens = [7, 1, 30]
    inp, Kc, Vc, start, ts, hs = _setup(9, B, Hq, Hkv, d, lens, cap, "bf16")
    par = np.array([-1, 0, 1, 1, 0, 4, 5], np.int32)
    path_nodes = np.full((B, 8), -1, np.int32)
    accept_len = np.array([2, 0, 3], np.int32)
    path_nodes[0, :3] = [0, 1, 3]
    path_nodes[1, :1] = [0]
    path_nodes[2, :4] = [0, 4, 5, 6]
    K0, V0 = Kc.copy(), Vc.copy()
    oracle.commit_path(inp["Kt"], inp["Vt"], Kc, Vc, start, lens, cap, ts, hs, path_nodes, accept_len, Hkv, d)
    touched = np.zeros(B * cap, bool)
    for b in range(B):
        for j in range(accept_len[b] + 1):
            pos = start[b] + lens[b] + j
            touched[pos] = True
            assert (Kc[pos] == inp["Kt"][b, path_nodes[b, j]]).all()
            assert (Vc[pos] == inp["Vt"][b, path_nodes[b, j]]).all()
    assert (Kc[~touched] == K0[~touched]).all() and (Vc[~touched] == V0[~touched]).all()
    assert not (inp["Kt"][0, 1] == inp["Kt"][0, 3]).all()      # the rows differ, so the order test means something


def test_commit_respects_capacity_and_strided_head_major_layout():
    B, Hkv, d, cap = 1, 2, 8, 10
    g = np.random.default_rng(3)
    Kt = g.standard_normal((B, MAX_NODES, Hkv, d)).astype(np.float32)
    Vt = g.standard_normal((B, MAX_NODES, Hkv, d)).astype(np.float32)
    # head-major cache [Hkv, cap, d]: token stride d, head stride cap*d
    Kc = np.zeros((Hkv, cap, d), np.float32)
    Vc = np.zeros_like(Kc)
    path_nodes = np.array([[0, 2, 5, 9, -1]], np.int32)
    oracle.commit_path(Kt, Vt, Kc, Vc, [0], [8], cap, d, cap * d, path_nodes, [3], Hkv, d)
    for j, node in enumerate([0, 2]):                          # positions 8, 9 fit; 10, 11 are dropped
        for h in range(Hkv):
            assert (Kc[h, 8 + j] == Kt[0, node, h]).all() and (Vc[h, 8 + j] == Vt[0, node, h]).all()
    assert (Kc[:, :8] == 0).all()
    assert list(oracle.advance_kv_len([8], [3], cap)) == [10]  # saturates at the capacity


# ---------------------------------------------------------------------------------------------------- O6

def _run(taus, d0, window=10, lo=2.0, hi=3.0, d_floor=3, d_cap=8):
    hist = np.zeros((1, window), np.int32)
    count = np.zeros(1, np.int32)
    d_max = np.full(1, d0, np.int32)
    out, avgs = [], []
    for t in taus:
        avgs.append(float(oracle.update_history([t], hist, count, d_max, window, lo, hi, d_floor, d_cap)[0]))
        out.append(int(d_max[0]))
    return out, avgs


def test_history_uses_the_papers_window_and_thresholds():
    hp = json.load(open(GOLDEN))
    assert hp["history_window"] == 10 and hp["history_low"] == 2 and hp["history_high"] == 3


def test_constant_acceptance_lengths():
    # always above the upper threshold: one level deeper per step up to the cap
    assert _run([5] * 6, 4)[0] == [5, 6, 7, 8, 8, 8]
    # always below the lower threshold: one level shallower per step down to the floor
    assert _run([0] * 6, 6)[0] == [5, 4, 3, 3, 3, 3]
    # inside the band, and exactly on either threshold (both strict): unchanged
    assert _run([2] * 5, 5)[0] == [5] * 5
    assert _run([3] * 5, 5)[0] == [5] * 5


def test_step_change_worked_by_hand():
    # ten steps of tau = 5 fill the window (depth climbs 3 -> 8 and stays), then tau = 0:
    # after z zeros the average is 5 (10 - z) / 10 = 4.5, 4.0, 3.5, 3.0, 2.5, 2.0, 1.5, 1.0, ...
    # > 3 for z <= 3 (already at the cap), held for z = 4, 5, 6 (3.0, 2.5, 2.0), < 2 from z = 7 on.
    d, avg = _run([5] * 10 + [0] * 10, 3)
    assert d[:10] == [4, 5, 6, 7, 8, 8, 8, 8, 8, 8]
    assert d[10:] == [8, 8, 8, 8, 8, 8, 7, 6, 5, 4]
    assert avg[10:16] == [4.5, 4.0, 3.5, 3.0, 2.5, 2.0]


def test_short_history_averages_what_is_there():
    # first step: the average is the value itself; second: the mean of two
    d, avg = _run([4, 0, 0], 5)
    assert avg[:2] == [4.0, 2.0] and abs(avg[2] - 4.0 / 3.0) < 1e-6
    assert d == [6, 6, 5]


@pytest.mark.parametrize("seed", range(10))
def test_ring_equals_full_history_recomputation(seed):
    g = np.random.default_rng(seed)
    window = int(g.integers(1, 13))
    lo, hi = 2.0, 3.0
    taus = g.integers(0, 8, 60)
    d, avg = _run(list(taus), 5, window=window, d_floor=2, d_cap=9)
    cur = 5
    for t in range(60):
        last = taus[max(0, t + 1 - window):t + 1]
        a = last.sum() / len(last)
        assert abs(avg[t] - a) < 1e-6
        if a < lo:
            cur -= 1
        elif a > hi:
            cur += 1
        cur = min(max(cur, 2), 9)
        assert d[t] == cur


def test_sequences_are_independent():
    hist = np.zeros((2, 10), np.int32)
    count = np.zeros(2, np.int32)
    d_max = np.array([5, 5], np.int32)
    for _ in range(3):
        oracle.update_history([7, 0], hist, count, d_max, 10, 2.0, 3.0, 3, 8)
    assert list(d_max) == [8, 3]


def test_build_tree_per_sequence_depth_limit():
    """A one-hot candidate distribution gives a chain as deep as Eq. (10) allows; with alpha = 1 that is D_max,
    so the per-sequence limit is visible directly in the chain length."""
    k = 4
    pt = np.zeros((3, k), np.float32)
    pt[:, 0] = 1.0
    prm = dict(d_min=2, d_max=6, w_min=1, w_max=4, k=k, n_max=64)
    base = oracle.build_tree(pt, np.ones(3, np.float32), prm)
    assert list(base["n_nodes"]) == [7, 7, 7]
    lim = oracle.build_tree(pt, np.ones(3, np.float32), prm, d_max_seq=np.array([3, 6, 1], np.int32))
    assert list(lim["n_nodes"]) == [4, 7, 3]                  # 1 is clamped up to d_min = 2
