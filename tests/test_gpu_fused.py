"""GPU parity of the calls that fold the second top-k pass into its consumer (sage_entropy_topk_slices +
sage_build_tree_from_slices / sage_verify_accept_from_slices): bit-identical to the separate calls on the same
inputs, and equal to the CPU oracle by the same rules as those (integers exact, floats to 1e-5)."""
import numpy as np
import pytest

import oracle
from helpers import MAX_NODES, pad_tree, random_parents
from paper_2602_00523_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_utils
    from paper_2602_00523_amd import sage
    print("\n[lib]", sage.sage_build_info(), flush=True)
    return gpu_utils


def same_bits(a, b, name):
    assert a.dtype == b.dtype and a.shape == b.shape, name
    assert (a.view(np.uint8) == b.view(np.uint8)).all(), name


@pytest.mark.parametrize("vocab,k,dtype,prm", [
    (152064, 10, "bf16", wl.CONFIGS["c2"]["tree"]),
    (152064, 16, "bf16", wl.CONFIGS["c3"]["tree"]),
    (4100, 8, "f32", wl.CONFIGS["toy"]["tree"]),
    (300000, 20, "bf16", dict(d_min=2, d_max=12, w_min=2, w_max=20, k=20, n_max=64)),    # more than 256 slices per row
    (1000, 1, "f32", dict(d_min=1, d_max=4, w_min=1, w_max=1, k=1, n_max=8)),
])
def test_plan_from_slices_equals_separate_calls_and_oracle(gu, vocab, k, dtype, prm):
    B = 9
    scales = np.array([0.2, 0.5, 1.0, 2.0, 3.0, 4.5, 6.0, 9.0, 30.0], np.float32)
    z = wl.rng(vocab * 3 + k).standard_normal((B, vocab), dtype=np.float32) * scales[:, None]
    z[4, 17] = z[4, 18] = z[4].max() + 1.0                                # an exact tie for the best token
    x = wl.to_storage(z, dtype)
    d_max_seq = np.array([prm["d_max"], prm["d_min"], 31, 0, 5, 7, 3, 9, 4], np.int32)
    for dms in (None, d_max_seq):
        a1, a2 = gu.gpu_plan_from_slices(x, k, prm, dms)
        s1 = gu.gpu_entropy_topk(x, k)
        s2 = gu.gpu_build_tree(s1["topk_renorm"], s1["alpha"], prm, s1["topk_idx"], dms)
        for key in s1:
            same_bits(a1[key], s1[key], key)
        n = s2["n_nodes"]
        same_bits(a2["n_nodes"], n, "n_nodes")
        for key in ("parent", "depth", "rank", "anc_mask", "cum_prob", "node_token"):
            for b in range(B):
                same_bits(a2[key][b, :n[b]], s2[key][b, :n[b]], f"{key}[{b}]")
                assert (a2[key][b, n[b]:] == (0 if key == "anc_mask" else -2)).all() or key == "cum_prob", key
        # the oracle on the same logits (a1) and on the GPU's own probabilities (a2, so that rounding cannot flip a tree)
        o1 = oracle.entropy_topk(x, k)
        np.testing.assert_array_equal(a1["topk_idx"], o1["topk_idx"])
        for key in ("entropy", "topk_prob", "topk_renorm", "topk_entropy", "alpha"):
            assert (np.abs(a1[key] - o1[key]) <= 1e-5 * np.maximum(np.abs(o1[key]), 1.0)).all(), key
        o2 = oracle.build_tree(a1["topk_renorm"], a1["alpha"], prm, a1["topk_idx"], dms)
        np.testing.assert_array_equal(a2["n_nodes"], o2["n_nodes"])
        for key in ("parent", "depth", "rank", "anc_mask", "node_token"):
            for b in range(B):
                np.testing.assert_array_equal(a2[key][b, :n[b]], o2[key][b, :n[b]], err_msg=f"{key}[{b}]")


@pytest.mark.parametrize("vocab,dtype,B", [(152064, "bf16", 4), (5000, "f32", 7), (300000, "bf16", 2)])
def test_accept_from_slices_equals_separate_calls_and_oracle(gu, vocab, dtype, B):
    g = wl.rng(vocab + B)
    rows = B * MAX_NODES
    parent = np.full((B, MAX_NODES), -7, np.int32)
    depth = np.full((B, MAX_NODES), -7, np.int32)
    mask = np.zeros((B, MAX_NODES), np.uint64)
    nn = np.zeros(B, np.int32)
    pars = []
    for b in range(B):
        n = (64, 1, 13, 33, 2, 50, 17)[b % 7]
        par = random_parents(g, n, chain_bias=0.6)
        p, d, m, _ = pad_tree(par)
        parent[b], depth[b], mask[b], nn[b] = p[0], d[0], m[0], n
        pars.append(par)
    z = g.standard_normal((rows, vocab), dtype=np.float32) * 3.0
    x = wl.to_storage(z, dtype)
    # the target's greedy token per live row, from the oracle; draft tokens match it along most edges
    o1 = oracle.entropy_topk(x, 1, nn, MAX_NODES)
    tgt = o1["topk_idx"][:, 0].reshape(B, MAX_NODES)
    tok = g.integers(0, vocab, (B, MAX_NODES)).astype(np.int32)
    for b in range(B):
        n = int(nn[b])
        for v in range(1, n):
            if g.random() < 0.8:
                tok[b, v] = tgt[b, pars[b][v]]
    cap = 40
    f = gu.gpu_accept_from_slices(x, tok, parent, depth, mask, nn, cap)
    s1 = gu.gpu_entropy_topk(x, 1, nn, MAX_NODES)
    s4 = gu.gpu_verify_accept(tok, s1["topk_idx"][:, 0].reshape(B, MAX_NODES), parent, depth, mask, nn, cap)
    live = (np.arange(MAX_NODES)[None, :] < nn[:, None]).reshape(-1)
    same_bits(f["target_argmax"][live], s1["topk_idx"][live, 0], "target_argmax")
    same_bits(f["entropy"][live], s1["entropy"][live], "entropy")
    assert (f["target_argmax"][~live] == -1).all() and np.isnan(f["entropy"][~live]).all()      # skipped rows untouched
    for key in ("accept_len", "best_node", "path_nodes", "out_tokens"):
        same_bits(f[key], s4[key], key)
    np.testing.assert_array_equal(f["target_argmax"][live], o1["topk_idx"][live, 0])
    assert (np.abs(f["entropy"][live] - o1["entropy"][live]) <= 1e-5 * np.maximum(np.abs(o1["entropy"][live]), 1.0)).all()
    o4 = oracle.verify_accept(tok, tgt, parent, depth, nn, cap)
    for key in ("accept_len", "best_node", "path_nodes", "out_tokens"):
        np.testing.assert_array_equal(f[key], o4[key], err_msg=key)
    assert o4["accept_len"].max() >= 3


@pytest.mark.parametrize("name,dtype,B,Hq,Hkv,d,lens,sizes,vocab,k,ldtype,prm", [
    # the benchmark's shape: one sequence, planning in the slab past the attention's 32 slots
    ("c2", "bf16", 1, 64, 8, 128, [4096], [13], 152064, 10, "bf16", wl.CONFIGS["c2"]["tree"]),
    # a ragged batch: ranges of one tile list, planning workgroups of all sequences in one slab
    ("batch", "bf16", 5, 64, 8, 128, [700, 0, 3000, 64, 1500], [8, 64, 1, 30, 47], 152064, 16, "bf16", wl.CONFIGS["c3"]["tree"]),
    # more sequences than KV heads: several planning slabs, the last one partly empty
    ("slabs", "bf16", 11, 28, 4, 128, [300] * 11, [5] * 11, 4100, 8, "f32", wl.CONFIGS["toy"]["tree"]),
    # more sequences than the batched decomposition takes: one launch slot per sequence
    ("many", "bf16", 70, 8, 2, 128, [90] * 70, [3] * 70, 2000, 4, "f32", dict(d_min=1, d_max=5, w_min=1, w_max=4, k=4, n_max=20)),
    # candidate lists too long for the planning workgroup: two launches, same results
    ("long", "bf16", 2, 64, 8, 128, [500, 200], [20, 9], 300000, 20, "bf16", dict(d_min=2, d_max=12, w_min=2, w_max=20, k=20, n_max=64)),
    # fp32 attention: two launches, same results
    ("toy", "f32", 2, 4, 1, 64, [256, 100], [16, 7], 1024, 8, "f32", wl.CONFIGS["toy"]["tree"]),
])
def test_attention_with_plan_equals_separate_calls_and_oracle(gu, name, dtype, B, Hq, Hkv, d, lens, sizes, vocab, k, ldtype, prm):
    """sage_tree_attention_with_plan against sage_tree_attention and sage_build_tree_from_slices on the same inputs (every
    output bit for bit) and against the oracle (attention to the tolerance of its dtype, top-k indices and tree exact)."""
    from test_gpu_parity import TOL, tree_batch
    g = wl.rng(len(name) * 1000 + B)
    inp = wl.attention_inputs(4000 + B, B, Hq, Hkv, d, lens, dtype, pad_tokens=2)
    mask, nn = tree_batch(g, B, sizes)
    scales = g.uniform(0.3, 9.0, size=(B, 1)).astype(np.float32)
    x = wl.to_storage(g.standard_normal((B, vocab), dtype=np.float32) * scales, ldtype)
    dms = g.integers(prm["d_min"], prm["d_max"] + 1, size=B).astype(np.int32)
    for d_max_seq in (None, dms):
        O, a1, a2 = gu.gpu_attention_with_plan(inp, mask, nn, Hq, Hkv, d, x, k, prm, d_max_seq)
        _, raw = gu.gpu_tree_attention(inp, mask, nn, Hq, Hkv, d)
        same_bits(O, gu.to_host(raw), "O")
        s1, s2 = gu.gpu_plan_from_slices(x, k, prm, d_max_seq)
        for key in s1:
            same_bits(a1[key], s1[key], key)
        for key in s2:
            same_bits(a2[key], s2[key], key)
        ref = oracle.tree_attention(inp["Q"], inp["Kc"], inp["Vc"], inp["Kt"], inp["Vt"], inp["kv_start"], inp["kv_len"],
                                    inp["kv_token_stride"], inp["kv_head_stride"], mask, nn, Hq, Hkv, d)
        gu.assert_attention_close(gu.widen(O), ref, nn, TOL[dtype])
        o1 = oracle.entropy_topk(x, k)
        np.testing.assert_array_equal(a1["topk_idx"], o1["topk_idx"])
        assert (np.abs(a1["alpha"] - o1["alpha"]) <= 1e-5).all()
        o2 = oracle.build_tree(a1["topk_renorm"], a1["alpha"], prm, a1["topk_idx"], d_max_seq)
        np.testing.assert_array_equal(a2["n_nodes"], o2["n_nodes"])
        for key in ("parent", "depth", "rank", "anc_mask", "node_token"):
            for b in range(B):
                n = int(o2["n_nodes"][b])
                np.testing.assert_array_equal(a2[key][b, :n], o2[key][b, :n], err_msg=f"{key}[{b}]")


@pytest.mark.parametrize("dtype,vocab,B,k", [("bf16", 152064, 1, 16), ("bf16", 152064, 8, 10), ("bf16", 5000, 3, 40),
                                             ("f32", 1024, 2, 8), ("bf16", 1032, 70, 2)])
def test_slices_pair_equals_the_two_separate_passes(gu, dtype, vocab, B, k):
    """sage_entropy_topk_slices_pair leaves both workspaces exactly as the two separate first passes do (same kernels'
    code, one launch), whatever the mix of live rows."""
    import torch
    from paper_2602_00523_amd import sage
    g = wl.rng(9100 + B)
    target = wl.draft_logits(9200 + B, B * MAX_NODES, vocab, dtype, 2.0)
    draft = wl.draft_logits(9300 + B, B, vocab, dtype, 3.0)
    n_nodes = g.integers(0, MAX_NODES + 1, size=B).astype(np.int32)
    n_nodes[0] = MAX_NODES
    T, Dr, nv = gu.to_dev(target), gu.to_dev(draft), gu.to_dev(n_nodes)
    size_a = sage.sage_entropy_topk_workspace_bytes(B * MAX_NODES, vocab, 1)
    size_b = sage.sage_entropy_topk_workspace_bytes(B, vocab, k)
    ws = [torch.zeros(n, device=gu.DEV, dtype=torch.uint8) for n in (size_a, size_b, size_a, size_b)]
    sage.sage_entropy_topk_slices(T, 1, ws[0], nv, MAX_NODES)
    sage.sage_entropy_topk_slices(Dr, k, ws[1])
    sage.sage_entropy_topk_slices_pair(T, nv, MAX_NODES, ws[2], Dr, k, ws[3])
    torch.cuda.synchronize()
    assert torch.equal(ws[0], ws[2]) and torch.equal(ws[1], ws[3])
    assert ws[0].any() and ws[1].any()
    # no live target row at all
    zero = gu.to_dev(np.zeros(B, np.int32))
    for w in ws[2:]:
        w.zero_()
    sage.sage_entropy_topk_slices_pair(T, zero, MAX_NODES, ws[2], Dr, k, ws[3])
    torch.cuda.synchronize()
    assert not ws[2].any() and torch.equal(ws[1], ws[3])
