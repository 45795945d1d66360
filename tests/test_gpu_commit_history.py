"""GPU parity of the path commit (Alg. 1 Phase 3), of adaptive history tracking (Sec. 3.3) and of the tree rule's
per-sequence maximum depth: byte- and integer-exact against the CPU oracle, plus a closed loop of several steps in
which cache, lengths, history and trees evolve on the device and on the host side by side."""
import numpy as np
import pytest

import oracle
from helpers import MAX_NODES, pad_tree, random_parents
from paper_2602_00523_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_utils
    return gpu_utils


def _path_of(par, node):
    p = []
    while node >= 0:
        p.append(int(node))
        node = par[node]
    return p[::-1]


def _random_paths(g, B, path_cap, max_nodes=24):
    path_nodes = np.full((B, path_cap), -1, np.int32)
    accept_len = np.zeros(B, np.int32)
    for b in range(B):
        n = int(g.integers(1, max_nodes))
        par = random_parents(g, n, chain_bias=0.5)
        p = _path_of(par, int(g.integers(0, n)))[:path_cap]
        path_nodes[b, :len(p)] = p
        accept_len[b] = len(p) - 1
    return path_nodes, accept_len


@pytest.mark.parametrize("dtype,Hkv,d,layout", [("bf16", 8, 128, "thd"), ("bf16", 2, 64, "htd"), ("f32", 1, 64, "thd"),
                                                 ("f32", 4, 32, "htd")])
def test_commit_path_bytes(gu, dtype, Hkv, d, layout):
    g = np.random.default_rng(11)
    B, cap, path_cap = 5, 96, 12
    lens = np.array([0, 17, 95, 88, 40], np.int32)             # empty cache, one slot left, overflow, ordinary
    np_dt = np.float32 if dtype == "f32" else np.uint16
    Kt = wl.gaussian(1, (B, MAX_NODES, Hkv, d), dtype)
    Vt = wl.gaussian(2, (B, MAX_NODES, Hkv, d), dtype)
    if layout == "thd":                                        # [token, head, dim]
        Kc = wl.gaussian(3, (B * cap, Hkv, d), dtype)
        Vc = wl.gaussian(4, (B * cap, Hkv, d), dtype)
        ts, hs = Hkv * d, d
        start = np.arange(B, dtype=np.int64) * cap
    else:                                                      # [head, token, dim]
        Kc = wl.gaussian(3, (Hkv, B * cap, d), dtype)
        Vc = wl.gaussian(4, (Hkv, B * cap, d), dtype)
        ts, hs = d, B * cap * d
        start = np.arange(B, dtype=np.int64) * cap
    assert Kc.dtype == np_dt
    path_nodes, accept_len = _random_paths(g, B, path_cap)
    accept_len[2] = max(accept_len[2], 3)                      # make sure sequence 2 really overflows its capacity
    path_nodes[2, :4] = [0, 1, 2, 3]
    Ko, Vo = Kc.copy(), Vc.copy()
    oracle.commit_path(Kt, Vt, Ko, Vo, start, lens, cap, ts, hs, path_nodes, accept_len, Hkv, d)
    lo = oracle.advance_kv_len(lens, accept_len, cap)
    Kg, Vg, lg = gu.gpu_commit_path(Kt, Vt, Kc, Vc, start, lens, cap, ts, hs, path_nodes, accept_len)
    assert (Kg == Ko).all() and (Vg == Vo).all()
    np.testing.assert_array_equal(lg, lo)
    assert not (Ko == Kc).all()                                # something was written


def test_update_history_integers(gu):
    import torch
    g = np.random.default_rng(2)
    B, window, steps = 7, 10, 40
    hist_o = np.zeros((B, window), np.int32); cnt_o = np.zeros(B, np.int32); dm_o = np.full(B, 5, np.int32)
    hist_g = torch.zeros((B, window), device="cuda:0", dtype=torch.int32)
    cnt_g = torch.zeros(B, device="cuda:0", dtype=torch.int32)
    dm_g = torch.full((B,), 5, device="cuda:0", dtype=torch.int32)
    means = g.uniform(0.5, 5.0, B)
    for t in range(steps):
        tau = np.clip(g.poisson(means), 0, 8).astype(np.int32)
        avg_o = oracle.update_history(tau, hist_o, cnt_o, dm_o, window, 2.0, 3.0, 3, 8)
        avg_g = gu.gpu_update_history(tau, hist_g, cnt_g, dm_g, 2.0, 3.0, 3, 8)
        np.testing.assert_array_equal(dm_g.cpu().numpy(), dm_o)
        np.testing.assert_array_equal(hist_g.cpu().numpy(), hist_o)
        np.testing.assert_array_equal(cnt_g.cpu().numpy(), cnt_o)
        np.testing.assert_array_equal(avg_g, avg_o)            # same fp32 division on both sides
    assert len(set(dm_o.tolist())) > 1                          # the sequences really went different ways


@pytest.mark.parametrize("window", [1, 3, 64])
def test_update_history_other_windows(gu, window):
    import torch
    g = np.random.default_rng(window)
    B = 3
    hist_o = np.zeros((B, window), np.int32); cnt_o = np.zeros(B, np.int32); dm_o = np.full(B, 4, np.int32)
    hist_g = torch.zeros((B, window), device="cuda:0", dtype=torch.int32)
    cnt_g = torch.zeros(B, device="cuda:0", dtype=torch.int32)
    dm_g = torch.full((B,), 4, device="cuda:0", dtype=torch.int32)
    for t in range(2 * window + 5):
        tau = g.integers(0, 7, B).astype(np.int32)
        oracle.update_history(tau, hist_o, cnt_o, dm_o, window, 1.5, 3.5, 2, 12)
        gu.gpu_update_history(tau, hist_g, cnt_g, dm_g, 1.5, 3.5, 2, 12)
        np.testing.assert_array_equal(dm_g.cpu().numpy(), dm_o)


def test_build_tree_per_sequence_depth(gu):
    g = np.random.default_rng(8)
    B, k = 24, 10
    prm = dict(d_min=3, d_max=8, w_min=2, w_max=10, k=k, n_max=64)
    raw = np.sort(g.dirichlet(np.full(k, 0.4), B), axis=1)[:, ::-1].astype(np.float32)
    alpha = g.random(B).astype(np.float32)
    d_seq = g.integers(1, 12, B).astype(np.int32)              # below d_min and above d_max on purpose
    o = oracle.build_tree(raw, alpha, prm, d_max_seq=d_seq)
    t = gu.gpu_build_tree(raw, alpha, prm, d_max_seq_np=d_seq)
    np.testing.assert_array_equal(t["n_nodes"], o["n_nodes"])
    for b in range(B):
        n = o["n_nodes"][b]
        for key in ("parent", "depth", "rank", "anc_mask"):
            np.testing.assert_array_equal(t[key][b, :n], o[key][b, :n], err_msg=key)
    base = oracle.build_tree(raw, alpha, prm)
    assert (o["n_nodes"] != base["n_nodes"]).any()              # the override changed something


def test_closed_loop_steps(gu):
    """Several SAGE steps with state carried on the device: tree (with the history-adapted depth) -> attention of
    one layer -> acceptance (synthetic target tokens) -> commit -> history.  The oracle runs the same loop on the host;
    integers and bytes must agree at every step, attention within the bf16 tolerance."""
    import torch
    from paper_2602_00523_amd import sage
    g = np.random.default_rng(21)
    B, Hq, Hkv, d, cap, k = 2, 8, 2, 128, 160, 6
    prm = dict(d_min=2, d_max=5, w_min=1, w_max=5, k=k, n_max=24)
    path_cap = 8
    lens = np.array([70, 9], np.int32)
    start = np.arange(B, dtype=np.int64) * cap
    Kc = wl.gaussian(31, (B * cap, Hkv, d), "bf16"); Vc = wl.gaussian(32, (B * cap, Hkv, d), "bf16")
    ts, hs = Hkv * d, d
    hist_o = np.zeros((B, 4), np.int32); cnt_o = np.zeros(B, np.int32); dm_o = np.full(B, 4, np.int32)
    hist_g = torch.zeros((B, 4), device="cuda:0", dtype=torch.int32)
    cnt_g = torch.zeros(B, device="cuda:0", dtype=torch.int32)
    dm_g = torch.full((B,), 4, device="cuda:0", dtype=torch.int32)
    Kc_g, Vc_g, lens_g = Kc.copy(), Vc.copy(), lens.copy()
    for step in range(6):
        pt = np.sort(g.dirichlet(np.full(k, 0.6), B), axis=1)[:, ::-1].astype(np.float32)
        alpha = g.random(B).astype(np.float32)
        ids = np.stack([g.choice(1000, k, replace=False) for _ in range(B)]).astype(np.int32)
        o2 = oracle.build_tree(pt, alpha, prm, ids, d_max_seq=dm_o)
        g2 = gu.gpu_build_tree(pt, alpha, prm, ids, d_max_seq_np=dm_g.cpu().numpy())
        np.testing.assert_array_equal(g2["n_nodes"], o2["n_nodes"])
        Q = wl.gaussian(100 + step, (B, MAX_NODES, Hq, d), "bf16")
        Kt = wl.gaussian(200 + step, (B, MAX_NODES, Hkv, d), "bf16")
        Vt = wl.gaussian(300 + step, (B, MAX_NODES, Hkv, d), "bf16")
        inp = dict(Q=Q, Kc=Kc_g, Vc=Vc_g, Kt=Kt, Vt=Vt, kv_start=start, kv_len=lens_g, kv_token_stride=ts, kv_head_stride=hs)
        Og, _ = gu.gpu_tree_attention(inp, g2["anc_mask"], g2["n_nodes"], Hq, Hkv, d)
        Oo = oracle.tree_attention(Q, Kc, Vc, Kt, Vt, start, lens, ts, hs, o2["anc_mask"], o2["n_nodes"], Hq, Hkv, d)
        for b in range(B):
            n = o2["n_nodes"][b]
            err = np.linalg.norm(Og[b, :n] - Oo[b, :n], axis=-1) / np.linalg.norm(Oo[b, :n], axis=-1)
            assert err.max() < 2e-2
        # synthetic target: agrees with the draft along a random prefix of every path
        tgt = g.integers(0, 1000, (B, MAX_NODES)).astype(np.int32)
        for b in range(B):
            for v in range(1, o2["n_nodes"][b]):
                if g.random() < 0.7:
                    tgt[b, o2["parent"][b, v]] = o2["node_token"][b, v]
        o4 = oracle.verify_accept(o2["node_token"], tgt, o2["parent"], o2["depth"], o2["n_nodes"], path_cap)
        g4 = gu.gpu_verify_accept(g2["node_token"], tgt, g2["parent"], g2["depth"], g2["anc_mask"], g2["n_nodes"], path_cap)
        for key in ("accept_len", "best_node", "path_nodes", "out_tokens"):
            np.testing.assert_array_equal(g4[key], o4[key], err_msg=key)
        oracle.commit_path(Kt, Vt, Kc, Vc, start, lens, cap, ts, hs, o4["path_nodes"], o4["accept_len"], Hkv, d)
        lens = oracle.advance_kv_len(lens, o4["accept_len"], cap)
        Kc_g, Vc_g, lens_g = gu.gpu_commit_path(Kt, Vt, Kc_g, Vc_g, start, lens_g, cap, ts, hs, g4["path_nodes"], g4["accept_len"])
        assert (Kc_g == Kc).all() and (Vc_g == Vc).all()
        np.testing.assert_array_equal(lens_g, lens)
        oracle.update_history(o4["accept_len"], hist_o, cnt_o, dm_o, 4, 1.0, 2.0, 2, 5)
        gu.gpu_update_history(g4["accept_len"], hist_g, cnt_g, dm_g, 1.0, 2.0, 2, 5)
        np.testing.assert_array_equal(dm_g.cpu().numpy(), dm_o)
    assert (lens > np.array([70, 9])).all()


@pytest.mark.parametrize("dtype,Hkv,d,two_limits", [("bf16", 8, 128, True), ("f32", 2, 64, False)])
def test_close_step_equals_commit_advance_history(gu, dtype, Hkv, d, two_limits):
    """sage_close_step over several steps against the oracle's commit, advance and history applied in that order: cache
    bytes, lengths, window, counts, depth limits and averages, all exact; with two depth-limit arrays the input one is
    left alone."""
    import torch
    from paper_2602_00523_amd import sage
    g = np.random.default_rng(23)
    B, cap, path_cap, window = 6, 80, 9, 10
    lens = np.array([0, 30, 76, 71, 12, 55], np.int32)         # empty cache, room, overflow within a few steps
    Kc = wl.gaussian(3, (B * cap, Hkv, d), dtype)
    Vc = wl.gaussian(4, (B * cap, Hkv, d), dtype)
    ts, hs = Hkv * d, d
    start = np.arange(B, dtype=np.int64) * cap
    Ko, Vo = Kc.copy(), Vc.copy()
    hist_o = np.zeros((B, window), np.int32); cnt_o = np.zeros(B, np.int32); dm_o = np.full(B, 6, np.int32)
    dev = dict(Kc=gu.to_dev(Kc), Vc=gu.to_dev(Vc), start=gu.to_dev(start), lens=gu.to_dev(lens.copy()),
               hist=torch.zeros((B, window), device="cuda:0", dtype=torch.int32),
               cnt=torch.zeros(B, device="cuda:0", dtype=torch.int32),
               dm=[torch.full((B,), 6, device="cuda:0", dtype=torch.int32) for _ in range(2)],
               avg=torch.zeros(B, device="cuda:0", dtype=torch.float32))
    for t in range(7):
        Kt = wl.gaussian(100 + t, (B, MAX_NODES, Hkv, d), dtype)
        Vt = wl.gaussian(200 + t, (B, MAX_NODES, Hkv, d), dtype)
        path_nodes, accept_len = _random_paths(g, B, path_cap)
        oracle.commit_path(Kt, Vt, Ko, Vo, start, lens, cap, ts, hs, path_nodes, accept_len, Hkv, d)
        lens = oracle.advance_kv_len(lens, accept_len, cap)
        avg_o = oracle.update_history(accept_len, hist_o, cnt_o, dm_o, window, 2.0, 3.0, 3, 8)
        d_in, d_out = (dev["dm"][t % 2], dev["dm"][(t + 1) % 2]) if two_limits else (dev["dm"][0], dev["dm"][0])
        before = d_in.clone()
        sage.sage_close_step(gu.to_dev(Kt), gu.to_dev(Vt), dev["Kc"], dev["Vc"], dev["start"], dev["lens"], cap, ts, hs,
                             gu.to_dev(path_nodes), gu.to_dev(accept_len), dev["hist"], dev["cnt"], d_in, d_out, 2.0, 3.0, 3, 8,
                             dev["avg"])
        torch.cuda.synchronize()
        assert (gu.to_host(dev["Kc"]) == Ko).all() and (gu.to_host(dev["Vc"]) == Vo).all(), t
        np.testing.assert_array_equal(dev["lens"].cpu().numpy(), lens)
        np.testing.assert_array_equal(dev["hist"].cpu().numpy(), hist_o)
        np.testing.assert_array_equal(dev["cnt"].cpu().numpy(), cnt_o)
        np.testing.assert_array_equal(d_out.cpu().numpy(), dm_o)
        np.testing.assert_array_equal(dev["avg"].cpu().numpy(), avg_o)
        if two_limits:
            assert torch.equal(d_in, before)
    assert lens.max() == cap and not (Ko == Kc).all()           # a sequence ran into its capacity; rows were written


@pytest.mark.parametrize("vocab,dtype", [(152064, "bf16"), (5000, "f32"),
                                         (300000, "bf16")])        # more than 256 slices per row
def test_accept_and_close_in_one_launch(gu, vocab, dtype):
    """sage_verify_accept_close_from_slices over several steps against sage_verify_accept_from_slices + sage_close_step
    on a second copy of the state (bit for bit) and against the oracle's acceptance, commit, advance and history."""
    import torch
    from paper_2602_00523_amd import sage
    g = np.random.default_rng(31)
    B, Hkv, d, cap, path_cap, window = 3, 2, 64, 120, 24, 10
    rows = B * MAX_NODES
    lens = np.array([5, 60, 101], np.int32)
    Kc0 = wl.gaussian(3, (B * cap, Hkv, d), dtype); Vc0 = wl.gaussian(4, (B * cap, Hkv, d), dtype)
    ts, hs = Hkv * d, d
    start = np.arange(B, dtype=np.int64) * cap
    Ko, Vo = Kc0.copy(), Vc0.copy()
    hist_o = np.zeros((B, window), np.int32); cnt_o = np.zeros(B, np.int32); dm_o = np.full(B, 6, np.int32)

    def state():
        return dict(Kc=gu.to_dev(Kc0), Vc=gu.to_dev(Vc0), lens=gu.to_dev(lens.copy()),
                    hist=torch.zeros((B, window), device="cuda:0", dtype=torch.int32),
                    cnt=torch.zeros(B, device="cuda:0", dtype=torch.int32),
                    dm=torch.full((B,), 6, device="cuda:0", dtype=torch.int32),
                    avg=torch.zeros(B, device="cuda:0", dtype=torch.float32))
    one, two = state(), state()
    startd = gu.to_dev(start)
    ws = torch.empty(sage.sage_entropy_topk_workspace_bytes(rows, vocab, 1), device="cuda:0", dtype=torch.uint8)
    lens_o = lens.copy()
    for t in range(5):
        parent = np.full((B, MAX_NODES), -7, np.int32); depth = np.full((B, MAX_NODES), -7, np.int32)
        mask = np.zeros((B, MAX_NODES), np.uint64); nn = np.zeros(B, np.int32); pars = []
        for b in range(B):
            n = int(g.integers(1, path_cap))                   # fewer nodes than path slots: no path is ever cut
            par = random_parents(g, n, chain_bias=0.7)
            p, dd, m, _ = pad_tree(par)
            parent[b], depth[b], mask[b], nn[b] = p[0], dd[0], m[0], n
            pars.append(par)
        x = wl.to_storage(g.standard_normal((rows, vocab), dtype=np.float32) * 3.0, dtype)
        o1 = oracle.entropy_topk(x, 1, nn, MAX_NODES)
        tgt = o1["topk_idx"][:, 0].reshape(B, MAX_NODES)
        tok = g.integers(0, vocab, (B, MAX_NODES)).astype(np.int32)
        for b in range(B):
            for v in range(1, int(nn[b])):
                if g.random() < 0.85:
                    tok[b, v] = tgt[b, pars[b][v]]
        Kt = wl.gaussian(100 + t, (B, MAX_NODES, Hkv, d), dtype); Vt = wl.gaussian(200 + t, (B, MAX_NODES, Hkv, d), dtype)
        # oracle
        o4 = oracle.verify_accept(tok, np.where(tgt < 0, 0, tgt), parent, depth, nn, path_cap)
        oracle.commit_path(Kt, Vt, Ko, Vo, start, lens_o, cap, ts, hs, o4["path_nodes"], o4["accept_len"], Hkv, d)
        lens_o = oracle.advance_kv_len(lens_o, o4["accept_len"], cap)
        avg_o = oracle.update_history(o4["accept_len"], hist_o, cnt_o, dm_o, window, 2.0, 3.0, 3, 8)
        # device: fused on `one`, two calls on `two`
        xd = gu.to_dev(x)
        dev_in = [gu.to_dev(np.ascontiguousarray(a, np.int32)) for a in (tok, parent, depth)]
        maskd, nnd = gu.to_dev(mask), gu.to_dev(nn)
        Ktd, Vtd = gu.to_dev(Kt), gu.to_dev(Vt)
        outs = []
        for st, fused in ((one, True), (two, False)):
            out = dict(entropy=torch.full((rows,), float("nan"), device="cuda:0"),
                       tgt=torch.full((rows,), -1, device="cuda:0", dtype=torch.int32),
                       acc=torch.full((B,), -9, device="cuda:0", dtype=torch.int32),
                       best=torch.full((B,), -9, device="cuda:0", dtype=torch.int32),
                       path=torch.full((B, path_cap), -9, device="cuda:0", dtype=torch.int32),
                       toks=torch.full((B, path_cap), -9, device="cuda:0", dtype=torch.int32))
            sage.sage_entropy_topk_slices(xd, 1, ws, nnd, MAX_NODES)
            if fused:
                sage.sage_verify_accept_close_from_slices(ws, vocab, dev_in[0], dev_in[1], dev_in[2], maskd, nnd, path_cap,
                                                          out["entropy"], out["tgt"], out["acc"], out["best"], out["path"],
                                                          out["toks"], Ktd, Vtd, st["Kc"], st["Vc"], startd, st["lens"], cap, ts,
                                                          hs, st["hist"], st["cnt"], st["dm"], st["dm"], 2.0, 3.0, 3, 8, st["avg"])
            else:
                sage.sage_verify_accept_from_slices(ws, vocab, dev_in[0], dev_in[1], dev_in[2], maskd, nnd, path_cap,
                                                    out["entropy"], out["tgt"], out["acc"], out["best"], out["path"], out["toks"])
                sage.sage_close_step(Ktd, Vtd, st["Kc"], st["Vc"], startd, st["lens"], cap, ts, hs, out["path"], out["acc"],
                                     st["hist"], st["cnt"], st["dm"], st["dm"], 2.0, 3.0, 3, 8, st["avg"])
            torch.cuda.synchronize()
            outs.append(out)
        for key in outs[0]:
            a, b2 = outs[0][key], outs[1][key]
            assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                               b2.view(torch.int32) if b2.dtype == torch.float32 else b2), key
        for key in one:
            assert torch.equal(one[key].view(torch.int16) if one[key].dtype == torch.bfloat16 else one[key],
                               two[key].view(torch.int16) if two[key].dtype == torch.bfloat16 else two[key]), key
        np.testing.assert_array_equal(outs[0]["acc"].cpu().numpy(), o4["accept_len"])
        np.testing.assert_array_equal(outs[0]["path"].cpu().numpy(), o4["path_nodes"])
        assert (gu.to_host(one["Kc"]) == Ko).all() and (gu.to_host(one["Vc"]) == Vo).all()
        np.testing.assert_array_equal(one["lens"].cpu().numpy(), lens_o)
        np.testing.assert_array_equal(one["hist"].cpu().numpy(), hist_o)
        np.testing.assert_array_equal(one["dm"].cpu().numpy(), dm_o)
        np.testing.assert_array_equal(one["avg"].cpu().numpy(), avg_o)
    assert cnt_o.max() >= 3                                     # enough steps really ran
