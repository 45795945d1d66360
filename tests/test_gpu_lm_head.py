"""GPU parity of sage_lm_head_topk (greedy token and softmax statistics straight from the output projection) against
oracle O7.  The kernel accumulates 16-bit x 16-bit products in fp32 (each product is exact, the sum is rounded), the
oracle in fp64, so the greedy token is compared as a decision under that rounding: it must be the oracle's token, or a
token whose fp64 logit is within the accumulation error of the oracle's maximum (several results are then correct)."""
import numpy as np
import pytest

import oracle
from paper_2602_00523_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_utils
    return gpu_utils


def check(gu, h, w, n_valid=None, rpg=1, rows_checked=None):
    rows = h.shape[0]
    g = gu.gpu_lm_head_topk(h, w, 1, n_valid, rpg)
    valid = np.ones(rows, bool) if n_valid is None else np.array([(r % rpg) < n_valid[r // rpg] for r in range(rows)])
    sel = np.flatnonzero(valid) if rows_checked is None else np.array(rows_checked)
    if len(sel) == 0:
        assert (g["topk_idx"] == -1).all() and np.isnan(g["entropy"]).all()
        return 0, 0
    o = oracle.lm_head_topk(np.ascontiguousarray(h[sel]), w, 1, return_logits=True)
    # fp32 accumulation of dim exact products: |error| <= dim * 2^-24 * sum|terms| is the worst case; a tenth of
    # that, relative to the row's logit scale, is already far above anything observed
    scale = np.abs(o["logits"]).max(axis=1)
    tol = 1e-5 * np.sqrt(h.shape[1]) * np.maximum(scale, 1.0)
    for j, r in enumerate(sel):
        gi, oi = int(g["topk_idx"][r, 0]), int(o["topk_idx"][j, 0])
        assert 0 <= gi < w.shape[0]
        assert gi == oi or o["logits"][j, gi] >= o["logits"][j, oi] - tol[j], (r, gi, oi)
        assert abs(g["entropy"][r] - o["entropy"][j]) <= 1e-3 * max(1.0, o["entropy"][j]), r
        assert g["alpha"][r] == 1.0 and g["topk_entropy"][r] == 0.0
    assert (g["topk_idx"][~valid] == -1).all() and np.isnan(g["entropy"][~valid]).all()
    exact = sum(int(g["topk_idx"][r, 0]) == int(o["topk_idx"][j, 0]) for j, r in enumerate(sel))
    return exact, len(sel)


@pytest.mark.parametrize("rows,dim,vocab", [(5, 256, 1000), (64, 512, 4096), (33, 128, 64), (70, 128, 700), (1, 1024, 130),
                                            (4, 384, 81920), (3, 384, 81900), (3, 128, 152064), (2, 640, 100003 * 1 + 5)])
def test_small_shapes(gu, rows, dim, vocab):
    h = wl.gaussian(rows, (rows, dim), "bf16", 1.0)
    w = wl.gaussian(vocab, (vocab, dim), "bf16", 3.0 / np.sqrt(dim))
    exact, n = check(gu, h, w)
    assert exact >= n - 1                                       # near-ties are rare on Gaussian logits


def test_row_groups_and_padded_strides(gu):
    g = np.random.default_rng(4)
    hfull = wl.gaussian(1, (128, 264), "bf16", 1.0)
    wfull = wl.gaussian(2, (900, 264), "bf16", 0.2)
    h, w = hfull[:, :256], wfull[:, :256]                       # row strides longer than the rows (still 16-byte aligned)
    import torch
    from paper_2602_00523_amd import sage
    hd, wd = gu.to_dev(hfull)[:, :256], gu.to_dev(wfull)[:, :256]
    rows, vocab = 128, 900
    out_idx = torch.full((rows, 1), -1, device="cuda:0", dtype=torch.int32)
    ent = torch.full((rows,), float("nan"), device="cuda:0")
    ws = torch.empty(sage.sage_lm_head_topk_workspace_bytes(rows, vocab, 1), device="cuda:0", dtype=torch.uint8)
    nv = gu.to_dev(np.array([10, 64], np.int32))
    sage.sage_lm_head_topk(hd, wd, 1, ent, out_idx, None, None, None, None, ws, nv, 64)
    torch.cuda.synchronize()
    o = oracle.lm_head_topk(h, w, 1, n_valid=[10, 64], rows_per_group=64)
    valid = np.array([r < 10 or r >= 64 for r in range(rows)])
    gi = out_idx.cpu().numpy()[:, 0]
    assert (gi[valid] == o["topk_idx"][valid, 0]).mean() > 0.97
    np.testing.assert_allclose(ent.cpu().numpy()[valid], o["entropy"][valid], rtol=1e-3, atol=1e-3)
    assert (gi[~valid] == -1).all()


@pytest.mark.parametrize("rows,rpg,n_valid", [
    (320, 64, [10, 0, 64, 3, 40]),            # live rows of several trees packed into two blocks of 64
    (200, 48, [48, 1, 0, 48, 5]),             # groups that are not the block size; the last group is short (8 rows)
    (512, 64, [64] * 8),                      # eight full blocks through one pass over the weights
    (130, 1, [1, 0] * 65),                    # one row per group
    (192, 64, [0, 0, 0]),                     # nothing live at all
    (600, 2, [2] * 300)])                     # more groups than threads in a workgroup
def test_more_rows_than_one_block(gu, rows, rpg, n_valid):
    """Rows beyond 64 go through the same pass over the weights; dead rows are packed away first.  The result of a
    row must not depend on which block and slot it lands in."""
    dim, vocab = 256, 2100
    h = wl.gaussian(rows, (rows, dim), "bf16", 1.0)
    w = wl.gaussian(vocab + 1, (vocab, dim), "bf16", 3.0 / np.sqrt(dim))
    n_valid = list(n_valid)
    if rows == 200:
        n_valid[4] = 30                        # asks for more rows than the short last group has: all 8 are live
    exact, n = check(gu, h, w, np.minimum(n_valid, [min(rpg, rows - g * rpg) for g in range(len(n_valid))]), rpg)
    assert exact >= n - 2
    if n:
        live = [r for r in range(rows) if (r % rpg) < n_valid[r // rpg]]
        alone = gu.gpu_lm_head_topk(np.ascontiguousarray(h[live[-1]:live[-1] + 1]), w, 1)
        packed = gu.gpu_lm_head_topk(h, w, 1, np.asarray(n_valid, np.int32), rpg)
        assert packed["topk_idx"][live[-1], 0] == alone["topk_idx"][0, 0]
        assert packed["entropy"][live[-1]] == alone["entropy"][0]


def test_planted_winner_and_ties(gu):
    """One vocabulary row is the hidden row itself scaled up: it must win; two identical weight rows tie exactly
    (same products, same order of accumulation), and the lower index must be reported."""
    dim, vocab = 256, 3000
    h = wl.gaussian(5, (4, dim), "bf16", 1.0)
    w = wl.gaussian(6, (vocab, dim), "bf16", 0.05)
    w[2500] = h[1]
    w[77] = h[2]
    w[1999] = h[2]
    g = gu.gpu_lm_head_topk(h, w, 1)
    assert g["topk_idx"][1, 0] == 2500
    assert g["topk_idx"][2, 0] == 77


@pytest.mark.parametrize("rows,n_valid,sampled", [(64, [50], (3, 40, 49)),
                                                  (512, [64, 9, 30, 64, 0, 17, 64, 41], (3, 64 + 8, 3 * 64 + 63, 7 * 64 + 40))])
def test_full_size_72b_projection_sampled_rows(gu, rows, n_valid, sampled):
    """The 72B output projection (hidden 8192, vocabulary 152064), the node rows of one tree and of a batch of eight, in
    the launch shapes bench.py times; the oracle recomputes a few of the rows over the whole vocabulary."""
    import torch
    from paper_2602_00523_amd import sage
    dim, vocab = 8192, 152064
    g = torch.Generator(device="cuda:0")
    g.manual_seed(wl.seed_for("c2", 0, 7))
    W = (torch.randn(vocab, dim, generator=g, device="cuda:0", dtype=torch.float32) * (3.0 / np.sqrt(dim))).to(torch.bfloat16)
    H = torch.randn(rows, dim, generator=g, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    ent = torch.full((rows,), float("nan"), device="cuda:0")
    idx = torch.full((rows, 1), -1, device="cuda:0", dtype=torch.int32)
    ws = torch.empty(sage.sage_lm_head_topk_workspace_bytes(rows, vocab, 1), device="cuda:0", dtype=torch.uint8)
    nv = torch.tensor(n_valid, device="cuda:0", dtype=torch.int32)     # only the first n_valid rows of each tree are live
    sage.sage_lm_head_topk(H, W, 1, ent, idx, None, None, None, None, ws, nv, 64)
    torch.cuda.synchronize()
    gi, ge = idx.cpu().numpy()[:, 0], ent.cpu().numpy()
    dead = np.array([(r % 64) >= n_valid[r // 64] for r in range(rows)])
    assert (gi[dead] == -1).all() and np.isnan(ge[dead]).all() and (gi[~dead] >= 0).all()
    ref = (H.float() @ W.float().T).argmax(1).cpu().numpy()            # a library matmul in fp32: agreement, not parity
    assert (gi[~dead] == ref[~dead]).mean() > 0.98
    w_np = gu.to_host(W)
    for r in sampled:
        o = oracle.lm_head_topk(gu.to_host(H[r:r + 1]), w_np, 1, return_logits=True)
        oi = int(o["topk_idx"][0, 0])
        tol = 1e-5 * np.sqrt(dim) * max(1.0, float(np.abs(o["logits"]).max()))
        assert gi[r] == oi or o["logits"][0, gi[r]] >= o["logits"][0, oi] - tol, (r, gi[r], oi)
        assert abs(ge[r] - o["entropy"][0]) <= 1e-3 * max(1.0, o["entropy"][0])


@pytest.mark.parametrize("rows,dim,vocab,k", [(5, 256, 1000, 10), (64, 512, 4096, 16), (1, 1024, 130, 8), (33, 128, 70, 16),
                                              (3, 128, 152064, 10), (16, 3584, 152064, 10), (2, 384, 81900, 2)])
def test_candidate_lists_of_a_draft_row(gu, rows, dim, vocab, k):
    """1 < k <= 16 (the draft side of Sec. 3.1): the k best tokens per row and Eq. 7-9 on them.  The order of two logits
    that differ by less than the fp32 accumulation error is not decidable, so position j must hold a token whose fp64
    logit equals the oracle's j-th largest within that error; the probabilities follow to 1e-3."""
    h = wl.gaussian(rows + k, (rows, dim), "bf16", 1.0)
    w = wl.gaussian(vocab + k, (vocab, dim), "bf16", 3.0 / np.sqrt(dim))
    g = gu.gpu_lm_head_topk(h, w, k)
    o = oracle.lm_head_topk(h, w, k, return_logits=True)
    exact = 0
    for r in range(rows):
        gi = g["topk_idx"][r]
        assert len(set(gi.tolist())) == k and gi.min() >= 0 and gi.max() < vocab
        tol = 1e-5 * np.sqrt(dim) * max(1.0, float(np.abs(o["logits"][r]).max()))
        want = np.sort(o["logits"][r])[::-1][:k]
        assert np.abs(o["logits"][r, gi] - want).max() <= tol, r
        exact += int((gi == o["topk_idx"][r]).all())
        for key in ("topk_prob", "topk_renorm"):
            np.testing.assert_allclose(np.sort(g[key][r])[::-1], np.sort(o[key][r])[::-1], rtol=2e-3, atol=1e-6, err_msg=key)
        for key in ("entropy", "topk_entropy", "alpha"):
            assert abs(g[key][r] - o[key][r]) <= 2e-3 * max(1.0, abs(o[key][r])), (key, r)
    assert exact >= rows - max(1, rows // 8)                    # near-ties among the k best are rare on Gaussian logits


def test_candidate_lists_with_exact_ties(gu):
    """Identical weight rows give identical logits (same products, same order of accumulation): the lower index comes
    first, across tiles and units alike."""
    dim, vocab, k = 256, 3000, 6
    h = wl.gaussian(15, (3, dim), "bf16", 1.0)
    w = wl.gaussian(16, (vocab, dim), "bf16", 0.02)
    for v in (2900, 70, 1500, 71):                             # four copies of the hidden row 1 scaled up: the four best
        w[v] = h[1]
    g = gu.gpu_lm_head_topk(h, w, k)
    assert g["topk_idx"][1, :4].tolist() == [70, 71, 1500, 2900]
    o = oracle.lm_head_topk(h, w, k)
    np.testing.assert_array_equal(g["topk_idx"][1, :4], o["topk_idx"][1, :4])


def test_candidate_lists_with_row_groups(gu):
    """k > 1 together with n_valid: the live rows are packed into the block, dead rows stay untouched, and a row's list
    does not depend on which slot it lands in."""
    rows, rpg, dim, vocab, k = 40, 8, 256, 5000, 4
    n_valid = np.array([3, 0, 8, 1, 5], np.int32)
    h = wl.gaussian(77, (rows, dim), "bf16", 1.0)
    w = wl.gaussian(78, (vocab, dim), "bf16", 3.0 / np.sqrt(dim))
    g = gu.gpu_lm_head_topk(h, w, k, n_valid, rpg)
    alone = gu.gpu_lm_head_topk(h, w, k)
    o = oracle.lm_head_topk(h, w, k, n_valid=n_valid, rows_per_group=rpg, return_logits=True)
    for r in range(rows):
        if (r % rpg) < n_valid[r // rpg]:
            np.testing.assert_array_equal(g["topk_idx"][r], alone["topk_idx"][r])
            np.testing.assert_array_equal(g["topk_renorm"][r], alone["topk_renorm"][r])
            tol = 1e-5 * np.sqrt(dim) * max(1.0, float(np.abs(o["logits"][r]).max()))
            want = np.sort(o["logits"][r])[::-1][:k]
            assert np.abs(o["logits"][r, g["topk_idx"][r]] - want).max() <= tol
            assert abs(g["alpha"][r] - o["alpha"][r]) <= 2e-3
        else:
            assert (g["topk_idx"][r] == -1).all() and np.isnan(g["entropy"][r])
