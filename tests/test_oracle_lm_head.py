"""Pins for oracle O7 (O1 on logits defined as hidden . weight^T, the target's output projection): a library matrix
product in fp64 followed by the separately pinned O1, and closed forms that need no implementation at all."""
import numpy as np
import pytest

import oracle
from paper_2602_00523_amd import workloads as wl


def _wide(a):
    return wl.bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,dim,vocab,k", [(3, 64, 500, 1), (5, 96, 1000, 7), (1, 16, 40, 40)])
def test_equals_library_matmul_then_o1(dtype, rows, dim, vocab, k):
    h = wl.gaussian(1, (rows, dim), dtype, 0.5)
    w = wl.gaussian(2, (vocab, dim), dtype, 0.5)
    got = oracle.lm_head_topk(h, w, k, return_logits=True)
    logits = _wide(h) @ _wide(w).T                             # numpy/BLAS, fp64
    np.testing.assert_allclose(got["logits"], logits, rtol=1e-12, atol=1e-12)
    # O1 takes stored logits; feed it the fp64 products rounded to fp32 only where that cannot change the order
    x = logits.astype(np.float32)
    srt = np.sort(logits, axis=1)
    gaps_ok = (np.diff(srt, axis=1).min() > 1e-5)              # fp32 rounding (~1e-7 relative) cannot reorder these
    ref = oracle.entropy_topk(x, k)
    np.testing.assert_allclose(got["entropy"], ref["entropy"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(got["topk_entropy"], ref["topk_entropy"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(got["topk_prob"], ref["topk_prob"], rtol=1e-5, atol=1e-9)
    if gaps_ok:
        np.testing.assert_array_equal(got["topk_idx"], ref["topk_idx"])
    order = np.argsort(-logits, axis=1, kind="stable")[:, :k]   # independent statement of the order
    np.testing.assert_array_equal(got["topk_idx"], order)


def test_closed_forms():
    rows, dim, vocab = 2, 8, 50
    h = np.ones((rows, dim), np.float32)
    # every weight row equal -> uniform logits -> H = ln V, argmax = index 0 (ties to the lowest index)
    w = np.full((vocab, dim), 0.25, np.float32)
    o = oracle.lm_head_topk(h, w, 1)
    np.testing.assert_allclose(o["entropy"], np.log(vocab), rtol=1e-12)
    assert (o["topk_idx"][:, 0] == 0).all() and (o["alpha"] == 1.0).all()
    # one weight row far above the others -> H = 0 and that row wins
    w2 = np.zeros((vocab, dim), np.float32)
    w2[17] = 200.0
    o = oracle.lm_head_topk(h, w2, 1)
    np.testing.assert_allclose(o["entropy"], 0.0, atol=1e-12)
    assert (o["topk_idx"][:, 0] == 17).all()
    # a one-hot hidden row reads out one column of the weight matrix as its logits
    g = np.random.default_rng(0)
    w3 = g.standard_normal((vocab, dim)).astype(np.float32)
    e = np.zeros((1, dim), np.float32)
    e[0, 3] = 1.0
    o = oracle.lm_head_topk(e, w3, 5, return_logits=True)
    np.testing.assert_array_equal(o["logits"][0], w3[:, 3].astype(np.float64))
    assert o["topk_idx"][0, 0] == int(np.argmax(w3[:, 3]))


def test_row_groups_and_strides():
    g = np.random.default_rng(3)
    hfull = g.standard_normal((8, 40)).astype(np.float32)
    wfull = g.standard_normal((30, 40)).astype(np.float32)
    h, w = hfull[:, :32], wfull[:, :32]                         # row strides larger than the row length
    a = oracle.lm_head_topk(h, w, 2, n_valid=[3, 1], rows_per_group=4)
    b = oracle.lm_head_topk(np.ascontiguousarray(h), np.ascontiguousarray(w), 2)
    valid = [0, 1, 2, 4]
    np.testing.assert_array_equal(a["topk_idx"][valid], b["topk_idx"][valid])
    np.testing.assert_allclose(a["entropy"][valid], b["entropy"][valid], rtol=1e-14)
    skipped = [3, 5, 6, 7]
    assert np.isnan(a["entropy"][skipped]).all() and (a["topk_idx"][skipped] == -1).all()
