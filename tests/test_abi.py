"""Host-side checks of the boundary: the built library loads without a GPU and exports every function that
include/sage.h declares; argument validation returns status codes without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_00523_amd", "libsage_hip.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2602_00523_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sage_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_calls():
    names = declared_functions()
    for need in ("sage_entropy_topk", "sage_build_tree", "sage_tree_attention", "sage_verify_accept",
                 "sage_commit_path", "sage_advance_kv_len", "sage_update_history"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name
    lib.sage_build_info.restype = ctypes.c_char_p
    assert b"gfx950" in lib.sage_build_info()


def test_workspace_sizes_are_pure_host_functions(lib):
    lib.sage_entropy_topk_workspace_bytes.restype = ctypes.c_size_t
    lib.sage_tree_attention_workspace_bytes.restype = ctypes.c_size_t
    a = lib.sage_entropy_topk_workspace_bytes(64, 152064, 1)
    b = lib.sage_entropy_topk_workspace_bytes(64, 152064, 10)
    assert 0 < a < b < (1 << 24)
    w1 = lib.sage_tree_attention_workspace_bytes(1, 1, 64, 8, 128, 4096)
    w2 = lib.sage_tree_attention_workspace_bytes(1, 1, 64, 8, 128, 32768)
    assert 0 < w1 <= w2 < (1 << 28)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    INVALID = 1
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(16)            # never dereferenced: validation fails first
    assert lib.sage_verify_accept(null, one, one, one, one, one, 1, 9, one, one, one, one, null) == INVALID
    assert lib.sage_verify_accept(one, one, one, one, one, one, 1, 0, one, one, one, one, null) == INVALID

    class P(ctypes.Structure):
        _fields_ = [(n, ctypes.c_int) for n in ("d_min", "d_max", "w_min", "w_max", "k", "n_max")]
    bad = [P(3, 8, 2, 10, 10, 65), P(3, 8, 2, 11, 10, 64), P(9, 8, 2, 10, 10, 64), P(3, 40, 2, 10, 10, 64),
           P(3, 8, 0, 10, 10, 64), P(3, 8, 2, 10, 9, 64)]
    for p in bad:
        assert lib.sage_build_tree(one, one, null, 1, 10, ctypes.byref(p), null, one, one, one, one, one, null, null, null) == INVALID
    ok = P(3, 8, 2, 10, 10, 64)
    assert lib.sage_build_tree(one, one, null, 1, 10, ctypes.byref(ok), null, one, one, one, one, one, null, one, null) == INVALID
    assert lib.sage_build_tree(one, one, null, 0, 10, ctypes.byref(ok), null, one, one, one, one, one, null, null, null) == 0

    lib.sage_entropy_topk.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_long,
                                      ctypes.c_int, ctypes.c_void_p, ctypes.c_int] + [ctypes.c_void_p] * 7 + \
                                     [ctypes.c_size_t, ctypes.c_void_p]
    args = lambda **kw: [kw.get("logits", 256), kw.get("dtype", 1), kw.get("rows", 1), kw.get("vocab", 1024),
                         kw.get("stride", 1024), kw.get("k", 10), None, 1, 256, kw.get("idx", 256), 256, 256, 256, 256,
                         kw.get("ws", 256), kw.get("wsb", 1 << 20), None]
    assert lib.sage_entropy_topk(*args(k=0)) == INVALID
    assert lib.sage_entropy_topk(*args(k=65)) == INVALID
    assert lib.sage_entropy_topk(*args(idx=None)) == INVALID
    assert lib.sage_entropy_topk(*args(stride=1001)) == INVALID            # rows must stay 16-byte aligned
    assert lib.sage_entropy_topk(*args(dtype=7)) == INVALID
    assert lib.sage_entropy_topk(*args(wsb=8)) == 3                        # WORKSPACE_TOO_SMALL
    assert lib.sage_entropy_topk(*args(rows=0)) == 0

    lib.sage_tree_attention.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int] * 5 + [ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int, ctypes.c_long, ctypes.c_long, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    att = lambda **kw: [256] * 6 + [kw.get("dtype", 1), kw.get("B", 1), kw.get("Hq", 64), kw.get("Hkv", 8), kw.get("d", 128),
                                    256, 256, kw.get("L", 4096), kw.get("ts", 1024), 128, 256, 256, None, kw.get("scale", 0.088),
                                    kw.get("ws", 256), kw.get("wsb", 1 << 30), None]
    assert lib.sage_tree_attention(*att(Hq=63)) == INVALID
    assert lib.sage_tree_attention(*att(scale=0.0)) == INVALID
    assert lib.sage_tree_attention(*att(d=96)) == 2                        # UNSUPPORTED head_dim on the bf16 path
    assert lib.sage_tree_attention(*att(Hq=136, Hkv=8)) == 2               # group size 17
    assert lib.sage_tree_attention(*att(ts=1004)) == INVALID               # token rows must stay 16-byte aligned
    assert lib.sage_tree_attention(*att(wsb=1024)) == 3
    assert lib.sage_tree_attention(*att(B=0)) == 0
    assert lib.sage_tree_attention(*att(ts=(1 << 24) + 8)) == 2            # 64 token rows must fit 32-bit byte offsets

    lib.sage_commit_path.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                    ctypes.c_long, ctypes.c_long, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    com = lambda **kw: [kw.get("kt", 256), 256, 256, 256, kw.get("dtype", 1), kw.get("B", 1), 8, kw.get("d", 128), 256, 256,
                        kw.get("cap", 4096), kw.get("ts", 1024), 128, 256, 256, kw.get("pc", 9), None]
    assert lib.sage_commit_path(*com(kt=None)) == INVALID
    assert lib.sage_commit_path(*com(dtype=5)) == INVALID
    assert lib.sage_commit_path(*com(d=4)) == INVALID                      # a head row must be whole 16-byte pieces
    assert lib.sage_commit_path(*com(ts=1004)) == INVALID
    assert lib.sage_commit_path(*com(pc=0)) == INVALID
    assert lib.sage_commit_path(*com(pc=65)) == 2
    assert lib.sage_commit_path(*com(B=0)) == 0
    lib.sage_lm_head_topk.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_long, ctypes.c_long, ctypes.c_int,
                                     ctypes.c_void_p, ctypes.c_int] + [ctypes.c_void_p] * 7 + [ctypes.c_size_t, ctypes.c_void_p]
    lm = lambda **kw: [256, kw.get("w", 256), kw.get("dtype", 1), kw.get("rows", 64), kw.get("dim", 8192), kw.get("vocab", 152064),
                       kw.get("hs", 8192), 8192, kw.get("k", 1), None, 1, 256, kw.get("idx", 256), None, None, 256, 256, 256,
                       kw.get("wsb", 1 << 24), None]
    assert lib.sage_lm_head_topk(*lm(w=None)) == INVALID
    assert lib.sage_lm_head_topk(*lm(idx=None)) == INVALID
    assert lib.sage_lm_head_topk(*lm(hs=100)) == INVALID                   # row stride shorter than a row
    assert lib.sage_lm_head_topk(*lm(hs=8196)) == INVALID                  # rows must stay 16-byte aligned
    assert lib.sage_lm_head_topk(*lm(k=17)) == 2                           # candidate lists of up to 16
    assert lib.sage_lm_head_topk(*lm(k=2, rows=65)) == 2                   # ... and only for up to 64 rows
    assert lib.sage_lm_head_topk(*lm(k=65)) == INVALID
    assert lib.sage_lm_head_topk(*lm(dtype=0)) == 2
    assert lib.sage_lm_head_topk(*lm(dim=8100)) == 2                          # hidden size must be whole 128-element chunks
    assert lib.sage_lm_head_topk(*lm(wsb=64)) == 3
    assert lib.sage_lm_head_topk(*lm(rows=0)) == 0
    lib.sage_lm_head_topk_workspace_bytes.restype = ctypes.c_size_t
    assert 0 < lib.sage_lm_head_topk_workspace_bytes(64, 152064, 1) < (1 << 22)
    lib.sage_advance_kv_len.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert lib.sage_advance_kv_len(None, 256, 1, 10, None) == INVALID
    assert lib.sage_advance_kv_len(256, 256, 0, 10, None) == 0
    lib.sage_update_history.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_float, ctypes.c_int,
                                       ctypes.c_int] + [ctypes.c_void_p] * 5
    his = lambda **kw: [256, kw.get("B", 1), kw.get("w", 10), kw.get("lo", 2.0), kw.get("hi", 3.0), kw.get("df", 3),
                        kw.get("dc", 8), kw.get("hist", 256), 256, 256, None, None]
    assert lib.sage_update_history(*his(w=0)) == INVALID
    assert lib.sage_update_history(*his(w=65)) == INVALID
    assert lib.sage_update_history(*his(lo=4.0)) == INVALID
    assert lib.sage_update_history(*his(df=9)) == INVALID
    assert lib.sage_update_history(*his(dc=32)) == INVALID
    assert lib.sage_update_history(*his(hist=None)) == INVALID
    assert lib.sage_update_history(*his(B=0)) == 0


def test_fused_calls_validate_on_the_host(lib):
    INVALID, UNSUPPORTED, TOO_SMALL = 1, 2, 3
    vp, ci, cl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_size_t
    null, one = vp(0), vp(4096)          # never dereferenced: validation fails first, or B == 0 returns early

    class P(ctypes.Structure):
        _fields_ = [(n, ci) for n in ("d_min", "d_max", "w_min", "w_max", "k", "n_max")]

    lib.sage_entropy_topk_slices.argtypes = [vp, ci, ci, ci, cl, ci, vp, ci, vp, sz, vp]
    sl = lambda logits=one, dtype=1, rows=1, vocab=1024, stride=1024, k=4, ws=one, wsb=1 << 20: \
        lib.sage_entropy_topk_slices(logits, dtype, rows, vocab, stride, k, null, 1, ws, wsb, null)
    assert sl(logits=null) == INVALID and sl(ws=null) == INVALID and sl(dtype=7) == INVALID
    assert sl(k=0) == INVALID and sl(k=65) == INVALID and sl(stride=1000) == INVALID
    assert sl(wsb=16) == TOO_SMALL
    assert sl(vocab=2_000_000, stride=2_000_000) == UNSUPPORTED
    assert sl(rows=0) == 0

    lib.sage_build_tree_from_slices.argtypes = [vp, ci, ci, ci, ctypes.POINTER(P)] + [vp] * 15
    good = P(3, 8, 2, 10, 10, 64)
    bt = lambda slices=one, vocab=152064, B=0, k=10, prm=good, idx=one, nn=one: lib.sage_build_tree_from_slices(
        slices, vocab, B, k, ctypes.byref(prm), null, one, idx, one, one, one, one, nn, one, one, one, one, null, null, null)
    assert bt() == 0
    assert bt(slices=null) == INVALID and bt(idx=null) == INVALID and bt(nn=null) == INVALID
    assert bt(k=9) == INVALID and bt(B=-1) == INVALID and bt(vocab=0) == INVALID
    assert bt(prm=P(3, 40, 2, 10, 10, 64)) == INVALID and bt(prm=P(3, 8, 2, 10, 10, 65)) == INVALID
    assert bt(slices=vp(4100)) == INVALID
    assert bt(vocab=2_000_000) == UNSUPPORTED

    lib.sage_verify_accept_from_slices.argtypes = [vp, ci, vp, vp, vp, vp, vp, ci, ci] + [vp] * 7
    va = lambda slices=one, vocab=152064, tok=one, B=0, cap=9, tgt=one: lib.sage_verify_accept_from_slices(
        slices, vocab, tok, one, one, one, one, B, cap, null, tgt, one, one, one, one, null)
    assert va() == 0
    assert va(slices=null) == INVALID and va(tok=null) == INVALID and va(tgt=null) == INVALID
    assert va(cap=0) == INVALID and va(B=-1) == INVALID and va(vocab=0) == INVALID
    assert va(B=2000) == UNSUPPORTED and va(vocab=2_000_000) == UNSUPPORTED


def test_close_step_validates_on_the_host(lib):
    INVALID, UNSUPPORTED = 1, 2
    vp, ci, cl, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float
    null, one = vp(0), vp(16)
    lib.sage_close_step.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp, ci, cl, cl, vp, vp, ci, ci, cf, cf, ci, ci, vp, vp, vp,
                                    vp, vp, vp]
    cs = lambda Kt=one, dtype=1, B=0, Hkv=8, d=128, lens=one, ts=1024, hs=128, cap=9, window=10, lo=2.0, hi=3.0, floor=3, top=8, \
                hist=one, dm_in=one, dm_out=one: lib.sage_close_step(Kt, one, one, one, dtype, B, Hkv, d, one, lens, 4096, ts, hs,
                                                                    one, one, cap, window, lo, hi, floor, top, hist, one, dm_in,
                                                                    dm_out, null, null)
    assert cs() == 0
    assert cs(Kt=null) == INVALID and cs(lens=null) == INVALID and cs(hist=null) == INVALID
    assert cs(dm_in=null) == INVALID and cs(dm_out=null) == INVALID
    assert cs(dtype=4) == INVALID and cs(B=-1) == INVALID and cs(d=0) == INVALID and cs(cap=0) == INVALID
    assert cs(ts=100) == INVALID and cs(hs=3) == INVALID and cs(d=60, ts=480, hs=60) == INVALID       # 120-byte rows
    assert cs(window=0) == INVALID and cs(window=65) == INVALID and cs(lo=4.0) == INVALID
    assert cs(floor=0) == INVALID and cs(floor=9) == INVALID and cs(top=40) == INVALID
    assert cs(B=70000) == UNSUPPORTED and cs(cap=65) == UNSUPPORTED


def test_accept_close_validates_on_the_host(lib):
    INVALID, UNSUPPORTED = 1, 2
    vp, ci, cl, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float
    null, one = vp(0), vp(16)
    lib.sage_verify_accept_close_from_slices.argtypes = ([vp, ci, vp, vp, vp, vp, vp, ci, ci] + [vp] * 6 +
                                                         [vp, vp, vp, vp, ci, ci, ci, vp, vp, ci, cl, cl, ci, cf, cf, ci, ci] +
                                                         [vp] * 6)
    ac = lambda slices=one, vocab=152064, tok=one, B=0, cap=9, tgt=one, Kt=one, dtype=1, d=128, lens=one, ts=1024, hs=128, \
                window=10, lo=2.0, floor=3, top=8, dm=one: lib.sage_verify_accept_close_from_slices(
        slices, vocab, tok, one, one, one, one, B, cap, null, tgt, one, one, one, one, Kt, one, one, one, dtype, 8, d, one, lens,
        4096, ts, hs, window, lo, 3.0, floor, top, one, one, dm, one, null, null)
    assert ac() == 0
    assert ac(slices=null) == INVALID and ac(tok=null) == INVALID and ac(tgt=null) == INVALID
    assert ac(Kt=null) == INVALID and ac(lens=null) == INVALID and ac(dm=null) == INVALID
    assert ac(cap=0) == INVALID and ac(B=-1) == INVALID and ac(vocab=0) == INVALID and ac(dtype=9) == INVALID
    assert ac(ts=100) == INVALID and ac(d=60, ts=480, hs=60) == INVALID
    assert ac(window=0) == INVALID and ac(lo=4.0) == INVALID and ac(floor=0) == INVALID and ac(top=40) == INVALID
    assert ac(B=2000) == UNSUPPORTED and ac(cap=65) == UNSUPPORTED and ac(vocab=2_000_000) == UNSUPPORTED


def test_attention_with_plan_validates_on_the_host(lib):
    """Both halves' checks run before anything is enqueued; B = 0 is a valid no-op."""
    INVALID, UNSUPPORTED = 1, 2
    vp, ci, cl, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float, ctypes.c_size_t
    null, one, two = vp(0), vp(16), vp(32)

    class P(ctypes.Structure):
        _fields_ = [(n, ctypes.c_int) for n in ("d_min", "d_max", "w_min", "w_max", "k", "n_max")]
    lib.sage_tree_attention_with_plan.argtypes = ([vp] * 6 + [ci] * 5 + [vp, vp, ci, cl, cl, vp, vp, cf, vp, sz] +
                                                  [vp, ci, ci, ctypes.POINTER(P)] + [vp] * 15)

    def call(Q=one, dtype=1, B=0, Hq=64, Hkv=8, d=128, lens=one, ts=1024, hs=128, mask=one, nn=one, scale=0.088, ws=one,
             slices=one, vocab=152064, k=10, prm=(3, 8, 2, 10, 10, 64), idx=one, next_nn=two, next_mask=two, next_par=two):
        return lib.sage_tree_attention_with_plan(Q, one, one, one, one, one, dtype, B, Hq, Hkv, d, one, lens, 4096, ts, hs, mask,
                                                 nn, scale, ws, 1 << 20, slices, vocab, k, ctypes.byref(P(*prm)), null, null, idx,
                                                 null, null, null, null, next_nn, next_par, two, two, next_mask, null, null, null)
    assert call() == 0
    assert call(Q=null) == INVALID and call(lens=null) == INVALID and call(mask=null) == INVALID and call(nn=null) == INVALID
    assert call(Hq=60) == INVALID and call(scale=0.0) == INVALID and call(dtype=7) == INVALID and call(hs=3) == INVALID
    assert call(slices=null) == INVALID and call(idx=null) == INVALID and call(next_par=null) == INVALID
    assert call(k=9) == INVALID and call(prm=(3, 40, 2, 10, 10, 64)) == INVALID and call(prm=(3, 8, 2, 10, 10, 65)) == INVALID
    assert call(next_nn=one) == INVALID and call(next_mask=one) == INVALID      # the planned tree aliases the verified one
    assert call(ws=null) == INVALID and call(ws=null, dtype=0) == 0             # fp32 needs no workspace
    assert call(vocab=2_000_000) == UNSUPPORTED and call(B=70000) == UNSUPPORTED
