"""ctypes front-end of the SAGE CPU oracle (oracle/sage_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package.  It shares nothing with
the HIP library; it takes numpy arrays (bf16 as uint16 bit patterns) and
returns numpy arrays, fp64 for every real-valued result of O1/O3.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sage_oracle.c")
_LIB = os.path.join(_HERE, "libsage_oracle.so")
MAX_NODES = 64
F32, BF16 = 0, 1


_LIB_SAN = os.path.join(_HERE, "libsage_oracle_san.so")
SANITIZE = os.environ.get("SAGE_ORACLE_SANITIZE", "") not in ("", "0")


def build(force: bool = False, sanitize: bool | None = None) -> str:
    """Compile the oracle with the host C compiler (no HIP, no contraction).

    With sanitize (or SAGE_ORACLE_SANITIZE=1 in the environment) the library is built with AddressSanitizer and
    UndefinedBehaviorSanitizer, any report fatal; the process that loads it must have the ASan runtime preloaded
    (tests/test_oracle_sanitized.py runs the oracle's own tests that way)."""
    sanitize = SANITIZE if sanitize is None else sanitize
    out = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
            if sanitize else ["-O2"]
        subprocess.check_call(
            ["gcc", *flags, "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
             "-o", out, _SRC, "-lm"])
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle inputs are float32 or bf16 bit patterns held as uint16")


class TreeParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("d_min", "d_max", "w_min", "w_max", "k", "n_max")]


def entropy_topk(logits: np.ndarray, k: int, n_valid: np.ndarray | None = None, rows_per_group: int = 1):
    """O1 (Sec. 3.1, Eq. 7-9).  logits [rows, V] float32 or uint16(bf16)."""
    assert logits.ndim == 2 and logits.strides[1] == logits.itemsize
    rows, vocab = logits.shape
    stride = logits.strides[0] // logits.itemsize
    out = dict(
        entropy=np.full(rows, np.nan), topk_idx=np.full((rows, k), -1, np.int32),
        topk_prob=np.full((rows, k), np.nan), topk_renorm=np.full((rows, k), np.nan),
        topk_entropy=np.full(rows, np.nan), alpha=np.full(rows, np.nan))
    if n_valid is not None:
        n_valid = np.ascontiguousarray(n_valid, np.int32)
    rc = lib().oracle_entropy_topk(
        _p(logits), _dtype_code(logits), rows, vocab, ctypes.c_long(stride), k, _p(n_valid), rows_per_group,
        _p(out["entropy"]), _p(out["topk_idx"]), _p(out["topk_prob"]), _p(out["topk_renorm"]),
        _p(out["topk_entropy"]), _p(out["alpha"]))
    if rc:
        raise ValueError(f"oracle_entropy_topk status {rc}")
    return out


def build_tree(topk_renorm: np.ndarray, alpha: np.ndarray, params: dict, topk_idx: np.ndarray | None = None,
               d_max_seq: np.ndarray | None = None):
    """O2 (Sec. 3.2, Eq. 10-12 and the membership rule).  fp32 inputs, bit-for-bit."""
    pr = np.ascontiguousarray(topk_renorm, np.float32)
    al = np.ascontiguousarray(alpha, np.float32)
    B, k = pr.shape
    tp = TreeParams(**{f: int(params[f]) for f, _ in TreeParams._fields_})
    out = dict(
        n_nodes=np.zeros(B, np.int32), parent=np.full((B, MAX_NODES), -2, np.int32),
        depth=np.full((B, MAX_NODES), -2, np.int32), rank=np.full((B, MAX_NODES), -2, np.int32),
        anc_mask=np.zeros((B, MAX_NODES), np.uint64), cum_prob=np.full((B, MAX_NODES), np.nan, np.float32),
        node_token=np.full((B, MAX_NODES), -2, np.int32))
    if topk_idx is not None:
        topk_idx = np.ascontiguousarray(topk_idx, np.int32)
    if d_max_seq is not None:
        d_max_seq = np.ascontiguousarray(d_max_seq, np.int32)
        assert d_max_seq.shape == (B,)
    rc = lib().oracle_build_tree(_p(pr), _p(al), _p(topk_idx), B, k, ctypes.byref(tp), _p(d_max_seq), _p(out["n_nodes"]),
                                 _p(out["parent"]), _p(out["depth"]), _p(out["rank"]), _p(out["anc_mask"]),
                                 _p(out["cum_prob"]), _p(out["node_token"]))
    if rc:
        raise ValueError(f"oracle_build_tree status {rc}")
    return out


def tree_attention(Q, Kc, Vc, Kt, Vt, kv_start, kv_len, kv_token_stride, kv_head_stride, anc_mask, n_nodes,
                   Hq: int, Hkv: int, d: int, scale: float | None = None):
    """O3.  Q [B,64,Hq,d]; Kt,Vt [B,64,Hkv,d]; Kc,Vc flat caches addressed by strides. Returns fp64 O."""
    B = Q.shape[0]
    code = _dtype_code(Q)
    for a in (Kc, Vc, Kt, Vt):
        assert _dtype_code(a) == code and a.flags["C_CONTIGUOUS"]
    assert Q.shape == (B, MAX_NODES, Hq, d) and Kt.shape == (B, MAX_NODES, Hkv, d) and Vt.shape == Kt.shape
    kv_start = np.ascontiguousarray(kv_start, np.int64)
    kv_len = np.ascontiguousarray(kv_len, np.int32)
    anc_mask = np.ascontiguousarray(anc_mask, np.uint64)
    n_nodes = np.ascontiguousarray(n_nodes, np.int32)
    O = np.full((B, MAX_NODES, Hq, d), np.nan)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    rc = lib().oracle_tree_attention(
        _p(Q), _p(Kc), _p(Vc), _p(Kt), _p(Vt), _p(O), code, B, Hq, Hkv, d, _p(kv_start), _p(kv_len),
        ctypes.c_long(kv_token_stride), ctypes.c_long(kv_head_stride), _p(anc_mask), _p(n_nodes),
        ctypes.c_double(scale))
    if rc:
        raise ValueError(f"oracle_tree_attention status {rc}")
    return O


def verify_accept(token, target_argmax, parent, depth, n_nodes, path_cap: int):
    """O4.  Integer arrays [B,64]; returns accept_len, best_node, path_nodes, out_tokens."""
    token = np.ascontiguousarray(token, np.int32)
    target_argmax = np.ascontiguousarray(target_argmax, np.int32)
    parent = np.ascontiguousarray(parent, np.int32)
    depth = np.ascontiguousarray(depth, np.int32)
    n_nodes = np.ascontiguousarray(n_nodes, np.int32)
    B = n_nodes.shape[0]
    out = dict(accept_len=np.zeros(B, np.int32), best_node=np.zeros(B, np.int32),
               path_nodes=np.full((B, path_cap), -1, np.int32), out_tokens=np.full((B, path_cap), -1, np.int32))
    rc = lib().oracle_verify_accept(_p(token), _p(target_argmax), _p(parent), _p(depth), _p(n_nodes), B, path_cap,
                                    _p(out["accept_len"]), _p(out["best_node"]), _p(out["path_nodes"]),
                                    _p(out["out_tokens"]))
    if rc:
        raise ValueError(f"oracle_verify_accept status {rc}")
    return out


def commit_path(Kt, Vt, Kc, Vc, kv_start, kv_len, kv_capacity: int, kv_token_stride: int, kv_head_stride: int,
                path_nodes, accept_len, Hkv: int, d: int):
    """O5 (Alg. 1 Phase 3).  Appends the K/V rows of the accepted path to the caches IN PLACE (one layer)."""
    code = _dtype_code(Kt)
    for a in (Kt, Vt, Kc, Vc):
        assert _dtype_code(a) == code and a.flags["C_CONTIGUOUS"]
    assert Kc.flags["WRITEABLE"] and Vc.flags["WRITEABLE"]
    B = Kt.shape[0]
    assert Kt.shape == (B, MAX_NODES, Hkv, d) and Vt.shape == Kt.shape
    kv_start = np.ascontiguousarray(kv_start, np.int64)
    kv_len = np.ascontiguousarray(kv_len, np.int32)
    path_nodes = np.ascontiguousarray(path_nodes, np.int32)
    accept_len = np.ascontiguousarray(accept_len, np.int32)
    rc = lib().oracle_commit_path(_p(Kt), _p(Vt), _p(Kc), _p(Vc), code, B, Hkv, d, _p(kv_start), _p(kv_len),
                                  int(kv_capacity), ctypes.c_long(kv_token_stride), ctypes.c_long(kv_head_stride),
                                  _p(path_nodes), _p(accept_len), path_nodes.shape[1])
    if rc:
        raise ValueError(f"oracle_commit_path status {rc}")


def advance_kv_len(kv_len, accept_len, kv_capacity: int):
    """O5: new sequence lengths after a commit (returns a new array)."""
    out = np.array(kv_len, np.int32, copy=True)
    accept_len = np.ascontiguousarray(accept_len, np.int32)
    rc = lib().oracle_advance_kv_len(_p(out), _p(accept_len), out.shape[0], int(kv_capacity))
    if rc:
        raise ValueError(f"oracle_advance_kv_len status {rc}")
    return out


def update_history(accept_len, hist, count, d_max, window: int, lo: float, hi: float, d_floor: int, d_cap: int):
    """O6 (Sec. 3.3 adaptive history tracking).  hist [B,window], count [B], d_max [B] are updated IN PLACE
    (int32, C-contiguous); returns the moving averages."""
    accept_len = np.ascontiguousarray(accept_len, np.int32)
    B = accept_len.shape[0]
    for a in (hist, count, d_max):
        assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    assert hist.shape == (B, window) and count.shape == (B,) and d_max.shape == (B,)
    avg = np.zeros(B, np.float32)
    rc = lib().oracle_update_history(_p(accept_len), B, window, ctypes.c_float(lo), ctypes.c_float(hi), d_floor, d_cap,
                                     _p(hist), _p(count), _p(d_max), _p(avg))
    if rc:
        raise ValueError(f"oracle_update_history status {rc}")
    return avg


def lm_head_topk(hidden: np.ndarray, weight: np.ndarray, k: int, n_valid=None, rows_per_group: int = 1,
                 return_logits: bool = False):
    """O7: O1 on logits = hidden @ weight.T evaluated in fp64 (hidden [rows, dim], weight [vocab, dim])."""
    assert hidden.ndim == 2 and weight.ndim == 2 and hidden.shape[1] == weight.shape[1]
    assert hidden.strides[1] == hidden.itemsize and weight.strides[1] == weight.itemsize
    code = _dtype_code(hidden)
    assert _dtype_code(weight) == code
    rows, dim = hidden.shape
    vocab = weight.shape[0]
    out = dict(
        entropy=np.full(rows, np.nan), topk_idx=np.full((rows, k), -1, np.int32),
        topk_prob=np.full((rows, k), np.nan), topk_renorm=np.full((rows, k), np.nan),
        topk_entropy=np.full(rows, np.nan), alpha=np.full(rows, np.nan))
    logits = np.full((rows, vocab), np.nan) if return_logits else None
    if n_valid is not None:
        n_valid = np.ascontiguousarray(n_valid, np.int32)
    rc = lib().oracle_lm_head_topk(
        _p(hidden), _p(weight), code, rows, dim, vocab, ctypes.c_long(hidden.strides[0] // hidden.itemsize),
        ctypes.c_long(weight.strides[0] // weight.itemsize), k, _p(n_valid), rows_per_group,
        _p(out["entropy"]), _p(out["topk_idx"]), _p(out["topk_prob"]), _p(out["topk_renorm"]),
        _p(out["topk_entropy"]), _p(out["alpha"]), _p(logits))
    if rc:
        raise ValueError(f"oracle_lm_head_topk status {rc}")
    if return_logits:
        out["logits"] = logits
    return out
