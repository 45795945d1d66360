"""Thin ctypes binding of libsage_hip.so (include/sage.h): same names, argument marshalling only.

Tensors are torch CUDA(HIP) tensors used as device buffers; nothing here computes anything.  The library is
loaded on first use and a missing library is an error (there is no fallback path of any kind).
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SAGE_HIP_LIBRARY") or os.path.join(_HERE, "libsage_hip.so")   # the in-tree build unless told otherwise
MAX_NODES = 64
F32, BF16 = 0, 1
STATUS = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE_TOO_SMALL", 4: "LAUNCH_FAILED"}


class SageError(RuntimeError):
    def __init__(self, call: str, code: int):
        super().__init__(f"{call} -> {STATUS.get(code, code)}")
        self.code = code


class TreeParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("d_min", "d_max", "w_min", "w_max", "k", "n_max")]


_lib = None
_vp, _ci, _cl, _cf, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float, ctypes.c_size_t


def lib():
    """Load the HIP library built in-tree by paper_2602_00523_amd.build; fail loudly when it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SageError(f"{LIB_PATH} is missing: run `python -m paper_2602_00523_amd.build`", -1)
        L = ctypes.CDLL(LIB_PATH)
        L.sage_entropy_topk_workspace_bytes.restype = _sz
        L.sage_entropy_topk_workspace_bytes.argtypes = [_ci, _ci, _ci]
        L.sage_entropy_topk.restype = _ci
        L.sage_entropy_topk.argtypes = [_vp, _ci, _ci, _ci, _cl, _ci, _vp, _ci, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.sage_build_tree.restype = _ci
        L.sage_build_tree.argtypes = [_vp, _vp, _vp, _ci, _ci, ctypes.POINTER(TreeParams), _vp, _vp, _vp, _vp, _vp, _vp,
                                      _vp, _vp, _vp]
        L.sage_tree_attention_workspace_bytes.restype = _sz
        L.sage_tree_attention_workspace_bytes.argtypes = [_ci, _ci, _ci, _ci, _ci, _ci]
        L.sage_tree_attention.restype = _ci
        L.sage_tree_attention.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl,
                                          _vp, _vp, _vp, _cf, _vp, _sz, _vp]
        L.sage_tree_attention_static_scratch_bytes.restype = _sz
        L.sage_tree_attention_static_scratch_bytes.argtypes = []
        L.sage_tree_attention_static.restype = _ci
        L.sage_tree_attention_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl,
                                                 _vp, _vp, _cf, _vp]
        L.sage_tree_attention_with_plan.restype = _ci
        L.sage_tree_attention_with_plan.argtypes = (
            [_vp, _vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl, _vp, _vp, _cf, _vp, _sz]
            + [_vp, _ci, _ci, ctypes.POINTER(TreeParams)] + [_vp] * 15)
        L.sage_verify_accept.restype = _ci
        L.sage_verify_accept.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _ci, _ci, _vp, _vp, _vp, _vp, _vp]
        L.sage_commit_path.restype = _ci
        L.sage_commit_path.argtypes = [_vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl, _vp, _vp, _ci, _vp]
        L.sage_advance_kv_len.restype = _ci
        L.sage_advance_kv_len.argtypes = [_vp, _vp, _ci, _ci, _vp]
        L.sage_update_history.restype = _ci
        L.sage_update_history.argtypes = [_vp, _ci, _ci, _cf, _cf, _ci, _ci, _vp, _vp, _vp, _vp, _vp]
        L.sage_lm_head_topk_workspace_bytes.restype = _sz
        L.sage_verify_accept_close_from_slices.restype = _ci
        L.sage_verify_accept_close_from_slices.argtypes = (
            [_vp, _ci, _vp, _vp, _vp, _vp, _vp, _ci, _ci] + [_vp] * 6 + [_vp, _vp, _vp, _vp, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl,
                                                                       _ci, _cf, _cf, _ci, _ci, _vp, _vp, _vp, _vp, _vp, _vp])
        L.sage_close_step.restype = _ci
        L.sage_close_step.argtypes = [_vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _cl, _cl, _vp, _vp, _ci, _ci, _cf, _cf,
                                      _ci, _ci, _vp, _vp, _vp, _vp, _vp, _vp]
        L.sage_entropy_topk_slices.restype = _ci
        L.sage_entropy_topk_slices.argtypes = [_vp, _ci, _ci, _ci, _cl, _ci, _vp, _ci, _vp, _sz, _vp]
        L.sage_entropy_topk_slices_pair.restype = _ci
        L.sage_entropy_topk_slices_pair.argtypes = [_vp, _ci, _cl, _vp, _ci, _vp, _sz, _vp, _ci, _cl, _ci, _vp, _sz, _ci, _ci, _vp]
        L.sage_build_tree_from_slices.restype = _ci
        L.sage_build_tree_from_slices.argtypes = [_vp, _ci, _ci, _ci, ctypes.POINTER(TreeParams)] + [_vp] * 15
        L.sage_verify_accept_from_slices.restype = _ci
        L.sage_verify_accept_from_slices.argtypes = [_vp, _ci, _vp, _vp, _vp, _vp, _vp, _ci, _ci] + [_vp] * 7
        L.sage_lm_head_topk_workspace_bytes.argtypes = [_ci, _ci, _ci]
        L.sage_lm_head_topk.restype = _ci
        L.sage_lm_head_topk.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _cl, _cl, _ci, _vp, _ci, _vp, _vp, _vp, _vp, _vp, _vp,
                                        _vp, _sz, _vp]
        L.sage_build_info.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("float32 or bfloat16 expected")


def _check(call: str, rc: int):
    if rc != 0:
        raise SageError(call, rc)


def tree_params(d_min, d_max, w_min, w_max, k, n_max) -> TreeParams:
    return TreeParams(d_min, d_max, w_min, w_max, k, n_max)


def sage_entropy_topk_workspace_bytes(rows: int, vocab: int, k: int) -> int:
    return int(lib().sage_entropy_topk_workspace_bytes(rows, vocab, k))


def sage_lm_head_topk_workspace_bytes(rows: int, vocab: int, k: int = 1) -> int:
    return int(lib().sage_lm_head_topk_workspace_bytes(rows, vocab, k))


def sage_tree_attention_workspace_bytes(dtype_code: int, B: int, Hq: int, Hkv: int, d: int, max_kv_len: int) -> int:
    return int(lib().sage_tree_attention_workspace_bytes(dtype_code, B, Hq, Hkv, d, max_kv_len))


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


# ---- argument marshalling: tensors -> the C argument list of each call -----------------------------------

def _args_entropy_topk(logits, k, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha, workspace,
                       n_valid=None, rows_per_group=1, stream=None):
    rows, vocab = logits.shape
    assert logits.stride(1) == 1
    return [_ptr(logits), _dtype_code(logits), rows, vocab, logits.stride(0), k, _ptr(n_valid), rows_per_group,
            _ptr(entropy), _ptr(topk_idx), _ptr(topk_prob), _ptr(topk_renorm), _ptr(topk_entropy), _ptr(alpha),
            _ptr(workspace), _nbytes(workspace), _stream(stream)]


def _args_build_tree(topk_renorm, alpha, params: TreeParams, n_nodes, parent, depth, rank, anc_mask, cum_prob=None,
                     topk_idx=None, node_token=None, stream=None, d_max_seq=None):
    B, k = topk_renorm.shape
    return [_ptr(topk_renorm), _ptr(alpha), _ptr(topk_idx), B, k, ctypes.byref(params), _ptr(d_max_seq), _ptr(n_nodes),
            _ptr(parent), _ptr(depth), _ptr(rank), _ptr(anc_mask), _ptr(cum_prob), _ptr(node_token), _stream(stream)]


def _args_attention_common(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                           n_nodes, scale, workspace, stream):
    """The argument list the three attention entry points share (without first_node, which only the plain call has)."""
    B, _, Hq, d = Q.shape
    Hkv = Kt.shape[2]
    return [_ptr(Q), _ptr(Kc), _ptr(Vc), _ptr(Kt), _ptr(Vt), _ptr(O), _dtype_code(Q), B, Hq, Hkv, d, _ptr(kv_start),
            _ptr(kv_len), max_kv_len, kv_token_stride, kv_head_stride, _ptr(anc_mask), _ptr(n_nodes), scale,
            _ptr(workspace), _nbytes(workspace), _stream(stream)]


def _args_tree_attention(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                         n_nodes, scale, workspace, stream=None, first_node=None):
    att = _args_attention_common(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                                 n_nodes, scale, workspace, stream)
    return att[:18] + [_ptr(first_node)] + att[18:]    # first_node follows n_nodes


def _args_tree_attention_static(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                                n_nodes, scale, stream=None):
    att = _args_attention_common(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                                 n_nodes, scale, None, stream)
    return att[:-3] + att[-1:]                         # no workspace pair


def _args_tree_attention_with_plan(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                                   n_nodes, scale, workspace, slices, vocab, params: TreeParams, entropy, topk_idx, topk_prob,
                                   topk_renorm, topk_entropy, alpha, next_n_nodes, next_parent, next_depth, next_rank,
                                   next_anc_mask, next_cum_prob=None, next_node_token=None, stream=None, d_max_seq=None):
    att = _args_attention_common(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_kv_len, kv_token_stride, kv_head_stride, anc_mask,
                                 n_nodes, scale, workspace, stream)
    plan = _args_build_tree_from_slices(slices, vocab, params, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha,
                                        next_n_nodes, next_parent, next_depth, next_rank, next_anc_mask, next_cum_prob,
                                        next_node_token, stream, d_max_seq)
    assert plan[2] == att[7], "one draft row per sequence"
    return att[:-1] + plan[:2] + plan[3:]              # the batch size travels once


def _args_verify_accept(token, target_argmax, parent, depth, anc_mask, n_nodes, path_cap, accept_len, best_node,
                        path_nodes, out_tokens, stream=None):
    B = n_nodes.shape[0]
    return [_ptr(token), _ptr(target_argmax), _ptr(parent), _ptr(depth), _ptr(anc_mask), _ptr(n_nodes), B, path_cap,
            _ptr(accept_len), _ptr(best_node), _ptr(path_nodes), _ptr(out_tokens), _stream(stream)]


def _args_commit_path(Kt, Vt, Kc, Vc, kv_start, kv_len, kv_capacity, kv_token_stride, kv_head_stride, path_nodes,
                      accept_len, stream=None):
    B, _, Hkv, d = Kt.shape
    return [_ptr(Kt), _ptr(Vt), _ptr(Kc), _ptr(Vc), _dtype_code(Kt), B, Hkv, d, _ptr(kv_start), _ptr(kv_len), kv_capacity,
            kv_token_stride, kv_head_stride, _ptr(path_nodes), _ptr(accept_len), path_nodes.shape[1], _stream(stream)]


def _args_advance_kv_len(kv_len, accept_len, kv_capacity, stream=None):
    return [_ptr(kv_len), _ptr(accept_len), kv_len.shape[0], kv_capacity, _stream(stream)]


def _args_update_history(accept_len, hist, count, d_max, lo, hi, d_floor, d_cap, avg_out=None, stream=None):
    B, window = hist.shape
    return [_ptr(accept_len), B, window, lo, hi, d_floor, d_cap, _ptr(hist), _ptr(count), _ptr(d_max), _ptr(avg_out),
            _stream(stream)]


def _args_lm_head_topk(hidden, weight, k, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy, alpha, workspace,
                       n_valid=None, rows_per_group=1, stream=None):
    rows, dim = hidden.shape
    vocab = weight.shape[0]
    return [_ptr(hidden), _ptr(weight), _dtype_code(hidden), rows, dim, vocab, hidden.stride(0), weight.stride(0), k,
            _ptr(n_valid), rows_per_group, _ptr(entropy), _ptr(topk_idx), _ptr(topk_prob), _ptr(topk_renorm),
            _ptr(topk_entropy), _ptr(alpha), _ptr(workspace), _nbytes(workspace), _stream(stream)]


def _args_entropy_topk_slices(logits, k, workspace, n_valid=None, rows_per_group=1, stream=None):
    rows, vocab = logits.shape
    assert logits.stride(1) == 1
    return [_ptr(logits), _dtype_code(logits), rows, vocab, logits.stride(0), k, _ptr(n_valid), rows_per_group,
            _ptr(workspace), _nbytes(workspace), _stream(stream)]


def _args_entropy_topk_slices_pair(logits_a, n_valid_a, rows_per_group_a, workspace_a, logits_b, k_b, workspace_b, stream=None):
    rows_a, vocab = logits_a.shape
    rows_b, vocab_b = logits_b.shape
    assert vocab_b == vocab and logits_a.dtype == logits_b.dtype and logits_a.stride(1) == 1 and logits_b.stride(1) == 1
    return [_ptr(logits_a), rows_a, logits_a.stride(0), _ptr(n_valid_a), rows_per_group_a, _ptr(workspace_a), _nbytes(workspace_a),
            _ptr(logits_b), rows_b, logits_b.stride(0), k_b, _ptr(workspace_b), _nbytes(workspace_b), _dtype_code(logits_a),
            vocab, _stream(stream)]


def _args_build_tree_from_slices(slices, vocab, params: TreeParams, entropy, topk_idx, topk_prob, topk_renorm, topk_entropy,
                                 alpha, n_nodes, parent, depth, rank, anc_mask, cum_prob=None, node_token=None, stream=None,
                                 d_max_seq=None):
    B, k = topk_idx.shape
    return [_ptr(slices), vocab, B, k, ctypes.byref(params), _ptr(d_max_seq), _ptr(entropy), _ptr(topk_idx), _ptr(topk_prob),
            _ptr(topk_renorm), _ptr(topk_entropy), _ptr(alpha), _ptr(n_nodes), _ptr(parent), _ptr(depth), _ptr(rank),
            _ptr(anc_mask), _ptr(cum_prob), _ptr(node_token), _stream(stream)]


def _args_verify_accept_from_slices(slices, vocab, token, parent, depth, anc_mask, n_nodes, path_cap, entropy, target_argmax,
                                    accept_len, best_node, path_nodes, out_tokens, stream=None):
    B = n_nodes.shape[0]
    return [_ptr(slices), vocab, _ptr(token), _ptr(parent), _ptr(depth), _ptr(anc_mask), _ptr(n_nodes), B, path_cap,
            _ptr(entropy), _ptr(target_argmax), _ptr(accept_len), _ptr(best_node), _ptr(path_nodes), _ptr(out_tokens),
            _stream(stream)]


def _args_close_step(Kt, Vt, Kc, Vc, kv_start, kv_len, kv_capacity, kv_token_stride, kv_head_stride, path_nodes, accept_len,
                     hist, count, d_max_in, d_max_out, lo, hi, d_floor, d_cap, avg_out=None, stream=None):
    B, _, Hkv, d = Kt.shape
    return [_ptr(Kt), _ptr(Vt), _ptr(Kc), _ptr(Vc), _dtype_code(Kt), B, Hkv, d, _ptr(kv_start), _ptr(kv_len), kv_capacity,
            kv_token_stride, kv_head_stride, _ptr(path_nodes), _ptr(accept_len), path_nodes.shape[1], hist.shape[1], lo, hi,
            d_floor, d_cap, _ptr(hist), _ptr(count), _ptr(d_max_in), _ptr(d_max_out), _ptr(avg_out), _stream(stream)]


def _args_verify_accept_close_from_slices(slices, vocab, token, parent, depth, anc_mask, n_nodes, path_cap, entropy, target_argmax,
                                          accept_len, best_node, path_nodes, out_tokens, Kt, Vt, Kc, Vc, kv_start, kv_len,
                                          kv_capacity, kv_token_stride, kv_head_stride, hist, count, d_max_in, d_max_out, lo, hi,
                                          d_floor, d_cap, avg_out=None, stream=None):
    B = n_nodes.shape[0]
    _, _, Hkv, d = Kt.shape
    return [_ptr(slices), vocab, _ptr(token), _ptr(parent), _ptr(depth), _ptr(anc_mask), _ptr(n_nodes), B, path_cap,
            _ptr(entropy), _ptr(target_argmax), _ptr(accept_len), _ptr(best_node), _ptr(path_nodes), _ptr(out_tokens),
            _ptr(Kt), _ptr(Vt), _ptr(Kc), _ptr(Vc), _dtype_code(Kt), Hkv, d, _ptr(kv_start), _ptr(kv_len), kv_capacity,
            kv_token_stride, kv_head_stride, hist.shape[1], lo, hi, d_floor, d_cap, _ptr(hist), _ptr(count), _ptr(d_max_in),
            _ptr(d_max_out), _ptr(avg_out), _stream(stream)]


_MARSHAL = {"sage_close_step": _args_close_step,
            "sage_tree_attention_with_plan": _args_tree_attention_with_plan,
            "sage_verify_accept_close_from_slices": _args_verify_accept_close_from_slices,
            "sage_entropy_topk_slices": _args_entropy_topk_slices,
            "sage_entropy_topk_slices_pair": _args_entropy_topk_slices_pair,
            "sage_build_tree_from_slices": _args_build_tree_from_slices,
            "sage_verify_accept_from_slices": _args_verify_accept_from_slices,
            "sage_entropy_topk": _args_entropy_topk, "sage_build_tree": _args_build_tree,
            "sage_tree_attention": _args_tree_attention, "sage_tree_attention_static": _args_tree_attention_static,
            "sage_verify_accept": _args_verify_accept,
            "sage_commit_path": _args_commit_path, "sage_advance_kv_len": _args_advance_kv_len,
            "sage_update_history": _args_update_history, "sage_lm_head_topk": _args_lm_head_topk}


def sage_entropy_topk(*a, **kw):
    _check("sage_entropy_topk", lib().sage_entropy_topk(*_args_entropy_topk(*a, **kw)))


def sage_build_tree(*a, **kw):
    _check("sage_build_tree", lib().sage_build_tree(*_args_build_tree(*a, **kw)))


def sage_tree_attention(*a, **kw):
    _check("sage_tree_attention", lib().sage_tree_attention(*_args_tree_attention(*a, **kw)))


def sage_tree_attention_static(*a, **kw):
    _check("sage_tree_attention_static", lib().sage_tree_attention_static(*_args_tree_attention_static(*a, **kw)))


def sage_tree_attention_static_scratch_bytes() -> int:
    return int(lib().sage_tree_attention_static_scratch_bytes())


def sage_tree_attention_with_plan(*a, **kw):
    _check("sage_tree_attention_with_plan", lib().sage_tree_attention_with_plan(*_args_tree_attention_with_plan(*a, **kw)))


def sage_verify_accept(*a, **kw):
    _check("sage_verify_accept", lib().sage_verify_accept(*_args_verify_accept(*a, **kw)))


def sage_commit_path(*a, **kw):
    _check("sage_commit_path", lib().sage_commit_path(*_args_commit_path(*a, **kw)))


def sage_advance_kv_len(*a, **kw):
    _check("sage_advance_kv_len", lib().sage_advance_kv_len(*_args_advance_kv_len(*a, **kw)))


def sage_update_history(*a, **kw):
    _check("sage_update_history", lib().sage_update_history(*_args_update_history(*a, **kw)))


def sage_verify_accept_close_from_slices(*a, **kw):
    _check("sage_verify_accept_close_from_slices",
           lib().sage_verify_accept_close_from_slices(*_args_verify_accept_close_from_slices(*a, **kw)))


def sage_close_step(*a, **kw):
    _check("sage_close_step", lib().sage_close_step(*_args_close_step(*a, **kw)))


def sage_lm_head_topk(*a, **kw):
    _check("sage_lm_head_topk", lib().sage_lm_head_topk(*_args_lm_head_topk(*a, **kw)))


def sage_entropy_topk_slices(*a, **kw):
    _check("sage_entropy_topk_slices", lib().sage_entropy_topk_slices(*_args_entropy_topk_slices(*a, **kw)))


def sage_entropy_topk_slices_pair(*a, **kw):
    _check("sage_entropy_topk_slices_pair", lib().sage_entropy_topk_slices_pair(*_args_entropy_topk_slices_pair(*a, **kw)))


def sage_build_tree_from_slices(*a, **kw):
    _check("sage_build_tree_from_slices", lib().sage_build_tree_from_slices(*_args_build_tree_from_slices(*a, **kw)))


def sage_verify_accept_from_slices(*a, **kw):
    _check("sage_verify_accept_from_slices",
           lib().sage_verify_accept_from_slices(*_args_verify_accept_from_slices(*a, **kw)))


def prepare(name: str, *a, **kw):
    """Marshal the arguments of call `name` once and return a zero-argument callable that enqueues it.

    For loops that issue the same call on the same buffers and stream many times: the per-call cost drops to
    one foreign-function call.  The tensors (and the TreeParams object) must outlive the callable.
    """
    fn = getattr(lib(), name)
    args = _MARSHAL[name](*a, **kw)
    keep = (a, kw)

    def call(_fn=fn, _args=args, _name=name, _keep=keep):
        rc = _fn(*_args)
        if rc != 0:
            raise SageError(_name, rc)
    return call


def sage_build_info() -> str:
    return lib().sage_build_info().decode()
