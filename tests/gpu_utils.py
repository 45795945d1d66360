"""Helpers of the GPU parity tests: move seeded numpy inputs to the device, call the C-ABI binding, compare."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_00523_amd import sage
from paper_2602_00523_amd import workloads as wl

MAX_NODES = 64
DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns; uint64 travels as int64 bits."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def widen(a: np.ndarray) -> np.ndarray:
    return a.astype(np.float64) if a.dtype != np.uint16 else wl.bf16_bits_to_f32(a).astype(np.float64)


def gpu_entropy_topk(logits_np, k, n_valid=None, rows_per_group=1):
    if logits_np.flags["C_CONTIGUOUS"]:
        x = to_dev(logits_np)
    else:                                            # a column slice of a padded buffer: keep the row stride
        full = logits_np.base
        assert full is not None and full.shape[0] == logits_np.shape[0]
        x = to_dev(full)[:, :logits_np.shape[1]]
    rows, vocab = x.shape
    f = lambda *s: torch.full(s, float("nan"), device=DEV, dtype=torch.float32)
    out = dict(entropy=f(rows), topk_idx=torch.full((rows, k), -1, device=DEV, dtype=torch.int32), topk_prob=f(rows, k),
               topk_renorm=f(rows, k), topk_entropy=f(rows), alpha=f(rows))
    ws = torch.empty(sage.sage_entropy_topk_workspace_bytes(rows, vocab, k), device=DEV, dtype=torch.uint8)
    nv = None if n_valid is None else to_dev(np.asarray(n_valid, np.int32))
    sage.sage_entropy_topk(x, k, out["entropy"], out["topk_idx"], out["topk_prob"], out["topk_renorm"],
                           out["topk_entropy"], out["alpha"], ws, nv, rows_per_group)
    torch.cuda.synchronize()
    return {key: v.cpu().numpy() for key, v in out.items()}


def gpu_build_tree(topk_renorm_np, alpha_np, prm: dict, topk_idx_np=None, d_max_seq_np=None):
    pt, al = to_dev(np.ascontiguousarray(topk_renorm_np, np.float32)), to_dev(np.ascontiguousarray(alpha_np, np.float32))
    B = pt.shape[0]
    i32 = lambda fill: torch.full((B, MAX_NODES), fill, device=DEV, dtype=torch.int32)
    out = dict(n_nodes=torch.zeros(B, device=DEV, dtype=torch.int32), parent=i32(-2), depth=i32(-2), rank=i32(-2),
               anc_mask=torch.zeros((B, MAX_NODES), device=DEV, dtype=torch.int64),
               cum_prob=torch.full((B, MAX_NODES), float("nan"), device=DEV, dtype=torch.float32),
               node_token=i32(-2))
    ti = None if topk_idx_np is None else to_dev(np.ascontiguousarray(topk_idx_np, np.int32))
    dm = None if d_max_seq_np is None else to_dev(np.ascontiguousarray(d_max_seq_np, np.int32))
    sage.sage_build_tree(pt, al, sage.tree_params(**prm), out["n_nodes"], out["parent"], out["depth"], out["rank"],
                         out["anc_mask"], out["cum_prob"], ti, out["node_token"] if ti is not None else None, d_max_seq=dm)
    torch.cuda.synchronize()
    res = {key: v.cpu().numpy() for key, v in out.items()}
    res["anc_mask"] = res["anc_mask"].view(np.uint64)
    return res


def gpu_tree_attention(inp: dict, anc_mask_np, n_nodes_np, Hq, Hkv, d, scale=None, fill=None, first_node_np=None):
    """inp as produced by workloads.attention_inputs.  Returns O widened to fp64 ([B,64,Hq,d]) and the raw tensor."""
    Q, Kc, Vc, Kt, Vt = (to_dev(inp[k]) for k in ("Q", "Kc", "Vc", "Kt", "Vt"))
    B = Q.shape[0]
    O = torch.zeros_like(Q)
    if fill is not None:
        O.fill_(fill)
    kv_start, kv_len = to_dev(np.asarray(inp["kv_start"], np.int64)), to_dev(np.asarray(inp["kv_len"], np.int32))
    mask, nn = to_dev(np.ascontiguousarray(anc_mask_np, np.uint64)), to_dev(np.asarray(n_nodes_np, np.int32))
    max_len = int(np.max(inp["kv_len"])) if B else 0
    code = sage.F32 if Q.dtype == torch.float32 else sage.BF16
    ws = torch.empty(sage.sage_tree_attention_workspace_bytes(code, B, Hq, Hkv, d, max_len), device=DEV, dtype=torch.uint8)
    if scale is None:
        scale = 1.0 / float(np.sqrt(d))
    first = None if first_node_np is None else to_dev(np.asarray(first_node_np, np.int32))
    sage.sage_tree_attention(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_len, inp["kv_token_stride"],
                             inp["kv_head_stride"], mask, nn, scale, ws, first_node=first)
    torch.cuda.synchronize()
    return widen(to_host(O)), O


def gpu_verify_accept(token, target_argmax, parent, depth, anc_mask, n_nodes, path_cap):
    B = len(n_nodes)
    args = [to_dev(np.ascontiguousarray(a, np.int32)) for a in (token, target_argmax, parent, depth)]
    mask, nn = to_dev(np.ascontiguousarray(anc_mask, np.uint64)), to_dev(np.ascontiguousarray(n_nodes, np.int32))
    out = dict(accept_len=torch.full((B,), -9, device=DEV, dtype=torch.int32),
               best_node=torch.full((B,), -9, device=DEV, dtype=torch.int32),
               path_nodes=torch.full((B, path_cap), -9, device=DEV, dtype=torch.int32),
               out_tokens=torch.full((B, path_cap), -9, device=DEV, dtype=torch.int32))
    sage.sage_verify_accept(*args, mask, nn, path_cap, out["accept_len"], out["best_node"], out["path_nodes"],
                            out["out_tokens"])
    torch.cuda.synchronize()
    return {key: v.cpu().numpy() for key, v in out.items()}


def assert_attention_close(gpu64, ref64, n_nodes, tol):
    """Per (node, head) row: relative L2 error and max error relative to the row's largest magnitude, both <= tol."""
    B = ref64.shape[0]
    worst = 0.0
    for b in range(B):
        n = int(n_nodes[b])
        g, r = gpu64[b, :n], ref64[b, :n]
        assert np.isfinite(g).all(), f"non-finite output in sequence {b}"
        l2 = np.linalg.norm(g - r, axis=-1) / np.maximum(np.linalg.norm(r, axis=-1), 1e-300)
        mx = np.abs(g - r).max(-1) / np.maximum(np.abs(r).max(-1), 1e-300)
        worst = max(worst, float(l2.max()), float(mx.max()))
        assert l2.max() <= tol, f"seq {b}: rel L2 {l2.max():.3e} > {tol}"
        assert mx.max() <= tol, f"seq {b}: rel max {mx.max():.3e} > {tol}"
    return worst


def gpu_commit_path(Kt_np, Vt_np, Kc_np, Vc_np, kv_start, kv_len, kv_capacity, ts, hs, path_nodes, accept_len):
    """Returns the caches after the commit and the advanced lengths (numpy)."""
    Kt, Vt, Kc, Vc = (to_dev(a) for a in (Kt_np, Vt_np, Kc_np, Vc_np))
    ks = to_dev(np.ascontiguousarray(kv_start, np.int64))
    kl = to_dev(np.ascontiguousarray(kv_len, np.int32))
    pn = to_dev(np.ascontiguousarray(path_nodes, np.int32))
    al = to_dev(np.ascontiguousarray(accept_len, np.int32))
    sage.sage_commit_path(Kt, Vt, Kc, Vc, ks, kl, int(kv_capacity), int(ts), int(hs), pn, al)
    sage.sage_advance_kv_len(kl, al, int(kv_capacity))
    torch.cuda.synchronize()
    return to_host(Kc), to_host(Vc), kl.cpu().numpy()


def gpu_update_history(accept_len, hist, count, d_max, lo, hi, d_floor, d_cap):
    """hist/count/d_max are device tensors updated in place; returns the averages (numpy)."""
    al = to_dev(np.ascontiguousarray(accept_len, np.int32))
    avg = torch.zeros(al.shape[0], device=DEV, dtype=torch.float32)
    sage.sage_update_history(al, hist, count, d_max, float(lo), float(hi), int(d_floor), int(d_cap), avg)
    torch.cuda.synchronize()
    return avg.cpu().numpy()


def gpu_lm_head_topk(hidden_np, weight_np, k, n_valid=None, rows_per_group=1):
    h, w = to_dev(hidden_np), to_dev(weight_np)
    rows, vocab = h.shape[0], w.shape[0]
    f = lambda *s: torch.full(s, float("nan"), device=DEV, dtype=torch.float32)
    out = dict(entropy=f(rows), topk_idx=torch.full((rows, k), -1, device=DEV, dtype=torch.int32), topk_prob=f(rows, k),
               topk_renorm=f(rows, k), topk_entropy=f(rows), alpha=f(rows))
    ws = torch.empty(sage.sage_lm_head_topk_workspace_bytes(rows, vocab, k), device=DEV, dtype=torch.uint8)
    nv = None if n_valid is None else to_dev(np.asarray(n_valid, np.int32))
    sage.sage_lm_head_topk(h, w, k, out["entropy"], out["topk_idx"], out["topk_prob"], out["topk_renorm"],
                           out["topk_entropy"], out["alpha"], ws, nv, rows_per_group)
    torch.cuda.synchronize()
    return {key: v.cpu().numpy() for key, v in out.items()}


def gpu_plan_from_slices(logits_np, k, prm: dict, d_max_seq_np=None):
    """sage_entropy_topk_slices + sage_build_tree_from_slices on B draft rows: the outputs of both separate calls."""
    x = to_dev(logits_np)
    B, vocab = x.shape
    f = lambda *s: torch.full(s, float("nan"), device=DEV, dtype=torch.float32)
    i32 = lambda fill: torch.full((B, MAX_NODES), fill, device=DEV, dtype=torch.int32)
    a1 = dict(entropy=f(B), topk_idx=torch.full((B, k), -1, device=DEV, dtype=torch.int32), topk_prob=f(B, k),
              topk_renorm=f(B, k), topk_entropy=f(B), alpha=f(B))
    a2 = dict(n_nodes=torch.zeros(B, device=DEV, dtype=torch.int32), parent=i32(-2), depth=i32(-2), rank=i32(-2),
              anc_mask=torch.zeros((B, MAX_NODES), device=DEV, dtype=torch.int64),
              cum_prob=torch.full((B, MAX_NODES), float("nan"), device=DEV, dtype=torch.float32), node_token=i32(-2))
    ws = torch.empty(sage.sage_entropy_topk_workspace_bytes(B, vocab, k), device=DEV, dtype=torch.uint8)
    dm = None if d_max_seq_np is None else to_dev(np.ascontiguousarray(d_max_seq_np, np.int32))
    sage.sage_entropy_topk_slices(x, k, ws)
    sage.sage_build_tree_from_slices(ws, vocab, sage.tree_params(**prm), a1["entropy"], a1["topk_idx"], a1["topk_prob"],
                                     a1["topk_renorm"], a1["topk_entropy"], a1["alpha"], a2["n_nodes"], a2["parent"],
                                     a2["depth"], a2["rank"], a2["anc_mask"], a2["cum_prob"], a2["node_token"], d_max_seq=dm)
    torch.cuda.synchronize()
    r1 = {key: v.cpu().numpy() for key, v in a1.items()}
    r2 = {key: v.cpu().numpy() for key, v in a2.items()}
    r2["anc_mask"] = r2["anc_mask"].view(np.uint64)
    return r1, r2


def gpu_attention_with_plan(inp: dict, anc_mask_np, n_nodes_np, Hq, Hkv, d, logits_np, k, prm: dict, d_max_seq_np=None):
    """sage_entropy_topk_slices + sage_tree_attention_with_plan: O (raw tensor bits as numpy) and the outputs of the planning
    half, laid out as gpu_plan_from_slices returns them."""
    Q, Kc, Vc, Kt, Vt = (to_dev(inp[key]) for key in ("Q", "Kc", "Vc", "Kt", "Vt"))
    B = Q.shape[0]
    O = torch.zeros_like(Q)
    kv_start, kv_len = to_dev(np.asarray(inp["kv_start"], np.int64)), to_dev(np.asarray(inp["kv_len"], np.int32))
    mask, nn = to_dev(np.ascontiguousarray(anc_mask_np, np.uint64)), to_dev(np.asarray(n_nodes_np, np.int32))
    max_len = int(np.max(inp["kv_len"])) if B else 0
    code = sage.F32 if Q.dtype == torch.float32 else sage.BF16
    ws3 = torch.empty(sage.sage_tree_attention_workspace_bytes(code, B, Hq, Hkv, d, max_len), device=DEV, dtype=torch.uint8)
    x = to_dev(logits_np)
    assert x.shape[0] == B
    vocab = x.shape[1]
    f = lambda *s: torch.full(s, float("nan"), device=DEV, dtype=torch.float32)
    i32 = lambda fill: torch.full((B, MAX_NODES), fill, device=DEV, dtype=torch.int32)
    a1 = dict(entropy=f(B), topk_idx=torch.full((B, k), -1, device=DEV, dtype=torch.int32), topk_prob=f(B, k),
              topk_renorm=f(B, k), topk_entropy=f(B), alpha=f(B))
    a2 = dict(n_nodes=torch.zeros(B, device=DEV, dtype=torch.int32), parent=i32(-2), depth=i32(-2), rank=i32(-2),
              anc_mask=torch.zeros((B, MAX_NODES), device=DEV, dtype=torch.int64),
              cum_prob=torch.full((B, MAX_NODES), float("nan"), device=DEV, dtype=torch.float32), node_token=i32(-2))
    ws1 = torch.empty(sage.sage_entropy_topk_workspace_bytes(B, vocab, k), device=DEV, dtype=torch.uint8)
    dm = None if d_max_seq_np is None else to_dev(np.ascontiguousarray(d_max_seq_np, np.int32))
    sage.sage_entropy_topk_slices(x, k, ws1)
    sage.sage_tree_attention_with_plan(Q, Kc, Vc, Kt, Vt, O, kv_start, kv_len, max_len, inp["kv_token_stride"],
                                       inp["kv_head_stride"], mask, nn, 1.0 / float(np.sqrt(d)), ws3, ws1, vocab,
                                       sage.tree_params(**prm), a1["entropy"], a1["topk_idx"], a1["topk_prob"], a1["topk_renorm"],
                                       a1["topk_entropy"], a1["alpha"], a2["n_nodes"], a2["parent"], a2["depth"], a2["rank"],
                                       a2["anc_mask"], a2["cum_prob"], a2["node_token"], d_max_seq=dm)
    torch.cuda.synchronize()
    r1 = {key: v.cpu().numpy() for key, v in a1.items()}
    r2 = {key: v.cpu().numpy() for key, v in a2.items()}
    r2["anc_mask"] = r2["anc_mask"].view(np.uint64)
    return to_host(O), r1, r2


def gpu_accept_from_slices(target_logits_np, token, parent, depth, anc_mask, n_nodes, path_cap):
    """sage_entropy_topk_slices (k = 1, rows grouped by sequence) + sage_verify_accept_from_slices."""
    x = to_dev(target_logits_np)
    rows, vocab = x.shape
    B = len(n_nodes)
    assert rows == B * MAX_NODES
    args = [to_dev(np.ascontiguousarray(a, np.int32)) for a in (token, parent, depth)]
    mask, nn = to_dev(np.ascontiguousarray(anc_mask, np.uint64)), to_dev(np.ascontiguousarray(n_nodes, np.int32))
    out = dict(entropy=torch.full((rows,), float("nan"), device=DEV, dtype=torch.float32),
               target_argmax=torch.full((rows,), -1, device=DEV, dtype=torch.int32),
               accept_len=torch.full((B,), -9, device=DEV, dtype=torch.int32),
               best_node=torch.full((B,), -9, device=DEV, dtype=torch.int32),
               path_nodes=torch.full((B, path_cap), -9, device=DEV, dtype=torch.int32),
               out_tokens=torch.full((B, path_cap), -9, device=DEV, dtype=torch.int32))
    ws = torch.empty(sage.sage_entropy_topk_workspace_bytes(rows, vocab, 1), device=DEV, dtype=torch.uint8)
    sage.sage_entropy_topk_slices(x, 1, ws, nn, MAX_NODES)
    sage.sage_verify_accept_from_slices(ws, vocab, args[0], args[1], args[2], mask, nn, path_cap, out["entropy"],
                                        out["target_argmax"], out["accept_len"], out["best_node"], out["path_nodes"],
                                        out["out_tokens"])
    torch.cuda.synchronize()
    return {key: v.cpu().numpy() for key, v in out.items()}
