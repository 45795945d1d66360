"""Test-side utilities: random tree topologies and independent re-derivations used to pin the oracle.

Nothing here is imported by the oracle or by the HIP library.
"""
from __future__ import annotations

import numpy as np

MAX_NODES = 64


def random_parents(rng: np.random.Generator, n: int, chain_bias: float = 0.0) -> np.ndarray:
    """parent[0] = -1, parent[v] uniform in [0, v) (or v-1 with probability chain_bias)."""
    par = np.full(n, -1, np.int32)
    for v in range(1, n):
        par[v] = v - 1 if rng.random() < chain_bias else rng.integers(0, v)
    return par


def depth_by_walk(par: np.ndarray) -> np.ndarray:
    dep = np.zeros(len(par), np.int32)
    for v in range(len(par)):
        u, c = v, 0
        while par[u] >= 0:
            u = par[u]
            c += 1
        dep[v] = c
    return dep


def ancestor_sets(par: np.ndarray):
    """List of ancestor-or-self sets obtained by walking parent pointers."""
    out = []
    for v in range(len(par)):
        s, u = {v}, v
        while par[u] >= 0:
            u = par[u]
            s.add(u)
        out.append(s)
    return out


def mask_by_walk(par: np.ndarray) -> np.ndarray:
    m = np.zeros(len(par), np.uint64)
    for v, s in enumerate(ancestor_sets(par)):
        bits = 0
        for u in s:
            bits |= 1 << int(u)
        m[v] = np.uint64(bits)
    return m


def pad_tree(par: np.ndarray, B: int = 1):
    """[B,64] parent/depth/mask arrays (same tree in every sequence) plus n_nodes."""
    n = len(par)
    parent = np.full((B, MAX_NODES), -7, np.int32)
    depth = np.full((B, MAX_NODES), -7, np.int32)
    mask = np.zeros((B, MAX_NODES), np.uint64)
    parent[:, :n] = par
    depth[:, :n] = depth_by_walk(par)
    mask[:, :n] = mask_by_walk(par)
    return parent, depth, mask, np.full(B, n, np.int32)


def chain_parents(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def star_parents(n: int) -> np.ndarray:
    p = np.zeros(n, np.int32)
    p[0] = -1
    return p


def level_order(par: np.ndarray) -> np.ndarray:
    """The same tree renumbered level by level (depth first, then old index), as a model that drafts one level per
    forward pass numbers it: parents of the new tree, every parent still before its children."""
    dep = depth_by_walk(par)
    order = np.lexsort((np.arange(len(par)), dep))         # old index of new node i
    new_of_old = np.empty(len(par), np.int64)
    new_of_old[order] = np.arange(len(par))
    return np.array([-1 if par[o] < 0 else new_of_old[par[o]] for o in order], np.int32)


def relayout_cache(inp: dict, layout: str) -> dict:
    """The packed cache [tokens, Hkv, d] of an attention input set (a dict as workloads.attention_inputs returns it)
    stored another way, same values: 'head_major' = [Hkv, tokens, d]; 'padded' = [tokens, Hkv, d + 8] with unrelated
    values in the padding; 'shifted' = the packed layout moved 29 tokens into a larger buffer (kv_start grows by 29);
    'reversed' = sequences stored in reverse order with gaps between them.  Returns a copy of inp with Kc, Vc,
    kv_start and the strides replaced."""
    out = dict(inp)
    Kc, Vc = inp["Kc"], inp["Vc"]
    T, Hkv, d = Kc.shape
    junk = np.random.default_rng(1234)

    def noise(shape):
        return (junk.integers(0, 2 ** 14, size=shape)).astype(Kc.dtype) if Kc.dtype == np.uint16 else \
            junk.standard_normal(shape).astype(Kc.dtype)
    if layout == "head_major":
        out["Kc"], out["Vc"] = (np.ascontiguousarray(a.transpose(1, 0, 2)) for a in (Kc, Vc))
        out["kv_token_stride"], out["kv_head_stride"] = d, T * d
    elif layout == "padded":
        bufs = []
        for a in (Kc, Vc):
            b = noise((T, Hkv, d + 8))
            b[:, :, :d] = a
            bufs.append(b)
        out["Kc"], out["Vc"] = bufs
        out["kv_token_stride"], out["kv_head_stride"] = Hkv * (d + 8), d + 8
    elif layout == "shifted":
        bufs = []
        for a in (Kc, Vc):
            b = noise((T + 40, Hkv, d))
            b[29:29 + T] = a
            bufs.append(b)
        out["Kc"], out["Vc"] = bufs
        out["kv_start"] = np.asarray(inp["kv_start"], np.int64) + 29
    elif layout == "reversed":
        lens = np.asarray(inp["kv_len"], np.int64)
        starts = np.asarray(inp["kv_start"], np.int64)
        new_start = np.zeros_like(starts)
        at = 5
        for b in range(len(lens) - 1, -1, -1):
            new_start[b] = at
            at += int(lens[b]) + 3
        bufs = []
        for a in (Kc, Vc):
            buf = noise((at + 1, Hkv, d))
            for b in range(len(lens)):
                buf[new_start[b]:new_start[b] + lens[b]] = a[starts[b]:starts[b] + lens[b]]
            bufs.append(buf)
        out["Kc"], out["Vc"] = bufs
        out["kv_start"] = new_start
    else:
        raise ValueError(layout)
    return out


CACHE_LAYOUTS = ("head_major", "padded", "shifted", "reversed")
