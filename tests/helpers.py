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
