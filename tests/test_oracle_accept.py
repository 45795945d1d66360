"""Pins for oracle O4 (acceptance: longest root-to-leaf prefix whose draft tokens equal the target's greedy
choices; Sec. 2.2, Sec. 3.3 Phase 2, Def. 4.1), against brute-force path enumeration and the closed form of
Thm. 4.6 for chains."""
import numpy as np
import pytest

import oracle
from helpers import MAX_NODES, chain_parents, depth_by_walk, pad_tree, random_parents


def brute_force(tok, tgt, par):
    """Enumerate every root-to-leaf path, count its matched prefix, keep the longest (ties: lowest end node)."""
    n = len(par)
    leaves = [v for v in range(n) if not any(par[c] == v for c in range(n))]
    best_len, best_end = 0, 0
    for leaf in leaves:
        path, u = [], leaf
        while u >= 0:
            path.append(u)
            u = par[u]
        path.reverse()                                  # root ... leaf
        m = 0
        for j in range(1, len(path)):
            if tok[path[j]] == tgt[path[j - 1]]:
                m += 1
            else:
                break
        end = path[m]
        if m > best_len or (m == best_len and end < best_end):
            best_len, best_end = m, end
    return best_len, best_end


@pytest.mark.parametrize("seed", range(40))
def test_matches_brute_force_on_small_trees(seed):
    g = np.random.default_rng(seed)
    n = int(g.integers(1, 13))
    par = random_parents(g, n, chain_bias=0.3)
    parent, depth, _, nn = pad_tree(par)
    alphabet = int(g.integers(1, 4))                    # tiny alphabets: frequent matches, duplicated sibling tokens
    tok = np.full((1, MAX_NODES), -5, np.int32)
    tgt = np.full((1, MAX_NODES), -6, np.int32)
    tok[0, :n] = g.integers(0, alphabet, n)
    tgt[0, :n] = g.integers(0, alphabet, n)
    o = oracle.verify_accept(tok, tgt, parent, depth, nn, path_cap=13)
    tau, end = brute_force(tok[0], tgt[0], par)
    assert o["accept_len"][0] == tau and o["best_node"][0] == end
    path = o["path_nodes"][0]
    assert path[0] == 0 and path[tau] == end and (path[tau + 1:] == -1).all()
    for j in range(1, tau + 1):
        assert par[path[j]] == path[j - 1]
        assert o["out_tokens"][0, j - 1] == tok[0, path[j]]
    # every emitted token is the target's greedy choice at the previous path node; the last one is the bonus token
    for j in range(tau + 1):
        assert o["out_tokens"][0, j] == tgt[0, path[j]]
    assert (o["out_tokens"][0, tau + 1:] == -1).all()


def test_all_match_and_none_match():
    g = np.random.default_rng(1)
    par = random_parents(g, 20, chain_bias=0.5)
    parent, depth, _, nn = pad_tree(par, B=2)
    tgt = np.zeros((2, MAX_NODES), np.int32)
    tgt[:, :20] = np.arange(100, 120)
    tok = np.zeros((2, MAX_NODES), np.int32)
    tok[0, 1:20] = tgt[0, par[1:]]                     # every node matches
    tok[1, :20] = -1                                   # nothing matches
    o = oracle.verify_accept(tok, tgt, parent, depth, nn, path_cap=21)
    dep = depth_by_walk(par)
    deepest = int(np.flatnonzero(dep == dep.max())[0])
    assert o["accept_len"][0] == dep.max() and o["best_node"][0] == deepest
    assert o["accept_len"][1] == 0 and o["best_node"][1] == 0
    assert o["out_tokens"][1, 0] == tgt[1, 0] and (o["out_tokens"][1, 1:] == -1).all()


def test_mismatch_blocks_descendants():
    # chain 0-1-2-3: node 2 mismatches, node 3 matches its parent: prefix semantics stop at depth 1
    parent, depth, _, nn = pad_tree(chain_parents(4))
    tgt = np.zeros((1, MAX_NODES), np.int32)
    tok = np.zeros((1, MAX_NODES), np.int32)
    tgt[0, :4] = [10, 11, 12, 13]
    tok[0, :4] = [0, 10, 99, 12]
    o = oracle.verify_accept(tok, tgt, parent, depth, nn, path_cap=5)
    assert o["accept_len"][0] == 1 and o["best_node"][0] == 1
    assert list(o["out_tokens"][0, :2]) == [10, 11]


def test_chain_expected_accept_length_closed_form():
    # i.i.d. acceptance with probability p on a chain of depth D: E[tau] = p (1 - p^D) / (1 - p)  (Thm. 4.6, gamma = 1)
    g = np.random.default_rng(2)
    D, p, trials = 8, 0.7, 4000
    parent, depth, _, nn = pad_tree(chain_parents(D + 1), B=trials)
    tgt = np.zeros((trials, MAX_NODES), np.int32)
    tgt[:, :D + 1] = 7
    tok = np.zeros((trials, MAX_NODES), np.int32)
    tok[:, 1:D + 1] = np.where(g.random((trials, D)) < p, 7, 8)
    o = oracle.verify_accept(tok, tgt, parent, depth, nn, path_cap=D + 1)
    want = p * (1 - p ** D) / (1 - p)
    assert abs(o["accept_len"].mean() - want) < 4 * 2.0 / np.sqrt(trials)
