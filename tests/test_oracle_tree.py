"""Pins for the oracle's integer work: tree mask / depth and the greedy accept walk.
Brute force on small trees, closed forms for chains and stars."""
import itertools

import numpy as np
import pytest

import moa_inputs as mi


def ancestors_or_self(par, i):
    out = set()
    while i >= 0:
        out.add(i)
        i = par[i]
    return out


def all_parent_arrays(M):
    return itertools.product(*[range(i) for i in range(1, M)])


def test_mask_and_depth_brute_force_all_trees_up_to_6(oracle):
    for M in range(1, 7):
        for tail in all_parent_arrays(M):
            par = np.array([-1, *tail], dtype=np.int32)
            mask, depth = oracle.tree_build(par[None])
            for i in range(M):
                anc = ancestors_or_self(par, i)
                bits = {j for j in range(M) if (int(mask[0, i, 0]) >> j) & 1}
                assert bits == anc
                assert depth[0, i] == len(anc) - 1


@pytest.mark.parametrize("M", [63, 64, 65, 128, 200, 256])
def test_mask_multiword(oracle, M):
    rng = np.random.default_rng(M)
    par = np.stack([mi.gen_tree(M, 10, 4, rng), mi.chain_tree(M), mi.star_tree(M)])
    mask, depth = oracle.tree_build(par)
    W = (M + 63) // 64
    assert mask.shape == (3, M, W)
    for b in range(3):
        for i in range(M):
            anc = ancestors_or_self(par[b], i)
            bits = {j for j in range(M) if (int(mask[b, i, j >> 6]) >> (j & 63)) & 1}
            assert bits == anc and depth[b, i] == len(anc) - 1
    # chain: row i = bits 0..i ; star: row i = {0, i}
    assert all(depth[1, i] == i for i in range(M))
    assert all(depth[2, i] == (i > 0) for i in range(M))


def test_tree_rejects_bad_parents(oracle):
    for bad in ([0, 0, 1], [-1, 1, 0], [-1, 0, 2], [-1, -1, 0]):
        with pytest.raises(oracle.OracleError) as e:
            oracle.tree_build(np.array([bad], dtype=np.int32))
        assert e.value.code == oracle.BAD_TREE


def brute_accept(par, tok, tgt):
    """Enumerate every root path; valid = each edge (p -> c) has tok[c] == tgt[p].
    Sibling tokens are distinct here, so the longest valid path is unique."""
    M = len(par)
    best = [0]
    for leaf in range(M):
        path = sorted(ancestors_or_self(par, leaf))      # indices increase along a root path
        if all(tok[c] == tgt[p] for p, c in zip(path[:-1], path[1:])) and len(path) > len(best):
            best = path
    return best


def test_accept_brute_force_small_trees(oracle):
    rng = np.random.default_rng(7)
    for M in range(1, 7):
        for tail in all_parent_arrays(M):
            par = np.array([-1, *tail], dtype=np.int32)
            kids = [np.nonzero(par == p)[0] for p in range(M)]
            tok = np.zeros(M, dtype=np.int32)
            for p in range(M):
                tok[kids[p]] = rng.permutation(4 * M)[: len(kids[p])]     # siblings distinct, small alphabet
            tgt = rng.integers(0, 4 * M, size=M).astype(np.int32)
            for p in range(M):
                if len(kids[p]) and rng.random() < 0.7:
                    tgt[p] = tok[rng.choice(kids[p])]
            path, n, bonus = oracle.tree_accept(par[None], tok[None], tgt[None])
            want = brute_accept(par, tok, tgt)
            assert n[0] == len(want)
            assert list(path[0, : n[0]]) == want and np.all(path[0, n[0]:] == -1)
            assert bonus[0] == tgt[want[-1]]


@pytest.mark.parametrize("seed", range(4))
def test_accept_chain_is_longest_common_prefix(oracle, seed):
    rng = np.random.default_rng(seed)
    M = 40
    par = mi.chain_tree(M)
    tgt = rng.integers(0, 50, size=M).astype(np.int32)
    tok = np.empty(M, dtype=np.int32)
    tok[0] = 3
    tok[1:] = tgt[:-1]
    k = int(rng.integers(1, M - 1))
    tok[k + 1] = tgt[k] + 1                    # first mismatch: node k+1 is not what the LLM says after node k
    path, n, bonus = oracle.tree_accept(par[None], tok[None], tgt[None])
    assert n[0] == k + 1 and list(path[0, : k + 1]) == list(range(k + 1)) and bonus[0] == tgt[k]


def test_accept_star_takes_at_most_one_child(oracle):
    M = 9
    par = mi.star_tree(M)
    tok = np.arange(100, 100 + M, dtype=np.int32)
    tgt = np.full(M, 7, dtype=np.int32)
    tgt[0] = 105
    tgt[5] = 42
    path, n, bonus = oracle.tree_accept(par[None], tok[None], tgt[None])
    assert n[0] == 2 and list(path[0, :2]) == [0, 5] and bonus[0] == 42
    tgt[0] = 5                                 # no child carries token 5
    path, n, bonus = oracle.tree_accept(par[None], tok[None], tgt[None])
    assert n[0] == 1 and path[0, 0] == 0 and bonus[0] == 5


def test_accept_on_generated_workload(oracle):
    c = mi.CONFIGS["C2"]
    par = mi.trees(c)
    tok, tgt = mi.tokens(c, par)
    path, n, bonus = oracle.tree_accept(par, tok, tgt)
    for b in range(c.B):
        want = brute_accept(par[b], tok[b], tgt[b])
        assert list(path[b, : n[b]]) == want and bonus[b] == tgt[b, want[-1]]
    assert n.max() > 1                         # the recipe does produce accepted drafts
