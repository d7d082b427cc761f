"""Pins for the oracle's draft-tree construction (Sec. 2.2: expand the B most probable tokens, per level rank the B*B
expansions by joint probability and keep the best B branches, at the end keep the m most probable of all
B + (D-1) B^2 candidates) and for the top-B log-probabilities that feed it.

Pinned by: a small example worked by hand; the paper's own count of candidates (328 at breadth 8, depth 6); an
independent re-implementation with Python sorting on every level of random inputs; structural facts (a kept node's
parent is kept, nodes are in depth order, breadth 1 gives a chain); tie handling; scipy's log_softmax."""
from pathlib import Path

import numpy as np
import pytest
from scipy.special import log_softmax

GOLD = {}
for line in (Path(__file__).parent / "golden" / "paper_hyperparameters.txt").read_text().splitlines():
    if line and not line.startswith("#"):
        k, v = line.split()
        GOLD[k] = int(v)


def build(oracle, levels, m, root_tok=1):
    """levels[l] = (child_logp [F, Bw], child_tok [F, Bw]) for level l+1, given as FUNCTIONS of the current frontier
    when they depend on it, else arrays."""
    D = len(levels)
    first = levels[0](None) if callable(levels[0]) else levels[0]
    Bw = np.asarray(first[0]).shape[-1]
    n = Bw + (D - 1) * Bw * Bw
    lp, tk, pr = np.zeros(n, np.float32), np.zeros(n, np.int32), np.zeros(n, np.int32)
    fr = np.full(Bw, -1, np.int32)
    trace = []
    for l, lev in enumerate(levels, start=1):
        clp, ctk = lev(fr.copy()) if callable(lev) else lev
        oracle.tree_expand_level(l, clp, ctk, lp, tk, pr, fr)
        trace.append(fr.copy())
    parent, tok, node_cand = oracle.tree_finalize(n, m, root_tok, lp, tk, pr)
    return parent, tok, node_cand, (lp, tk, pr), trace


def test_hand_worked_example(oracle):
    """Breadth 2, depth 3, keep 5: every number below was computed by hand from the definition."""
    levels = [
        (np.array([[-0.1, -2.0]]), np.array([[5, 6]])),
        (np.array([[-0.2, -1.0], [-0.05, -3.0]]), np.array([[7, 8], [9, 10]])),        # rows: children of candidates 0, 1
        (np.array([[-0.5, -0.6], [-0.1, -4.0]]), np.array([[11, 12], [13, 14]])),      # rows: children of candidates 2, 3
    ]
    parent, tok, node_cand, (lp, tk, pr), trace = build(oracle, levels, m=5, root_tok=99)
    assert [list(t) for t in trace] == [[0, 1], [2, 3], [6, 7]]
    assert np.allclose(lp, [-0.1, -2.0, -0.3, -1.1, -2.05, -5.0, -0.8, -0.9, -1.2, -5.1], atol=1e-6)
    assert list(pr) == [-1, -1, 0, 0, 1, 1, 2, 2, 3, 3]
    assert list(node_cand) == [-1, 0, 2, 3, 6, 7]
    assert list(parent) == [-1, 0, 1, 1, 2, 2]
    assert list(tok) == [99, 5, 7, 8, 11, 12]


def test_candidate_count_of_the_paper(oracle):
    Bw, D, m = GOLD["tree_breadth"], GOLD["tree_depth"], GOLD["tree_max_tokens"]
    assert Bw + (D - 1) * Bw * Bw == GOLD["tree_candidates"]
    rng = np.random.default_rng(1)

    def level(fr):
        F = 1 if fr is None or fr[0] < 0 else Bw
        return log_softmax(rng.standard_normal((F, 50)) * 2, axis=1)[:, :Bw].astype(np.float32), rng.integers(0, 1000, (F, Bw))

    parent, tok, node_cand, state, _ = build(oracle, [level] * D, m)
    assert len(parent) == 1 + m and node_cand.max() < GOLD["tree_candidates"]


def python_reference(levels_data, Bw, m, root_tok):
    """The same construction with Python lists and sorted(); float32 additions."""
    cand = []                       # (logp, tok, parent)
    frontier = []
    for l, (clp, ctk) in enumerate(levels_data, start=1):
        clp = np.minimum(np.asarray(clp, dtype=np.float32), np.float32(0))
        new = []
        rows = 1 if l == 1 else Bw
        for f in range(rows):
            for j in range(Bw):
                base = np.float32(0) if l == 1 else cand[frontier[f]][0]
                new.append((np.float32(base + clp[f, j]), int(ctk[f, j]), -1 if l == 1 else frontier[f]))
        start = len(cand)
        cand.extend(new)
        order = sorted(range(start, len(cand)), key=lambda c: (-cand[c][0], c))
        frontier = order[:Bw]
    kept = sorted(sorted(range(len(cand)), key=lambda c: (-cand[c][0], c))[:m])
    node = {c: i + 1 for i, c in enumerate(kept)}
    parent = [-1] + [0 if cand[c][2] < 0 else node[cand[c][2]] for c in kept]
    tok = [root_tok] + [cand[c][1] for c in kept]
    return parent, tok, [-1] + kept


@pytest.mark.parametrize("Bw,D,m,seed", [(2, 4, 7, 0), (3, 3, 100, 1), (4, 5, 20, 2), (8, 6, 59, 3), (8, 6, 61, 4), (5, 2, 1, 5)])
def test_matches_independent_python_construction(oracle, Bw, D, m, seed):
    rng = np.random.default_rng(seed)
    data = []
    for l in range(1, D + 1):
        F = 1 if l == 1 else Bw
        lp = np.sort(log_softmax(rng.standard_normal((F, 4 * Bw)) * 3, axis=1), axis=1)[:, ::-1][:, :Bw]
        data.append((np.ascontiguousarray(lp, dtype=np.float32), rng.integers(0, 128256, (F, Bw))))
    parent, tok, node_cand, _, _ = build(oracle, data, m, root_tok=7)
    wp, wt, wc = python_reference(data, Bw, m, 7)
    assert list(parent) == wp and list(tok) == wt and list(node_cand) == wc
    # structure: parents come first, a kept node's parent is kept, depth never decreases along the node order
    depth = [0] * len(parent)
    for i in range(1, len(parent)):
        assert 0 <= parent[i] < i
        depth[i] = depth[parent[i]] + 1
    assert depth == sorted(depth) and max(depth) <= D


def test_ties_go_to_the_lower_index_and_breadth_one_is_a_chain(oracle):
    # all expansions equally likely: the first Bw of each level stay, and the first m candidates are kept
    Bw, D = 3, 3
    eq = [(np.full((1 if l == 0 else Bw, Bw), -1.0, np.float32), np.arange((1 if l == 0 else Bw) * Bw).reshape(-1, Bw)) for l in range(D)]
    parent, tok, node_cand, _, trace = build(oracle, eq, m=5)
    assert [list(t) for t in trace] == [[0, 1, 2], [3, 4, 5], [12, 13, 14]]
    assert list(node_cand) == [-1, 0, 1, 2, 3, 4]                      # level 1 (logp -1) first, then level 2 (-2) in index order
    assert list(parent) == [-1, 0, 0, 0, 1, 1]
    chain = [(np.array([[-0.5]], np.float32), np.array([[10 + l]])) for l in range(6)]
    parent, tok, _, _, _ = build(oracle, chain, m=10)
    assert list(parent) == [-1, 0, 1, 2, 3, 4, 5] and list(tok) == [1, 10, 11, 12, 13, 14, 15]


def test_positive_log_probabilities_are_clamped(oracle):
    lv = [(np.array([[0.7, -1.0]], np.float32), np.array([[1, 2]])), (np.array([[0.3, -0.2], [-0.1, -0.4]], np.float32), np.array([[3, 4], [5, 6]]))]
    _, _, _, (lp, _, _), _ = build(oracle, lv, m=6)
    assert np.allclose(lp, [0.0, -1.0, 0.0, -0.2, -1.1, -1.4], atol=1e-6)       # a child is never more likely than its parent


def test_topk_logprob_against_library(oracle):
    rng = np.random.default_rng(9)
    logits = rng.standard_normal((5, 1000)) * 4
    logits[2, 17] = logits[2, 400] = logits[2].max() + 1.0                       # a tie for the first place
    tok, logp = oracle.topk_logprob(logits, 8)
    ref = log_softmax(logits, axis=1)
    for f in range(5):
        order = sorted(range(1000), key=lambda v: (-logits[f, v], v))[:8]
        assert list(tok[f]) == order
        assert np.allclose(logp[f], ref[f, order], atol=1e-12)
    assert list(tok[2, :2]) == [17, 400]
    assert np.allclose(np.exp(oracle.topk_logprob(logits[:1, :6], 6)[1]).sum(), 1.0, atol=1e-12)


def test_lm_head_argmax_pins(oracle):
    """One-hot head rows select a component of x, so the greedy token is the position of its largest entry; a general
    head agrees with numpy; equal logits go to the lower id."""
    rng = np.random.default_rng(21)
    x = rng.standard_normal((7, 12))
    tgt, best = oracle.lm_head_argmax(x, np.eye(12))
    assert list(tgt) == list(np.argmax(x, axis=1)) and np.allclose(best, x.max(axis=1))
    w = rng.standard_normal((300, 12))
    w[250] = w[40]                                                            # two tokens with the same logits
    tgt, best = oracle.lm_head_argmax(x, w)
    logits = x @ w.T
    assert list(tgt) == list(np.argmax(logits, axis=1)) and np.allclose(best, logits.max(axis=1), atol=1e-12)
    x2 = w[40:41] * 3.0                                                       # this row prefers token 40 = 250
    assert list(oracle.lm_head_argmax(x2, w)[0]) == [40]
