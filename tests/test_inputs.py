"""Input recipe checks: shapes the paper fixes (tests/golden/paper_hyperparameters.txt) and
structural guarantees of the seeded generators."""
from pathlib import Path

import numpy as np
import pytest

import moa_inputs as mi

GOLD = {}
for line in (Path(__file__).parent / "golden" / "paper_hyperparameters.txt").read_text().splitlines():
    if line and not line.startswith("#"):
        k, v = line.split()
        GOLD[k] = int(v)


def test_llama8b_config_matches_paper_table():
    c = mi.CONFIGS["C1"]
    assert c.L == GOLD["L"] and c.d == GOLD["E"] and c.E_kv == GOLD["E_kv"]
    # LSA works on K||V of one layer: width 2*E_kv = the table's LSA embedding size
    assert c.d_lsa_in == 2 * GOLD["E_kv"] == GOLD["lsa_embed"]
    assert c.E_kv == GOLD["lsa_kv_embed"] == GOLD["ca_kv_embed"]
    assert c.H * c.dh == GOLD["ca_embed"]


def test_candidate_count_formula():
    B, D = GOLD["tree_breadth"], GOLD["tree_depth"]
    assert B + (D - 1) * B * B == GOLD["tree_candidates"]


@pytest.mark.parametrize("seed", range(5))
def test_beam_tree_shape(seed):
    rng = np.random.default_rng(seed)
    m = GOLD["tree_max_tokens"]
    par = mi.beam_tree(GOLD["tree_breadth"], GOLD["tree_depth"], m, rng)
    assert len(par) == m and par[0] == -1
    assert all(0 <= par[i] < i for i in range(1, m))
    depth = np.zeros(m, dtype=int)
    for i in range(1, m):
        depth[i] = depth[par[i]] + 1
    assert depth.max() <= GOLD["tree_depth"]
    assert np.bincount(par[1:], minlength=m).max() <= GOLD["tree_breadth"]


@pytest.mark.parametrize("name", ["C0", "C1", "C2", "C3", "C4"])
def test_gen_tree_limits(name):
    c = mi.CONFIGS[name]
    par = mi.trees(c)
    assert par.shape == (c.B, c.M)
    for b in range(c.B):
        p = par[b]
        assert p[0] == -1 and all(0 <= p[i] < i for i in range(1, c.M))
        depth = np.zeros(c.M, dtype=int)
        for i in range(1, c.M):
            depth[i] = depth[p[i]] + 1
        assert depth.max() == c.D
        assert np.bincount(p[1:], minlength=c.M).max() <= c.max_branch
        assert np.all(np.diff(depth) >= 0)          # relabelled in depth order


def test_tokens_siblings_distinct():
    c = mi.CONFIGS["C2"]
    par = mi.trees(c)
    tok, tgt = mi.tokens(c, par)
    for b in range(c.B):
        for p in range(c.M):
            kids = np.nonzero(par[b] == p)[0]
            assert len(set(tok[b, kids])) == len(kids)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.14159], dtype=np.float32)
    q = mi.quantize(x, "bf16")
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even mantissa (1.0); 1+3*2^-8 ties up to 1+2^-6
    assert q[0] == 1.0 and q[1] == 1.0 and q[2] == 1.0 + 2 ** -7 and q[3] == 1.0 + 2 ** -6
    assert np.all(np.abs(q - x) <= np.abs(x) * 2 ** -8)
    assert np.array_equal(mi.quantize(q, "bf16"), q)


def test_seeds_are_reproducible_and_ragged():
    c = mi.CONFIGS["C2"]
    p1, p2 = mi.prefix_lengths(c), mi.prefix_lengths(c)
    assert np.array_equal(p1, p2) and p1.min() >= 512 and p1.max() <= 2048 and len(set(p1)) > 1


@pytest.mark.parametrize("lsa_tokens,per_seq", [("tree", None), ("prefix", None), (5, 5)])
def test_step_workload_lsa_token_regimes(lsa_tokens, per_seq):
    """The three token counts the Layer Self-Attention sees (Alg. 1: whole prompt first, then what the last cycle
    verified): rows of the LSA input, the per-sequence offsets and the memory length before the append must agree."""
    cfg = mi.Config(name="R", index=12, dtype="f32", B=3, P_min=20, P_max=50, M=9, D=3, max_branch=3, L=2,
                    d=128, H=2, Hkv=2, dh=64, d_lsa_in=128, rms_norm=False)
    w = mi.step_workload(cfg, 1, lsa_tokens=lsa_tokens)
    plen = w["prefix_len"].astype(np.int64)
    new = {"tree": np.full(cfg.B, cfg.M), "prefix": plen}.get(lsa_tokens, np.full(cfg.B, per_seq))
    assert w["lsa_hs"].shape == (int(new.sum()), cfg.L, cfg.d_lsa_in)
    assert np.array_equal(w["tok_off"], np.concatenate([[0], np.cumsum(new)]))
    assert np.array_equal(w["ca_len0"] + new, plen)
    with pytest.raises(ValueError):
        mi.step_workload(cfg, 1, lsa_tokens=int(plen.min()) + 1)
