"""Pins for the oracle's draft Self-Attention layer (Sec. 3.1 "Self-Attention"; Alg. 1, q <- SA_layer(token_embed(y))).

The paper prints no numbers for it.  What its definition fixes: it is a causal self-attention over the token
sequence that leads to a node (verified tokens, then the drafted tokens on the node's own path), so
 * on a chain it is rows P.. of plain causal self-attention over all P + M embeddings (library routine, fp64);
 * on a tree, every node equals the last row of causal self-attention over prefix ++ path(root..node), computed
   here token by token with numpy;
 * level-by-level calls with a growing draft cache give what one call over the whole tree gives;
 * a drafted token is visible to its descendants and to nobody else (the reason the layer exists: cross-attention
   alone is input-independent);
 * zero query weights give the mean of the visible values; the widths of the appendix table fix 4 KV heads of 128."""
from pathlib import Path

import numpy as np
import pytest
import torch

import moa_inputs as mi

TOL = 1e-11


def rnd(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


def sa_rand(rng, B, P, M, d, H, Hkv, dh, d_out=None):
    """Embeddings of P verified and M drafted tokens per sequence, SA weights, and the cache of the verified
    tokens' keys / values (their embeddings projected, as the layer itself would have stored them)."""
    d_out = d_out or d
    a = dict(emb_prefix=rnd(rng, B, P, d), emb=rnd(rng, B, M, d), wq=rnd(rng, H * dh, d, scale=0.3),
             wk=rnd(rng, Hkv * dh, d, scale=0.3), wv=rnd(rng, Hkv * dh, d), wo=rnd(rng, d_out, H * dh, scale=0.3))
    kc = (a["emb_prefix"] @ a["wk"].T).reshape(B, P, Hkv, dh).transpose(0, 2, 1, 3)
    vc = (a["emb_prefix"] @ a["wv"].T).reshape(B, P, Hkv, dh).transpose(0, 2, 1, 3)
    a["kcache"], a["vcache"] = np.ascontiguousarray(kc), np.ascontiguousarray(vc)
    return a


def run_sa(oracle, a, parent, plen, H, Hkv, dh, node0=0, Mn=None, caches=None):
    B, M = parent.shape
    Mn = M - node0 if Mn is None else Mn
    if caches is None:
        caches = (np.zeros((B, Hkv, M, dh)), np.zeros((B, Hkv, M, dh)))
    out = oracle.self_attn_draft(a["emb"][:, node0:node0 + Mn], parent, node0, a["wq"], a["wk"], a["wv"], a["wo"],
                                 a["kcache"], a["vcache"], plen, caches[0], caches[1], H, Hkv, dh)
    return out, caches


def causal_last_row(x, wq, wk, wv, wo, H, Hkv, dh):
    """Textbook causal self-attention, last position only: x [n, d] -> [d_out]."""
    G = H // Hkv
    q = (x[-1] @ wq.T).reshape(H, dh)
    k = (x @ wk.T).reshape(-1, Hkv, dh)
    v = (x @ wv.T).reshape(-1, Hkv, dh)
    heads = []
    for h in range(H):
        s = k[:, h // G] @ q[h] / np.sqrt(dh)
        p = np.exp(s - s.max())
        p /= p.sum()
        heads.append(p @ v[:, h // G])
    return np.concatenate(heads) @ wo.T


def test_sa_chain_is_causal_self_attention_by_library(oracle):
    rng = np.random.default_rng(41)
    B, P, M, d, H, Hkv, dh = 2, 9, 7, 32, 4, 2, 8
    a = sa_rand(rng, B, P, M, d, H, Hkv, dh)
    parent = np.tile(mi.chain_tree(M), (B, 1))
    plen = np.full(B, P, dtype=np.int32)
    out, _ = run_sa(oracle, a, parent, plen, H, Hkv, dh)
    x = np.concatenate([a["emb_prefix"], a["emb"]], axis=1)                       # [B, P+M, d]
    q = torch.from_numpy((x @ a["wq"].T).reshape(B, P + M, H, dh).transpose(0, 2, 1, 3).copy())
    k = torch.from_numpy(np.repeat((x @ a["wk"].T).reshape(B, P + M, Hkv, dh).transpose(0, 2, 1, 3), H // Hkv, axis=1).copy())
    v = torch.from_numpy(np.repeat((x @ a["wv"].T).reshape(B, P + M, Hkv, dh).transpose(0, 2, 1, 3), H // Hkv, axis=1).copy())
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).numpy()
    ref = ref.transpose(0, 2, 1, 3).reshape(B, P + M, H * dh)[:, P:] @ a["wo"].T
    assert np.allclose(out, ref, atol=TOL)


@pytest.mark.parametrize("M,D,P", [(13, 4, 6), (40, 6, 0), (70, 5, 3)])
def test_sa_tree_is_causal_attention_along_each_path(oracle, M, D, P):
    rng = np.random.default_rng(100 + M)
    B, d, H, Hkv, dh = 2, 24, 4, 2, 8
    a = sa_rand(rng, B, max(P, 1), M, d, H, Hkv, dh)
    parent = np.stack([mi.gen_tree(M, D, 3, rng) for _ in range(B)])
    plen = np.array([P, max(P - 2, 0)], dtype=np.int32)
    out, (kd, vd) = run_sa(oracle, a, parent, plen, H, Hkv, dh)
    for b in range(B):
        for i in range(M):
            path = []
            j = i
            while j >= 0:
                path.append(j)
                j = parent[b, j]
            x = np.concatenate([a["emb_prefix"][b, :plen[b]], a["emb"][b, path[::-1]]], axis=0)
            ref = causal_last_row(x, a["wq"], a["wk"], a["wv"], a["wo"], H, Hkv, dh)
            assert np.allclose(out[b, i], ref, atol=TOL), (b, i)
    # the draft cache holds the nodes' own projected keys / values
    assert np.allclose(kd, (a["emb"] @ a["wk"].T).reshape(B, M, Hkv, dh).transpose(0, 2, 1, 3), atol=TOL)
    assert np.allclose(vd, (a["emb"] @ a["wv"].T).reshape(B, M, Hkv, dh).transpose(0, 2, 1, 3), atol=TOL)


def test_sa_level_by_level_equals_whole_tree(oracle):
    rng = np.random.default_rng(7)
    B, P, M, D, d, H, Hkv, dh = 2, 5, 37, 5, 24, 4, 2, 8
    a = sa_rand(rng, B, P, M, d, H, Hkv, dh)
    parent = np.stack([mi.gen_tree(M, D, 4, rng) for _ in range(B)])
    plen = np.array([P, P - 1], dtype=np.int32)
    whole, (kw, vw) = run_sa(oracle, a, parent, plen, H, Hkv, dh)
    # trees are labelled in depth order, so a level is a node range (the same for every sequence only if the level
    # sizes agree; cut at arbitrary points instead: any cut keeps ancestors before descendants)
    caches = (np.full((B, Hkv, M, dh), np.nan), np.full((B, Hkv, M, dh), np.nan))
    pieces = []
    cuts = [0, 1, 4, 5, 19, 30, M]
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        o, caches = run_sa(oracle, a, parent, plen, H, Hkv, dh, node0=lo, Mn=hi - lo, caches=caches)
        pieces.append(o)
    assert np.array_equal(np.concatenate(pieces, axis=1), whole)
    assert np.array_equal(caches[0], kw) and np.array_equal(caches[1], vw)


def test_sa_a_drafted_token_is_seen_by_its_descendants_only(oracle):
    rng = np.random.default_rng(11)
    B, P, M, D, d, H, Hkv, dh = 1, 4, 25, 4, 16, 2, 1, 8
    a = sa_rand(rng, B, P, M, d, H, Hkv, dh)
    parent = mi.gen_tree(M, D, 3, rng)[None]
    plen = np.array([P], dtype=np.int32)
    base, _ = run_sa(oracle, a, parent, plen, H, Hkv, dh)
    for j in (0, 2, 7, M - 1):
        b2 = dict(a)
        b2["emb"] = a["emb"].copy()
        b2["emb"][0, j] += 1.0
        got, _ = run_sa(oracle, b2, parent, plen, H, Hkv, dh)
        changed = np.abs(got - base).max(axis=2)[0] > 1e-9
        desc = np.zeros(M, dtype=bool)
        for i in range(M):
            k = i
            while k >= 0:
                if k == j:
                    desc[i] = True
                k = parent[0, k]
        assert np.array_equal(changed, desc), j


def test_sa_zero_query_weight_is_mean_of_visible_values(oracle):
    rng = np.random.default_rng(13)
    B, P, M, d, H, Hkv, dh = 1, 3, 9, 16, 4, 2, 4
    a = sa_rand(rng, B, P, M, d, H, Hkv, dh)
    a["wq"] = np.zeros_like(a["wq"])
    parent = mi.star_tree(M)[None]
    plen = np.array([P], dtype=np.int32)
    out, _ = run_sa(oracle, a, parent, plen, H, Hkv, dh)
    v_all = np.concatenate([a["emb_prefix"][0], a["emb"][0]]) @ a["wv"].T          # [P+M, Hkv*dh]
    for i in range(M):
        vis = list(range(P)) + ([P] if i == 0 else [P, P + i])                     # star: root and the leaf itself
        mean = v_all[vis].mean(axis=0).reshape(Hkv, dh)
        heads = np.concatenate([mean[h // (H // Hkv)] for h in range(H)])
        assert np.allclose(out[0, i], heads @ a["wo"].T, atol=TOL)


def test_sa_widths_of_the_paper_give_four_kv_heads(oracle):
    gold = {}
    for line in (Path(__file__).parent / "golden" / "paper_hyperparameters.txt").read_text().splitlines():
        if line and not line.startswith("#"):
            k, v = line.split()
            gold[k] = int(v)
    cfg = mi.CONFIGS["C1"]
    assert gold["sa_embed"] == cfg.d and gold["sa_kv_embed"] == mi.sa_kv_heads(cfg) * cfg.dh
    assert mi.sa_kv_heads(cfg) == 4 and cfg.H % mi.sa_kv_heads(cfg) == 0


def test_sa_rejects_bad_arguments(oracle):
    rng = np.random.default_rng(3)
    B, P, M, d, H, Hkv, dh = 1, 2, 5, 8, 2, 1, 4
    a = sa_rand(rng, B, P, M, d, H, Hkv, dh)
    plen = np.array([P], dtype=np.int32)
    bad_parent = np.array([[-1, 0, 3, 1, 2]], dtype=np.int32)                      # node 2 names a later node
    with pytest.raises(oracle.OracleError):
        run_sa(oracle, a, bad_parent, plen, H, Hkv, dh)
    z = np.zeros((B, Hkv, M, dh))
    with pytest.raises(oracle.OracleError):                                        # nodes 3..6 of a 5-node tree
        oracle.self_attn_draft(a["emb"][:, :4], np.tile(mi.chain_tree(M), (B, 1)), 3, a["wq"], a["wk"], a["wv"], a["wo"],
                               a["kcache"], a["vcache"], plen, z, z.copy(), H, Hkv, dh)
