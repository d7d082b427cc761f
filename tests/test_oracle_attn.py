"""Pins for the oracle's floating-point functions (LSA with mean, CA, tree verification).

The paper prints no numeric example for them, so they are pinned by what its definitions
fix: closed forms of special cases, invariances, a library attention routine
(torch.nn.functional.scaled_dot_product_attention on CPU in fp64), token-by-token
sequential decoding, and the softmax normalisation."""
import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

import moa_inputs as mi

TOL = 1e-11


def rnd(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


def sdpa(q, k, v, mask=None):
    """Library routine: q [.., n, dh], k/v [.., m, dh] in fp64."""
    q, k, v = (torch.from_numpy(np.ascontiguousarray(a)) for a in (q, k, v))
    m = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask))
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m).numpy()


# ------------------------------------------------------------------ softmax primitive

def test_softmax_rows_sum_to_one_and_match_library(oracle):
    rng = np.random.default_rng(0)
    for n in (1, 2, 7, 64, 1000):
        s = rnd(rng, n, scale=5.0)
        p, psum = oracle.softmax_weighted_sum(s, np.eye(n))     # identity values -> the probabilities
        assert abs(psum - 1.0) < 1e-12 and np.all(p >= 0)
        assert np.allclose(p, sp_softmax(s), atol=1e-15)
    # huge scores must not overflow (max subtraction)
    p, psum = oracle.softmax_weighted_sum(np.array([1000.0, 999.0]), np.eye(2))
    assert abs(psum - 1) < 1e-12 and abs(p[0] - 1 / (1 + np.exp(-1))) < 1e-14


@pytest.mark.parametrize("chunk", [1, 3, 32, 64, 1000])
def test_chunked_merge_equals_two_pass(oracle, chunk):
    rng = np.random.default_rng(chunk)
    s, v = rnd(rng, 333, scale=4.0), rnd(rng, 333, 16)
    full, _ = oracle.softmax_weighted_sum(s, v)
    assert np.allclose(oracle.softmax_weighted_sum_chunked(s, v, chunk), full, atol=1e-13)


# ------------------------------------------------------------------ LSA

LSA_SHAPE = dict(T=3, L=5, d_in=24, Hq=4, Hkv=2, dh=8)


def lsa_rand(rng, T, L, d_in, Hq, Hkv, dh, d_out=None):
    d_out = d_out or Hq * dh
    return dict(hs=rnd(rng, T, L, d_in), wq=rnd(rng, Hq * dh, d_in, scale=0.3), wk=rnd(rng, Hkv * dh, d_in, scale=0.3),
                wv=rnd(rng, Hkv * dh, d_in), wo=rnd(rng, d_out, Hq * dh))


def run_lsa(oracle, a, Hq, Hkv, dh):
    return oracle.lsa(a["hs"], a["wq"], a["wk"], a["wv"], a["wo"], Hq, Hkv, dh)


def test_lsa_single_layer_is_projected_value(oracle):
    """L = 1: the softmax over one score is 1, so out = Wo * repeat_G(Wv x)."""
    rng = np.random.default_rng(1)
    s = dict(LSA_SHAPE, L=1)
    a = lsa_rand(rng, **s, d_out=20)
    out = run_lsa(oracle, a, s["Hq"], s["Hkv"], s["dh"])
    G = s["Hq"] // s["Hkv"]
    for t in range(s["T"]):
        v = a["wv"] @ a["hs"][t, 0]                                        # [Hkv*dh]
        concat = np.concatenate([v[(h // G) * s["dh"]:(h // G + 1) * s["dh"]] for h in range(s["Hq"])])
        assert np.allclose(out[t], a["wo"] @ concat, atol=TOL)


def test_lsa_zero_query_weight_is_uniform_average(oracle):
    """Wq = 0: uniform attention -> out = Wo * repeat_G(Wv * mean_l x_l); V differs per KV head."""
    rng = np.random.default_rng(2)
    s = LSA_SHAPE
    a = lsa_rand(rng, **s)
    a["wq"][:] = 0
    out = run_lsa(oracle, a, s["Hq"], s["Hkv"], s["dh"])
    G = s["Hq"] // s["Hkv"]
    for t in range(s["T"]):
        v = a["wv"] @ a["hs"][t].mean(axis=0)
        concat = np.concatenate([v[(h // G) * s["dh"]:(h // G + 1) * s["dh"]] for h in range(s["Hq"])])
        assert np.allclose(out[t], a["wo"] @ concat, atol=TOL)


def test_lsa_identical_layers_and_layer_permutation(oracle):
    rng = np.random.default_rng(3)
    s = LSA_SHAPE
    a = lsa_rand(rng, **s)
    base = run_lsa(oracle, a, s["Hq"], s["Hkv"], s["dh"])
    # full mask, no positions on the layer axis: permuting layers changes nothing
    perm = rng.permutation(s["L"])
    b = dict(a, hs=a["hs"][:, perm])
    assert np.allclose(run_lsa(oracle, b, s["Hq"], s["Hkv"], s["dh"]), base, atol=TOL)
    # all layers equal -> same as one layer
    c = dict(a, hs=np.repeat(a["hs"][:, :1], s["L"], axis=1))
    d = dict(a, hs=a["hs"][:, :1])
    assert np.allclose(run_lsa(oracle, c, s["Hq"], s["Hkv"], s["dh"]),
                       run_lsa(oracle, d, s["Hq"], s["Hkv"], s["dh"]), atol=TOL)
    # tokens are independent: a token alone gives its own row
    e = dict(a, hs=a["hs"][1:2])
    assert np.allclose(run_lsa(oracle, e, s["Hq"], s["Hkv"], s["dh"])[0], base[1], atol=TOL)


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (4, 4), (6, 1)])
def test_lsa_matches_library_attention(oracle, Hq, Hkv):
    """Bidirectional attention over the layer axis by the library routine, then Wo, then the mean."""
    rng = np.random.default_rng(4)
    T, L, d_in, dh, d_out = 4, 7, 20, 8, 12
    a = lsa_rand(rng, T, L, d_in, Hq, Hkv, dh, d_out)
    out = run_lsa(oracle, a, Hq, Hkv, dh)
    G = Hq // Hkv
    q = (a["hs"] @ a["wq"].T).reshape(T, L, Hq, dh).transpose(0, 2, 1, 3)
    k = (a["hs"] @ a["wk"].T).reshape(T, L, Hkv, dh).transpose(0, 2, 1, 3).repeat(G, axis=1)
    v = (a["hs"] @ a["wv"].T).reshape(T, L, Hkv, dh).transpose(0, 2, 1, 3).repeat(G, axis=1)
    o = sdpa(q, k, v).transpose(0, 2, 1, 3).reshape(T, L, Hq * dh)
    want = (o @ a["wo"].T).mean(axis=1)
    assert np.allclose(out, want, atol=TOL)


def test_lsa_identity_weights(oracle):
    rng = np.random.default_rng(5)
    T, L, dh = 2, 6, 8
    hs = rnd(rng, T, L, dh)
    out = oracle.lsa(hs, None, None, None, None, 1, 1, dh)
    want = sdpa(hs, hs, hs).mean(axis=1)
    assert np.allclose(out, want, atol=TOL)


# ------------------------------------------------------------------ CA

def ca_rand(rng, B, Mq, d, H, Hkv, dh, P_cap, d_out=None):
    E = H * dh
    return dict(xq=rnd(rng, B, Mq, d), wq=rnd(rng, E, d, scale=0.3), wo=rnd(rng, d_out or d, E),
                kc=rnd(rng, B, Hkv, P_cap, dh), vc=rnd(rng, B, Hkv, P_cap, dh))


def test_ca_matches_library_and_ignores_rows_past_len(oracle):
    rng = np.random.default_rng(10)
    B, Mq, d, H, Hkv, dh, P_cap = 3, 5, 24, 4, 2, 8, 19
    a = ca_rand(rng, B, Mq, d, H, Hkv, dh, P_cap, d_out=10)
    ca_len = np.array([19, 1, 7], dtype=np.int32)
    out = oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], ca_len, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        n = ca_len[b]
        q = (a["xq"][b] @ a["wq"].T).reshape(Mq, H, dh).transpose(1, 0, 2)
        k = a["kc"][b, :, :n].repeat(G, axis=0)
        v = a["vc"][b, :, :n].repeat(G, axis=0)
        o = sdpa(q, k, v).transpose(1, 0, 2).reshape(Mq, H * dh)
        assert np.allclose(out[b], o @ a["wo"].T, atol=TOL)
    # rows beyond ca_len never matter
    a["kc"][0, :, 19:] = 1e6
    a["kc"][2, :, 7:] += 100.0
    a["vc"][2, :, 7:] -= 50.0
    out2 = oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], ca_len, H, Hkv, dh)
    assert np.array_equal(out, out2)


def test_ca_input_independence_and_single_key(oracle):
    """Input-independence property of the CA layer: a batch of queries equals the queries one by one.
    With one cached row every query returns Wo * repeat_G(Vc[0])."""
    rng = np.random.default_rng(11)
    B, Mq, d, H, Hkv, dh, P_cap = 2, 6, 16, 4, 2, 8, 9
    a = ca_rand(rng, B, Mq, d, H, Hkv, dh, P_cap)
    ca_len = np.array([9, 4], dtype=np.int32)
    out = oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], ca_len, H, Hkv, dh)
    for m in range(Mq):
        one = oracle.cross_attn(a["xq"][:, m:m + 1], a["wq"], a["wo"], a["kc"], a["vc"], ca_len, H, Hkv, dh)
        assert np.allclose(one[:, 0], out[:, m], atol=TOL)
    ones = np.ones(B, dtype=np.int32)
    out1 = oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], ones, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        concat = np.concatenate([a["vc"][b, h // G, 0] for h in range(H)])
        assert np.allclose(out1[b], np.tile(a["wo"] @ concat, (Mq, 1)), atol=TOL)


def test_ca_zero_query_weight_is_mean_of_values(oracle):
    rng = np.random.default_rng(12)
    B, Mq, d, H, Hkv, dh, P_cap = 2, 3, 16, 4, 2, 8, 11
    a = ca_rand(rng, B, Mq, d, H, Hkv, dh, P_cap)
    a["wq"][:] = 0
    ca_len = np.array([11, 5], dtype=np.int32)
    out = oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], ca_len, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        concat = np.concatenate([a["vc"][b, h // G, :ca_len[b]].mean(axis=0) for h in range(H)])
        assert np.allclose(out[b], np.tile(a["wo"] @ concat, (Mq, 1)), atol=TOL)


def test_ca_empty_memory_is_an_error(oracle):
    rng = np.random.default_rng(13)
    a = ca_rand(rng, 1, 2, 16, 2, 2, 8, 4)
    with pytest.raises(oracle.OracleError) as e:
        oracle.cross_attn(a["xq"], a["wq"], a["wo"], a["kc"], a["vc"], np.zeros(1, np.int32), 2, 2, 8)
    assert e.value.code == oracle.EMPTY


def test_ca_kv_append_projects_and_places_rows(oracle):
    rng = np.random.default_rng(14)
    B, Hkv, dh, d_mem, P_cap = 3, 2, 4, 10, 12
    wk, wv = rnd(rng, Hkv * dh, d_mem), rnd(rng, Hkv * dh, d_mem)
    kc = np.full((B, Hkv, P_cap, dh), 777.0)
    vc = np.full((B, Hkv, P_cap, dh), 888.0)
    ca_len = np.array([0, 5, 9], dtype=np.int32)
    tok_off = np.array([0, 4, 4, 7], dtype=np.int32)             # 4, 0 and 3 new rows
    mem = rnd(rng, 7, d_mem)
    oracle.ca_kv_append(mem, tok_off, wk, wv, kc, vc, ca_len, Hkv, dh)
    assert list(ca_len) == [4, 5, 12]
    K, V = mem @ wk.T, mem @ wv.T
    for b, (start, rows) in enumerate([(0, range(0, 4)), (5, range(0)), (9, range(4, 7))]):
        for i, r in enumerate(rows):
            for g in range(Hkv):
                assert np.allclose(kc[b, g, start + i], K[r, g * dh:(g + 1) * dh], atol=TOL)
                assert np.allclose(vc[b, g, start + i], V[r, g * dh:(g + 1) * dh], atol=TOL)
    untouched = np.ones((B, P_cap), dtype=bool)
    untouched[0, 0:4] = False
    untouched[2, 9:12] = False
    assert np.all(kc.transpose(0, 2, 1, 3)[untouched] == 777.0) and np.all(vc.transpose(0, 2, 1, 3)[untouched] == 888.0)
    with pytest.raises(oracle.OracleError):                      # overflow of the cache
        oracle.ca_kv_append(mem, tok_off, wk, wv, kc, vc, ca_len, Hkv, dh)


# ------------------------------------------------------------------ tree verification

def verify_rand(rng, B, M, d, H, Hkv, dh, P_cap, d_out=None):
    E, Ekv = H * dh, Hkv * dh
    return dict(x=rnd(rng, B, M, d), wq=rnd(rng, E, d, scale=0.3), wk=rnd(rng, Ekv, d, scale=0.3),
                wv=rnd(rng, Ekv, d), wo=rnd(rng, d_out or d, E),
                kc=rnd(rng, B, Hkv, P_cap, dh), vc=rnd(rng, B, Hkv, P_cap, dh))


def run_verify(oracle, a, plen, mask, H, Hkv, dh):
    return oracle.tree_verify_attn(a["x"], a["wq"], a["wk"], a["wv"], a["wo"], a["kc"], a["vc"], plen, mask, H, Hkv, dh)


def walk_mask(par):
    """Boolean [M, M] visibility by explicit ancestor walks (independent of the bitset code)."""
    M = len(par)
    vis = np.zeros((M, M), dtype=bool)
    for i in range(M):
        j = i
        while j >= 0:
            vis[i, j] = True
            j = par[j]
    return vis


def test_verify_chain_is_causal_attention(oracle):
    """A chain-shaped tree is plain causal attention over prefix ++ chain."""
    rng = np.random.default_rng(20)
    B, M, d, H, Hkv, dh, P = 2, 7, 24, 4, 2, 8, 13
    a = verify_rand(rng, B, M, d, H, Hkv, dh, P + 3, d_out=9)
    par = np.stack([mi.chain_tree(M)] * B)
    mask, _ = oracle.tree_build(par)
    plen = np.array([P, 5], dtype=np.int32)
    out, kt, vt = run_verify(oracle, a, plen, mask, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        n = plen[b]
        q = (a["x"][b] @ a["wq"].T).reshape(M, H, dh).transpose(1, 0, 2)
        knew = (a["x"][b] @ a["wk"].T).reshape(M, Hkv, dh).transpose(1, 0, 2)
        vnew = (a["x"][b] @ a["wv"].T).reshape(M, Hkv, dh).transpose(1, 0, 2)
        assert np.allclose(kt[b], knew, atol=TOL) and np.allclose(vt[b], vnew, atol=TOL)
        k = np.concatenate([a["kc"][b, :, :n], knew], axis=1).repeat(G, axis=0)
        v = np.concatenate([a["vc"][b, :, :n], vnew], axis=1).repeat(G, axis=0)
        # textbook causal rule: query at absolute position n+i sees positions <= n+i
        causal = np.arange(n + M)[None, :] <= (n + np.arange(M))[:, None]
        o = sdpa(q, k, v, np.broadcast_to(causal, (H, M, n + M))).transpose(1, 0, 2).reshape(M, H * dh)
        assert np.allclose(out[b], o @ a["wo"].T, atol=TOL)


@pytest.mark.parametrize("M,Dmax", [(12, 4), (70, 9)])
def test_verify_tree_is_sequential_decoding(oracle, M, Dmax):
    """Every node's row equals token-by-token decoding along its root path: append the K/V of each
    path node to the cache, then attend with the last one.  Written with plain numpy, one token at a time."""
    rng = np.random.default_rng(21)
    B, d, H, Hkv, dh = 2, 16, 4, 2, 8
    plen = np.array([6, 0], dtype=np.int32)            # second sequence: empty prefix (tree-only keys)
    a = verify_rand(rng, B, M, d, H, Hkv, dh, 6)
    par = np.stack([mi.gen_tree(M, Dmax, 3, rng) for _ in range(B)])
    mask, _ = oracle.tree_build(par)
    out, _, _ = run_verify(oracle, a, plen, mask, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        for i in range(M):
            path = []
            j = i
            while j >= 0:
                path.append(j)
                j = par[b, j]
            path.reverse()
            kcache = [a["kc"][b, :, p] for p in range(plen[b])]      # list of [Hkv, dh]
            vcache = [a["vc"][b, :, p] for p in range(plen[b])]
            last = None
            for node in path:                                        # decode one token at a time
                xt = a["x"][b, node]
                kcache.append((a["wk"] @ xt).reshape(Hkv, dh))
                vcache.append((a["wv"] @ xt).reshape(Hkv, dh))
                qt = (a["wq"] @ xt).reshape(H, dh)
                Kc, Vc = np.stack(kcache, axis=1), np.stack(vcache, axis=1)   # [Hkv, n, dh]
                heads = []
                for h in range(H):
                    w = sp_softmax(Kc[h // G] @ qt[h] / np.sqrt(dh))
                    heads.append(w @ Vc[h // G])
                last = a["wo"] @ np.concatenate(heads)
            assert np.allclose(out[b, i], last, atol=TOL)


def test_verify_random_tree_matches_library_with_walked_mask(oracle):
    rng = np.random.default_rng(22)
    B, M, d, H, Hkv, dh, P_cap = 2, 66, 24, 6, 3, 8, 10     # M > 64: two mask words
    a = verify_rand(rng, B, M, d, H, Hkv, dh, P_cap)
    par = np.stack([mi.gen_tree(M, 8, 4, rng) for _ in range(B)])
    mask, _ = oracle.tree_build(par)
    plen = np.array([10, 3], dtype=np.int32)
    out, _, _ = run_verify(oracle, a, plen, mask, H, Hkv, dh)
    G = H // Hkv
    for b in range(B):
        n = plen[b]
        q = (a["x"][b] @ a["wq"].T).reshape(M, H, dh).transpose(1, 0, 2)
        knew = (a["x"][b] @ a["wk"].T).reshape(M, Hkv, dh).transpose(1, 0, 2)
        vnew = (a["x"][b] @ a["wv"].T).reshape(M, Hkv, dh).transpose(1, 0, 2)
        k = np.concatenate([a["kc"][b, :, :n], knew], axis=1).repeat(G, axis=0)
        v = np.concatenate([a["vc"][b, :, :n], vnew], axis=1).repeat(G, axis=0)
        vis = np.concatenate([np.ones((M, n), dtype=bool), walk_mask(par[b])], axis=1)
        o = sdpa(q, k, v, np.broadcast_to(vis, (H, M, n + M))).transpose(1, 0, 2).reshape(M, H * dh)
        assert np.allclose(out[b], o @ a["wo"].T, atol=TOL)


def test_verify_zero_query_weight_is_mean_over_visible_set(oracle):
    rng = np.random.default_rng(23)
    B, M, d, H, Hkv, dh, P = 1, 9, 16, 4, 2, 8, 5
    a = verify_rand(rng, B, M, d, H, Hkv, dh, P)
    a["wq"][:] = 0
    par = mi.gen_tree(M, 3, 3, rng)[None]
    mask, _ = oracle.tree_build(par)
    out, _, vt = run_verify(oracle, a, np.array([P], np.int32), mask, H, Hkv, dh)
    vis = walk_mask(par[0])
    G = H // Hkv
    for i in range(M):
        concat = np.concatenate([np.concatenate([a["vc"][0, h // G, :P], vt[0, h // G][vis[i]]]).mean(axis=0)
                                 for h in range(H)])
        assert np.allclose(out[0, i], a["wo"] @ concat, atol=TOL)


def test_verify_gqa_equals_mha_with_replicated_heads(oracle):
    rng = np.random.default_rng(24)
    B, M, d, H, Hkv, dh, P = 1, 6, 16, 4, 2, 8, 7
    a = verify_rand(rng, B, M, d, H, Hkv, dh, P)
    par = mi.gen_tree(M, 2, 3, rng)[None]
    mask, _ = oracle.tree_build(par)
    plen = np.array([P], np.int32)
    out, _, _ = run_verify(oracle, a, plen, mask, H, Hkv, dh)
    G = H // Hkv
    rep = lambda w: w.reshape(Hkv, dh, d).repeat(G, axis=0).reshape(H * dh, d)
    b2 = dict(a, wk=rep(a["wk"]), wv=rep(a["wv"]), kc=a["kc"].repeat(G, axis=1), vc=a["vc"].repeat(G, axis=1))
    out2, _, _ = run_verify(oracle, b2, plen, mask, H, H, dh)
    assert np.allclose(out, out2, atol=TOL)


def test_verify_root_alone_with_empty_prefix_returns_its_own_value(oracle):
    rng = np.random.default_rng(25)
    d, H, Hkv, dh = 16, 2, 1, 8
    a = verify_rand(rng, 1, 1, d, H, Hkv, dh, 1)
    mask, _ = oracle.tree_build(np.array([[-1]], np.int32))
    out, _, vt = run_verify(oracle, a, np.array([0], np.int32), mask, H, Hkv, dh)
    assert np.allclose(out[0, 0], a["wo"] @ np.tile(vt[0, 0, 0], H), atol=TOL)


def test_verify_preprojected_inputs(oracle):
    """NULL weights: the input is taken as already projected (H*dh == Hkv*dh == d here)."""
    rng = np.random.default_rng(26)
    B, M, dh, P = 1, 5, 8, 4
    x = rnd(rng, B, M, dh)
    kc, vc = rnd(rng, B, 1, P, dh), rnd(rng, B, 1, P, dh)
    par = mi.chain_tree(M)[None]
    mask, _ = oracle.tree_build(par)
    out, kt, vt = oracle.tree_verify_attn(x, None, None, None, None, kc, vc, np.array([P], np.int32), mask, 1, 1, dh)
    assert np.array_equal(kt[0, 0], x[0]) and np.array_equal(vt[0, 0], x[0])
    k = np.concatenate([kc[0, 0], x[0]])
    v = np.concatenate([vc[0, 0], x[0]])
    causal = np.arange(P + M)[None, :] <= (P + np.arange(M))[:, None]
    assert np.allclose(out[0], sdpa(x[0], k, v, causal), atol=TOL)
