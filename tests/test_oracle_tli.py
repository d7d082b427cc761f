"""Pins for the oracle's reused decoder layer under Target Layer Inference (Sec. 3.2: the last layers of the LLM,
f^l_decoder, run on the drafted tokens with their KV cache of the verified ones).

The paper prints no numbers; the layer is the LLM's own (a Llama-family pre-norm block), so it is pinned by
 * rotary embedding: norm preserved, identity at position 0, scores depend on the position difference only, and
   equality with multiplication by exp(i * pos * theta_c) in complex arithmetic;
 * on a chain, rows P.. of the same layer evaluated on the whole sequence with library routines in fp64
   (torch rms_norm, scaled_dot_product_attention with is_causal, silu);
 * on a tree, every node equals the last row of that library evaluation over prefix ++ path(root..node);
 * level-by-level calls equal one call over the whole tree; zero W_o and W_down make the layer the identity."""
import numpy as np
import pytest
import torch

import moa_inputs as mi

TOL = 1e-10
EPS, THETA = 1e-5, 10000.0


def rnd(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


def layer_rand(rng, d, H, Hkv, dh, d_ff):
    return dict(g_attn=1.0 + 0.1 * rnd(rng, d), wq=rnd(rng, H * dh, d, scale=0.3), wk=rnd(rng, Hkv * dh, d, scale=0.3),
                wv=rnd(rng, Hkv * dh, d, scale=0.5), wo=rnd(rng, d, H * dh, scale=0.2), g_mlp=1.0 + 0.1 * rnd(rng, d),
                w_gate=rnd(rng, d_ff, d, scale=0.3), w_up=rnd(rng, d_ff, d, scale=0.3), w_down=rnd(rng, d, d_ff, scale=0.2))


def rope_complex(x, pos, dh):
    """x [..., n, dh], pos [n]: the rotation as a complex product, pairs (c, c + dh/2)."""
    half = dh // 2
    inv = torch.tensor(THETA, dtype=torch.float64) ** (-2.0 * torch.arange(half, dtype=torch.float64) / dh)
    ang = pos.to(torch.float64)[:, None] * inv[None, :]
    z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], dim=-1)


def library_layer(x, w, H, Hkv, dh):
    """The block on one whole sequence x [n, d] with library routines; returns out [n, d] and the rotated keys and
    the values [n, Hkv, dh] (what a KV cache of this layer holds)."""
    F = torch.nn.functional
    t = {k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in w.items()}
    x = torch.from_numpy(np.ascontiguousarray(x))
    n, d = x.shape
    pos = torch.arange(n)
    n1 = F.rms_norm(x, (d,), weight=t["g_attn"], eps=EPS)
    q = (n1 @ t["wq"].T).view(n, H, dh).transpose(0, 1)
    k = (n1 @ t["wk"].T).view(n, Hkv, dh).transpose(0, 1)
    v = (n1 @ t["wv"].T).view(n, Hkv, dh).transpose(0, 1)
    q, k = rope_complex(q, pos, dh), rope_complex(k, pos, dh)
    kk, vv = k.repeat_interleave(H // Hkv, dim=0), v.repeat_interleave(H // Hkv, dim=0)
    a = F.scaled_dot_product_attention(q[None], kk[None], vv[None], is_causal=True)[0]
    h1 = x + a.transpose(0, 1).reshape(n, H * dh) @ t["wo"].T
    n2 = F.rms_norm(h1, (d,), weight=t["g_mlp"], eps=EPS)
    out = h1 + (F.silu(n2 @ t["w_gate"].T) * (n2 @ t["w_up"].T)) @ t["w_down"].T
    return out.numpy(), k.transpose(0, 1).numpy(), v.transpose(0, 1).numpy()


def cache_from(ks, vs, P_cap):
    """[P, Hkv, dh] -> [1, Hkv, P_cap, dh]"""
    P, Hkv, dh = ks.shape
    kc = np.zeros((1, Hkv, P_cap, dh))
    vc = np.zeros((1, Hkv, P_cap, dh))
    kc[0, :, :P], vc[0, :, :P] = ks.transpose(1, 0, 2), vs.transpose(1, 0, 2)
    return kc, vc


def run_layer(oracle, x, parent, w, kc, vc, plen, H, Hkv, dh, node0=0, Mn=None, caches=None):
    B, M = parent.shape
    Mn = M - node0 if Mn is None else Mn
    if caches is None:
        caches = (np.zeros((B, Hkv, M, dh)), np.zeros((B, Hkv, M, dh)))
    out = oracle.tli_decoder_layer(x[:, node0:node0 + Mn], parent, node0, w, kc, vc, plen, caches[0], caches[1],
                                   H, Hkv, dh, EPS, THETA)
    return out, caches


def test_rope_properties(oracle):
    rng = np.random.default_rng(5)
    dh = 16
    q, k = rnd(rng, dh), rnd(rng, dh)
    assert np.array_equal(oracle.rope(q, 0, THETA), q)
    for pos in (1, 7, 1000, 32768 + 6):
        r = oracle.rope(q, pos, THETA)
        assert abs(np.linalg.norm(r) - np.linalg.norm(q)) < 1e-12
        want = rope_complex(torch.from_numpy(q)[None, None], torch.tensor([pos]), dh)[0, 0].numpy()
        assert np.allclose(r, want, atol=1e-12)
    base = oracle.rope(q, 40, THETA) @ oracle.rope(k, 33, THETA)
    for shift in (1, 10, 500):
        assert abs(oracle.rope(q, 40 + shift, THETA) @ oracle.rope(k, 33 + shift, THETA) - base) < 1e-10
    assert abs(oracle.rope(q, 41, THETA) @ oracle.rope(k, 33, THETA) - base) > 1e-6       # and not on the sum


def test_tli_chain_is_the_layer_on_the_whole_sequence_by_library(oracle):
    rng = np.random.default_rng(17)
    P, M, d, H, Hkv, dh, d_ff = 11, 6, 32, 4, 2, 8, 48
    w = layer_rand(rng, d, H, Hkv, dh, d_ff)
    x_all = rnd(rng, P + M, d)
    ref, ks, vs = library_layer(x_all, w, H, Hkv, dh)
    kc, vc = cache_from(ks[:P], vs[:P], P + 3)
    out, (kd, vd) = run_layer(oracle, x_all[None, P:], mi.chain_tree(M)[None], w, kc, vc, np.array([P], dtype=np.int32),
                              H, Hkv, dh)
    assert np.allclose(out[0], ref[P:], atol=TOL)
    assert np.allclose(kd[0], ks[P:].transpose(1, 0, 2), atol=TOL)          # the draft cache holds rotated keys
    assert np.allclose(vd[0], vs[P:].transpose(1, 0, 2), atol=TOL)


@pytest.mark.parametrize("M,D,P", [(12, 4, 5), (30, 6, 0)])
def test_tli_tree_is_the_layer_along_each_path(oracle, M, D, P):
    rng = np.random.default_rng(200 + M)
    d, H, Hkv, dh, d_ff = 24, 4, 2, 6, 40
    w = layer_rand(rng, d, H, Hkv, dh, d_ff)
    x_prefix, x = rnd(rng, max(P, 1), d)[:P], rnd(rng, M, d)
    parent = mi.gen_tree(M, D, 3, rng)[None]
    if P:
        _, ks, vs = library_layer(x_prefix, w, H, Hkv, dh)
        kc, vc = cache_from(ks, vs, P + 1)
    else:
        kc, vc = np.zeros((1, Hkv, 1, dh)), np.zeros((1, Hkv, 1, dh))
    out, _ = run_layer(oracle, x[None], parent, w, kc, vc, np.array([P], dtype=np.int32), H, Hkv, dh)
    for i in range(M):
        path, j = [], i
        while j >= 0:
            path.append(j)
            j = parent[0, j]
        ref, _, _ = library_layer(np.concatenate([x_prefix, x[path[::-1]]]), w, H, Hkv, dh)
        assert np.allclose(out[0, i], ref[-1], atol=TOL), i


def test_tli_level_by_level_equals_whole_tree(oracle):
    rng = np.random.default_rng(23)
    B, P, M, D, d, H, Hkv, dh, d_ff = 2, 4, 29, 5, 16, 4, 2, 4, 24
    w = layer_rand(rng, d, H, Hkv, dh, d_ff)
    x = rnd(rng, B, M, d)
    parent = np.stack([mi.gen_tree(M, D, 4, rng) for _ in range(B)])
    kc, vc = rnd(rng, B, Hkv, P + 2, dh), rnd(rng, B, Hkv, P + 2, dh)
    plen = np.array([P, P - 3], dtype=np.int32)
    whole, (kw, vw) = run_layer(oracle, x, parent, w, kc, vc, plen, H, Hkv, dh)
    caches = (np.full((B, Hkv, M, dh), np.nan), np.full((B, Hkv, M, dh), np.nan))
    pieces = []
    cuts = [0, 1, 3, 11, 12, 25, M]
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        o, caches = run_layer(oracle, x, parent, w, kc, vc, plen, H, Hkv, dh, node0=lo, Mn=hi - lo, caches=caches)
        pieces.append(o)
    assert np.array_equal(np.concatenate(pieces, axis=1), whole)
    assert np.array_equal(caches[0], kw) and np.array_equal(caches[1], vw)


def test_tli_zero_output_weights_make_the_layer_the_identity(oracle):
    rng = np.random.default_rng(29)
    d, H, Hkv, dh, d_ff, M = 16, 2, 1, 8, 20, 7
    w = layer_rand(rng, d, H, Hkv, dh, d_ff)
    x = rnd(rng, 1, M, d)
    parent = mi.star_tree(M)[None]
    kc, vc = rnd(rng, 1, Hkv, 3, dh), rnd(rng, 1, Hkv, 3, dh)
    plen = np.array([3], dtype=np.int32)
    w0 = dict(w, wo=np.zeros_like(w["wo"]), w_down=np.zeros_like(w["w_down"]))
    out, _ = run_layer(oracle, x, parent, w0, kc, vc, plen, H, Hkv, dh)
    assert np.array_equal(out, x)
    # and with only W_down zero the second residual passes the attention block's result through
    w1 = dict(w, w_down=np.zeros_like(w["w_down"]))
    h1, _ = run_layer(oracle, x, parent, w1, kc, vc, plen, H, Hkv, dh)
    full, _ = run_layer(oracle, x, parent, w, kc, vc, plen, H, Hkv, dh)
    assert np.abs(h1 - x).max() > 1e-3 and np.abs(full - h1).max() > 1e-3


def test_tli_rejects_bad_arguments(oracle):
    rng = np.random.default_rng(31)
    d, H, Hkv, dh, d_ff, M = 8, 2, 1, 4, 8, 5
    w = layer_rand(rng, d, H, Hkv, dh, d_ff)
    x = rnd(rng, 1, M, d)
    kc, vc = rnd(rng, 1, Hkv, 2, dh), rnd(rng, 1, Hkv, 2, dh)
    plen = np.array([2], dtype=np.int32)
    with pytest.raises(oracle.OracleError):
        run_layer(oracle, x, np.array([[-1, 0, 3, 1, 2]], dtype=np.int32), w, kc, vc, plen, H, Hkv, dh)
    with pytest.raises(oracle.OracleError):                                       # more prefix rows than the cache has
        run_layer(oracle, x, mi.chain_tree(M)[None], w, kc, vc, np.array([3], dtype=np.int32), H, Hkv, dh)
