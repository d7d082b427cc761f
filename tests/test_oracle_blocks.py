"""Pins for the oracle's pre-norm residual MLP sub-block and RMS norm: the wrappers of the drafter's own layers
(appendix architecture table: an MLP after Layer Self-Attention, Self-Attention and Cross-Attention; form not stated
in the paper, the LLM's own block form is taken).

Pinned by: an example worked by hand; torch's CPU routines in double precision (rms_norm, silu, linear); closed
forms (a zero down- or gate-projection leaves the stream unchanged; with eps = 0 the MLP term does not depend on the
scale of the stream); agreement with the reused-decoder-layer oracle when that layer's attention contributes nothing."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def weights(rng, d, d_ff):
    return (rng.standard_normal(d) * 0.2 + 1.0, rng.standard_normal((d_ff, d)) / np.sqrt(d),
            rng.standard_normal((d_ff, d)) / np.sqrt(d), rng.standard_normal((d, d_ff)) / np.sqrt(d_ff))


def test_hand_worked_scalar_block(oracle):
    """d = d_ff = 1, eps = 0: h = 2 -> n = h / |h| = 1; gate = 1 -> silu(1) = 1 / (1 + 1/e) = 0.731058578630...;
    up = 3 -> 2.193175735890...; down weight 0.5 -> 1.096587867945...; out = 2 + that."""
    one = np.ones((1, 1))
    args = (np.array([1.0]), one, 3 * one, 0.5 * one, 0.0)
    assert abs(oracle.mlp_block(np.array([[2.0]]), None, *args)[0, 0] - 3.0965878679450073) < 1e-13
    assert abs(oracle.mlp_block(np.array([[1.5]]), np.array([[0.5]]), *args)[0, 0] - 3.0965878679450073) < 1e-13
    # a negative stream value flips the sign of n: gate = -1, silu(-1) = -1 / (1 + e) = -0.268941421369...; up = -3
    assert abs(oracle.mlp_block(np.array([[-2.0]]), None, *args)[0, 0] - (-2.0 + 0.5 * 0.2689414213699951 * 3.0)) < 1e-13


@pytest.mark.parametrize("R,d,d_ff,with_res,seed", [(5, 16, 24, True, 0), (3, 64, 8, False, 1), (1, 7, 13, True, 2)])
def test_block_against_torch_routines(oracle, R, d, d_ff, with_res, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((R, d)) * 2.0
    res = rng.standard_normal((R, d)) if with_res else None
    g, wg, wu, wd = weights(rng, d, d_ff)
    eps = 1e-5
    got = oracle.mlp_block(x, res, g, wg, wu, wd, eps)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    h = t(x) + (t(res) if with_res else 0.0)
    n = F.rms_norm(h, (d,), weight=t(g), eps=eps)
    want = h + F.linear(F.silu(F.linear(n, t(wg))) * F.linear(n, t(wu)), t(wd))
    assert np.max(np.abs(got - want.numpy())) < 1e-12
    assert np.max(np.abs(oracle.rmsnorm(x, g, eps) - F.rms_norm(t(x), (d,), weight=t(g), eps=eps).numpy())) < 1e-13


def test_closed_forms(oracle):
    rng = np.random.default_rng(7)
    R, d, d_ff = 4, 12, 20
    x, res = rng.standard_normal((R, d)), rng.standard_normal((R, d))
    g, wg, wu, wd = weights(rng, d, d_ff)
    assert np.array_equal(oracle.mlp_block(x, res, g, wg, wu, np.zeros_like(wd), 1e-5), x + res)
    assert np.array_equal(oracle.mlp_block(x, res, g, np.zeros_like(wg), wu, wd, 1e-5), x + res)       # silu(0) = 0
    assert np.array_equal(oracle.mlp_block(x, None, g, wg, np.zeros_like(wu), wd, 1e-5), x)
    # eps = 0: the normalised stream, hence the MLP term, does not see the stream's scale
    base = oracle.mlp_block(x, None, g, wg, wu, wd, 0.0) - x
    for c in (0.25, 3.0, 1000.0):
        assert np.max(np.abs(oracle.mlp_block(c * x, None, g, wg, wu, wd, 0.0) - c * x - base)) < 1e-9
    # unit gain, eps = 0: every normalised row has mean square 1; the gain multiplies feature by feature
    n = oracle.rmsnorm(x, np.ones(d), 0.0)
    assert np.allclose((n * n).mean(axis=1), 1.0, atol=1e-13)
    assert np.allclose(oracle.rmsnorm(x, g, 0.0), n * g, atol=1e-14)
    # splitting the stream between x and res changes nothing
    assert np.max(np.abs(oracle.mlp_block(x, res, g, wg, wu, wd, 1e-5) - oracle.mlp_block(x + res, None, g, wg, wu, wd, 1e-5))) < 1e-13


def test_block_is_the_second_half_of_the_reused_decoder_layer(oracle):
    """With a zero output projection the decoder layer's attention adds nothing: what is left is this block."""
    rng = np.random.default_rng(11)
    B, M, d, H, Hkv, dh, d_ff = 2, 5, 32, 4, 2, 8, 40
    x = rng.standard_normal((B, M, d))
    g, wg, wu, wd = weights(rng, d, d_ff)
    w = dict(g_attn=np.ones(d), wq=rng.standard_normal((H * dh, d)), wk=rng.standard_normal((Hkv * dh, d)),
             wv=rng.standard_normal((Hkv * dh, d)), wo=np.zeros((d, H * dh)), g_mlp=g, w_gate=wg, w_up=wu, w_down=wd)
    parent = np.array([[-1, 0, 0, 1, 2]] * B, dtype=np.int32)
    kc = rng.standard_normal((B, Hkv, 6, dh))
    kd = np.zeros((B, Hkv, M, dh))
    out = oracle.tli_decoder_layer(x, parent, 0, w, kc, kc.copy(), np.array([6, 3], np.int32), kd, kd.copy(), H, Hkv, dh, 1e-5, 1e4)
    assert np.max(np.abs(out - oracle.mlp_block(x, None, g, wg, wu, wd, 1e-5))) < 1e-12


def test_bad_arguments(oracle):
    g, wg, wu, wd = weights(np.random.default_rng(0), 4, 6)
    x = np.zeros((2, 4))
    with pytest.raises(ValueError):
        oracle.mlp_block(x, np.zeros((2, 5)), g, wg, wu, wd, 1e-5)
    with pytest.raises(ValueError):
        oracle.mlp_block(x, None, g, wg, wu[:, :3], wd, 1e-5)
    with pytest.raises(oracle.OracleError):
        oracle.mlp_block(x, None, g, wg, wu, wd, -1.0)
    assert oracle.mlp_block(np.zeros((0, 4)), None, g, wg, wu, wd, 1e-5).shape == (0, 4)
