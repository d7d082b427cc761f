"""GPU parity of a reused LLM decoder layer under Target Layer Inference (moa_tli_decoder_layer) against the fp64
oracle: whole trees in one call and level-by-level calls that grow the layer's draft cache."""
import numpy as np
import pytest
import torch

import moa_inputs as mi

pytestmark = pytest.mark.gpu

EPS, THETA = 1e-5, 500000.0           # Llama-3 values


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


@pytest.fixture(scope="module")
def moa(G):
    import paper_2410_03804_amd as m
    return m


def small_cfg(dtype, **kw):
    base = dict(name="TLI", index=16, dtype=dtype, B=3, P_min=1, P_max=200, M=37, D=5, max_branch=4, L=2, d=512,
                H=8, Hkv=2, dh=128, d_lsa_in=512, rms_norm=True)
    base.update(kw)
    return mi.Config(**base)


CASES = {
    "C0_f32": mi.CONFIGS["C0"],
    "small_f32": small_cfg("f32", d=192, H=6, Hkv=3, dh=32, M=19, D=4),
    "small_bf16": small_cfg("bf16"),
    "bf16_dh64_M70": small_cfg("bf16", B=2, dh=64, H=8, Hkv=4, M=70, D=7, P_max=150),
    "bf16_long_prefix": small_cfg("bf16", B=1, P_min=3000, P_max=3000, M=21, D=5),    # angles of thousands of radians
    "C1_bf16": mi.CONFIGS["C1"],          # d 4096, 32/8 heads of 128, MLP 14336, prefix 1024, 60 nodes
}


def setup(oracle, cfg):
    w = mi.tli_weights(cfg)
    x = mi.verify_inputs(cfg)
    kc, vc = mi.kv_cache(cfg, which=7)
    plen = mi.prefix_lengths(cfg)
    parent = mi.trees(cfg)
    mask_np, depth_np = oracle.tree_build(parent)
    return w, x, kc, vc, plen, parent, mask_np, depth_np


def run_gpu(G, moa, cfg, w, x, kc, vc, plen, mask_np, depth_np, cuts):
    dt = cfg.dtype
    tdt = G.TDT[dt]
    shape = G.shape_of(cfg)
    dcfg = moa.DecoderCfg(mi.tli_d_ff(cfg), EPS, THETA)
    P_cap = kc.shape[2]
    ws = torch.empty(max(moa.tli_workspace_bytes(shape, dcfg, cfg.B, P_cap, cfg.M), 256), dtype=torch.uint8, device="cuda")
    kd = torch.full((cfg.B, cfg.Hkv, cfg.M, cfg.dh), float("nan"), dtype=tdt, device="cuda")
    vd = torch.full_like(kd, float("nan"))
    st = G.status_word()
    mask, depth = G.dev(mask_np.view(np.int64)), G.dev(depth_np)
    wd = {k: G.dev(v, dt) for k, v in w.items()}
    kcd, vcd, pl = G.dev(kc, dt), G.dev(vc, dt), G.dev(plen)
    outs = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        out = torch.empty((cfg.B, hi - lo, cfg.d), dtype=tdt, device="cuda")
        moa.tli_decoder_layer(shape, dcfg, G.dev(np.ascontiguousarray(x[:, lo:hi]), dt), lo, wd, kcd, vcd, pl, P_cap, mask,
                              depth, out, kd, vd, ws, st)
        outs.append(out)
    torch.cuda.synchronize()
    assert st.item() == 0
    return torch.cat(outs, dim=1), kd, vd


def run_oracle(oracle, cfg, w, x, kc, vc, plen, parent):
    kd = np.zeros((cfg.B, cfg.Hkv, cfg.M, cfg.dh))
    vd = np.zeros_like(kd)
    out = oracle.tli_decoder_layer(x, parent, 0, w, kc, vc, plen, kd, vd, cfg.H, cfg.Hkv, cfg.dh, EPS, THETA)
    return out, kd, vd


@pytest.mark.parametrize("case", list(CASES))
def test_tli_layer_whole_tree_parity(G, moa, oracle, case):
    cfg = CASES[case]
    w, x, kc, vc, plen, parent, mask_np, depth_np = setup(oracle, cfg)
    print(f"[case] tli_layer whole {case} B={cfg.B} M={cfg.M} d={cfg.d} d_ff={mi.tli_d_ff(cfg)} len={list(plen)}", flush=True)
    out, kd, vd = run_gpu(G, moa, cfg, w, x, kc, vc, plen, mask_np, depth_np, [0, cfg.M])
    want, wk, wv = run_oracle(oracle, cfg, w, x, kc, vc, plen, parent)
    G.check_close(G.host(kd), wk, cfg.dtype, f"tli.k_draft[{case}]", residual_stream=True)
    G.check_close(G.host(vd), wv, cfg.dtype, f"tli.v_draft[{case}]")
    G.check_close(G.host(out), want, cfg.dtype, f"tli.out[{case}]", residual_stream=True)


@pytest.mark.parametrize("case", ["small_f32", "small_bf16", "C1_bf16"])
def test_tli_layer_level_by_level_parity(G, moa, oracle, case):
    cfg = CASES[case]
    w, x, kc, vc, plen, parent, mask_np, depth_np = setup(oracle, cfg)
    cuts = sorted({0, cfg.M} | {int(np.searchsorted(depth_np[0], dlev, side="right")) for dlev in range(int(depth_np[0].max()) + 1)})
    assert len(cuts) >= 3
    print(f"[case] tli_layer levels {case} cuts={cuts}", flush=True)
    out, kd, vd = run_gpu(G, moa, cfg, w, x, kc, vc, plen, mask_np, depth_np, cuts)
    want, wk, wv = run_oracle(oracle, cfg, w, x, kc, vc, plen, parent)
    G.check_close(G.host(kd), wk, cfg.dtype, f"tli.levels.k_draft[{case}]", residual_stream=True)
    G.check_close(G.host(vd), wv, cfg.dtype, f"tli.levels.v_draft[{case}]")
    G.check_close(G.host(out), want, cfg.dtype, f"tli.levels.out[{case}]", residual_stream=True)


def test_tli_layer_rejects_bad_arguments(G, moa, oracle):
    cfg = small_cfg("bf16", B=1, M=9, D=3)
    w, x, kc, vc, plen, parent, mask_np, depth_np = setup(oracle, cfg)
    shape = G.shape_of(cfg)
    dcfg = moa.DecoderCfg(mi.tli_d_ff(cfg), EPS, THETA)
    tdt = G.TDT[cfg.dtype]
    P_cap = kc.shape[2]
    ws = torch.empty(moa.tli_workspace_bytes(shape, dcfg, 1, P_cap, cfg.M), dtype=torch.uint8, device="cuda")
    kd = torch.zeros((1, cfg.Hkv, cfg.M, cfg.dh), dtype=tdt, device="cuda")
    out = torch.zeros((1, cfg.M, cfg.d), dtype=tdt, device="cuda")
    wd = {k: G.dev(v, cfg.dtype) for k, v in w.items()}
    args = (G.dev(kc, cfg.dtype), G.dev(vc, cfg.dtype), G.dev(plen), P_cap, G.dev(mask_np.view(np.int64)), G.dev(depth_np),
            out, kd, kd.clone())
    with pytest.raises(moa.MoaError):                       # workspace one byte short
        moa.tli_decoder_layer(shape, dcfg, G.dev(x, cfg.dtype), 0, wd, *args, ws[:-256], G.status_word())
    with pytest.raises(moa.MoaError):                       # nodes 5..13 of a 9-node tree
        moa.tli_decoder_layer(shape, dcfg, G.dev(x, cfg.dtype), 5, wd, *args, ws, G.status_word())
    with pytest.raises(moa.MoaError):
        moa.tli_decoder_layer(shape, moa.DecoderCfg(0, EPS, THETA), G.dev(x, cfg.dtype), 0, wd, *args, ws, G.status_word())
    torch.cuda.synchronize()
    assert torch.count_nonzero(out).item() == 0             # nothing was launched
