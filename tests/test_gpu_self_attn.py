"""GPU parity of the draft Self-Attention layer (moa_self_attn_draft) against the fp64 oracle: whole trees in
one call, and level-by-level calls that grow the per-cycle draft cache, through both MFMA forms of the attention
core and the generic one."""
import numpy as np
import pytest
import torch

import moa_inputs as mi

pytestmark = pytest.mark.gpu


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


@pytest.fixture(params=["split", "whole"])
def attn_kernel(request, moa):
    moa.debug_force_attn_kernel(request.param)
    yield request.param
    moa.debug_force_attn_kernel("auto")


def small_cfg(dtype, **kw):
    base = dict(name="SA", index=13, dtype=dtype, B=3, P_min=1, P_max=200, M=37, D=5, max_branch=4, L=2, d=512,
                H=8, Hkv=4, dh=128, d_lsa_in=512, rms_norm=True)
    base.update(kw)
    return mi.Config(**base)


# Hkv is the LLM's; the layer itself has mi.sa_kv_heads(cfg) = Hkv / 2 KV heads (appendix table: 512 against 1024)
CASES = {
    "C0_f32": mi.CONFIGS["C0"],
    "small_f32": small_cfg("f32", d=192, H=6, Hkv=6, dh=32, M=19, D=4),
    "small_bf16": small_cfg("bf16"),
    "bf16_dh64_M70": small_cfg("bf16", B=2, dh=64, H=8, Hkv=4, M=70, D=7, P_max=150),
    "bf16_M130_three_words": small_cfg("bf16", B=2, H=4, Hkv=2, M=130, D=10, P_max=97),
    "C1_bf16": mi.CONFIGS["C1"],          # embedding 4096, 32 query heads, 4 KV heads of 128, prefix 1024, 60 nodes
}


def sa_shape(G, moa, cfg):
    return moa.Shape(cfg.L, cfg.d, cfg.H, mi.sa_kv_heads(cfg), cfg.dh, cfg.d_lsa_in, cfg.lsa_heads, cfg.Hkv, G.MDT[cfg.dtype])


def setup(G, moa, oracle, cfg):
    w = mi.sa_weights(cfg)
    emb, kc, vc = mi.sa_inputs(cfg)
    plen = mi.prefix_lengths(cfg)
    parent = mi.trees(cfg)
    mask_np, _ = oracle.tree_build(parent)
    return w, emb, kc, vc, plen, parent, mask_np


def run_gpu(G, moa, cfg, w, emb, kc, vc, plen, mask_np, cuts):
    """One call per node range [cuts[i], cuts[i+1]); the draft cache starts as NaN so a row read before it was
    written would show."""
    dt = cfg.dtype
    tdt = G.TDT[dt]
    hkv = mi.sa_kv_heads(cfg)
    shape = sa_shape(G, moa, cfg)
    P_cap = kc.shape[2]
    ws = G.workspace(shape, cfg.B, P_cap, cfg.M, 0)
    kd = torch.full((cfg.B, hkv, cfg.M, cfg.dh), float("nan"), dtype=tdt, device="cuda")
    vd = torch.full_like(kd, float("nan"))
    st = G.status_word()
    mask = G.dev(mask_np.view(np.int64))
    wd = [G.dev(w[k], dt) for k in ("wq", "wk", "wv", "wo")]
    kcd, vcd, pl = G.dev(kc, dt), G.dev(vc, dt), G.dev(plen)
    outs = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        out = torch.empty((cfg.B, hi - lo, cfg.d), dtype=tdt, device="cuda")
        moa.self_attn_draft(shape, G.dev(np.ascontiguousarray(emb[:, lo:hi]), dt), lo, *wd, kcd, vcd, pl, P_cap, mask, out,
                            kd, vd, ws, st)
        outs.append(out)
    torch.cuda.synchronize()
    assert st.item() == 0
    return torch.cat(outs, dim=1), kd, vd


def run_oracle(oracle, cfg, w, emb, kc, vc, plen, parent):
    hkv = mi.sa_kv_heads(cfg)
    kd = np.zeros((cfg.B, hkv, cfg.M, cfg.dh))
    vd = np.zeros_like(kd)
    out = oracle.self_attn_draft(emb, parent, 0, w["wq"], w["wk"], w["wv"], w["wo"], kc, vc, plen, kd, vd,
                                 cfg.H, hkv, cfg.dh)
    return out, kd, vd


@pytest.mark.parametrize("case", list(CASES))
def test_self_attn_whole_tree_parity(G, moa, oracle, case, attn_kernel):
    cfg = CASES[case]
    w, emb, kc, vc, plen, parent, mask_np = setup(G, moa, oracle, cfg)
    print(f"[case] self_attn whole {case} B={cfg.B} M={cfg.M} H={cfg.H}/{mi.sa_kv_heads(cfg)} len={list(plen)}", flush=True)
    out, kd, vd = run_gpu(G, moa, cfg, w, emb, kc, vc, plen, mask_np, [0, cfg.M])
    want, wk, wv = run_oracle(oracle, cfg, w, emb, kc, vc, plen, parent)
    G.check_close(G.host(kd), wk, cfg.dtype, f"self_attn.k_draft[{case}]")
    G.check_close(G.host(vd), wv, cfg.dtype, f"self_attn.v_draft[{case}]")
    G.check_close(G.host(out), want, cfg.dtype, f"self_attn[{case}]")


@pytest.mark.parametrize("case", ["small_f32", "small_bf16", "bf16_M130_three_words", "C1_bf16"])
def test_self_attn_level_by_level_parity(G, moa, oracle, case, attn_kernel):
    """Drafting order: the root, then one call per depth level (nodes are labelled in depth order; with several
    sequences the cuts follow the first tree's levels, any cut keeps ancestors first), the draft cache growing."""
    cfg = CASES[case]
    w, emb, kc, vc, plen, parent, mask_np = setup(G, moa, oracle, cfg)
    _, depth = oracle.tree_build(parent)
    cuts = [0] + [int(np.searchsorted(depth[0], dlev, side="right")) for dlev in range(int(depth[0].max()) + 1)]
    cuts = sorted(set(cuts))
    assert cuts[0] == 0 and cuts[-1] == cfg.M and len(cuts) >= 3
    print(f"[case] self_attn levels {case} cuts={cuts}", flush=True)
    out, kd, vd = run_gpu(G, moa, cfg, w, emb, kc, vc, plen, mask_np, cuts)
    want, wk, wv = run_oracle(oracle, cfg, w, emb, kc, vc, plen, parent)
    G.check_close(G.host(kd), wk, cfg.dtype, f"self_attn.levels.k_draft[{case}]")
    G.check_close(G.host(vd), wv, cfg.dtype, f"self_attn.levels.v_draft[{case}]")
    G.check_close(G.host(out), want, cfg.dtype, f"self_attn.levels[{case}]")
    # and against the library's own whole-tree call, to rounding (other row counts take other projection kernels)
    out1, kd1, vd1 = run_gpu(G, moa, cfg, w, emb, kc, vc, plen, mask_np, [0, cfg.M])
    for a, b in ((kd, kd1), (vd, vd1), (out, out1)):
        assert torch.allclose(a.float(), b.float(), atol=G.ABS_TOL[cfg.dtype], rtol=G.REL_TOL[cfg.dtype])


def test_self_attn_single_node_and_empty_prefix(G, moa, oracle):
    """The root alone with nothing verified yet attends only itself: out = W_o W_v emb."""
    cfg = small_cfg("bf16", B=2, M=1, D=0, P_min=0, P_max=9)
    w, emb, kc, vc, plen, parent, mask_np = setup(G, moa, oracle, cfg)
    plen = np.array([0, 9], dtype=np.int32)
    out, kd, vd = run_gpu(G, moa, cfg, w, emb, kc, vc, plen, mask_np, [0, 1])
    want, wk, wv = run_oracle(oracle, cfg, w, emb, kc, vc, plen, parent)
    G.check_close(G.host(out), want, cfg.dtype, "self_attn[single node]")
    G.check_close(G.host(kd), wk, cfg.dtype, "self_attn.k_draft[single node]")


def test_self_attn_rejects_node_range_outside_tree(G, moa, oracle):
    cfg = small_cfg("bf16", B=1, M=9, D=3)
    w, emb, kc, vc, plen, parent, mask_np = setup(G, moa, oracle, cfg)
    shape = sa_shape(G, moa, cfg)
    tdt = G.TDT[cfg.dtype]
    ws = G.workspace(shape, 1, kc.shape[2], cfg.M, 0)
    kd = torch.zeros((1, mi.sa_kv_heads(cfg), cfg.M, cfg.dh), dtype=tdt, device="cuda")
    out = torch.zeros((1, 4, cfg.d), dtype=tdt, device="cuda")
    with pytest.raises(moa.MoaError):
        moa.self_attn_draft(shape, G.dev(np.ascontiguousarray(emb[:, :4]), cfg.dtype), 7,
                            *(G.dev(w[k], cfg.dtype) for k in ("wq", "wk", "wv", "wo")), G.dev(kc, cfg.dtype),
                            G.dev(vc, cfg.dtype), G.dev(plen), kc.shape[2], G.dev(mask_np.view(np.int64)), out,
                            kd, kd.clone(), ws, G.status_word())
    torch.cuda.synchronize()
    assert torch.count_nonzero(out).item() == 0          # nothing was launched
