"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle, element by element, on the
same seeded inputs.  Integer results (mask, depth, path, bonus) are bit-exact; floating point is held
to max-abs 1e-4 (fp32) / 2e-2 (bf16) plus a tighter max-abs/rms bound."""
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


# ------------------------------------------------------------------ integer kernels

def tree_cases():
    rng = np.random.default_rng(99)
    yield "C0", mi.trees(mi.CONFIGS["C0"])
    yield "C1", mi.trees(mi.CONFIGS["C1"])
    yield "C2", mi.trees(mi.CONFIGS["C2"])
    yield "C4", mi.trees(mi.CONFIGS["C4"])
    yield "chain256", mi.chain_tree(256)[None]
    yield "star200", mi.star_tree(200)[None]
    yield "single", np.array([[-1]], dtype=np.int32)
    yield "beam62", mi.beam_tree(8, 6, 62, rng)[None]
    yield "full3x4", mi.full_tree(3, 4)[None]
    yield "rand65", np.stack([mi.gen_tree(65, 12, 3, rng) for _ in range(5)])


@pytest.mark.parametrize("name,parent", list(tree_cases()), ids=[n for n, _ in tree_cases()])
def test_tree_build_bit_exact(G, moa, oracle, name, parent):
    print(f"[case] tree_build {name} shape={parent.shape}", flush=True)
    B, M = parent.shape
    W = (M + 63) // 64
    mask = torch.full((B, M, W), -1, dtype=torch.int64, device="cuda")
    depth = torch.full((B, M), -7, dtype=torch.int32, device="cuda")
    st = G.status_word()
    moa.tree_build(G.dev(parent), mask, depth, st)
    torch.cuda.synchronize()
    want_mask, want_depth = oracle.tree_build(parent)
    assert np.array_equal(G.mask_u64(mask), want_mask)
    assert np.array_equal(depth.cpu().numpy(), want_depth)
    assert st.item() == 0


def test_tree_build_flags_bad_parent(G, moa):
    parent = np.array([[-1, 0, 1, 3, 2]], dtype=np.int32)        # node 3 names itself
    mask = torch.zeros((1, 5, 1), dtype=torch.int64, device="cuda")
    depth = torch.zeros((1, 5), dtype=torch.int32, device="cuda")
    st = G.status_word()
    moa.tree_build(G.dev(parent), mask, depth, st)
    torch.cuda.synchronize()
    assert st.item() & moa.DEV_BAD_PARENT


@pytest.mark.parametrize("name", ["C0", "C1", "C2", "C3", "C4"])
def test_tree_accept_bit_exact(G, moa, oracle, name):
    cfg = mi.CONFIGS[name]
    parent = mi.trees(cfg)
    tok, tgt = mi.tokens(cfg, parent)
    print(f"[case] tree_accept {name}", flush=True)
    B, M = parent.shape
    path = torch.zeros((B, M), dtype=torch.int32, device="cuda")
    n_path = torch.zeros((B,), dtype=torch.int32, device="cuda")
    bonus = torch.zeros((B,), dtype=torch.int32, device="cuda")
    moa.tree_accept(G.dev(parent), G.dev(tok), G.dev(tgt), path, n_path, bonus)
    torch.cuda.synchronize()
    wp, wn, wb = oracle.tree_accept(parent, tok, tgt)
    assert np.array_equal(path.cpu().numpy(), wp)
    assert np.array_equal(n_path.cpu().numpy(), wn) and np.array_equal(bonus.cpu().numpy(), wb)


def test_tree_accept_chain_and_no_match(G, moa, oracle):
    M = 256
    parent = mi.chain_tree(M)[None]
    tgt = np.arange(1000, 1000 + M, dtype=np.int32)[None]
    tok = np.concatenate([[5], tgt[0, :-1]]).astype(np.int32)[None]          # everything accepted
    tok2 = tok.copy()
    tok2[0, 1] += 1                                                            # nothing accepted
    for t in (tok, tok2):
        path = torch.zeros((1, M), dtype=torch.int32, device="cuda")
        n_path = torch.zeros((1,), dtype=torch.int32, device="cuda")
        bonus = torch.zeros((1,), dtype=torch.int32, device="cuda")
        moa.tree_accept(G.dev(parent), G.dev(t), G.dev(tgt), path, n_path, bonus)
        torch.cuda.synchronize()
        wp, wn, wb = oracle.tree_accept(parent, t, tgt)
        assert np.array_equal(path.cpu().numpy(), wp) and n_path.item() == wn[0] and bonus.item() == wb[0]


# ------------------------------------------------------------------ floating-point entry points

def small_cfg(dtype, **kw):
    base = dict(name="S", index=7, dtype=dtype, B=3, P_min=1, P_max=333, M=37, D=5, max_branch=4, L=6, d=512,
                H=8, Hkv=2, dh=128, d_lsa_in=512, rms_norm=True)
    base.update(kw)
    return mi.Config(**base)


CASES = {
    "C0_f32": mi.CONFIGS["C0"],
    "small_f32": small_cfg("f32", d=192, H=6, Hkv=3, dh=32, d_lsa_in=96, L=5, M=19, D=4),
    "small_bf16_dh128": small_cfg("bf16"),
    "small_bf16_dh64": small_cfg("bf16", dh=64, H=8, Hkv=4, d=512, d_lsa_in=256, M=61, D=6),
    "bf16_two_rowtiles_M70": small_cfg("bf16", B=2, H=8, Hkv=2, M=70, D=7, P_max=150),
    "bf16_M130_three_words": small_cfg("bf16", B=2, H=4, Hkv=2, d=512, M=130, D=10, P_max=97),
    "bf16_generic_dh32": small_cfg("bf16", d=256, H=8, Hkv=4, dh=32, d_lsa_in=128, M=21, D=4),
    "bf16_M256_largest_tree": small_cfg("bf16", B=1, H=4, Hkv=2, d=512, M=256, D=20, P_max=70, L=2),
    "C1_bf16": mi.CONFIGS["C1"],
}


def run_lsa(G, moa, oracle, cfg, T):
    shape = G.shape_of(cfg)
    w = mi.lsa_weights(cfg)
    hs = mi.lsa_inputs(cfg, T)
    ws = G.workspace(shape, cfg.B, cfg.P_cap, cfg.M, T)
    out = torch.empty((T, cfg.d_lsa), dtype=G.TDT[cfg.dtype], device="cuda")
    moa.lsa(shape, G.dev(hs, cfg.dtype), *(G.dev(w[k], cfg.dtype) for k in ("wq", "wk", "wv", "wo")), out, ws)
    torch.cuda.synchronize()
    want = oracle.lsa(hs, w["wq"], w["wk"], w["wv"], w["wo"], cfg.lsa_heads, cfg.Hkv, cfg.dh)
    return G.host(out), want


@pytest.fixture(params=["fused", "separate"])
def lsa_kernel(request, moa):
    """Both forms of the Layer Self-Attention on every case: projection, attention over the layers and mean in one
    kernel (taken wherever the shapes allow: bf16, head_dim 128), or as three kernels with the projected rows in the
    workspace (forced)."""
    moa.debug_force_lsa_kernel(request.param)
    yield request.param
    moa.debug_force_lsa_kernel("auto")


@pytest.mark.parametrize("case", list(CASES))
def test_lsa_parity(G, moa, oracle, case, lsa_kernel):
    cfg = CASES[case]
    T = 60 if case == "C1_bf16" else 7
    print(f"[case] lsa {case} T={T} L={cfg.L} d_in={cfg.d_lsa_in} heads={cfg.lsa_heads}/{cfg.Hkv} dh={cfg.dh}", flush=True)
    got, want = run_lsa(G, moa, oracle, cfg, T)
    G.check_close(got, want, cfg.dtype, f"lsa[{case}]")


def test_lsa_many_tokens_tiled_projection(G, moa, oracle, lsa_kernel):
    """More than 128 projected rows takes the LDS-tiled MFMA GEMM; more than 256 tokens takes two chunks."""
    cfg = small_cfg("bf16", L=3, d_lsa_in=256, dh=128, Hkv=1)       # LSA heads 2/1, N = 256 + 128 + 128
    T = 300
    print(f"[case] lsa tiled T={T}", flush=True)
    got, want = run_lsa(G, moa, oracle, cfg, T)
    G.check_close(got, want, cfg.dtype, "lsa[tiled,T=300]")


@pytest.mark.parametrize("L,dh", [(80, 128), (40, 64), (33, 128), (96, 64)])
def test_lsa_layer_counts_beyond_one_block(G, moa, oracle, L, dh, lsa_kernel):
    """Llama-2-70B stacks 80 layers: more than one 32-layer block on the layer axis, ragged last block."""
    cfg = small_cfg("bf16", L=L, d_lsa_in=2 * dh, dh=dh, Hkv=1)
    print(f"[case] lsa L={L} dh={dh}", flush=True)
    got, want = run_lsa(G, moa, oracle, cfg, 5)
    G.check_close(got, want, cfg.dtype, f"lsa[L={L},dh={dh}]")


@pytest.mark.parametrize("L,d_in,Hkv,T", [(32, 512, 2, 9), (64, 1024, 2, 5), (17, 256, 1, 6), (96, 512, 4, 3), (2, 128, 1, 4),
                                           (32, 1024, 4, 600), (32, 512, 2, 401), (64, 512, 2, 201), (32, 320, 1, 7),
                                           (64, 576, 1, 600), (96, 1024, 4, 3)])
def test_lsa_one_kernel_form_shapes(G, moa, oracle, L, d_in, Hkv, T):
    """The one-kernel form across its template variants (one, two and three blocks of 32 layers), groups of two and of
    four query heads per KV head (a group of four is cut into two parts that recompute K and V), odd token counts (a
    half-filled token tile), the shortest input width it takes, and enough tokens for the tiles of three and four tokens
    (two at two blocks of layers) with a ragged last tile, and input widths whose tile count is not a multiple of the
    packed form's register stages (5 and 9 tiles of 64); it must also give the bits of the three-kernel form, from
    plain and from packed weights."""
    cfg = small_cfg("bf16", L=L, d_lsa_in=d_in, dh=128, Hkv=Hkv)
    print(f"[case] lsa one-kernel L={L} d_in={d_in} heads={cfg.lsa_heads}/{Hkv} T={T}", flush=True)
    shape = G.shape_of(cfg)
    w = mi.lsa_weights(cfg)
    hs = mi.lsa_inputs(cfg, T)
    ws = G.workspace(shape, cfg.B, cfg.P_cap, cfg.M, T)
    dw = [G.dev(w[k], cfg.dtype) for k in ("wq", "wk", "wv", "wo")]
    outs = {}
    for form in ("fused", "separate"):
        moa.debug_force_lsa_kernel(form)
        try:
            out = torch.full((T, cfg.d_lsa), float("nan"), dtype=G.TDT[cfg.dtype], device="cuda")
            moa.lsa(shape, G.dev(hs, cfg.dtype), *dw, out, ws)
            torch.cuda.synchronize()
        finally:
            moa.debug_force_lsa_kernel("auto")
        outs[form] = out
    want = oracle.lsa(hs, w["wq"], w["wk"], w["wv"], w["wo"], cfg.lsa_heads, cfg.Hkv, cfg.dh)
    G.check_close(G.host(outs["fused"]), want, cfg.dtype, f"lsa one-kernel[L={L},d_in={d_in},Hkv={Hkv}]")
    if d_in % 128 == 0:     # then the three-kernel form projects on the matrix cores too, in the same order along d_in
        assert torch.equal(outs["fused"], outs["separate"]), "same products in the same order, same roundings"
    else:
        G.check_close(G.host(outs["separate"]), want, cfg.dtype, f"lsa three kernels[L={L},d_in={d_in},Hkv={Hkv}]")
    # the same kernel fed from weights packed into MFMA-operand order: registers instead of LDS for the weight tile
    if (cfg.lsa_heads // Hkv) % 2:
        with pytest.raises(moa.MoaError):       # a shape the one-kernel form does not take has no packed form
            moa.lsa_pack_weights(shape, *dw[:3])
        return
    packed = moa.lsa_pack_weights(shape, *dw[:3])
    out = torch.full((T, cfg.d_lsa), float("nan"), dtype=G.TDT[cfg.dtype], device="cuda")
    moa.lsa_packed(shape, G.dev(hs, cfg.dtype), packed, dw[3], out, ws)
    torch.cuda.synchronize()
    G.check_close(G.host(out), want, cfg.dtype, f"lsa one-kernel, packed weights[L={L},d_in={d_in},Hkv={Hkv}]")
    assert torch.equal(outs["fused"], out), "packing changes where a weight is read from, not the arithmetic"


def ca_setup(cfg, Mq):
    w = mi.ca_weights(cfg)
    xq = mi.ca_queries(cfg, Mq)
    P_cap = cfg.P_max + 5
    kc, vc = mi.kv_cache(cfg, which=1000, P_cap=P_cap)
    ca_len = mi.prefix_lengths(cfg)
    return w, xq, kc, vc, ca_len, P_cap


@pytest.fixture(params=["split", "whole"])
def attn_kernel(request, moa):
    """Both MFMA forms of the attention core (split-KV + merge, whole key range per workgroup) on every case;
    without the override the library picks by key-range length.  No effect on the generic (fp32, odd head_dim) path."""
    moa.debug_force_attn_kernel(request.param)
    yield request.param
    moa.debug_force_attn_kernel("auto")


@pytest.mark.parametrize("case", list(CASES))
def test_cross_attn_parity(G, moa, oracle, case, attn_kernel):
    cfg = CASES[case]
    Mq = cfg.M
    w, xq, kc, vc, ca_len, P_cap = ca_setup(cfg, Mq)
    print(f"[case] cross_attn {case} B={cfg.B} Mq={Mq} len={list(ca_len)} P_cap={P_cap}", flush=True)
    shape = G.shape_of(cfg)
    ws = G.workspace(shape, cfg.B, P_cap, Mq, 0)
    out = torch.empty((cfg.B, Mq, cfg.d), dtype=G.TDT[cfg.dtype], device="cuda")
    st = G.status_word()
    moa.cross_attn_draft(shape, G.dev(xq, cfg.dtype), G.dev(w["wq"], cfg.dtype), G.dev(w["wo"], cfg.dtype),
                         G.dev(kc, cfg.dtype), G.dev(vc, cfg.dtype), G.dev(ca_len), P_cap, out, ws, st)
    torch.cuda.synchronize()
    want = oracle.cross_attn(xq, w["wq"], w["wo"], kc, vc, ca_len, cfg.H, cfg.Hkv, cfg.dh)
    G.check_close(G.host(out), want, cfg.dtype, f"cross_attn[{case}]")
    assert st.item() == 0


@pytest.mark.parametrize("case", list(CASES))
def test_tree_verify_parity(G, moa, oracle, case, attn_kernel):
    cfg = CASES[case]
    w = mi.verify_weights(cfg)
    x = mi.verify_inputs(cfg)
    P_cap = cfg.P_max + 3
    kc, vc = mi.kv_cache(cfg, which=0, P_cap=P_cap)
    plen = mi.prefix_lengths(cfg)
    parent = mi.trees(cfg)
    mask_np, _ = oracle.tree_build(parent)
    print(f"[case] tree_verify {case} B={cfg.B} M={cfg.M} len={list(plen)} P_cap={P_cap}", flush=True)
    shape = G.shape_of(cfg)
    ws = G.workspace(shape, cfg.B, P_cap, cfg.M, 0)
    tdt = G.TDT[cfg.dtype]
    out = torch.empty((cfg.B, cfg.M, cfg.d), dtype=tdt, device="cuda")
    kt = torch.empty((cfg.B, cfg.Hkv, cfg.M, cfg.dh), dtype=tdt, device="cuda")
    vt = torch.empty_like(kt)
    st = G.status_word()
    mask = G.dev(mask_np.view(np.int64))
    moa.tree_verify_attn(shape, G.dev(x, cfg.dtype), *(G.dev(w[k], cfg.dtype) for k in ("wq", "wk", "wv", "wo")),
                         G.dev(kc, cfg.dtype), G.dev(vc, cfg.dtype), G.dev(plen), P_cap, mask, out, kt, vt, ws, st)
    torch.cuda.synchronize()
    want, wkt, wvt = oracle.tree_verify_attn(x, w["wq"], w["wk"], w["wv"], w["wo"], kc, vc, plen, mask_np,
                                             cfg.H, cfg.Hkv, cfg.dh)
    G.check_close(G.host(kt), wkt, cfg.dtype, f"tree_verify.k_tree[{case}]")
    G.check_close(G.host(vt), wvt, cfg.dtype, f"tree_verify.v_tree[{case}]")
    G.check_close(G.host(out), want, cfg.dtype, f"tree_verify[{case}]")
    assert st.item() == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tree_verify_empty_prefix_and_peaked_scores(G, moa, oracle, dtype, attn_kernel):
    """prefix_len = 0 (tree-only keys) for one sequence; queries scaled so the softmax is peaked."""
    cfg = small_cfg(dtype, B=2, M=33, D=6, P_max=40, dh=64, H=4, Hkv=2, d=256)
    w = mi.verify_weights(cfg)
    w["wq"] = mi.quantize(w["wq"] * 4.0, dtype)
    x = mi.verify_inputs(cfg)
    P_cap = 48
    kc, vc = mi.kv_cache(cfg, which=0, P_cap=P_cap)
    plen = np.array([0, 40], dtype=np.int32)
    parent = mi.trees(cfg)
    mask_np, _ = oracle.tree_build(parent)
    print(f"[case] tree_verify empty-prefix/peaked {dtype}", flush=True)
    shape = G.shape_of(cfg)
    ws = G.workspace(shape, cfg.B, P_cap, cfg.M, 0)
    tdt = G.TDT[dtype]
    out = torch.empty((cfg.B, cfg.M, cfg.d), dtype=tdt, device="cuda")
    kt = torch.empty((cfg.B, cfg.Hkv, cfg.M, cfg.dh), dtype=tdt, device="cuda")
    vt = torch.empty_like(kt)
    st = G.status_word()
    moa.tree_verify_attn(shape, G.dev(x, dtype), *(G.dev(w[k], dtype) for k in ("wq", "wk", "wv", "wo")),
                         G.dev(kc, dtype), G.dev(vc, dtype), G.dev(plen), P_cap, G.dev(mask_np.view(np.int64)),
                         out, kt, vt, ws, st)
    torch.cuda.synchronize()
    want, _, _ = oracle.tree_verify_attn(x, w["wq"], w["wk"], w["wv"], w["wo"], kc, vc, plen, mask_np,
                                         cfg.H, cfg.Hkv, cfg.dh)
    G.check_close(G.host(out), want, dtype, f"tree_verify[empty-prefix,{dtype}]")
    assert st.item() == 0


@pytest.mark.parametrize("case", ["C0_f32", "small_bf16_dh128", "small_bf16_dh64"])
def test_ca_kv_append_parity(G, moa, oracle, case):
    cfg = CASES[case]
    w = mi.ca_weights(cfg)
    B, P_cap = cfg.B, 50
    rng = mi.rng_for(cfg, mi.S_LSA, extra=5)
    counts = rng.integers(0, 9, size=B)
    counts[0] = 8
    tok_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    T = int(tok_off[-1])
    mem = mi.normal(rng, (T, cfg.d_lsa), cfg.dtype)
    kc0, vc0 = mi.kv_cache(cfg, which=1000, P_cap=P_cap)
    ca_len0 = rng.integers(0, 30, size=B).astype(np.int32)
    print(f"[case] ca_kv_append {case} counts={list(counts)} ca_len={list(ca_len0)}", flush=True)
    shape = G.shape_of(cfg)
    kc, vc, ca_len = G.dev(kc0, cfg.dtype), G.dev(vc0, cfg.dtype), G.dev(ca_len0)
    st = G.status_word()
    # with a workspace the bf16 projection takes the split-K weight-streaming kernel, without it the fallback
    ws = G.workspace(shape, B, P_cap, cfg.M, T) if case.endswith("dh128") else None
    moa.ca_kv_append(shape, G.dev(mem, cfg.dtype), G.dev(tok_off), G.dev(w["wk"], cfg.dtype), G.dev(w["wv"], cfg.dtype),
                     kc, vc, ca_len, P_cap, st, ws)
    torch.cuda.synchronize()
    wk_, wv_, wl = kc0.astype(np.float64), vc0.astype(np.float64), ca_len0.copy()
    oracle.ca_kv_append(mem, tok_off, w["wk"], w["wv"], wk_, wv_, wl, cfg.Hkv, cfg.dh)
    assert np.array_equal(ca_len.cpu().numpy(), wl)
    G.check_close(G.host(kc), wk_, cfg.dtype, f"ca_kv_append.k[{case}]")
    G.check_close(G.host(vc), wv_, cfg.dtype, f"ca_kv_append.v[{case}]")
    assert st.item() == 0


def test_ca_kv_append_overflow_is_flagged_and_clamped(G, moa):
    cfg = CASES["small_bf16_dh128"]
    w = mi.ca_weights(cfg)
    B, P_cap = cfg.B, 16
    tok_off = np.array([0, 4, 8, 12], dtype=np.int32)
    mem = mi.normal(np.random.default_rng(1), (12, cfg.d_lsa), cfg.dtype)
    kc = torch.zeros((B, cfg.Hkv, P_cap, cfg.dh), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    ca_len = G.dev(np.array([0, 14, 16], dtype=np.int32))
    st = G.status_word()
    moa.ca_kv_append(G.shape_of(cfg), G.dev(mem, "bf16"), G.dev(tok_off), G.dev(w["wk"], "bf16"), G.dev(w["wv"], "bf16"),
                     kc, vc, ca_len, P_cap, st)
    torch.cuda.synchronize()
    assert list(ca_len.cpu().numpy()) == [4, 16, 16]
    assert st.item() & moa.DEV_CACHE_FULL


def test_cross_attn_empty_memory_is_flagged(G, moa, attn_kernel):
    cfg = CASES["small_bf16_dh128"]
    w, xq, kc, vc, ca_len, P_cap = ca_setup(cfg, 4)
    ca_len = ca_len.copy()
    ca_len[1] = 0
    shape = G.shape_of(cfg)
    ws = G.workspace(shape, cfg.B, P_cap, 4, 0)
    out = torch.full((cfg.B, 4, cfg.d), 9.0, dtype=torch.bfloat16, device="cuda")
    st = G.status_word()
    moa.cross_attn_draft(shape, G.dev(xq, "bf16"), G.dev(w["wq"], "bf16"), G.dev(w["wo"], "bf16"),
                         G.dev(kc, "bf16"), G.dev(vc, "bf16"), G.dev(ca_len), P_cap, out, ws, st)
    torch.cuda.synchronize()
    assert st.item() & moa.DEV_EMPTY_KEYS
    assert torch.all(out[1] == 0)


def test_cross_attn_input_independence(G, moa):
    """Property 3 (input-independence): a batch of queries equals the same queries one at a time, bit for bit
    per row here because each row's arithmetic does not depend on its neighbours."""
    cfg = CASES["small_bf16_dh128"]
    w, xq, kc, vc, ca_len, P_cap = ca_setup(cfg, 9)
    shape = G.shape_of(cfg)
    ws = G.workspace(shape, cfg.B, P_cap, 9, 0)
    args = [G.dev(w["wq"], "bf16"), G.dev(w["wo"], "bf16"), G.dev(kc, "bf16"), G.dev(vc, "bf16"), G.dev(ca_len), P_cap]
    out = torch.empty((cfg.B, 9, cfg.d), dtype=torch.bfloat16, device="cuda")
    moa.cross_attn_draft(shape, G.dev(xq, "bf16"), *args, out, ws)
    for m in (0, 4, 8):
        one = torch.empty((cfg.B, 1, cfg.d), dtype=torch.bfloat16, device="cuda")
        moa.cross_attn_draft(shape, G.dev(xq[:, m:m + 1], "bf16"), *args, one, ws)
        torch.cuda.synchronize()
        diff = (one[:, 0].float() - out[:, m].float()).abs().max().item()
        print(f"[parity] input-independence row {m}: max diff {diff:.3e}", flush=True)
        assert diff <= 2e-2
