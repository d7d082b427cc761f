"""One whole drafting cycle in tree form on the GPU, entry point by entry point (Alg. 1, inner loop): per level the new
branches' token embeddings go through the Self-Attention layer, the Cross-Attention over the memory, one reused LLM
decoder layer (Target Layer Inference with one layer), the head's logits, the top-B log-probabilities and the tree
expansion; at the end the best m candidates become the tree that verification takes.  The same cycle is run with the
oracle's functions; the two must build the same tree (every discrete decision) and agree on the hidden states.

The driver below is plumbing (gathers, reshapes, bookkeeping of node numbers); every step of the method is a library
call on one side and an oracle call on the other."""
import numpy as np
import pytest
import torch

import moa_inputs as mi

pytestmark = pytest.mark.gpu

EPS, THETA = 1e-5, 10000.0


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


def make_problem(seed, dtype):
    rng = np.random.default_rng(seed)
    p = dict(B=2, P=20, d=256, H=4, Hkv=2, Hkv_sa=1, dh=64, V=512, Bw=4, D=3, m=12, dtype=dtype)
    d, H, dh, V = p["d"], p["H"], p["dh"], p["V"]
    E, ekv, ekv_sa, dff = H * dh, p["Hkv"] * dh, p["Hkv_sa"] * dh, 7 * d // 2
    q = lambda a: mi.quantize(np.asarray(a, dtype=np.float32), dtype)
    w = lambda o, i: q(rng.standard_normal((o, i)) / np.sqrt(i))
    p["embed"] = q(rng.standard_normal((V, d)))
    p["sa_w"] = dict(wq=w(E, d), wk=w(ekv_sa, d), wv=w(ekv_sa, d), wo=w(d, E))
    p["ca_w"] = dict(wq=w(E, d), wo=w(d, E))
    p["tli_w"] = dict(g_attn=q(1 + 0.1 * rng.standard_normal(d)), wq=w(E, d), wk=w(ekv, d), wv=w(ekv, d), wo=w(d, E),
                      g_mlp=q(1 + 0.1 * rng.standard_normal(d)), w_gate=w(dff, d), w_up=w(dff, d), w_down=w(d, dff))
    p["head"] = q(rng.standard_normal((V, d)) * 4.0 / np.sqrt(d))            # peaked enough for clear rankings
    cache = lambda hk: (q(rng.standard_normal((p["B"], hk, p["P"] + 4, dh))), q(rng.standard_normal((p["B"], hk, p["P"] + 4, dh))))
    p["sa_cache"], p["ca_mem"], p["tli_cache"] = cache(p["Hkv_sa"]), cache(p["Hkv"]), cache(p["Hkv"])
    p["plen"] = np.array([p["P"], p["P"] - 7], dtype=np.int32)
    p["root_tok"] = rng.integers(0, V, p["B"]).astype(np.int32)
    return p


def node_bookkeeping(level, Bw, frontier, cand_parent, prev_frontier):
    """Draft-time node numbers of the level's branches and of their parents (root = 0; level l branch f = 1 + (l-1) Bw + f)."""
    B = frontier.shape[0]
    parents = np.zeros((B, Bw), dtype=np.int32)
    if level > 1:
        for b in range(B):
            where = {int(c): f for f, c in enumerate(prev_frontier[b])}
            parents[b] = [1 + (level - 2) * Bw + where[int(cand_parent[b, c])] for c in frontier[b]]
    return parents


def run_cycle(p, side, G=None, moa=None, oracle=None):
    """side = "gpu" or "oracle".  Returns the final tree and the hidden states of every forwarded node."""
    B, Bw, D, m, d, H, dh, V = p["B"], p["Bw"], p["D"], p["m"], p["d"], p["H"], p["dh"], p["V"]
    dt = p["dtype"]
    Md = 1 + (D - 1) * Bw                                  # nodes that get a forward pass: root + branches of levels 1..D-1
    n_max = Bw + (D - 1) * Bw * Bw
    parent_d = np.zeros((B, Md), dtype=np.int32)
    parent_d[:, 0] = -1
    tok_d = np.zeros((B, Md), dtype=np.int32)
    tok_d[:, 0] = p["root_tok"]
    hidden = np.zeros((B, Md, d))
    lp, tk, pr = np.zeros((B, n_max), np.float32), np.zeros((B, n_max), np.int32), np.zeros((B, n_max), np.int32)
    fr = np.full((B, Bw), -1, np.int32)
    if side == "gpu":
        tdt = G.TDT[dt]
        dev = lambda a: G.dev(a, dt)
        sh = lambda hkv: moa.Shape(1, d, H, hkv, dh, d, H, hkv, G.MDT[dt])
        shape_sa, shape = sh(p["Hkv_sa"]), sh(p["Hkv"])
        dcfg = moa.DecoderCfg(7 * d // 2, EPS, THETA)
        P_cap = p["P"] + 4
        ws = torch.empty(max(moa.workspace_bytes(shape, B, P_cap, Md, 0), moa.workspace_bytes(shape_sa, B, P_cap, Md, 0),
                             moa.tli_workspace_bytes(shape, dcfg, B, P_cap, Md), 4096),
                         dtype=torch.uint8, device="cuda")
        tws = torch.empty(max(moa.topk_workspace_bytes(B * Bw, V, Bw), 256), dtype=torch.uint8, device="cuda")
        W = {k: {kk: dev(vv) for kk, vv in p[k].items()} for k in ("sa_w", "ca_w", "tli_w")}
        head, embed = dev(p["head"]), dev(p["embed"])
        caches = {k: (dev(p[k][0]), dev(p[k][1])) for k in ("sa_cache", "ca_mem", "tli_cache")}
        plen = G.dev(p["plen"])
        mask = torch.zeros((B, Md, (Md + 63) // 64), dtype=torch.int64, device="cuda")
        depth = torch.zeros((B, Md), dtype=torch.int32, device="cuda")
        kd_sa = torch.zeros((B, p["Hkv_sa"], Md, dh), dtype=tdt, device="cuda")
        vd_sa = torch.zeros_like(kd_sa)
        kd_t = torch.zeros((B, p["Hkv"], Md, dh), dtype=tdt, device="cuda")
        vd_t = torch.zeros_like(kd_t)
        dlp, dtk, dpr, dfr = (G.dev(a) for a in (lp, tk, pr, fr))
        st = G.status_word()
    else:
        kd_sa, vd_sa = np.zeros((B, p["Hkv_sa"], Md, dh)), np.zeros((B, p["Hkv_sa"], Md, dh))
        kd_t, vd_t = np.zeros((B, p["Hkv"], Md, dh)), np.zeros((B, p["Hkv"], Md, dh))
    n0, Mn, prev_fr = 0, 1, None
    for level in range(1, D + 1):
        emb = p["embed"][tok_d[:, n0:n0 + Mn]]                                   # [B, Mn, d]
        if side == "gpu":
            moa.tree_build(G.dev(parent_d), mask, depth, st)
            q_sa = torch.empty((B, Mn, d), dtype=tdt, device="cuda")
            moa.self_attn_draft(shape_sa, dev(emb), n0, W["sa_w"]["wq"], W["sa_w"]["wk"], W["sa_w"]["wv"], W["sa_w"]["wo"],
                                *caches["sa_cache"], plen, P_cap, mask, q_sa, kd_sa, vd_sa, ws, st)
            o = torch.empty_like(q_sa)
            moa.cross_attn_draft(shape, q_sa, W["ca_w"]["wq"], W["ca_w"]["wo"], *caches["ca_mem"], plen, P_cap, o, ws, st)
            h = torch.empty_like(q_sa)
            moa.tli_decoder_layer(shape, dcfg, o, n0, W["tli_w"], *caches["tli_cache"], plen, P_cap, mask, depth, h, kd_t, vd_t, ws, st)
            logits = torch.empty((B * Mn, V), dtype=tdt, device="cuda")
            moa.linear(h.view(B * Mn, d), head, logits)
            ctk = torch.zeros((B * Mn, Bw), dtype=torch.int32, device="cuda")
            clp = torch.zeros((B * Mn, Bw), dtype=torch.float32, device="cuda")
            moa.topk_logprob(logits, Bw, ctk, clp, tws)
            moa.tree_expand_level(level, clp.view(B, Mn, Bw), ctk.view(B, Mn, Bw), dlp, dtk, dpr, dfr)
            torch.cuda.synchronize()
            assert st.item() == 0
            hidden[:, n0:n0 + Mn] = G.host(h)
            fr, pr_now, tk_now = dfr.cpu().numpy(), dpr.cpu().numpy(), dtk.cpu().numpy()
        else:
            sw, cw = p["sa_w"], p["ca_w"]
            q_sa = oracle.self_attn_draft(emb, parent_d, n0, sw["wq"], sw["wk"], sw["wv"], sw["wo"], *p["sa_cache"], p["plen"],
                                          kd_sa, vd_sa, H, p["Hkv_sa"], dh)
            o = oracle.cross_attn(q_sa, cw["wq"], cw["wo"], *p["ca_mem"], p["plen"], H, p["Hkv"], dh)
            h = oracle.tli_decoder_layer(o, parent_d, n0, p["tli_w"], *p["tli_cache"], p["plen"], kd_t, vd_t, H, p["Hkv"], dh, EPS, THETA)
            logits = h.reshape(B * Mn, d) @ p["head"].astype(np.float64).T
            ctk, clp = oracle.topk_logprob(logits, Bw)
            ctk, clp = ctk.reshape(B, Mn, Bw), clp.reshape(B, Mn, Bw).astype(np.float32)
            for b in range(B):
                oracle.tree_expand_level(level, clp[b], ctk[b], lp[b], tk[b], pr[b], fr[b])
            hidden[:, n0:n0 + Mn] = h
            pr_now, tk_now = pr, tk
        if level < D:                                                           # the new branches get node numbers and a forward pass
            parents = node_bookkeeping(level, Bw, fr, pr_now, prev_fr)
            n0, Mn = 1 + (level - 1) * Bw, Bw
            parent_d[:, n0:n0 + Mn] = parents
            tok_d[:, n0:n0 + Mn] = np.take_along_axis(tk_now, fr.astype(np.int64), axis=1)
            prev_fr = fr.copy()
    if side == "gpu":
        parent = torch.zeros((B, 1 + m), dtype=torch.int32, device="cuda")
        tok = torch.zeros_like(parent)
        nc = torch.zeros_like(parent)
        moa.tree_finalize(n_max, m, G.dev(p["root_tok"]), dlp, dtk, dpr, parent, tok, nc, st)
        torch.cuda.synchronize()
        assert st.item() == 0
        tree = (parent.cpu().numpy(), tok.cpu().numpy(), nc.cpu().numpy())
        cand_lp = dlp.cpu().numpy()
    else:
        outs = [oracle.tree_finalize(n_max, m, p["root_tok"][b], lp[b], tk[b], pr[b]) for b in range(B)]
        tree = tuple(np.stack([o[i] for o in outs]) for i in range(3))
        cand_lp = lp
    return tree, hidden, parent_d, tok_d, cand_lp


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_draft_cycle_builds_the_same_tree(G, moa, oracle, seed):
    p = make_problem(seed, "f32")
    print(f"[case] draft_cycle f32 seed={seed} B={p['B']} breadth={p['Bw']} depth={p['D']} keep={p['m']}", flush=True)
    (gp, gt, gc), gh, gpd, gtd, glp = run_cycle(p, "gpu", G=G, moa=moa)
    (wp, wt, wc), wh, wpd, wtd, wlp = run_cycle(p, "oracle", oracle=oracle)
    # the branches that were forwarded (tokens, parents) and the final tree: every discrete decision
    assert np.array_equal(gtd, wtd) and np.array_equal(gpd, wpd)
    assert np.array_equal(gc, wc) and np.array_equal(gp, wp) and np.array_equal(gt, wt)
    G.check_close(gh, wh, "f32", "draft_cycle.hidden[f32]", residual_stream=True)
    assert np.max(np.abs(glp.astype(np.float64) - wlp)) < 1e-4             # joint log-probabilities of all candidates
    for b in range(p["B"]):                                                # what verification takes: a tree in depth order
        assert gp[b, 0] == -1 and all(0 <= gp[b, i] < i for i in range(1, gp.shape[1]))


def test_draft_cycle_bf16_runs_and_gives_a_valid_tree(G, moa, oracle):
    """In bf16 the logits themselves are rounded, so rankings may legitimately differ from the fp64 cycle after the first
    level; what must hold: the root level agrees with the oracle, and the cycle ends in a valid tree of known tokens."""
    p = make_problem(3, "bf16")
    (gp, gt, gc), gh, gpd, gtd, glp = run_cycle(p, "gpu", G=G, moa=moa)
    (_, _, _), wh, _, _, _ = run_cycle(p, "oracle", oracle=oracle)
    G.check_close(gh[:, :1], wh[:, :1], "bf16", "draft_cycle.hidden[bf16, root]", residual_stream=True)
    assert np.all(np.isfinite(gh)) and np.all(glp <= 0)
    for b in range(p["B"]):
        assert gp[b, 0] == -1 and all(0 <= gp[b, i] < i for i in range(1, gp.shape[1]))
        assert gt[b, 0] == p["root_tok"][b] and np.all((gt[b] >= 0) & (gt[b] < p["V"]))
