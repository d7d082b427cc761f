"""One whole draft step on the CPU oracle (TEST INFRASTRUCTURE ONLY): the same sequence of stages the
GPU library's moa_draft_step runs, on the numpy inputs of moa_inputs.step_workload."""
from __future__ import annotations

import time

import numpy as np

import oracle as orc


def run_step(work, timings: dict | None = None):
    cfg = work["cfg"]
    t = time.perf_counter()

    def lap(name):
        nonlocal t
        now = time.perf_counter()
        if timings is not None:
            timings[name] = timings.get(name, 0.0) + (now - t)
        t = now

    mask, depth = orc.tree_build(work["parent"])
    lap("tree_build")
    w = work["lsa_w"]
    lsa_out = orc.lsa(work["lsa_hs"], w["wq"], w["wk"], w["wv"], w["wo"], cfg.lsa_heads, cfg.Hkv, cfg.dh)
    lap("lsa")
    ca_k = np.array(work["ca_k"], dtype=np.float64)
    ca_v = np.array(work["ca_v"], dtype=np.float64)
    ca_len = work["ca_len0"].copy()
    cw = work["ca_w"]
    orc.ca_kv_append(lsa_out, work["tok_off"], cw["wk"], cw["wv"], ca_k, ca_v, ca_len, cfg.Hkv, cfg.dh)
    lap("ca_kv_append")
    ca_xq, sa_res = work["ca_xq"], {}
    if work.get("sa") is not None:            # Alg. 1: q <- SA_layer(token_embed(y)); o <- CA_layer(q, kv)
        sa = work["sa"]
        hkv_s = sa["w"]["wk"].shape[0] // cfg.dh
        kd = np.zeros((cfg.B, hkv_s, cfg.M, cfg.dh))
        vd = np.zeros_like(kd)
        ca_xq = orc.self_attn_draft(sa["emb"], work["parent"], 0, sa["w"]["wq"], sa["w"]["wk"], sa["w"]["wv"], sa["w"]["wo"],
                                    sa["kcache"], sa["vcache"], work["prefix_len"], kd, vd, cfg.H, hkv_s, cfg.dh)
        sa_res = dict(sa_out=ca_xq, sa_k_draft=kd, sa_v_draft=vd)
        lap("self_attn")
    ca_out = orc.cross_attn(ca_xq, cw["wq"], cw["wo"], ca_k, ca_v, ca_len, cfg.H, cfg.Hkv, cfg.dh)
    lap("cross_attn")
    v_out, v_kt, v_vt = [], [], []
    for lay in work["layers"]:
        lw = lay["w"]
        o, kt, vt = orc.tree_verify_attn(lay["x"], lw["wq"], lw["wk"], lw["wv"], lw["wo"], lay["kcache"], lay["vcache"],
                                         work["prefix_len"], mask, cfg.H, cfg.Hkv, cfg.dh)
        v_out.append(o)
        v_kt.append(kt)
        v_vt.append(vt)
    lap("tree_verify")
    path, n_path, bonus = orc.tree_accept(work["parent"], work["tok"], work["tgt"])
    lap("tree_accept")
    return dict(mask=mask, depth=depth, lsa_out=lsa_out, ca_k=ca_k, ca_v=ca_v, ca_len=ca_len, ca_out=ca_out,
                v_out=v_out, v_ktree=v_kt, v_vtree=v_vt, path=path, n_path=n_path, bonus=bonus, **sa_res)
