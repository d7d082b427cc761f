#!/usr/bin/env python3
"""Benchmark of the Mixture-of-Attentions draft step on one MI355X.

A "step" is one pass of the whole hot path through moa_draft_step: tree mask -> LSA of the B*M newly
verified tokens -> CA memory append -> CA of the M tree tokens -> n tree-verify attention layers ->
accept walk.  Inputs are synthetic (seeded, Llama-3-8B shape by default) and resident in HBM before the
timed region; several independent buffer sets are rotated so that a step's weights and caches are not
served from the 256 MiB Infinity Cache.

Prints ONE JSON line: metric = draft-tree tokens/s (B*M / step time), plus
  "roofline"     : the kernel with the largest share of the step, timed with hipEvents recorded by the
                   library around that kernel's launches inside the timed region;
  "cpu_baseline" : the fp64 CPU oracle timed on the same workload on this machine's host cores;
  "pieces"       : per launch site time, algorithmic bytes / flops and the roofline that bounds it.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak
VEC_F32_PEAK_TFLOPS = 157.3

# HBM bytes per launch as counted by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the counters read for a
# plain device copy of known size) are kept in a tracked summary that names the commit it was measured at and the
# kernels the step launched then; the figure is reported only while the step still launches exactly those kernels.
PMC_TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "c1_draft_step_hbm_traffic.json")


def recorded_traffic(kernel, kernels_seen, default_workload):
    """HBM bytes per launch of `kernel` from the tracked counter summary, or None when the summary does not describe
    this run (another workload, a kernel set that has changed since, no summary)."""
    if not default_workload:
        return None, "not the workload the counters were collected on"
    try:
        with open(PMC_TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, "no tracked counter summary"
    if sorted(rec.get("kernel_set", [])) != sorted(kernels_seen):
        return None, f"kernel set changed since the counters were collected at {rec.get('commit')}"
    mib = rec.get("traffic_MiB_per_launch", {}).get(kernel)
    if mib is None:
        return None, "kernel not in the tracked counter summary"
    return int(mib * 2 ** 20), f"rocprofv3 FETCH_SIZE/WRITE_SIZE at {rec.get('commit')}"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C1", help="C0..C4 (moa_inputs.CONFIGS); C1 is the headline workload")
    ap.add_argument("--verify-layers", type=int, default=1, help="tree-verify attention layers per step")
    ap.add_argument("--sets", type=int, default=3, help="independent buffer sets rotated between steps")
    ap.add_argument("--profile-steps", type=int, default=12, help="untimed steps with events around every kernel")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the two probes of the practical HBM / MFMA ceilings")
    ap.add_argument("--sample-every", type=int, default=7,
                    help="in the timed region, put events around every n-th launch of the dominant kernel only "
                         "(an event pair costs the stream a few microseconds)")
    ap.add_argument("--schedule", choices=list(SCHEDULES), default="grouped",
                    help="grouped: independent same-shape calls share a launch (default); two-stream: fork the "
                         "step's independent branch onto a second stream (kernels then overlap, so per-kernel "
                         "durations no longer describe one kernel alone); sequential: one launch per stage")
    ap.add_argument("--d-lsa-in", type=int, default=0, help="override the LSA input width (default 2*E_kv)")
    ap.add_argument("--lsa-tokens", default="tree",
                    help="tokens per sequence that are new to the Layer Self-Attention in a step: 'tree' (M, the "
                         "headline), 'prefix' (first cycle: the whole prompt) or an integer (accepted tokens, ~5)")
    ap.add_argument("--with-sa", action="store_true",
                    help="run the drafter's Self-Attention layer in front of the cross-attention (its output becomes "
                         "the CA queries); not part of the headline step")
    ap.add_argument("--no-pack", action="store_true",
                    help="feed the LSA kernel the plain Wq / Wk / Wv instead of the copy packed once into MFMA-operand order")
    ap.add_argument("--no-fold", action="store_true",
                    help="keep the memory's K/V projection a launch of its own instead of folding ca_wk/ca_wv with lsa_wo")
    ap.add_argument("--drafter-blocks", action="store_true",
                    help="also time the MLP sub-blocks behind the drafter's LSA / SA / CA layers (moa_mlp_block at the "
                         "sizes of the appendix table) on the tree tokens; reported under 'drafter_blocks'")
    ap.add_argument("--tli-layers", type=int, default=0,
                    help="after the timed region, also time this many reused LLM decoder layers (Target Layer Inference) "
                         "on the tree tokens, each with its own weights; reported under 'tli', not in the headline")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run three plain device copies of this many MiB (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


SCHEDULES = {"grouped": 0, "two-stream": 1, "sequential": 2}


def lsa_token_count(cfg, lsa_tokens):
    import moa_inputs as mi
    if lsa_tokens == "tree":
        return cfg.B * cfg.M
    if lsa_tokens == "prefix":
        return int(mi.prefix_lengths(cfg).sum())
    return cfg.B * int(lsa_tokens)


def site_costs(cfg, n_layers, schedule="grouped", lsa_tokens="tree", with_sa=False, fold=True):
    """Algorithmic bytes and flops per launch site for one step: what the call must read and write once
    (inputs, weights, caches, outputs) and 2*MACs of the contractions as defined."""
    es = 2 if cfg.dtype == "bf16" else 4
    B, M, L, d, H, Hkv, dh = cfg.B, cfg.M, cfg.L, cfg.d, cfg.H, cfg.Hkv, cfg.dh
    T = B * M
    Tl = lsa_token_count(cfg, lsa_tokens)           # rows of the LSA and of the memory append
    d_in, eq, ekv = cfg.d_lsa_in, cfg.lsa_heads * dh, cfg.Hkv * dh
    E = H * dh
    import moa_inputs as mi
    plen = mi.prefix_lengths(cfg).astype(float)

    def lin(R, K, N):
        return dict(bytes=(R * K + N * K + R * N) * es, flops=2.0 * R * K * N)

    c = {}
    c["tree_build"] = dict(bytes=B * M * 4 + B * M * ((M + 63) // 64) * 8 + B * M * 4, flops=0.0)
    attn_flops = 2.0 * Tl * cfg.lsa_heads * L * L * dh + 2.0 * Tl * cfg.lsa_heads * L * dh
    # three-kernel form: the projected rows the first kernel writes and the second reads back are traffic the method
    # does not need (Sec. 3.1.1: a token's layer rows are self-contained), so they are not algorithmic bytes of either
    c["lsa.qkv_proj"] = dict(bytes=(Tl * L * d_in + (eq + 2 * ekv) * d_in) * es, flops=2.0 * Tl * L * d_in * (eq + 2 * ekv))
    c["lsa.layer_attn"] = dict(bytes=Tl * eq * es, flops=attn_flops)
    # one-kernel form: layer rows and weights in, mean-folded heads out
    c["lsa.fused"] = dict(bytes=(Tl * L * d_in + (eq + 2 * ekv) * d_in + Tl * eq) * es,
                          flops=2.0 * Tl * L * d_in * (eq + 2 * ekv) + attn_flops)
    folded = fold and schedule != "sequential" and Tl <= 4096       # one launch: LSA output + the memory's new K/V rows
    c["lsa.o_proj"] = lin(Tl, eq, eq + 2 * ekv) if folded else lin(Tl, eq, eq)
    c["ca_append.kv_proj"] = lin(Tl, eq, 2 * ekv)
    c["ca_append.lengths"] = dict(bytes=B * 12, flops=0.0)
    c["ca.q_proj"] = lin(T, d, E)
    cache_ca = 2.0 * Hkv * dh * es * float(plen.sum())
    core_flops_ca = 4.0 * M * H * dh * float(plen.sum())
    c["ca.core"] = dict(bytes=cache_ca + 2 * T * E * es, flops=core_flops_ca)
    c["ca.o_proj"] = lin(T, E, d)
    cache_v = 2.0 * Hkv * dh * es * float(plen.sum()) + 2.0 * B * Hkv * M * dh * es
    core_flops_v = 4.0 * M * H * dh * float((plen + M).sum())
    one = {"verify.qkv_proj": lin(T, d, E + 2 * ekv),
           "verify.core": dict(bytes=cache_v + 2 * T * E * es, flops=core_flops_v),
           "verify.o_proj": lin(T, E, d)}
    c["tree_accept"] = dict(bytes=B * M * 16 + B * 8, flops=0.0)
    if with_sa:
        ekv_s = mi.sa_kv_heads(cfg) * dh
        c["sa.qkv_proj"] = lin(T, d, E + 2 * ekv_s)
        c["sa.core"] = dict(bytes=2.0 * ekv_s * es * float(plen.sum()) + 2.0 * B * ekv_s * M * es + 2 * T * E * es,
                            flops=core_flops_v)
        c["sa.o_proj"] = lin(T, E, d)

    def add(*parts):
        return dict(bytes=sum(p["bytes"] for p in parts), flops=sum(p["flops"] for p in parts))

    # grouped: the first verification layer is launched together with the cross-attention; two-stream: only its
    # projections are (cores and output projections run on different streams)
    paired = {"grouped": set(one), "two-stream": {"verify.qkv_proj"}}.get(schedule, set())
    for k, v in one.items():
        alone = n_layers - 1 if k in paired else n_layers
        c[k] = {kk: vv * alone for kk, vv in v.items()}
    # what one whole step must move once: LSA rows, every weight matrix, the two caches, inputs and outputs -- no
    # intermediate (projected queries, heads, partial sums) counts
    w_lsa = ((eq + 2 * ekv) * d_in + eq * eq + 2 * ekv * eq) * es
    lsa_io = (Tl * L * d_in + Tl * eq + 2 * Tl * ekv) * es
    ca_b = (2 * E * d) * es + cache_ca + 2 * T * d * es
    ver_b = ((2 * E + 2 * ekv) * d) * es + cache_v + 2 * T * d * es + 2 * T * ekv * es
    sa_b = 0.0
    if with_sa:
        ekv_s2 = mi.sa_kv_heads(cfg) * dh
        sa_b = ((2 * E + 2 * ekv_s2) * d) * es + c["sa.core"]["bytes"] - 2 * T * E * es + 2 * T * d * es
    c["__step__"] = dict(bytes=w_lsa + lsa_io + ca_b + n_layers * ver_b + sa_b + c["tree_build"]["bytes"] + c["tree_accept"]["bytes"],
                         flops=c["lsa.fused"]["flops"] + c["lsa.o_proj"]["flops"] + c["ca.q_proj"]["flops"] + core_flops_ca +
                         c["ca.o_proj"]["flops"] + n_layers * sum(v["flops"] for v in one.values()))
    if paired:
        c["tree_build+accept+lengths"] = add(c["tree_build"], c["tree_accept"], c["ca_append.lengths"])
        c["ca.q_proj+verify.qkv_proj"] = add(c["ca.q_proj"], one["verify.qkv_proj"])
        c["ca.core+verify.core"] = add(c["ca.core"], one["verify.core"])
        c["ca.o_proj+verify.o_proj"] = add(c["ca.o_proj"], one["verify.o_proj"])
    return c


def time_tli_layers(cfg, n_layers, stream, moa, mi, reps=20):
    """n_layers reused LLM decoder layers back to back on the tree tokens (each with its own weights and KV cache, so
    nothing is cache-resident when it is touched again), timed as a whole and per kernel."""
    import torch
    from paper_2410_03804_amd.workload import shape_of
    import numpy as np
    dt = cfg.dtype
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    shape = shape_of(cfg)
    dcfg = moa.DecoderCfg(mi.tli_d_ff(cfg), 1e-5, 500000.0)
    B, M = cfg.B, cfg.M
    dev = lambda a, t=None: (torch.from_numpy(np.ascontiguousarray(a)).to(t) if t else torch.from_numpy(np.ascontiguousarray(a))).cuda()
    parent = mi.trees(cfg)
    W = (M + 63) // 64
    mask = torch.zeros((B, M, W), dtype=torch.int64, device="cuda")
    depth = torch.zeros((B, M), dtype=torch.int32, device="cuda")
    moa.tree_build(dev(parent), mask, depth)
    plen = dev(mi.prefix_lengths(cfg))
    layers = []
    for l in range(n_layers):
        w = {k: dev(v, tdt) for k, v in mi.tli_weights(cfg, l).items()}
        kc, vc = mi.kv_cache(cfg, which=20 + l)
        layers.append((w, dev(kc, tdt), dev(vc, tdt),
                       torch.zeros((B, cfg.Hkv, M, cfg.dh), dtype=tdt, device="cuda"),
                       torch.zeros((B, cfg.Hkv, M, cfg.dh), dtype=tdt, device="cuda")))
    P_cap = cfg.P_cap
    ws = torch.empty(moa.tli_workspace_bytes(shape, dcfg, B, P_cap, M), dtype=torch.uint8, device="cuda")
    xs = [dev(mi.verify_inputs(cfg), tdt), torch.zeros((B, M, cfg.d), dtype=tdt, device="cuda")]
    st = torch.zeros(1, dtype=torch.int32, device="cuda")

    def once():
        for l, (w, kc, vc, kd, vd) in enumerate(layers):
            moa.tli_decoder_layer(shape, dcfg, xs[l & 1], 0, w, kc, vc, plen, P_cap, mask, depth, xs[(l + 1) & 1], kd, vd, ws, st, stream)

    for _ in range(3):
        once()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        once()
    torch.cuda.synchronize()
    us_layer = (time.perf_counter() - t0) * 1e6 / (reps * n_layers)
    moa.profile_enable(True)
    for _ in range(4):
        once()
    torch.cuda.synchronize()
    rows = moa.profile_collect()
    moa.profile_enable(False)
    es = 2 if dt == "bf16" else 4
    E, ekv, d, dff = cfg.H * cfg.dh, cfg.E_kv, cfg.d, mi.tli_d_ff(cfg)
    plen_sum = float(mi.prefix_lengths(cfg).sum())
    byt = (E * d * 2 + 2 * ekv * d + 3 * dff * d) * es + 2 * ekv * es * plen_sum + 2 * B * M * d * es
    pieces = sorted(({"site": s_, "kernel": k_, "us_per_layer": round(ms * 1e3 / (4 * n_layers), 2)} for s_, k_, n, ms in rows),
                    key=lambda p: -p["us_per_layer"])
    return {"layers": n_layers, "us_per_layer": round(us_layer, 2), "alg_MiB_per_layer": round(byt / 2 ** 20, 1),
            "gbs": round(byt / (us_layer * 1e-6) / 1e9, 1), "frac_of_hbm_peak": round(byt / (us_layer * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "tokens_per_s": round(B * M / (us_layer * 1e-6), 1), "pieces": pieces}


def time_drafter_blocks(cfg, stream, moa, mi, reps=30):
    """moa_mlp_block behind each of the drafter's three attention layers, on B*M rows, rotating through enough weight
    sets that none is cache-resident when it is touched again."""
    import torch
    import numpy as np
    dt = cfg.dtype
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    mdt = moa.BF16 if dt == "bf16" else moa.F32
    es = 2 if dt == "bf16" else 4
    R = cfg.B * cfg.M
    out = {}
    for which, (d, dff) in mi.drafter_mlp_sizes(cfg).items():
        w0 = mi.drafter_mlp_weights(cfg, which)
        wbytes = 3 * d * dff * es
        nsets = max(2, int(math.ceil(600e6 / wbytes)))
        rng = torch.Generator(device="cuda").manual_seed(7)
        sets = []
        for i in range(nsets):      # the first set is the seeded one; the others only have to be different memory
            sets.append([torch.from_numpy(np.ascontiguousarray(w0[k])).to(tdt).cuda() if i == 0 else
                         (torch.randn(w0[k].shape, device="cuda", generator=rng) * float(np.std(w0[k]))).to(tdt)
                         for k in ("g", "w_gate", "w_up", "w_down")])
        x = torch.randn((R, d), device="cuda", generator=rng).to(tdt)
        res = (0.5 * torch.randn((R, d), device="cuda", generator=rng)).to(tdt)
        y = torch.empty_like(x)
        ws = torch.empty(max(moa.mlp_block_workspace_bytes(mdt, R, d, dff), 256), dtype=torch.uint8, device="cuda")
        for i in range(min(nsets, 3)):
            moa.mlp_block(mdt, x, res, *sets[i], 1e-5, y, ws, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(reps):
            moa.mlp_block(mdt, x, res, *sets[i % nsets], 1e-5, y, ws, stream)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / reps
        byt = wbytes + d * es + 3 * R * d * es
        out[which] = {"rows": R, "d": d, "d_ff": dff, "us": round(us, 2), "alg_MiB": round(byt / 2 ** 20, 1),
                      "gbs": round(byt / (us * 1e-6) / 1e9, 1), "frac_of_hbm_peak": round(byt / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                      "weight_sets": nsets}
        del sets
    return out


def bound_of(bytes_, flops, peak_tflops):
    t_hbm = bytes_ / (HBM_PEAK_GBS * 1e9)
    t_mfma = flops / (peak_tflops * 1e12)
    return ("mfma", t_mfma) if t_mfma > t_hbm else ("hbm", t_hbm)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures the single-GPU draft step only: --gpus {args.gpus} is not supported "
              "(no collectives or sharding are part of this build; run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import moa_inputs as mi
    import paper_2410_03804_amd as moa
    from paper_2410_03804_amd.workload import DeviceStep

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)

    cfg = mi.CONFIGS[args.config]
    if args.d_lsa_in:
        cfg = mi.scaled(cfg, d_lsa_in=args.d_lsa_in)
    K, Wm, P, NL = args.steps, args.warmup, args.profile_steps, args.verify_layers
    nsets = max(1, args.sets)
    total = Wm + P + K
    hot_steps = min(K, 50)
    slots = math.ceil(total / nsets) + 1 + hot_steps      # one fresh length slot per step a set runs

    t_setup = time.perf_counter()
    lsa_tokens = args.lsa_tokens if args.lsa_tokens in ("tree", "prefix") else int(args.lsa_tokens)
    works = [mi.step_workload(cfg, NL, variant=i, lsa_tokens=lsa_tokens, with_sa=args.with_sa) for i in range(nsets)]
    sets = []
    ws = None
    for w in works:
        s = DeviceStep(w, n_len_slots=slots, ws=ws, fold=not args.no_fold, pack=not args.no_pack)
        ws = s.ws
        sets.append(s)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    counter = [0]
    # a stream of our own: the legacy default stream synchronises implicitly with other streams
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(stream)

    plans = [sets[i % nsets].plan(len_slot=i // nsets, schedule=SCHEDULES[args.schedule]) for i in range(total)]

    def one_step():
        i = counter[0]
        counter[0] += 1
        plans[i].run(stream)

    for _ in range(Wm):
        one_step()
    torch.cuda.synchronize()

    # untimed pass with events around every kernel: where does a step's time go
    moa.profile_enable(True)
    for _ in range(P):
        one_step()
    torch.cuda.synchronize()
    rows = moa.profile_collect()
    moa.profile_enable(False)
    per_kernel = {}
    for site, kern, n, ms in rows:
        per_kernel[kern] = per_kernel.get(kern, 0.0) + ms
    dominant = max(per_kernel, key=per_kernel.get) if per_kernel else None

    # timed region: exactly K steps, events only around the dominant kernel's launches
    dom_lps = max(1, round(sum(n for site, kern, n, ms in rows if kern == dominant) / P))
    every = max(1, args.sample_every)
    while math.gcd(every, dom_lps) != 1:       # so that the samples rotate through the kernel's launch sites
        every += 1
    moa.profile_enable(True, only_kernel=dominant, every=every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        one_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_rows = moa.profile_collect()
    moa.profile_enable(False)

    # the same steps again on ONE buffer set: weights and caches then sit in the 256 MiB Infinity Cache (labelled
    # hot-cache figure, not the headline)
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    hot_plans = [sets[0].plan(len_slot=slots - 1 - i, schedule=SCHEDULES[args.schedule]) for i in range(hot_steps)]
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    for pl in hot_plans:
        pl.run(stream)
    torch.cuda.synchronize()
    hot_ms = (time.perf_counter() - h0) * 1e3 / hot_steps

    # what this device delivers in practice: a plain 1 GiB streaming read and a register-resident bf16 MFMA loop
    ceilings = None
    if not args.no_ceilings:
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        big.fill_(1)
        sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
        for _ in range(2):
            moa.probe_read(big, sink, stream)
            mf = moa.probe_mfma(2000, sink, stream)
        torch.cuda.synchronize()
        moa.profile_enable(True)
        for _ in range(10):
            moa.probe_read(big, sink, stream)
            mf = moa.probe_mfma(2000, sink, stream)
        torch.cuda.synchronize()
        pr = {kern: ms / n for site, kern, n, ms in moa.profile_collect()}
        moa.profile_enable(False)
        ceilings = dict(hbm_read_gbs=round(big.numel() / (pr["k_probe_read"] * 1e-3) / 1e9, 1),
                        mfma_bf16_tflops=round(mf / (pr["k_probe_mfma"] * 1e-3) / 1e12, 1),
                        how="plain coalesced 1 GiB read; 4096 wavefronts x 4 independent 32x32x16 bf16 MFMA chains")
        del big

    drafter_blocks = time_drafter_blocks(cfg, stream, moa, mi) if args.drafter_blocks else None
    tli = None
    if args.tli_layers > 0:
        tli = time_tli_layers(cfg, args.tli_layers, stream, moa, mi)

    if args.calibrate_copy_mib > 0:
        n = args.calibrate_copy_mib * (1 << 20)
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    bad = sum(int(s.dev_status.item()) for s in sets)
    if bad:
        print(f"device status word non-zero ({bad}): the workload tripped a device-side check", file=sys.stderr)
        sys.exit(1)

    ms_per_step = (t1 - t0) * 1e3 / K
    tokens = cfg.B * cfg.M
    value = tokens / (ms_per_step * 1e-3)

    costs = site_costs(cfg, NL, schedule=args.schedule, lsa_tokens=lsa_tokens, with_sa=args.with_sa, fold=not args.no_fold)
    peak_mm = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else VEC_F32_PEAK_TFLOPS
    pieces = []
    for site, kern, n, ms in sorted(rows, key=lambda r: -r[3]):
        c = costs.get(site, dict(bytes=0.0, flops=0.0))
        if "reduce" in kern or "merge" in kern:      # second pass of a site: its algorithmic cost is counted once, above
            c = dict(bytes=0.0, flops=0.0)
        us = ms * 1e3 / P                       # per step, all launches of this site
        bnd, t_min = bound_of(c["bytes"], c["flops"], peak_mm)
        pieces.append(dict(site=site, kernel=kern, launches_per_step=n / P, us_per_step=round(us, 3),
                           alg_MiB=round(c["bytes"] / 2 ** 20, 3), gflop=round(c["flops"] / 1e9, 3), bound=bnd,
                           gbs=round(c["bytes"] / (us * 1e-6) / 1e9, 1) if us > 0 else None,
                           tflops=round(c["flops"] / (us * 1e-6) / 1e12, 2) if us > 0 else None,
                           frac_of_bound=round(t_min / (us * 1e-6), 4) if us > 0 else None))
    kernel_us_sum = sum(p["us_per_step"] for p in pieces)

    roofline = None
    if dominant and dom_rows:
        launches = sum(r[2] for r in dom_rows)
        tot_ms = sum(r[3] for r in dom_rows)
        avg_us = tot_ms * 1e3 / launches
        sites = sorted({r[0] for r in dom_rows})
        # launches per step of each site (from the profiling pass); the timed region samples every n-th launch,
        # so bytes and flops are weighted by the launches that were actually bracketed
        site_lps = {site: n / P for site, kern, n, ms in rows if kern == dominant}
        per_step_launches = sum(site_lps.values())
        byt = sum(r[2] * costs[r[0]]["bytes"] / site_lps[r[0]] for r in dom_rows) / launches
        flo = sum(r[2] * costs[r[0]]["flops"] / site_lps[r[0]] for r in dom_rows) / launches
        bnd, _ = bound_of(byt, flo, peak_mm)
        if bnd == "hbm":
            ach = byt / (avg_us * 1e-6) / 1e9
            roofline = dict(bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                            frac=round(ach / HBM_PEAK_GBS, 4), traffic=None)
        else:
            ach = flo / (avg_us * 1e-6) / 1e12
            roofline = dict(bound="mfma", achieved=round(ach, 2), peak=peak_mm, unit="TFLOP/s",
                            frac=round(ach / peak_mm, 4), traffic=None)
        default_workload = (cfg.name == "C1" and not args.d_lsa_in and NL == 1 and args.schedule == "grouped"
                            and lsa_tokens == "tree" and not args.with_sa and not args.no_fold)
        roofline["traffic"], roofline["traffic_source"] = recorded_traffic(dominant, list(per_kernel), default_workload)
        if ceilings:
            ceil = ceilings["hbm_read_gbs"] if roofline["bound"] == "hbm" else ceilings["mfma_bf16_tflops"]
            roofline["frac_of_measured_ceiling"] = round(roofline["achieved"] / ceil, 4)
        roofline.update(kernel=dominant, sites=sites, avg_launch_us=round(avg_us, 3),
                        launches_per_step=per_step_launches, alg_bytes_per_launch=int(byt),
                        flops_per_launch=int(flo), sampled_launches=launches, share_of_kernel_time=round(per_kernel[dominant] / sum(per_kernel.values()), 4))

    # the whole step against the HBM roofline: the bytes the method must move once per step over the step time
    sb, sf = costs["__step__"]["bytes"], costs["__step__"]["flops"]
    step_gbs = sb / (ms_per_step * 1e-3) / 1e9
    step_roofline = dict(bound="hbm", alg_bytes_per_step=int(sb), achieved=round(step_gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                         frac=round(step_gbs / HBM_PEAK_GBS, 4), gflop_per_step=round(sf / 1e9, 2),
                         mfma_frac=round(sf / (ms_per_step * 1e-3) / 1e12 / peak_mm, 4),
                         note="algorithmic bytes of one whole step / step time / 8 TB/s: the '% HBM peak' of the metric")

    cpu = None
    if not args.no_cpu_baseline:
        from oracle.step import run_step
        import oracle as orc
        orc.build()
        tm = {}
        c0 = time.perf_counter()
        run_step(works[0], tm)
        c1 = time.perf_counter()
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = dict(value=round(tokens / (c1 - c0), 3), unit="tokens/s", cores=cores, kind="oracle",
                   sample=f"the whole {cfg.name} step once (all {tokens} tree tokens, {NL} verify layer(s)), fp64, "
                          f"{c1 - c0:.2f} s",
                   seconds=round(c1 - c0, 3), stage_seconds={k: round(v, 4) for k, v in tm.items()})
        # the same once more on a single thread when that stays within the budget of this leg (~30 s)
        if (c1 - c0) * cores <= 30.0:
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            s0 = time.perf_counter()
            run_step(works[0])
            s1 = time.perf_counter()
            gomp.omp_set_num_threads(cores)
            cpu["one_thread"] = dict(value=round(tokens / (s1 - s0), 3), seconds=round(s1 - s0, 3))
        try:
            model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
        except (OSError, StopIteration):
            model = "unknown"
        cpu["host"] = dict(cpu_model=model, logical_cpus=os.cpu_count())

    out = {
        "metric": "draft-tree tokens/sec (draft step + verify attn) at Llama-3-8B shape; % HBM peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} prefix={cfg.P_min}..{cfg.P_max} tree M={cfg.M} depth={cfg.D} "
                               f"L={cfg.L} d={cfg.d} H={cfg.H}/{cfg.Hkv} dh={cfg.dh} d_lsa_in={cfg.d_lsa_in}; "
                               f"LSA on T={lsa_token_count(cfg, lsa_tokens)} tokens ({lsa_tokens}), {NL} tree-verify layer(s)"
                               + ("; Self-Attention layer in front of the CA" if args.with_sa else ""),
                   "verify_layers": NL, "buffer_sets": nsets, "profile_steps": P},
        "roofline": roofline, "step_roofline": step_roofline, "cpu_baseline": cpu, "ceilings": ceilings,
        "tli": tli, "drafter_blocks": drafter_blocks,
        "hot_cache": {"ms_per_step": round(hot_ms, 5), "steps": hot_steps,
                      "note": "one buffer set reused: operands stay in the Infinity Cache; not the headline"},
        "kernel_us_per_step": round(kernel_us_sum, 2), "setup_s": round(setup_s, 1), "pieces": pieces,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
