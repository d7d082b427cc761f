"""moa_draft_step (the whole path on one stream) against the oracle's step, stage by stage."""
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


STEP_CASES = {
    "C0_f32": (mi.CONFIGS["C0"], 2),
    "small_bf16": (mi.Config(name="S", index=8, dtype="bf16", B=3, P_min=80, P_max=300, M=37, D=5, max_branch=4, L=6,
                             d=512, H=8, Hkv=2, dh=128, d_lsa_in=512, rms_norm=True), 2),
    "C1_bf16": (mi.CONFIGS["C1"], 1),
    # the 8B widths on few rows: the grouped projections run with the activation slice resident (two classes of
    # segments, 18 of a workgroup's 64 rows in use), two sequences
    "wide_few_rows_bf16": (mi.Config(name="W18", index=16, dtype="bf16", B=2, P_min=100, P_max=260, M=9, D=3, max_branch=3,
                                     L=8, d=4096, H=32, Hkv=8, dh=128, d_lsa_in=2048, rms_norm=True), 2),
    # degenerate trees: the root alone (M = 1: nothing drafted, the bonus token is the only result) and a prefix
    # shorter than one key tile
    "single_node_bf16": (mi.Config(name="M1", index=9, dtype="bf16", B=2, P_min=5, P_max=40, M=1, D=0, max_branch=4, L=3,
                                   d=256, H=4, Hkv=2, dh=64, d_lsa_in=256, rms_norm=True), 1),
    "single_node_f32": (mi.Config(name="M1f", index=10, dtype="f32", B=1, P_min=3, P_max=3, M=1, D=0, max_branch=4, L=2,
                                  d=128, H=2, Hkv=2, dh=64, d_lsa_in=128, rms_norm=False), 2),
    # the other two token counts the Layer Self-Attention sees (Sec. 3, Alg. 1): the whole prompt on the first cycle
    # (empty memory before the append) and only the accepted tokens of the last cycle (5 per sequence)
    "first_cycle_bf16": (mi.Config(name="FC", index=11, dtype="bf16", B=2, P_min=70, P_max=200, M=37, D=5, max_branch=4,
                                   L=6, d=512, H=8, Hkv=2, dh=128, d_lsa_in=512, rms_norm=True), 1, "prefix"),
    "accepted_only_bf16": (mi.CONFIGS["C1"], 1, 5),
    # the drafter's Self-Attention layer in front of the cross-attention (Alg. 1: q <- SA_layer(token_embed(y)))
    "small_f32_with_sa": (mi.Config(name="SAf", index=14, dtype="f32", B=2, P_min=20, P_max=90, M=19, D=4, max_branch=3, L=3,
                                    d=192, H=6, Hkv=3, dh=32, d_lsa_in=96, rms_norm=True), 1, "tree", True),
    "small_bf16_with_sa": (mi.Config(name="SAb", index=15, dtype="bf16", B=3, P_min=80, P_max=300, M=37, D=5, max_branch=4,
                                     L=6, d=512, H=8, Hkv=4, dh=128, d_lsa_in=512, rms_norm=True), 2, "tree", True),
    "C1_bf16_with_sa": (mi.CONFIGS["C1"], 1, "tree", True),
}


def _case(case):
    cfg, nlayers, *rest = STEP_CASES[case]
    return cfg, nlayers, (rest[0] if rest else "tree"), (rest[1] if len(rest) > 1 else False)


SCHEDULES = {"grouped": 0, "two_stream": 1, "sequential": 2}


@pytest.mark.parametrize("schedule", ["grouped", "two_stream", "sequential"])
@pytest.mark.parametrize("case", list(STEP_CASES))
def test_draft_step_parity(G, oracle, case, schedule):
    from oracle.step import run_step
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers, lsa_tokens, with_sa = _case(case)
    print(f"[case] draft_step {case} {schedule} B={cfg.B} M={cfg.M} layers={nlayers} lsa_tokens={lsa_tokens} sa={with_sa}", flush=True)
    work = mi.step_workload(cfg, n_verify_layers=nlayers, lsa_tokens=lsa_tokens, with_sa=with_sa)
    step = DeviceStep(work)
    step.run(schedule=SCHEDULES[schedule])
    torch.cuda.synchronize()
    want = run_step(work)
    dt = cfg.dtype
    assert step.dev_status.item() == 0
    assert np.array_equal(G.mask_u64(step.mask), want["mask"])
    assert np.array_equal(step.depth.cpu().numpy(), want["depth"])
    G.check_close(G.host(step.lsa_out), want["lsa_out"], dt, f"step.lsa[{case}]")
    assert np.array_equal(step.ca_len[0].cpu().numpy(), want["ca_len"])
    G.check_close(G.host(step.ca_k), want["ca_k"], dt, f"step.ca_k[{case}]")
    G.check_close(G.host(step.ca_v), want["ca_v"], dt, f"step.ca_v[{case}]")
    if with_sa:
        G.check_close(G.host(step.sa["out"]), want["sa_out"], dt, f"step.sa_out[{case}]")
        G.check_close(G.host(step.sa["k_draft"]), want["sa_k_draft"], dt, f"step.sa_k_draft[{case}]")
        G.check_close(G.host(step.sa["v_draft"]), want["sa_v_draft"], dt, f"step.sa_v_draft[{case}]")
    G.check_close(G.host(step.ca_out), want["ca_out"], dt, f"step.ca_out[{case}]")
    for l in range(nlayers):
        G.check_close(G.host(step.v_out[l]), want["v_out"][l], dt, f"step.verify{l}[{case}]")
        G.check_close(G.host(step.v_ktree[l]), want["v_ktree"][l], dt, f"step.k_tree{l}[{case}]")
        G.check_close(G.host(step.v_vtree[l]), want["v_vtree"][l], dt, f"step.v_tree{l}[{case}]")
    assert np.array_equal(step.path.cpu().numpy(), want["path"])
    assert np.array_equal(step.n_path.cpu().numpy(), want["n_path"])
    assert np.array_equal(step.bonus.cpu().numpy(), want["bonus"])


def test_draft_step_bad_argument_launches_nothing(G):
    """A stage that fails its host checks must stop the whole step before the first launch."""
    import paper_2410_03804_amd as moa
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, _ = STEP_CASES["small_bf16"]
    step = DeviceStep(mi.step_workload(cfg, 1))
    step.mask.fill_(-1)
    step.ws = torch.empty(256, dtype=torch.uint8, device="cuda")      # far too small for the later stages
    with pytest.raises(moa.MoaError) as e:
        step.run()
    torch.cuda.synchronize()
    assert e.value.status == -6
    assert torch.all(step.mask == -1)                                  # tree_build (the first stage) never ran


def _step_outputs(step):
    exact = [step.lsa_out, step.ca_k, step.ca_v, step.ca_len[0], step.mask, step.depth, step.path, step.n_path, step.bonus,
             *step.v_ktree, *step.v_vtree]
    merged = [step.ca_out, *step.v_out]          # results that pass through the split-KV merge
    return [t.clone() for t in exact], [t.clone() for t in merged]


@pytest.mark.parametrize("case", ["small_bf16", "C1_bf16", "small_bf16_with_sa"])
def test_schedules_agree(G, case):
    """The step's result must not depend on how its independent pieces are launched: what does not pass through a merge
    of key slices is bit-identical under all three schedules; the grouped and the two-stream schedule launch the two
    attention cores as one pair and agree bit for bit in everything (unless the Self-Attention layer is there: then
    the two-stream schedule has one core per branch); the sequential one may give the cores another
    number of key slices (its merged outputs then agree with theirs to rounding)."""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers, lsa_tokens, with_sa = _case(case)
    work = mi.step_workload(cfg, n_verify_layers=nlayers, lsa_tokens=lsa_tokens, with_sa=with_sa)
    outs = {}
    for name in ("sequential", "two_stream", "two_stream", "grouped", "grouped"):
        print(f"[case] schedules {case} {name}", flush=True)
        step = DeviceStep(work, fold=False)         # the folded memory projection is another arithmetic: tested below
        step.run(schedule=SCHEDULES[name])
        torch.cuda.synchronize()
        assert step.dev_status.item() == 0
        outs.setdefault(name, []).append(_step_outputs(step))
    ref_exact, ref_merged = outs["sequential"][0]
    for name, runs in outs.items():
        for exact, merged in runs:
            for a, b in zip(ref_exact, exact):
                assert torch.equal(a, b), name
            for a, b in zip(ref_merged, merged):
                assert torch.allclose(a.float(), b.float(), atol=G.ABS_TOL[cfg.dtype], rtol=G.REL_TOL[cfg.dtype]), name
    # the pair schedules agree with each other, and each is deterministic; with the Self-Attention layer the two-stream
    # schedule launches each core on its own branch, so there it is only compared bit for bit with itself
    for name in ("grouped", "two_stream"):
        pair_ref = outs[name if with_sa else "grouped"][0][1]
        for _, merged in outs[name]:
            for a, b in zip(pair_ref, merged):
                assert torch.equal(a, b), name


@pytest.mark.parametrize("case", ["small_bf16", "C1_bf16", "C0_f32"])
def test_folded_memory_projection_agrees_with_the_two_projections(G, case):
    """With ca_wk lsa_wo and ca_wv lsa_wo folded once, the memory's new rows come straight from LSA's mean-folded heads
    ((a Wo^T) Wk^T = a (Wk Wo)^T): same rows to rounding, the integer results bit for bit."""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers, lsa_tokens, with_sa = _case(case)
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    res = []
    for fold in (False, True):
        step = DeviceStep(work, fold=fold)
        step.run()
        torch.cuda.synchronize()
        assert step.dev_status.item() == 0
        res.append(step)
    a, b = res
    for name in ("mask", "path", "n_path", "bonus"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    # the LSA output comes from a launch twice as wide when the folded projections share it, which may take another
    # slicing of K: the same sums in another order
    assert torch.allclose(a.lsa_out.float(), b.lsa_out.float(), atol=G.ABS_TOL[cfg.dtype] / 4, rtol=G.REL_TOL[cfg.dtype] / 4)
    assert torch.equal(a.ca_len[0], b.ca_len[0])
    for x, y in ((a.ca_k, b.ca_k), (a.ca_v, b.ca_v), (a.ca_out, b.ca_out)):
        assert torch.allclose(x.float(), y.float(), atol=G.ABS_TOL[cfg.dtype], rtol=G.REL_TOL[cfg.dtype])
    assert not torch.equal(a.ca_k, b.ca_k) or cfg.dtype == "f32"      # the folded path really ran (bf16 rounds differently)


def test_grouped_schedule_full_memory_flags_and_matches_sequential(G):
    """A cross-attention memory that cannot take all new rows: both schedules drop the same rows and raise the
    same device flag."""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers = STEP_CASES["small_bf16"]
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    res = []
    for name in ("sequential", "grouped"):
        step = DeviceStep(work, fold=False)
        step.ca_len[0].fill_(step.ca_P_cap - 5)                      # room for 5 of the M new rows per sequence
        step.run(schedule=SCHEDULES[name])
        torch.cuda.synchronize()
        res.append((step.dev_status.item(), _step_outputs(step)))
    assert res[0][0] == res[1][0] and res[0][0] != 0
    for a, b in zip(res[0][1][0], res[1][1][0]):
        assert torch.equal(a, b)


@pytest.mark.parametrize("case,schedule", [("small_bf16", "grouped"), ("small_bf16", "two_stream"),
                                           ("C1_bf16_with_sa", "two_stream")])
def test_step_captured_in_a_hip_graph_replays_like_eager(G, case, schedule):
    """The step allocates nothing, synchronises nothing and reads its lengths on the device, so it can be captured;
    every replay (with other eager work and synchronisations in between) must reproduce the eager step bit for bit."""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers, lsa_tokens, with_sa = _case(case)
    work = mi.step_workload(cfg, n_verify_layers=nlayers, lsa_tokens=lsa_tokens, with_sa=with_sa)
    ref = DeviceStep(work)
    ref.run(schedule=SCHEDULES[schedule])
    torch.cuda.synchronize()
    want_exact, want_merged = _step_outputs(ref)

    step = DeviceStep(work)
    saved = [t.clone() for t in (step.ca_len[0], step.ca_k, step.ca_v)]

    def reset():
        for dst, src in zip((step.ca_len[0], step.ca_k, step.ca_v), saved):
            dst.copy_(src)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step.run(stream=stream, schedule=SCHEDULES[schedule])      # warm-up outside the capture (library-owned stream/events)
        stream.synchronize()
        reset()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step.plan(0, SCHEDULES[schedule]).run(torch.cuda.current_stream())
        for rep in range(3):
            reset()
            for t in (step.ca_out, step.lsa_out, *step.v_out):
                t.zero_()
            graph.replay()
            torch.cuda.synchronize()
            got_exact, got_merged = _step_outputs(step)
            for a, b in zip(want_exact + want_merged, got_exact + got_merged):
                assert torch.equal(a, b), f"replay {rep}"
            x = torch.randn(256, 256, device="cuda")                 # unrelated eager work between replays
            (x @ x).sum().item()
    assert step.dev_status.item() == 0


@pytest.mark.parametrize("schedule", ["grouped", "two_stream", "sequential"])
def test_step_from_packed_and_plain_lsa_weights_gives_the_same_bits(G, schedule):
    """The LSA weights packed once into MFMA-operand order change where the kernel reads a weight from, not the
    arithmetic: a step fed the packed copy and one fed the plain matrices agree bit for bit in every output.  (The other
    step cases run with the packed copy, as the benchmark does; this one also runs the plain path through a step.)"""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers = STEP_CASES["C1_bf16"]
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    outs = {}
    for pack in (True, False):
        step = DeviceStep(work, pack=pack)
        assert (step.lsa_w_packed is not None) == pack
        step.run(schedule=SCHEDULES[schedule])
        torch.cuda.synchronize()
        assert step.dev_status.item() == 0
        exact, merged = _step_outputs(step)
        outs[pack] = exact + merged
    for a, b in zip(outs[True], outs[False]):
        assert torch.equal(a, b)


def test_measurement_aid_times_kernels_and_samples(G):
    """The profiling aid attributes device time to kernels; sampling every n-th launch keeps a share of them;
    the two ceiling probes run and report plausible rates for this device."""
    import paper_2410_03804_amd as moa
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers = STEP_CASES["small_bf16"]
    step = DeviceStep(mi.step_workload(cfg, n_verify_layers=nlayers), n_len_slots=12)
    step.run(len_slot=0)
    torch.cuda.synchronize()
    moa.profile_enable(True)
    for i in range(4):
        step.run(len_slot=1 + i)
    torch.cuda.synchronize()
    rows = moa.profile_collect()
    moa.profile_enable(False)
    assert rows and all(n > 0 and 0.0 < ms < 1e3 for _, _, n, ms in rows)
    kern = rows[0][1]
    full = sum(n for _, k, n, _ in rows if k == kern)
    moa.profile_enable(True, only_kernel=kern, every=3)
    for i in range(4):
        step.run(len_slot=5 + i)
    torch.cuda.synchronize()
    sampled = moa.profile_collect()
    moa.profile_enable(False)
    assert {k for _, k, _, _ in sampled} == {kern}
    assert sum(n for _, _, n, _ in sampled) == (full + 2) // 3
    assert moa.profile_collect() == []                                  # off: nothing is recorded

    buf = torch.ones(64 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    moa.probe_read(buf, sink)
    moa.probe_mfma(200, sink)
    torch.cuda.synchronize()
    moa.profile_enable(True)
    moa.probe_read(buf, sink)
    flops = moa.probe_mfma(200, sink)
    torch.cuda.synchronize()
    t = {k: ms for _, k, n, ms in moa.profile_collect()}
    moa.profile_enable(False)
    assert 0.2e12 < buf.numel() / (t["k_probe_read"] * 1e-3) < 40e12     # between a fifth of a TB/s and L2 speed
    assert 0.2e15 < flops / (t["k_probe_mfma"] * 1e-3) < 2.6e15
    assert torch.all(sink == 0)
