"""moa_draft_step on the launch configurations it takes at the batched and long-context workloads: the grouped
projection through the tiled kernel (four segments with their own activations, the integer work riding in its
grid), a carried slice-summing pass over several row tiles, both attention cores in one split-KV launch + merge,
two-word tree masks.  The library runs the whole batch as the benchmark does; the oracle recomputes sampled
sequences (each sequence of a step is independent of the others, so the sample is exact for the rows it covers)."""
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


def _cfg(name, index, **kw):
    base = dict(name=name, index=index, dtype="bf16", B=4, P_min=100, P_max=700, M=64, D=6, max_branch=4, L=6, d=512,
                H=8, Hkv=2, dh=128, d_lsa_in=512, rms_norm=True)
    base.update(kw)
    return mi.Config(**base)


# name -> (config, verify layers, sampled sequences, attention form forced for the run)
LARGE_CASES = {
    # 256 rows: the grouped projection takes the tiled kernel (several row tiles, four segments, riding integer work)
    "tiled_pair_256_rows": (_cfg("T256", 21), 2, 4, "auto"),
    # 180 rows: weight-streaming projection over three row tiles whose slice-summing pass (180 rows) is carried by
    # the LSA projection's tiled launch
    "carried_sum_180_rows": (_cfg("S180", 22, B=3, M=60, d=1024, H=8, Hkv=2, d_lsa_in=512, L=8), 1, 3, "auto"),
    # both cores of the step in one split-KV launch + one merge, at a size that would otherwise take the other form
    "split_pair_forced": (_cfg("SP", 23, B=3, M=37, P_min=80, P_max=300), 2, 3, "split"),
    # two-word masks (M = 128) through the whole-key-range form and through the split form
    "two_word_masks_whole": (_cfg("M128w", 24, B=2, M=128, D=10, P_min=140, P_max=400), 1, 2, "whole"),
    "two_word_masks_split": (_cfg("M128s", 25, B=2, M=128, D=10, P_min=140, P_max=400), 1, 2, "split"),
    # the batched and long-context workloads themselves
    "C2": (mi.CONFIGS["C2"], 1, 3, "auto"),
    "C3": (mi.CONFIGS["C3"], 1, 2, "auto"),
    "C4": (mi.CONFIGS["C4"], 1, 2, "auto"),
}


@pytest.mark.parametrize("case", list(LARGE_CASES))
def test_draft_step_large_paths_against_oracle(G, oracle, case):
    import paper_2410_03804_amd as moa
    from oracle.step import run_step
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers, nseq, form = LARGE_CASES[case]
    print(f"[case] draft_step large {case}: B={cfg.B} M={cfg.M} P={cfg.P_min}..{cfg.P_max} d={cfg.d} L={cfg.L} "
          f"layers={nlayers} attention form={form}", flush=True)
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    print("[step] workload drawn", flush=True)
    step = DeviceStep(work)
    moa.debug_force_attn_kernel(form)
    try:
        step.run()
        torch.cuda.synchronize()
    finally:
        moa.debug_force_attn_kernel("auto")
    print("[step] moa_draft_step done", flush=True)
    dt = cfg.dtype
    assert step.dev_status.item() == 0
    seqs = G.sample_sequences(work["prefix_len"], nseq)
    sub, rows = G.slice_step_work(work, seqs)
    want = run_step(sub)
    print(f"[step] oracle done on sequences {seqs}", flush=True)
    assert np.array_equal(G.mask_u64(step.mask)[seqs], want["mask"])
    assert np.array_equal(step.depth.cpu().numpy()[seqs], want["depth"])
    G.check_close(G.host(step.lsa_out[torch.from_numpy(rows).cuda()]), want["lsa_out"], dt, f"step.lsa[{case}]")
    assert np.array_equal(step.ca_len[0].cpu().numpy()[seqs], want["ca_len"])
    sel = torch.tensor(seqs, device="cuda")
    G.check_close(G.host(step.ca_k[sel]), want["ca_k"], dt, f"step.ca_k[{case}]")
    G.check_close(G.host(step.ca_v[sel]), want["ca_v"], dt, f"step.ca_v[{case}]")
    G.check_close(G.host(step.ca_out[sel]), want["ca_out"], dt, f"step.ca_out[{case}]")
    for l in range(nlayers):
        G.check_close(G.host(step.v_out[l][sel]), want["v_out"][l], dt, f"step.verify{l}[{case}]")
        G.check_close(G.host(step.v_ktree[l][sel]), want["v_ktree"][l], dt, f"step.k_tree{l}[{case}]")
        G.check_close(G.host(step.v_vtree[l][sel]), want["v_vtree"][l], dt, f"step.v_tree{l}[{case}]")
    assert np.array_equal(step.path.cpu().numpy()[seqs], want["path"])
    assert np.array_equal(step.n_path.cpu().numpy()[seqs], want["n_path"])
    assert np.array_equal(step.bonus.cpu().numpy()[seqs], want["bonus"])
