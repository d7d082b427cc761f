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
}


@pytest.mark.parametrize("case", list(STEP_CASES))
def test_draft_step_parity(G, oracle, case):
    from oracle.step import run_step
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers = STEP_CASES[case]
    print(f"[case] draft_step {case} B={cfg.B} M={cfg.M} layers={nlayers}", flush=True)
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    step = DeviceStep(work)
    step.run()
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
    G.check_close(G.host(step.ca_out), want["ca_out"], dt, f"step.ca_out[{case}]")
    for l in range(nlayers):
        G.check_close(G.host(step.v_out[l]), want["v_out"][l], dt, f"step.verify{l}[{case}]")
        G.check_close(G.host(step.v_ktree[l]), want["v_ktree"][l], dt, f"step.k_tree{l}[{case}]")
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


@pytest.mark.parametrize("case", ["small_bf16", "C1_bf16"])
def test_two_stream_schedule_is_bit_identical_to_serial(G, case):
    """The step forks its independent branches onto a second stream; the result must not depend on it."""
    from paper_2410_03804_amd.workload import DeviceStep
    cfg, nlayers = STEP_CASES[case]
    work = mi.step_workload(cfg, n_verify_layers=nlayers)
    outs = []
    for two in (False, True, True):
        step = DeviceStep(work)
        step.run(two_stream=two)
        torch.cuda.synchronize()
        assert step.dev_status.item() == 0
        outs.append([step.lsa_out.clone(), step.ca_k.clone(), step.ca_out.clone(), step.mask.clone(), step.path.clone(),
                     *[o.clone() for o in step.v_out], *[o.clone() for o in step.v_ktree]])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)
