"""The sequence-slicing helper the large GPU step tests rely on: the oracle's step on a slice of the sequences equals
the matching rows of its step on the whole batch (sequences are independent), so a sampled comparison is exact."""
import numpy as np

import moa_inputs as mi


def test_oracle_step_on_a_slice_equals_rows_of_the_whole(oracle):
    import gpu_util as G
    from oracle.step import run_step
    cfg = mi.Config(name="SL", index=31, dtype="bf16", B=4, P_min=20, P_max=90, M=11, D=3, max_branch=3, L=3, d=128,
                    H=4, Hkv=2, dh=32, d_lsa_in=64, rms_norm=True)
    for lsa_tokens, with_sa in (("tree", False), (3, True)):
        work = mi.step_workload(cfg, n_verify_layers=2, lsa_tokens=lsa_tokens, with_sa=with_sa)
        full = run_step(work)
        seqs = G.sample_sequences(work["prefix_len"], 3)
        assert len(seqs) == 3 and int(np.argmin(work["prefix_len"])) in seqs and int(np.argmax(work["prefix_len"])) in seqs
        sub, rows = G.slice_step_work(work, seqs)
        part = run_step(sub)
        assert np.array_equal(part["lsa_out"], full["lsa_out"][rows])
        for k in ("mask", "depth", "ca_k", "ca_v", "ca_len", "ca_out", "path", "n_path", "bonus"):
            assert np.array_equal(part[k], full[k][seqs]), k
        for l in range(2):
            for k in ("v_out", "v_ktree", "v_vtree"):
                assert np.array_equal(part[k][l], full[k][l][seqs]), (k, l)
        if with_sa:
            assert np.array_equal(part["sa_out"], full["sa_out"][seqs])
