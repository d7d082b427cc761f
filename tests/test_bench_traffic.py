"""bench.py's roofline.traffic comes from the tracked rocprofv3 summary and is withheld when that summary does not
describe the run (CPU only: the lookup, not a measurement)."""
import importlib.util
import json
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent


def _bench():
    spec = importlib.util.spec_from_file_location("moa_bench", ROOT / "bench.py")
    mod = importlib.util.module_from_spec(spec)
    sys.modules["moa_bench"] = mod
    spec.loader.exec_module(mod)
    return mod


def test_traffic_is_read_from_the_tracked_summary_or_withheld(tmp_path, monkeypatch):
    bench = _bench()
    rec = dict(commit="abc123", workload="C1", kernel_set=["k_a<1>", "k_b"],
               traffic_MiB_per_launch={"k_a<1>": 2.5, "k_b": 1.0, "k_setup": 9.0})
    f = tmp_path / "traffic.json"
    f.write_text(json.dumps(rec))
    monkeypatch.setattr(bench, "PMC_TRAFFIC_FILE", str(f))
    val, src = bench.recorded_traffic("k_a<1>", ["k_b", "k_a<1>"], True)
    assert val == int(2.5 * 2 ** 20) and "abc123" in src
    val, src = bench.recorded_traffic("k_a<1>", ["k_a<1>", "k_b", "k_new"], True)          # a kernel joined the step
    assert val is None and "kernel set changed" in src
    val, src = bench.recorded_traffic("k_a<1>", ["k_a<1>", "k_b"], False)                  # another workload
    assert val is None
    val, src = bench.recorded_traffic("k_c", ["k_a<1>", "k_b"], True)
    assert val is None
    monkeypatch.setattr(bench, "PMC_TRAFFIC_FILE", str(tmp_path / "missing.json"))
    val, src = bench.recorded_traffic("k_a<1>", ["k_a<1>", "k_b"], True)
    assert val is None and "no tracked" in src


def test_tracked_summary_names_its_commit_and_the_step_kernels():
    rec = json.loads((ROOT / "profiles" / "c1_draft_step_hbm_traffic.json").read_text())
    assert rec["workload"] == "C1" and len(rec["commit"]) >= 7
    assert rec["kernel_set"] and all(k in rec["traffic_MiB_per_launch"] for k in rec["kernel_set"])
    assert not any(k.startswith(("k_probe", "k_fold", "k_lsa_pack")) for k in rec["kernel_set"])
