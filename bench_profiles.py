#!/usr/bin/env python3
"""Turns rocprofv3 result databases into the short summaries kept under profiles/.

rocprofv3 (ROCm 7) writes one SQLite file per run (`<dir>/<name>_results.db`).  Nothing here touches a GPU: the
databases are produced on the MI355X machine by commands like the ones each summary quotes, and summarised afterwards.

  python bench_profiles.py trace    --db gpurun_out/prof/c1_results.db --cmd "<command>" --title "..." --out profiles/x.md
  python bench_profiles.py traffic  --fetch F.db --write W.db --cmd "<commands>" --title "..." --workload "..." \
                                    --out profiles/x            (writes x.md and x.json; bench.py reads the .json)
  python bench_profiles.py counters --db A.db B.db ... --cmd "<commands>" --title "..." --out profiles/x.md
  python bench_profiles.py regimes  --line "label=bench_output.json" ... --cmd "<commands>" --title "..." --out profiles/x.md
                                    (one table row per bench.py JSON line: step time, dominant kernel, rooflines)

Counter rows of one dispatch (one per shader engine / XCD instance) are summed; a kernel's figure is the mean over
its dispatches.
"""
from __future__ import annotations

import argparse
import json
import re
import sqlite3
import subprocess
from collections import defaultdict
from pathlib import Path

ROOT = Path(__file__).resolve().parent


def short_name(n: str) -> str:
    """`void moa::k_x<2, 2>(moa::Args)` -> `k_x<2, 2>`; mangled leftovers are demangled by hand."""
    m = re.match(r"_ZN3moa\d+(k_[a-z0-9_]+?)I((?:Li\d+E)+)E", n)
    if m:
        return m.group(1) + "<" + ", ".join(re.findall(r"Li(\d+)E", m.group(2))) + ">"
    n = re.sub(r"^void\s+", "", n)
    depth, cut = 0, len(n)
    for i, ch in enumerate(n):                  # drop the argument list: the first '(' outside template brackets
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            cut = i
            break
    return n[:cut].replace("moa::", "").strip()


COMMIT_OVERRIDE = ""


def head_commit() -> str:
    """The commit the summarised run was made from: --commit if given, else the current HEAD."""
    if COMMIT_OVERRIDE:
        return COMMIT_OVERRIDE
    try:
        return subprocess.check_output(["git", "-C", str(ROOT), "rev-parse", "--short=12", "HEAD"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return "unknown"


def per_kernel_counters(db: str):
    """{kernel: {counter: (dispatches, mean over dispatches of the per-dispatch sum)}}"""
    con = sqlite3.connect(db)
    q = ("select name, counter_name, dispatch_id, sum(counter_value) from pmc_events "
         "group by name, counter_name, dispatch_id")
    acc = defaultdict(lambda: defaultdict(list))
    for name, counter, _disp, value in con.execute(q):
        acc[short_name(name)][counter].append(float(value))
    return {k: {c: (len(v), sum(v) / len(v)) for c, v in cs.items()} for k, cs in acc.items()}


def kernel_durations(db: str):
    """{kernel: [durations in us]} from the dispatch begin / end timestamps."""
    con = sqlite3.connect(db)
    out = defaultdict(list)
    for name, start, end in con.execute("select name, start, end from kernels"):
        out[short_name(name)].append((end - start) / 1e3)
    return out


# kernels a benchmark run launches outside its steps: ceiling probes, the one-time weight fold and weight packing
SETUP_KERNELS = ("k_probe", "k_fold", "k_lsa_pack")


def ours(name: str) -> bool:
    return name.startswith("k_")


def cmd_trace(a):
    dur = kernel_durations(a.db[0])
    total = sum(sum(v) for v in dur.values())
    lines = [f"# {a.title}", "", "Command (from the repository root on the MI355X box):", "", "```", a.cmd, "```", "",
             f"Library commit: `{head_commit()}`. Durations are the dispatch begin / end timestamps rocprofv3 records, over "
             "every launch of the run (warm-up, the per-kernel profiling pass and the timed steps launch the same kernels).", "",
             "| kernel | calls | avg us | min us | max us | total ms | % |", "|---|---|---|---|---|---|---|"]
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if sum(v) / total < 0.002:
            continue
        lines.append(f"| `{k}` | {len(v)} | {sum(v) / len(v):.2f} | {min(v):.2f} | {max(v):.2f} | {sum(v) / 1e3:.3f} | {100 * sum(v) / total:.2f} |")
    if a.note:
        lines += ["", a.note]
    Path(a.out).write_text("\n".join(lines) + "\n")
    print("\n".join(lines))


def cmd_traffic(a):
    fetch = per_kernel_counters(a.fetch)
    write = per_kernel_counters(a.write)
    copy = "__amd_rocclr_copyBuffer"
    # the largest copy of the run is the calibration copy of known size (bench.py --calibrate-copy-mib)
    def calib(db, counter):
        con = sqlite3.connect(db)
        row = con.execute("select max(s) from (select sum(counter_value) s from pmc_events where name = ? and counter_name = ? "
                          "group by dispatch_id)", (copy, counter)).fetchone()
        return float(row[0]) if row and row[0] else None
    cf, cw = calib(a.fetch, "FETCH_SIZE"), calib(a.write, "WRITE_SIZE")
    known_kib = a.copy_mib * 1024.0
    sf = known_kib / cf if cf else 1.0
    sw = known_kib / cw if cw else 1.0
    alg = json.loads(a.alg) if a.alg else {}
    lines = [f"# {a.title}", "", "Commands (one counter per run, from the repository root on the MI355X box):", "", "```", a.cmd, "```", "",
             f"Library commit: `{head_commit()}`. Workload: {a.workload}.", "",
             f"Calibration: the plain {a.copy_mib} MiB device copy at the end of each run (`{copy}`, known traffic {a.copy_mib} MiB "
             f"each way) reads FETCH_SIZE = {cf:.0f} KiB and WRITE_SIZE = {cw:.0f} KiB, so the counters are scaled by "
             f"**{sf:.3f}** (fetch) and **{sw:.3f}** (write).", "",
             "| kernel | launches | FETCH_SIZE KiB (raw mean) | WRITE_SIZE KiB (raw mean) | scaled traffic MiB / launch | algorithmic MiB / launch | ratio |",
             "|---|---|---|---|---|---|---|"]
    table = {}
    for k in sorted(set(fetch) | set(write), key=lambda k: -(fetch.get(k, {}).get("FETCH_SIZE", (0, 0))[1])):
        if not ours(k):
            continue
        nf, f = fetch.get(k, {}).get("FETCH_SIZE", (0, 0.0))
        _, w = write.get(k, {}).get("WRITE_SIZE", (0, 0.0))
        mib = (f * sf + w * sw) / 1024.0
        table[k] = round(mib, 3)
        am = alg.get(k)
        lines.append(f"| `{k}` | {nf} | {f:.1f} | {w:.1f} | {mib:.2f} | {am if am is not None else ''} | "
                     f"{(mib / am if am else 0):.2f} |" if am else f"| `{k}` | {nf} | {f:.1f} | {w:.1f} | {mib:.2f} |  |  |")
    if a.note:
        lines += ["", a.note]
    out = Path(a.out)
    out.with_suffix(".md").write_text("\n".join(lines) + "\n")
    out.with_suffix(".json").write_text(json.dumps(dict(
        commit=head_commit(), workload=a.workload, fetch_scale=round(sf, 4), write_scale=round(sw, 4),
        kernel_set=sorted(k for k in table if not k.startswith(SETUP_KERNELS)),
        traffic_MiB_per_launch=table), indent=1) + "\n")
    print("\n".join(lines))


DERIVED = [
    # (label, needed counters, formula)
    ("MFMA pipe busy, % of SIMD time", ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES"),
     lambda c: 100.0 * c["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * c["SQ_BUSY_CU_CYCLES"])),
    ("bf16 MFMA flop / launch (MOPS x 512)", ("SQ_INSTS_VALU_MFMA_MOPS_BF16",), lambda c: 512.0 * c["SQ_INSTS_VALU_MFMA_MOPS_BF16"]),
    ("mean waves per busy CU", ("SQ_WAVE_CYCLES", "SQ_BUSY_CU_CYCLES"), lambda c: 4.0 * c["SQ_WAVE_CYCLES"] / c["SQ_BUSY_CU_CYCLES"]),
    ("wave time waiting on an instruction, %", ("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"), lambda c: 100.0 * c["SQ_WAIT_INST_ANY"] / c["SQ_WAVE_CYCLES"]),
    ("wave time waiting on anything, %", ("SQ_WAIT_ANY", "SQ_WAVE_CYCLES"), lambda c: 100.0 * c["SQ_WAIT_ANY"] / c["SQ_WAVE_CYCLES"]),
    ("wave time waiting on LDS, %", ("SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES"), lambda c: 100.0 * c["SQ_WAIT_INST_LDS"] / c["SQ_WAVE_CYCLES"]),
    ("LDS bank-conflict cycles / LDS active cycles, %", ("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE"),
     lambda c: 100.0 * c["SQ_LDS_BANK_CONFLICT"] / max(c["SQ_LDS_IDX_ACTIVE"], 1.0)),
    ("LDS active, % of CU time", ("SQ_LDS_IDX_ACTIVE", "SQ_BUSY_CU_CYCLES"), lambda c: 100.0 * c["SQ_LDS_IDX_ACTIVE"] / c["SQ_BUSY_CU_CYCLES"]),
    ("L2 hit rate, %", ("TCC_HIT_sum", "TCC_MISS_sum"), lambda c: 100.0 * c["TCC_HIT_sum"] / max(c["TCC_HIT_sum"] + c["TCC_MISS_sum"], 1.0)),
    ("mean vector-memory latency, cycles", ("SQ_INST_LEVEL_VMEM", "SQ_INSTS_VMEM"),
     lambda c: c["SQ_INST_LEVEL_VMEM"] / max(c["SQ_INSTS_VMEM"], 1.0)),
]


def cmd_counters(a):
    merged = defaultdict(dict)
    launches = {}
    for db in a.db:
        for k, cs in per_kernel_counters(db).items():
            if not ours(k) or k.startswith(SETUP_KERNELS):
                continue
            for c, (n, v) in cs.items():
                merged[k][c] = v
                launches[k] = n
    only = set(s.strip() for s in a.kernels.split(";")) if a.kernels else None
    lines = [f"# {a.title}", "", "Commands (one counter set per run, from the repository root on the MI355X box):", "", "```", a.cmd, "```", "",
             f"Library commit: `{head_commit()}`. Every figure is per launch: the counter summed over the chip's shader "
             "engines, then averaged over the launches of the run. SQ_WAVE_CYCLES, SQ_WAIT_* and SQ_ACTIVE_* count in units of "
             "four clocks; SQ_BUSY_CU_CYCLES and SQ_VALU_MFMA_BUSY_CYCLES in clocks (a 32x32x16 bf16 MFMA holds its pipe for 32).", ""]
    for k in sorted(merged, key=lambda k: -merged[k].get("SQ_BUSY_CU_CYCLES", 0.0)):
        if only and k not in only:
            continue
        c = merged[k]
        lines += [f"## `{k}` ({launches[k]} launches)", "", "| counter | per launch |", "|---|---|"]
        for name in sorted(c):
            lines.append(f"| {name} | {c[name]:.4g} |")
        for label, need, fn in DERIVED:
            if all(n in c for n in need) and all(c[n] is not None for n in need):
                try:
                    lines.append(f"| **{label}** | **{fn(c):.4g}** |")
                except ZeroDivisionError:
                    pass
        lines.append("")
    if a.note:
        lines += [a.note]
    Path(a.out).write_text("\n".join(lines) + "\n")
    print("\n".join(lines))


def cmd_regimes(a):
    lines = [f"# {a.title}", "", "Commands (from the repository root on the MI355X box; `bench.py` prints one JSON line each):", "", "```", a.cmd, "```", "",
             f"Library commit: `{head_commit()}`. `frac` is the dominant kernel's achieved rate over the published peak of its bound "
             "(HBM 8 TB/s, dense bf16 MFMA 2.5 PFLOP/s); `step frac` is the whole step's algorithmic bytes (or flops) over the "
             "step time against the same peaks.", "",
             "| workload | ms / step | tokens / s | dominant kernel | us / launch | bound | achieved | frac | step bound | step frac |",
             "|---|---|---|---|---|---|---|---|---|---|"]
    for item in a.line:
        label, path = item.split("=", 1)
        j = None
        for text in Path(path).read_text().splitlines():
            if text.startswith("{"):
                j = json.loads(text)
        if j is None:
            raise SystemExit(f"no JSON line in {path}")
        r, sr = j["roofline"], j.get("step_roofline") or {}
        lines.append(f"| {label} | {j['ms_per_step']:.4f} | {j['value']:.0f} | `{r.get('kernel', '')}` | {r.get('avg_launch_us', 0):.1f} | "
                     f"{r['bound']} | {r['achieved']:.0f} {r['unit']} | {r['frac']:.3f} | {sr.get('bound', '')} | {sr.get('frac', 0):.3f} |")
    if a.note:
        lines += ["", a.note]
    Path(a.out).write_text("\n".join(lines) + "\n")
    print("\n".join(lines))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    for name in ("trace", "traffic", "counters", "regimes"):
        p = sub.add_parser(name)
        p.add_argument("--commit", default="", help="commit the run was made from (default: the current HEAD)")
        p.add_argument("--title", required=True)
        p.add_argument("--cmd", required=True, help="the full command(s) that produced the databases")
        p.add_argument("--out", required=True)
        p.add_argument("--note", default="")
        if name == "traffic":
            p.add_argument("--fetch", required=True)
            p.add_argument("--write", required=True)
            p.add_argument("--workload", required=True)
            p.add_argument("--copy-mib", type=int, default=512)
            p.add_argument("--alg", default="", help="JSON {kernel: algorithmic MiB per launch}")
        elif name == "regimes":
            p.add_argument("--line", nargs="+", required=True, help="label=path of a file holding bench.py's JSON line")
        else:
            p.add_argument("--db", nargs="+", required=True)
        if name == "counters":
            p.add_argument("--kernels", default="", help="semicolon-separated short kernel names to keep (default: all of ours)")
    a = ap.parse_args()
    global COMMIT_OVERRIDE
    COMMIT_OVERRIDE = a.commit
    {"trace": cmd_trace, "traffic": cmd_traffic, "counters": cmd_counters, "regimes": cmd_regimes}[a.what](a)


if __name__ == "__main__":
    main()
