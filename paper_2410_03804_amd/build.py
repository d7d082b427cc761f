"""Builds libmoa.so (hand-written HIP for gfx950) in-tree with hipcc.  No torch involved."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libmoa.so"
SOURCES = ["moa_api.hip", "moa_tree.hip", "moa_gemm.hip", "moa_attn.hip", "moa_lsa.hip", "moa_lsa_fused.hip", "moa_block.hip", "moa_draft_tree.hip", "moa_lm_head.hip", "moa_msg.hip", "moa_gzip.hip", "moa_prof.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in cand or os.path.exists(cand):
            return cand
    return "hipcc"


def _compile(src: str, objdir: Path) -> Path:
    obj = objdir / (Path(src).stem + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> Path:
    """Compile every source (always: a stale library must never be picked up) and link."""
    objdir = HERE / "_build"
    objdir.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir), SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs), "-lz"])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    return LIB


HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_host_check_driver(out_dir=None) -> Path:
    """The library's HOST code under AddressSanitizer + UndefinedBehaviorSanitizer, linked with csrc/host_check_driver.cpp
    into an executable that a CPU test runs (no GPU: argument checks, workspace carving, the checks-only pass of a whole
    step, the gzip pass).  Only the host side of every source is compiled; the device code objects the host stubs refer to
    are replaced by empty ones, which is all a run without a device ever looks at."""
    out = Path(out_dir or (HERE / "_build_host_check"))
    out.mkdir(parents=True, exist_ok=True)
    common = [_hipcc(), "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", *HOST_SANITIZE]

    def host_obj(src: str) -> Path:
        obj = out / (Path(src).stem + ".o")
        r = subprocess.run([*common, "-c", str(CSRC / src), "-o", str(obj)], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"host-only compile failed for {src}:\n{r.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(host_obj, SOURCES))
    drv = out / "host_check_driver.o"
    subprocess.check_call([*common, "-x", "c++", "-c", str(CSRC / "host_check_driver.cpp"), "-o", str(drv)])
    # the device code objects the kernels' host stubs point at: one empty, page-aligned object per source
    syms = subprocess.check_output(["nm", *map(str, objs)], text=True)
    names = sorted({l.split()[-1] for l in syms.splitlines() if " U __hip_fatbin_" in l})
    stubs = out / "fatbin_stubs.cpp"
    stubs.write_text("".join(
        f'extern "C" __attribute__((section(".hip_fatbin"), aligned(4096), visibility("default"))) const unsigned char {n}[4096];\n'
        f"const unsigned char {n}[4096] = {{0}};\n" for n in names))
    stub_obj = out / "fatbin_stubs.o"
    subprocess.check_call(["g++", "-c", str(stubs), "-o", str(stub_obj)])
    exe = out / "moa_host_check"
    subprocess.check_call([_hipcc(), "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", str(exe), *map(str, objs), str(drv),
                           str(stub_obj), "-lz"])
    return exe


if __name__ == "__main__":
    build(verbose=True)
