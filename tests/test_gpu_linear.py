"""GPU parity of the bare projection (moa_linear) across the kernels it dispatches to -- weight streaming with the
activation slice resident in LDS or re-read in chunks (at most 64 rows, K in 1024s or 512s), weight streaming in one
shot (up to 192 rows), the tiled GEMM, the narrow and
the generic forms -- against the oracle's projection, with ragged row counts and the smallest and largest row count of each
form."""
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


@pytest.fixture(scope="module")
def moa(G):
    import paper_2410_03804_amd as m
    return m


# (dtype, rows, K, N): what decides the kernel is in the comment
CASES = [
    ("bf16", 1, 4096, 4096),      # chunks of a 1024-wide slice: 64 tiles x 4 slices, one row
    ("bf16", 33, 4096, 8192),     # the same, ragged rows
    ("bf16", 64, 1024, 16384),    # a single slice: nothing to add up but the chunks
    ("bf16", 60, 2048, 4096),     # 512-wide slices in two chunks (64 tiles x 4)
    ("bf16", 60, 14336, 4096),    # 14 slices (activation slice resident: 18 workgroups per slice, 15 wavefronts each)
    ("bf16", 60, 4096, 10240),    # activation slice resident, one group of 16 features per wavefront, ten wavefronts
    ("bf16", 64, 4096, 28672),    # the same with two groups per wavefront
    ("bf16", 5, 2048, 14336),     # two slices, seven wavefronts
    ("bf16", 47, 4096, 6208),     # groups do not divide: the last workgroup of a slice has idle wavefronts
    ("bf16", 65, 4096, 4096),     # one row more: two row tiles, one shot per 512-wide slice
    ("bf16", 128, 2048, 2048),
    ("bf16", 160, 2048, 6144),    # three row tiles, wide slices
    ("bf16", 193, 2048, 2048),    # tiled GEMM
    ("bf16", 700, 512, 1024),
    ("bf16", 60, 4096, 1024),     # too few tiles for chunks: one shot
    ("bf16", 17, 384, 96),        # K not in 512s, N in 32s: narrow form
    ("bf16", 9, 200, 50),         # nothing aligned: generic
    ("f32", 19, 320, 70),
]


@pytest.mark.parametrize("dtype,R,K,N", CASES)
def test_linear_parity(G, moa, oracle, dtype, R, K, N):
    rng = np.random.default_rng(R * 7 + K + N)
    x = mi.quantize(rng.standard_normal((R, K)).astype(np.float32), dtype)
    w = mi.quantize((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32), dtype)
    print(f"[case] linear {dtype} R={R} K={K} N={N}", flush=True)
    mdt = G.MDT[dtype]
    y = torch.full((R, N), float("nan"), dtype=G.TDT[dtype], device="cuda")
    ws = torch.empty(max(moa.linear_workspace_bytes(mdt, R, K, N), 256), dtype=torch.uint8, device="cuda")
    moa.linear(G.dev(x, dtype), G.dev(w, dtype), y, ws)
    torch.cuda.synchronize()
    want = oracle.linear(x, w)
    G.check_close(G.host(y), want, dtype, f"linear[{dtype} {R}x{K}x{N}]", residual_stream=True)
    # the same call again gives the same bits (fixed summation order whatever the scheduling)
    y2 = torch.empty_like(y)
    moa.linear(G.dev(x, dtype), G.dev(w, dtype), y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
