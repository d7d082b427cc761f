"""GPU parity of the client-server message codec against the oracle: every byte, every unpacked value, bit for bit."""
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


@pytest.mark.parametrize("case", ["C1", "C2", "M256"])
def test_tree_message_bit_exact(G, moa, oracle, case):
    rng = np.random.default_rng(5)
    if case == "M256":
        parent = np.stack([mi.gen_tree(256, 25, 4, rng) for _ in range(3)])
        tok = rng.integers(0, 1 << 24, parent.shape).astype(np.int32)
    else:
        cfg = mi.CONFIGS[case]
        parent = mi.trees(cfg)
        tok, _ = mi.tokens(cfg, parent)
    B, M = parent.shape
    print(f"[case] msg_tree {case} B={B} M={M}", flush=True)
    msg = torch.zeros((B, 4 * M), dtype=torch.uint8, device="cuda")
    st = G.status_word()
    moa.msg_pack_tree(G.dev(tok), G.dev(parent), msg, st)
    t2 = torch.full((B, M), -9, dtype=torch.int32, device="cuda")
    p2 = torch.full((B, M), -9, dtype=torch.int32, device="cuda")
    moa.msg_unpack_tree(msg, t2, p2)
    torch.cuda.synchronize()
    assert st.item() == 0
    assert np.array_equal(msg.cpu().numpy(), oracle.msg_pack_tree(tok, parent))
    assert np.array_equal(t2.cpu().numpy(), tok) and np.array_equal(p2.cpu().numpy(), parent)


def test_tree_message_flags_a_token_that_does_not_fit(G, moa):
    tok = torch.tensor([[5, 1 << 24]], dtype=torch.int32, device="cuda")
    parent = torch.tensor([[-1, 0]], dtype=torch.int32, device="cuda")
    msg = torch.zeros((1, 8), dtype=torch.uint8, device="cuda")
    st = G.status_word()
    moa.msg_pack_tree(tok, parent, msg, st)
    torch.cuda.synchronize()
    assert st.item() == moa.DEV_BAD_MESSAGE


@pytest.mark.parametrize("dtype,A,n_vec,n", [("f32", 5, 2, 2048), ("bf16", 5, 2, 2048), ("bf16", 60, 4, 2048), ("f32", 3, 1, 37), ("f32", 1, 3, 1)])
def test_accept_message_bit_exact(G, moa, oracle, dtype, A, n_vec, n):
    """n_vec = TLI + 1 vectors of n = 2 E_kv values per accepted token (the appendix table's 2 A E_kv (TLI+1))."""
    rng = np.random.default_rng(A * n)
    x = mi.quantize((rng.standard_normal((A, n_vec, n)) * rng.uniform(0.05, 40, (A, n_vec, 1))).astype(np.float32), dtype)
    if A > 1:
        x[1, 0] = 0.0
    tok = rng.integers(0, 128256, A).astype(np.int32)
    print(f"[case] msg_accept {dtype} A={A} n_vec={n_vec} n={n}", flush=True)
    nbytes = moa.msg_accept_bytes(A, n_vec, n)
    assert nbytes == A * (3 + n_vec * (4 + n))
    msg = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    st = G.status_word()
    moa.msg_pack_accept(G.dev(tok), G.dev(x, dtype), msg, st)
    t2 = torch.full((A,), -9, dtype=torch.int32, device="cuda")
    y = torch.zeros((A, n_vec, n), dtype=torch.float32, device="cuda")
    moa.msg_unpack_accept(msg, t2, y)
    torch.cuda.synchronize()
    assert st.item() == 0
    want = oracle.msg_pack_accept(tok, x)
    assert np.array_equal(msg.cpu().numpy().reshape(want.shape), want)
    wt, wy = oracle.msg_unpack_accept(want, n_vec, n)
    assert np.array_equal(t2.cpu().numpy(), wt)
    assert np.array_equal(y.cpu().numpy().view(np.uint32), wy.view(np.uint32))
    scale = np.abs(x).max(axis=2, keepdims=True) / np.float32(127)
    assert np.all(np.abs(y.cpu().numpy() - x) <= scale * (0.5 + 2e-5) + 1e-30)
