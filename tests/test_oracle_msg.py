"""Pins for the oracle's client-server message codec (Sec. 4.2; appendix table of message lengths).

The paper fixes the sizes (4 M bytes from the client; 3 A bytes of tokens plus 2 A E_kv (TLI+1) activation values from
the server) and the field widths (3-byte token id, 1-byte tree position); the 8-bit quantiser itself is not described,
so value-level parity with the authors' quantiser is unpinned.  Pinned here: the sizes, a message worked by hand, exact
round trips of the integer fields, the quantiser's error bound and its fixed points."""
from pathlib import Path

import numpy as np
import pytest

import moa_inputs as mi

GOLD = {}
for line in (Path(__file__).parent / "golden" / "paper_hyperparameters.txt").read_text().splitlines():
    if line and not line.startswith("#"):
        k, v = line.split()
        GOLD[k] = int(v)


def test_message_sizes_of_the_paper(oracle):
    M, A, tli, ekv = 60, 5, 1, GOLD["E_kv"]
    cfg = mi.CONFIGS["C1"]
    parent = mi.trees(cfg)
    tok, _ = mi.tokens(cfg, parent)
    assert oracle.msg_pack_tree(tok, parent).size == 4 * M                       # "4M"
    n_vec, n = tli + 1, 2 * ekv
    x = np.zeros((A, n_vec, n), np.float32)
    msg = oracle.msg_pack_accept(np.arange(A), x)
    values = 2 * A * ekv * (tli + 1)                                             # "3A + 2 A E_kv (TLI+1)" before quantisation
    assert msg.size == 3 * A + values + 4 * A * n_vec                            # one byte per value, one 4-byte scale per vector


def test_tree_message_by_hand_and_round_trip(oracle):
    tok = np.array([[0x010203, 128255, 7]], dtype=np.int32)
    parent = np.array([[-1, 0, 1]], dtype=np.int32)
    msg = oracle.msg_pack_tree(tok, parent)
    assert list(msg[0]) == [0x03, 0x02, 0x01, 0xFF, 0xFF, 0xF4, 0x01, 0x00, 0x07, 0x00, 0x00, 0x01]
    rng = np.random.default_rng(0)
    parent = np.stack([mi.gen_tree(256, 20, 4, rng) for _ in range(3)])
    tok = rng.integers(0, 1 << 24, parent.shape).astype(np.int32)
    t2, p2 = oracle.msg_unpack_tree(oracle.msg_pack_tree(tok, parent))
    assert np.array_equal(t2, tok) and np.array_equal(p2, parent)
    with pytest.raises(oracle.OracleError):
        oracle.msg_pack_tree(np.array([[1 << 24]], dtype=np.int32), np.array([[-1]], dtype=np.int32))


def test_quantiser_error_bound_and_fixed_points(oracle):
    rng = np.random.default_rng(3)
    A, n_vec, n = 4, 2, 2048
    x = (rng.standard_normal((A, n_vec, n)) * rng.uniform(0.1, 30, (A, n_vec, 1))).astype(np.float32)
    x[1, 0] = 0.0                                                                # an all-zero vector
    tok = rng.integers(0, 128256, A).astype(np.int32)
    msg = oracle.msg_pack_accept(tok, x)
    t2, y = oracle.msg_unpack_accept(msg, n_vec, n)
    assert np.array_equal(t2, tok)
    scale = np.abs(x).max(axis=2, keepdims=True) / np.float32(127)
    assert np.all(np.abs(y - x) <= scale * (0.5 + 2e-5) + 1e-30)    # round to nearest (+ the rounding of x/scale and code*scale)
    assert np.all(y[1, 0] == 0)
    # the largest magnitude is reproduced exactly, and values already on the grid are fixed points
    idx = np.abs(x[0, 0]).argmax()
    assert abs(y[0, 0, idx]) == np.float32(127) * scale[0, 0, 0]
    t3, y2 = oracle.msg_unpack_accept(oracle.msg_pack_accept(tok, y), n_vec, n)
    assert np.array_equal(y2, y)
    # by hand: absmax 127 -> scale 1 -> codes are the rounded values, ties to even
    v = np.array([[[127.0, -3.5, 2.5, 0.49, -126.6]]], np.float32)
    m = oracle.msg_pack_accept(np.array([9]), v)
    assert list(m[0, :3]) == [9, 0, 0] and m[0, 3:7].view(np.float32)[0] == 1.0
    assert list(m[0, 7:].view(np.int8)) == [127, -4, 2, 0, -127]
