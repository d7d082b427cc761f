"""The gzip pass over the first message of a conversation (Sec. 4.2): the oracle's (Python's gzip) pinned against the
published container format, and the library's host functions against the oracle.  Several compressed byte strings are
correct for one message, so what is compared is what is unique -- the decompressed message -- and each stream is
checked to be valid.  CPU only: these are host functions."""
import struct

import numpy as np
import pytest

import moa_inputs as mi


def crc32_bitwise(data: bytes) -> int:
    """CRC-32 of RFC 1952 (reflected polynomial 0xEDB88320), bit by bit: independent of any library table."""
    crc = 0xFFFFFFFF
    for byte in data:
        crc ^= byte
        for _ in range(8):
            crc = (crc >> 1) ^ (0xEDB88320 if crc & 1 else 0)
    return crc ^ 0xFFFFFFFF


def stored_gzip(data: bytes) -> bytes:
    """A gzip stream written out by hand with one uncompressed DEFLATE block (RFC 1951, block type 00)."""
    assert len(data) < 65536
    header = bytes([0x1F, 0x8B, 8, 0, 0, 0, 0, 0, 0, 255])
    block = bytes([0x01]) + struct.pack("<HH", len(data), len(data) ^ 0xFFFF) + data
    return header + block + struct.pack("<II", crc32_bitwise(data), len(data))


def check_container(gz: bytes, msg: bytes):
    assert gz[:3] == bytes([0x1F, 0x8B, 8]), "gzip magic and the DEFLATE method byte"
    assert gz[3] == 0 and gz[4:8] == b"\0\0\0\0", "no optional header fields, no time stamp"
    crc, size = struct.unpack("<II", gz[-8:])
    assert crc == crc32_bitwise(msg) and size == len(msg) % (1 << 32)


def first_message(oracle, n_tokens=40, tli=1, e_kv=64, seed=3):
    """The server's first message: every prompt token's id and its (TLI+1) x 2 E_kv activations at 8 bits."""
    rng = np.random.default_rng(seed)
    tok = rng.integers(0, mi.VOCAB, size=n_tokens).astype(np.int32)
    x = (rng.standard_normal((n_tokens, tli + 1, 2 * e_kv)) * rng.uniform(0.05, 40.0, size=(n_tokens, tli + 1, 1))).astype(np.float32)
    return oracle.msg_pack_accept(tok, x).tobytes(), tok, x


MESSAGES = {
    "empty": b"",
    "one_byte": b"\x07",
    "zeros": bytes(5000),
    "text": b"mixture of attentions " * 37,
}


def test_oracle_gunzip_reads_a_hand_written_stored_block(oracle):
    for data in (b"", b"a", bytes(range(256)) * 3):
        assert oracle.msg_gunzip(stored_gzip(data)) == data


@pytest.mark.parametrize("name", list(MESSAGES) + ["first_message"])
def test_oracle_gzip_is_a_valid_stream_of_the_message(oracle, name):
    msg = MESSAGES[name] if name in MESSAGES else first_message(oracle)[0]
    gz = oracle.msg_gzip(msg)
    check_container(gz, msg)
    assert oracle.msg_gunzip(gz) == msg
    assert oracle.msg_gzip(msg) == gz                                 # no time stamp: a function of the message


def test_first_message_size_before_compression_follows_the_table(oracle):
    """3 bytes per token + (TLI+1) vectors of 2 E_kv values at one byte each (appendix table of message lengths: 3A +
    2 A E_kv (TLI+1) values), plus this quantiser's 4-byte scale per vector."""
    for n_tokens, tli, e_kv in ((40, 1, 64), (7, 0, 1024), (1, 3, 16)):
        msg, _, _ = first_message(oracle, n_tokens, tli, e_kv)
        assert len(msg) == 3 * n_tokens + 2 * n_tokens * e_kv * (tli + 1) + 4 * n_tokens * (tli + 1)


@pytest.fixture(scope="module")
def moa():
    import paper_2410_03804_amd as m
    return m


@pytest.mark.parametrize("name", list(MESSAGES) + ["first_message"])
def test_library_gzip_against_the_oracle(moa, oracle, name):
    msg = MESSAGES[name] if name in MESSAGES else first_message(oracle)[0]
    gz = moa.msg_gzip(msg)
    check_container(gz, msg)
    assert oracle.msg_gunzip(gz) == msg                                # the library's stream, read by the oracle
    assert moa.msg_gunzip(oracle.msg_gzip(msg), len(msg)) == msg       # the oracle's stream, read by the library
    assert moa.msg_gunzip(stored_gzip(msg[:60000]), 60000) == msg[:60000]
    assert moa.msg_gzip(msg) == gz


def test_first_message_survives_the_whole_codec(moa, oracle):
    """quantise -> gzip -> gunzip -> dequantise gives the oracle's dequantised activations bit for bit."""
    msg, tok, x = first_message(oracle, 33, 2, 48)
    back = moa.msg_gunzip(moa.msg_gzip(msg), len(msg))
    rows = np.frombuffer(back, dtype=np.uint8).reshape(33, -1)
    tok2, x2 = oracle.msg_unpack_accept(rows, 3, 96)
    want_tok, want_x = oracle.msg_unpack_accept(np.frombuffer(msg, dtype=np.uint8).reshape(33, -1), 3, 96)
    assert np.array_equal(tok2, tok) and np.array_equal(tok2, want_tok) and np.array_equal(x2, want_x)
    assert len(moa.msg_gzip(msg)) < len(msg)                           # 8-bit codes of bell-shaped values do compress


def test_library_gunzip_errors(moa, oracle):
    msg = first_message(oracle)[0]
    gz = moa.msg_gzip(msg)
    with pytest.raises(moa.MoaError) as e:
        moa.msg_gunzip(gz[:-5], len(msg))                              # truncated
    assert e.value.status == -2
    bad = bytearray(gz)
    bad[len(bad) // 2] ^= 0x40                                         # corrupt payload: the CRC or the code stream breaks
    with pytest.raises(moa.MoaError) as e:
        moa.msg_gunzip(bytes(bad), len(msg))
    assert e.value.status == -2
    with pytest.raises(moa.MoaError) as e:
        moa.msg_gunzip(gz, len(msg) - 1)                               # does not fit
    assert e.value.status == -4
    with pytest.raises(moa.MoaError) as e:
        moa.msg_gunzip(b"not a gzip stream at all", 100)
    assert e.value.status == -2
