"""The C-ABI library loads, exports every symbol the header declares, and rejects bad host
arguments before touching a device (no GPU needed: nothing is launched)."""
import ctypes as C
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "moa.h").read_text()


@pytest.fixture(scope="module")
def moa():
    import paper_2410_03804_amd as m
    return m


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(moa_[a-z_]+)\s*\(", body)))


def test_header_functions_are_exported(moa):
    names = declared_functions()
    assert "moa_lsa" in names and "moa_cross_attn_draft" in names and "moa_tree_verify_attn" in names
    assert "moa_draft_step" in names
    lib = C.CDLL(moa.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/moa.h but not exported"
    assert sorted(moa.exported_symbols()) == names


def test_every_entry_point_cites_the_paper():
    # each declaration is preceded by a comment naming the section / algorithm that defines it
    for fn in ("moa_tree_build", "moa_tree_accept", "moa_lsa", "moa_ca_kv_append", "moa_cross_attn_draft",
               "moa_tree_verify_attn", "moa_draft_step"):
        i = HEADER.index(f"int32_t {fn}(")
        prev = HEADER.rfind(");\n", 0, i)                    # end of the previous declaration
        comments = " ".join(re.findall(r"/\*.*?\*/", HEADER[prev:i], flags=re.S))
        assert re.search(r"Sec\.|Alg\.", comments), fn


def test_status_strings(moa):
    assert moa.status_str(0) == "MOA_OK" and moa.status_str(-6) == "MOA_ERR_WORKSPACE"


def test_workspace_query_and_shape_errors(moa):
    s = moa.Shape(32, 4096, 32, 8, 128, 2048, 16, 8, moa.BF16)
    assert moa.workspace_bytes(s, 1, 1084, 60, 60) > 0
    big = moa.workspace_bytes(s, 8, 32768 + 128, 128, 1024)
    assert big >= moa.workspace_bytes(s, 1, 1084, 60, 60)
    for bad in (moa.Shape(32, 4096, 32, 5, 128, 2048, 16, 8, moa.BF16),      # H % Hkv
                moa.Shape(32, 4096, 32, 8, 512, 2048, 16, 8, moa.BF16),      # head_dim
                moa.Shape(32, 4096, 32, 8, 128, 2048, 16, 8, 7)):            # dtype
        with pytest.raises(moa.MoaError):
            moa.workspace_bytes(bad, 1, 1024, 60, 0)


def test_null_and_range_errors_launch_nothing(moa):
    lib = C.CDLL(moa.library_path())
    lib.moa_tree_build.restype = C.c_int32
    assert lib.moa_tree_build(None, 1, 8, None, None, None, None) == -1            # MOA_ERR_NULL
    fake = C.c_void_p(256)                                                         # never dereferenced
    lib.moa_tree_build.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    assert lib.moa_tree_build(fake, 1, moa.MAX_TREE + 1, fake, fake, None, None) == -2   # MOA_ERR_SHAPE
    assert lib.moa_tree_build(fake, 0, 8, fake, fake, None, None) == -2
    s = moa.Shape(4, 256, 4, 2, 64, 256, 4, 2, moa.F32)
    lib.moa_lsa.restype = C.c_int32
    lib.moa_lsa.argtypes = [C.c_void_p, C.c_void_p, C.c_int64] + [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
    assert lib.moa_lsa(C.byref(s), None, 4, fake, fake, fake, fake, fake, fake, 1 << 30, None) == -1
    assert lib.moa_lsa(C.byref(s), fake, 4, fake, fake, fake, fake, fake, None, 0, None) == -6      # no workspace
    assert lib.moa_lsa(C.byref(s), fake, 4, fake, fake, fake, fake, fake, fake, 16, None) == -6     # too small
    lib.moa_last_error.restype = C.c_char_p
    assert b"workspace" in lib.moa_last_error()
    lib.moa_draft_step.restype = C.c_int32
    assert lib.moa_draft_step(None) == -1


def test_packed_lsa_weights_sizes_and_refusals(moa):
    """The packed copy of the LSA weights: its size is that of the rows the one-kernel form reads (two query heads, a key
    head and a value head per unit: a group of four query heads stores its K and V rows twice); shapes that form does not
    take have no packed form; bad pointers and short buffers are refused before anything is launched."""
    s = moa.Shape(32, 4096, 32, 8, 128, 2048, 16, 8, moa.BF16)                 # Llama-3-8B: 16 LSA heads over 8 KV heads
    assert moa.lsa_packed_weight_bytes(s) == (16 + 8 + 8) * 128 * 2048 * 2
    s4 = moa.Shape(32, 4096, 32, 8, 128, 4096, 32, 8, moa.BF16)                # d_in = d: groups of four query heads
    assert moa.lsa_packed_weight_bytes(s4) == (32 + 16 + 16) * 128 * 4096 * 2
    for bad in (moa.Shape(32, 4096, 32, 8, 128, 2048, 16, 8, moa.F32),         # fp32
                moa.Shape(32, 4096, 32, 8, 64, 2048, 32, 16, moa.BF16),        # head_dim 64
                moa.Shape(32, 4096, 32, 8, 128, 2048, 16, 16, moa.BF16),       # one query head per KV head
                moa.Shape(128, 4096, 32, 8, 128, 2048, 16, 8, moa.BF16),       # more than 96 layers
                moa.Shape(32, 4096, 32, 8, 128, 2080, 16, 8, moa.BF16)):       # d_lsa_in not in 64s
        with pytest.raises(moa.MoaError) as e:
            moa.lsa_packed_weight_bytes(bad)
        assert e.value.status == -2
    lib = C.CDLL(moa.library_path())
    fake = C.c_void_p(256)
    need = moa.lsa_packed_weight_bytes(s)
    lib.moa_lsa_pack_weights.restype = C.c_int32
    lib.moa_lsa_pack_weights.argtypes = [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p]
    assert lib.moa_lsa_pack_weights(C.byref(s), fake, fake, None, fake, need, None) == -1
    assert lib.moa_lsa_pack_weights(C.byref(s), fake, fake, fake, fake, need - 1, None) == -6
    assert lib.moa_lsa_pack_weights(C.byref(s), fake, fake, fake, C.c_void_p(264), need, None) == -2     # misaligned
    lib.moa_lsa_packed.restype = C.c_int32
    lib.moa_lsa_packed.argtypes = [C.c_void_p, C.c_void_p, C.c_int64] + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
    assert lib.moa_lsa_packed(C.byref(s), fake, 4, None, fake, fake, fake, 1 << 30, None) == -1
    assert lib.moa_lsa_packed(C.byref(s), fake, -1, fake, fake, fake, fake, 1 << 30, None) == -2
    assert lib.moa_lsa_packed(C.byref(s), fake, 4, fake, fake, fake, fake, 16, None) == -6
    assert lib.moa_lsa_packed(C.byref(s), fake, 0, fake, fake, fake, None, 0, None) == 0                 # nothing to do


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N above 1 must exit with a message that says so (before any GPU use)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""


def test_product_path_does_not_use_the_oracle():
    """The oracle is test infrastructure: nothing in the package may import, load or call it (and the other way round)."""
    pkg = ROOT / "paper_2410_03804_amd"
    for f in list(pkg.glob("*.py")) + list((pkg / "csrc").glob("*")):
        text = f.read_text()
        assert not re.search(r"\boracle\b|moa_ref", text), f
    for f in (ROOT / "oracle").glob("*"):
        if f.suffix in (".py", ".c", ".h"):
            assert "paper_2410_03804_amd" not in f.read_text() and "libmoa.so" not in f.read_text(), f
    gen = (ROOT / "moa_inputs" / "__init__.py").read_text()          # the shared input generators import neither side
    assert not re.search(r"^\s*(import|from)\s+(oracle|paper_2410_03804_amd)", gen, flags=re.M)


def test_draft_step_rejects_unknown_schedule_before_any_launch(moa):
    import ctypes as C
    from paper_2410_03804_amd import binding
    args = binding._StepArgs()
    shape = moa.Shape(4, 256, 4, 2, 64, 256, 4, 2, moa.F32)
    args.shape = C.pointer(shape)
    args.schedule = 7
    rc = binding._lib.moa_draft_step(C.byref(args))
    assert rc == -2 and "schedule" in moa.last_error()
