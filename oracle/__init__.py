"""ctypes front-end of the fp64 CPU oracle (``moa_ref.c``).

TEST INFRASTRUCTURE ONLY.  Importable from ``tests/``, from the smoke check and
from the benchmark's ``cpu_baseline`` leg -- never from the product package.
Nothing here imports the GPU package; the two share no code.

Every wrapper converts its numpy inputs to C-contiguous float64 / int32 / uint64
(an exact conversion for fp32 and bf16-representable values) and returns fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "moa_ref.c"
_LIB = _HERE / "libmoa_ref.so"

OK, BAD_ARG, BAD_TREE, EMPTY = 0, 1, 2, 3


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: oracle status {code}")
        self.code = code


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP).  Building the checker is not using it."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < max(
            _SRC.stat().st_mtime, (_HERE / "moa_ref.h").stat().st_mtime):
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


SANITIZE_FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                  "-fno-omit-frame-pointer", "-static-libasan"]


def build_sanitize_driver(out_dir=None) -> Path:
    """Compile moa_ref.c together with sanitize_driver.c under AddressSanitizer + UndefinedBehaviorSanitizer into
    an executable (host code only; a CPU test runs it).  The sanitizer runtime is linked statically so that the
    program does not depend on the order of preloaded libraries."""
    exe = Path(out_dir or _HERE) / "moa_ref_sanitize"
    tmp = exe.with_suffix(f".tmp{os.getpid()}")
    subprocess.check_call(["gcc", *SANITIZE_FLAGS, "-fopenmp", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC),
                           str(_HERE / "sanitize_driver.c"), "-lm"])
    os.replace(tmp, exe)
    return exe


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(_LIB))
    return _lib


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, ct=C.c_double):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _check(rc, where):
    if rc != OK:
        raise OracleError(rc, where)


def tree_build(parent):
    parent = _i32(parent)
    B, M = parent.shape
    W = (M + 63) // 64
    mask = np.zeros((B, M, W), dtype=np.uint64)
    depth = np.zeros((B, M), dtype=np.int32)
    rc = lib().moa_ref_tree_build(_p(parent, C.c_int32), B, M, _p(mask, C.c_uint64), _p(depth, C.c_int32))
    _check(rc, "tree_build")
    return mask, depth


def linear(x, w):
    x = _f64(x)
    w = _f64(w)
    R, K = x.shape
    N = K if w is None else w.shape[0]
    y = np.empty((R, N), dtype=np.float64)
    _check(lib().moa_ref_linear(_p(x), C.c_int64(R), K, _p(w), N, _p(y)), "linear")
    return y


def lsa(hs, wq, wk, wv, wo, Hq, Hkv, dh):
    hs = _f64(hs)
    T, L, d_in = hs.shape
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    d_out = Hq * dh if wo is None else wo.shape[0]
    out = np.empty((T, d_out), dtype=np.float64)
    rc = lib().moa_ref_lsa(_p(hs), C.c_int64(T), L, d_in, Hq, Hkv, dh, _p(wq), _p(wk), _p(wv), _p(wo),
                           d_out, _p(out))
    _check(rc, "lsa")
    return out


def ca_kv_append(mem_new, tok_off, wk, wv, kc, vc, ca_len, Hkv, dh):
    """Appends in place into kc / vc (float64 [B,Hkv,P_cap,dh]) and ca_len (int32 [B])."""
    mem_new = _f64(mem_new)
    tok_off = _i32(tok_off)
    wk, wv = _f64(wk), _f64(wv)
    assert kc.dtype == np.float64 and vc.dtype == np.float64 and ca_len.dtype == np.int32
    assert kc.flags.c_contiguous and vc.flags.c_contiguous and ca_len.flags.c_contiguous
    B, hk, P_cap, dd = kc.shape
    assert hk == Hkv and dd == dh and tok_off.shape == (B + 1,)
    rc = lib().moa_ref_ca_kv_append(_p(mem_new), mem_new.shape[1], _p(tok_off, C.c_int32), B, Hkv, dh,
                                    _p(wk), _p(wv), _p(kc), _p(vc), _p(ca_len, C.c_int32), P_cap)
    _check(rc, "ca_kv_append")


def cross_attn(xq, wq, wo, kc, vc, ca_len, H, Hkv, dh):
    xq = _f64(xq)
    B, Mq, d = xq.shape
    wq, wo, kc, vc = _f64(wq), _f64(wo), _f64(kc), _f64(vc)
    ca_len = _i32(ca_len)
    P_cap = kc.shape[2]
    d_out = H * dh if wo is None else wo.shape[0]
    out = np.empty((B, Mq, d_out), dtype=np.float64)
    rc = lib().moa_ref_cross_attn(_p(xq), B, Mq, d, H, Hkv, dh, _p(wq), _p(wo), d_out, _p(kc), _p(vc),
                                  _p(ca_len, C.c_int32), P_cap, _p(out))
    _check(rc, "cross_attn")
    return out


def tree_verify_attn(x, wq, wk, wv, wo, kcache, vcache, prefix_len, mask, H, Hkv, dh):
    x = _f64(x)
    B, M, d = x.shape
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    kcache, vcache = _f64(kcache), _f64(vcache)
    prefix_len = _i32(prefix_len)
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    P_cap = 0 if kcache is None else kcache.shape[2]
    d_out = H * dh if wo is None else wo.shape[0]
    out = np.empty((B, M, d_out), dtype=np.float64)
    kt = np.empty((B, Hkv, M, dh), dtype=np.float64)
    vt = np.empty((B, Hkv, M, dh), dtype=np.float64)
    rc = lib().moa_ref_tree_verify_attn(_p(x), B, M, d, H, Hkv, dh, _p(wq), _p(wk), _p(wv), _p(wo), d_out,
                                        _p(kcache), _p(vcache), _p(prefix_len, C.c_int32), P_cap,
                                        _p(mask, C.c_uint64), _p(out), _p(kt), _p(vt))
    _check(rc, "tree_verify_attn")
    return out, kt, vt


def self_attn_draft(emb, parent, node0, wq, wk, wv, wo, kcache, vcache, prefix_len, k_draft, v_draft, H, Hkv, dh):
    """SA layer on the embeddings of the tree nodes node0 .. node0+Mn-1 (emb [B, Mn, d]); k_draft / v_draft
    [B, Hkv, M, dh] (float64, C-contiguous) are updated in place.  Returns out [B, Mn, d_out]."""
    emb = _f64(emb)
    B, Mn, d = emb.shape
    parent = _i32(parent)
    M = parent.shape[1]
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    kcache, vcache = _f64(kcache), _f64(vcache)
    prefix_len = _i32(prefix_len)
    for a in (k_draft, v_draft):
        if a.dtype != np.float64 or not a.flags.c_contiguous or a.shape != (B, Hkv, M, dh):
            raise ValueError("draft cache must be C-contiguous float64 [B, Hkv, M, dh]")
    P_cap = 0 if kcache is None else kcache.shape[2]
    d_out = H * dh if wo is None else wo.shape[0]
    out = np.empty((B, Mn, d_out), dtype=np.float64)
    rc = lib().moa_ref_self_attn_draft(_p(emb), B, M, int(node0), Mn, d, H, Hkv, dh, _p(wq), _p(wk), _p(wv), _p(wo),
                                       d_out, _p(kcache), _p(vcache), _p(prefix_len, C.c_int32), P_cap,
                                       _p(parent, C.c_int32), _p(out), _p(k_draft), _p(v_draft))
    _check(rc, "self_attn_draft")
    return out


def rope(v, pos, theta):
    """Rotary embedding of one head vector (returns a rotated copy)."""
    v = np.array(v, dtype=np.float64)
    lib().moa_ref_rope.restype = None
    lib().moa_ref_rope(_p(v), int(v.shape[0]), C.c_double(float(pos)), C.c_double(float(theta)))
    return v


def tli_decoder_layer(x, parent, node0, w, kcache, vcache, prefix_len, k_draft, v_draft, H, Hkv, dh, rms_eps, rope_theta):
    """One reused LLM decoder layer on the tree nodes node0 .. node0+Mn-1 (x [B, Mn, d]); w = dict(g_attn, wq, wk, wv,
    wo, g_mlp, w_gate, w_up, w_down); k_draft / v_draft [B, Hkv, M, dh] float64, updated in place."""
    x = _f64(x)
    B, Mn, d = x.shape
    parent = _i32(parent)
    M = parent.shape[1]
    ww = {k: _f64(v) for k, v in w.items()}
    kcache, vcache = _f64(kcache), _f64(vcache)
    prefix_len = _i32(prefix_len)
    for a in (k_draft, v_draft):
        if a.dtype != np.float64 or not a.flags.c_contiguous or a.shape != (B, Hkv, M, dh):
            raise ValueError("draft cache must be C-contiguous float64 [B, Hkv, M, dh]")
    P_cap = 0 if kcache is None else kcache.shape[2]
    d_ff = ww["w_gate"].shape[0]
    out = np.empty((B, Mn, d), dtype=np.float64)
    rc = lib().moa_ref_tli_decoder_layer(
        _p(x), B, M, int(node0), Mn, d, H, Hkv, dh, d_ff, C.c_double(rms_eps), C.c_double(rope_theta),
        _p(ww["g_attn"]), _p(ww["wq"]), _p(ww["wk"]), _p(ww["wv"]), _p(ww["wo"]), _p(ww["g_mlp"]), _p(ww["w_gate"]),
        _p(ww["w_up"]), _p(ww["w_down"]), _p(kcache), _p(vcache), _p(prefix_len, C.c_int32), P_cap,
        _p(parent, C.c_int32), _p(out), _p(k_draft), _p(v_draft))
    _check(rc, "tli_decoder_layer")
    return out


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = _f64(x)
    g = _f64(g)
    d = x.shape[-1]
    out = np.empty_like(x)
    rc = lib().moa_ref_rmsnorm(_p(x), C.c_int64(x.size // d), d, _p(g), C.c_double(eps), _p(out))
    _check(rc, "rmsnorm")
    return out


def mlp_block(x, res, g, w_gate, w_up, w_down, eps):
    """h = x + res (res may be None); out = h + W_down(silu(W_gate n) * W_up n), n = rmsnorm(h) * g."""
    x = _f64(x)
    res = None if res is None else _f64(res)
    if res is not None and res.shape != x.shape:
        raise ValueError("res must have the shape of x")
    g, w_gate, w_up, w_down = _f64(g), _f64(w_gate), _f64(w_up), _f64(w_down)
    d = x.shape[-1]
    d_ff = w_gate.shape[0]
    if w_gate.shape != (d_ff, d) or w_up.shape != (d_ff, d) or w_down.shape != (d, d_ff) or g.shape != (d,):
        raise ValueError("mlp_block: weight shapes")
    out = np.empty_like(x)
    rc = lib().moa_ref_mlp_block(_p(x), _p(res), C.c_int64(x.size // d), d, d_ff, _p(g), _p(w_gate), _p(w_up),
                                 _p(w_down), C.c_double(eps), _p(out))
    _check(rc, "mlp_block")
    return out


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def tree_expand_level(level, child_logp, child_tok, cand_logp, cand_tok, cand_parent, frontier):
    """One level of the draft-tree construction for ONE sequence; the cand_* arrays (float32 / int32, length
    >= Bw + (D-1) Bw^2) and frontier (int32 [Bw]) are updated in place."""
    child_logp, child_tok = _f32(child_logp), _i32(child_tok)
    Bw = child_logp.shape[-1]
    for a, t in ((cand_logp, np.float32), (cand_tok, np.int32), (cand_parent, np.int32), (frontier, np.int32)):
        if a.dtype != t or not a.flags.c_contiguous:
            raise ValueError("state arrays must be C-contiguous float32 / int32")
    rc = lib().moa_ref_tree_expand_level(int(level), Bw, _p(child_logp, C.c_float), _p(child_tok, C.c_int32),
                                         _p(cand_logp, C.c_float), _p(cand_tok, C.c_int32),
                                         _p(cand_parent, C.c_int32), _p(frontier, C.c_int32))
    _check(rc, "tree_expand_level")


def tree_finalize(n_cand, m, root_tok, cand_logp, cand_tok, cand_parent):
    """-> parent [M], tok [M], node_cand [M] of the kept tree (root first), M = 1 + min(m, n_cand)."""
    cand_logp, cand_tok, cand_parent = _f32(cand_logp), _i32(cand_tok), _i32(cand_parent)
    parent = np.full(1 + m, -9, dtype=np.int32)
    tok = np.full(1 + m, -9, dtype=np.int32)
    node_cand = np.full(1 + m, -9, dtype=np.int32)
    M = C.c_int32(0)
    rc = lib().moa_ref_tree_finalize(int(n_cand), int(m), int(root_tok), _p(cand_logp, C.c_float), _p(cand_tok, C.c_int32),
                                     _p(cand_parent, C.c_int32), _p(parent, C.c_int32), _p(tok, C.c_int32),
                                     _p(node_cand, C.c_int32), C.byref(M))
    _check(rc, "tree_finalize")
    return parent[:M.value], tok[:M.value], node_cand[:M.value]


def topk_logprob(logits, Bw):
    """-> tok [F, Bw] int32, logp [F, Bw] float64: the Bw most probable tokens of each row and their log-probabilities."""
    logits = _f64(logits)
    F, V = logits.shape
    tok = np.empty((F, Bw), dtype=np.int32)
    logp = np.empty((F, Bw), dtype=np.float64)
    _check(lib().moa_ref_topk_logprob(_p(logits), F, V, int(Bw), _p(tok, C.c_int32), _p(logp)), "topk_logprob")
    return tok, logp


def lm_head_argmax(x, w):
    """-> tgt [R] int32 (arg max over the vocabulary of x @ w.T, lower id on ties), best [R] (the winning logit)."""
    x, w = _f64(x), _f64(w)
    R, d = x.shape
    V = w.shape[0]
    tgt = np.empty(R, dtype=np.int32)
    best = np.empty(R, dtype=np.float64)
    _check(lib().moa_ref_lm_head_argmax(_p(x), R, d, _p(w), V, _p(tgt, C.c_int32), _p(best)), "lm_head_argmax")
    return tgt, best


def msg_pack_tree(tok, parent):
    tok, parent = _i32(tok), _i32(parent)
    B, M = tok.shape
    msg = np.empty((B, 4 * M), dtype=np.uint8)
    _check(lib().moa_ref_msg_pack_tree(_p(tok, C.c_int32), _p(parent, C.c_int32), B, M, _p(msg, C.c_uint8)), "msg_pack_tree")
    return msg


def msg_unpack_tree(msg):
    msg = np.ascontiguousarray(msg, dtype=np.uint8)
    B, M = msg.shape[0], msg.shape[1] // 4
    tok = np.empty((B, M), dtype=np.int32)
    parent = np.empty((B, M), dtype=np.int32)
    _check(lib().moa_ref_msg_unpack_tree(_p(msg, C.c_uint8), B, M, _p(tok, C.c_int32), _p(parent, C.c_int32)), "msg_unpack_tree")
    return tok, parent


def msg_pack_accept(tok, x):
    """tok [A], x [A, n_vec, n] (float32) -> bytes [A, 3 + n_vec (4 + n)]"""
    tok, x = _i32(tok), _f32(x)
    A, n_vec, n = x.shape
    msg = np.empty((A, 3 + n_vec * (4 + n)), dtype=np.uint8)
    _check(lib().moa_ref_msg_pack_accept(_p(tok, C.c_int32), _p(x, C.c_float), A, n_vec, n, _p(msg, C.c_uint8)), "msg_pack_accept")
    return msg


def msg_unpack_accept(msg, n_vec, n):
    msg = np.ascontiguousarray(msg, dtype=np.uint8)
    A = msg.shape[0]
    tok = np.empty(A, dtype=np.int32)
    x = np.empty((A, n_vec, n), dtype=np.float32)
    _check(lib().moa_ref_msg_unpack_accept(_p(msg, C.c_uint8), A, n_vec, n, _p(tok, C.c_int32), _p(x, C.c_float)), "msg_unpack_accept")
    return tok, x


def msg_gzip(msg: bytes) -> bytes:
    """The gzip pass over the server's first message (Sec. 4.2): the standard library's gzip, no file name, no time
    stamp.  Any valid gzip stream of the message is a correct result; what is unique is what it decompresses to."""
    import gzip
    return gzip.compress(bytes(msg), mtime=0)


def msg_gunzip(gz: bytes) -> bytes:
    import gzip
    return gzip.decompress(bytes(gz))


def tree_accept(parent, tok, tgt):
    parent, tok, tgt = _i32(parent), _i32(tok), _i32(tgt)
    B, M = parent.shape
    path = np.empty((B, M), dtype=np.int32)
    n_path = np.empty((B,), dtype=np.int32)
    bonus = np.empty((B,), dtype=np.int32)
    rc = lib().moa_ref_tree_accept(_p(parent, C.c_int32), _p(tok, C.c_int32), _p(tgt, C.c_int32), B, M,
                                   _p(path, C.c_int32), _p(n_path, C.c_int32), _p(bonus, C.c_int32))
    _check(rc, "tree_accept")
    return path, n_path, bonus


def softmax_weighted_sum(scores, values):
    scores, values = _f64(scores), _f64(values)
    n, dh = values.shape
    o = np.empty((dh,), dtype=np.float64)
    ps = C.c_double(0.0)
    _check(lib().moa_ref_softmax_weighted_sum(_p(scores), _p(values), n, dh, _p(o), C.byref(ps)),
           "softmax_weighted_sum")
    return o, ps.value


def softmax_weighted_sum_chunked(scores, values, chunk):
    scores, values = _f64(scores), _f64(values)
    n, dh = values.shape
    o = np.empty((dh,), dtype=np.float64)
    _check(lib().moa_ref_softmax_weighted_sum_chunked(_p(scores), _p(values), n, dh, chunk, _p(o)),
           "softmax_weighted_sum_chunked")
    return o
