"""ctypes binding of libmoa.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors (PyTorch is used for device memory and streams, nothing else);
every computation happens inside the library's kernels.  Each wrapper checks that the tensors it
hands over are contiguous, on the GPU, of the call's dtype and at least as large as the C
function will touch -- the kernels trust their sizes.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libmoa.so"
if not _LIB_PATH.exists():
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2410_03804_amd.build` "
                      "(there is no fallback path)")
_lib = C.CDLL(str(_LIB_PATH))

F32, BF16 = 0, 1
MAX_TREE = 256
DEV_BAD_PARENT, DEV_BAD_LENGTH, DEV_EMPTY_KEYS, DEV_CACHE_FULL, DEV_BAD_MESSAGE = 1, 2, 4, 8, 16
_TORCH_DTYPE = {F32: torch.float32, BF16: torch.bfloat16}


class MoaError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"{status_str(status)}: {detail}")
        self.status = status


class Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_lsa_in", "lsa_q_heads", "lsa_kv_heads", "dtype")]


class _StepArgs(C.Structure):
    _fields_ = [
        ("shape", C.POINTER(Shape)), ("B", C.c_int32), ("M", C.c_int32), ("Mq", C.c_int32),
        ("parent", C.c_void_p), ("mask", C.c_void_p), ("depth", C.c_void_p),
        ("lsa_hs", C.c_void_p), ("T_lsa", C.c_int64),
        ("lsa_wq", C.c_void_p), ("lsa_wk", C.c_void_p), ("lsa_wv", C.c_void_p), ("lsa_wo", C.c_void_p),
        ("lsa_out", C.c_void_p),
        ("tok_off", C.c_void_p),
        ("ca_wk", C.c_void_p), ("ca_wv", C.c_void_p), ("ca_k", C.c_void_p), ("ca_v", C.c_void_p),
        ("ca_len", C.c_void_p), ("ca_P_cap", C.c_int32),
        ("ca_xq", C.c_void_p), ("ca_wq", C.c_void_p), ("ca_wo", C.c_void_p), ("ca_out", C.c_void_p),
        ("n_verify_layers", C.c_int32),
        ("v_x_host", C.POINTER(C.c_void_p)), ("v_wq_host", C.POINTER(C.c_void_p)),
        ("v_wk_host", C.POINTER(C.c_void_p)), ("v_wv_host", C.POINTER(C.c_void_p)),
        ("v_wo_host", C.POINTER(C.c_void_p)), ("v_kcache_host", C.POINTER(C.c_void_p)),
        ("v_vcache_host", C.POINTER(C.c_void_p)), ("v_out_host", C.POINTER(C.c_void_p)),
        ("v_ktree_host", C.POINTER(C.c_void_p)), ("v_vtree_host", C.POINTER(C.c_void_p)),
        ("prefix_len", C.c_void_p), ("P_cap", C.c_int32),
        ("tok", C.c_void_p), ("tgt", C.c_void_p), ("path", C.c_void_p), ("n_path", C.c_void_p),
        ("bonus", C.c_void_p),
        ("dev_status", C.c_void_p), ("ws", C.c_void_p), ("ws_bytes", C.c_size_t), ("stream", C.c_void_p),
        ("schedule", C.c_int32),
        ("sa_shape", C.POINTER(Shape)), ("sa_emb", C.c_void_p),
        ("sa_wq", C.c_void_p), ("sa_wk", C.c_void_p), ("sa_wv", C.c_void_p), ("sa_wo", C.c_void_p),
        ("sa_kcache", C.c_void_p), ("sa_vcache", C.c_void_p), ("sa_P_cap", C.c_int32),
        ("sa_k_draft", C.c_void_p), ("sa_v_draft", C.c_void_p), ("sa_out", C.c_void_p),
        ("ca_wk_lsa_wo", C.c_void_p), ("ca_wv_lsa_wo", C.c_void_p),
        ("lsa_w_packed", C.c_void_p),
    ]


SCHED_GROUPED, SCHED_TWO_STREAM, SCHED_SEQUENTIAL = 0, 1, 2

_SYMBOLS = ["moa_status_str", "moa_last_error", "moa_workspace_bytes", "moa_tree_build", "moa_tree_accept",
            "moa_lsa", "moa_ca_kv_append", "moa_cross_attn_draft", "moa_tree_verify_attn", "moa_draft_step",
            "moa_self_attn_draft", "moa_tli_workspace_bytes", "moa_tli_decoder_layer", "moa_tree_expand_level", "moa_tree_finalize", "moa_topk_logprob", "moa_topk_workspace_bytes", "moa_lm_head_workspace_bytes", "moa_lm_head_argmax", "moa_msg_pack_tree", "moa_msg_unpack_tree", "moa_msg_accept_bytes", "moa_msg_pack_accept",
            "moa_msg_unpack_accept", "moa_msg_gzip_bound", "moa_msg_gzip", "moa_msg_gunzip", "moa_linear_workspace_bytes", "moa_linear", "moa_fold_projection", "moa_lsa_packed_weight_bytes", "moa_lsa_pack_weights", "moa_lsa_packed", "moa_mlp_block_workspace_bytes", "moa_mlp_block", "moa_rmsnorm", "moa_profile_enable", "moa_profile_sample_every", "moa_profile_collect", "moa_profile_kernel_name", "moa_profile_site_name", "moa_probe_read", "moa_probe_mfma",
            "moa_debug_force_attn_kernel", "moa_debug_force_lsa_kernel", "moa_tree_verify_attn_noalloc"]

_lib.moa_status_str.restype = C.c_char_p
_lib.moa_status_str.argtypes = [C.c_int32]
_lib.moa_last_error.restype = C.c_char_p
_lib.moa_last_error.argtypes = []
_vp, _i32, _i64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
_lib.moa_workspace_bytes.argtypes = [C.POINTER(Shape), _i32, _i32, _i32, _i64, C.POINTER(_sz)]
_lib.moa_tree_build.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.moa_tree_accept.argtypes = [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.moa_lsa.argtypes = [C.POINTER(Shape), _vp, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moa_lsa_packed_weight_bytes.argtypes = [C.POINTER(Shape), C.POINTER(_sz)]
_lib.moa_lsa_pack_weights.argtypes = [C.POINTER(Shape), _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moa_lsa_packed.argtypes = [C.POINTER(Shape), _vp, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moa_ca_kv_append.argtypes = [C.POINTER(Shape), _vp, _i64, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
_lib.moa_cross_attn_draft.argtypes = [C.POINTER(Shape), _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.moa_tree_verify_attn.argtypes = [C.POINTER(Shape), _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp,
                                      _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moa_tree_verify_attn_noalloc.argtypes = [C.POINTER(Shape), _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp,
                                              _vp, _vp, _vp, _vp, _vp]
_lib.moa_draft_step.argtypes = [C.POINTER(_StepArgs)]
_lib.moa_self_attn_draft.argtypes = [C.POINTER(Shape), _vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp,
                                     _vp, _vp, _vp, _vp, _vp, _sz, _vp]


class DecoderCfg(C.Structure):
    """moa_decoder_cfg_t: MLP width, RMS-norm epsilon and rotary base of a reused LLM decoder layer."""
    _fields_ = [("d_ff", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


_lib.moa_tli_workspace_bytes.argtypes = [C.POINTER(Shape), C.POINTER(DecoderCfg), _i32, _i32, _i32, C.POINTER(_sz)]
_lib.moa_tli_decoder_layer.argtypes = [C.POINTER(Shape), C.POINTER(DecoderCfg), _vp, _i32, _i32, _i32, _i32] + [_vp] * 11 + [
    _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moa_tree_expand_level.argtypes = [_i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.moa_tree_finalize.argtypes = [_i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.moa_topk_logprob.argtypes = [_i32, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.moa_topk_workspace_bytes.argtypes = [_i32, _i32, _i32, C.POINTER(_sz)]
_lib.moa_lm_head_workspace_bytes.argtypes = [_i32, C.POINTER(_sz)]
_lib.moa_lm_head_argmax.argtypes = [_i32, _vp, _i32, _i32, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.moa_msg_pack_tree.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp, _vp]
_lib.moa_msg_unpack_tree.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp]
_lib.moa_msg_accept_bytes.argtypes = [_i32, _i32, _i32, C.POINTER(_sz)]
_lib.moa_msg_pack_accept.argtypes = [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.moa_msg_unpack_accept.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.moa_msg_gzip_bound.argtypes = [_sz, C.POINTER(_sz)]
_lib.moa_msg_gzip.argtypes = [C.c_char_p, _sz, _vp, _sz, C.POINTER(_sz)]
_lib.moa_msg_gunzip.argtypes = [C.c_char_p, _sz, _vp, _sz, C.POINTER(_sz)]
_lib.moa_linear_workspace_bytes.argtypes = [_i32, _i64, _i32, _i32, C.POINTER(_sz)]
_lib.moa_linear.argtypes = [_i32, _vp, _i64, _i32, _vp, _i32, _vp, _vp, _sz, _vp]
_lib.moa_fold_projection.argtypes = [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _vp]
_lib.moa_mlp_block_workspace_bytes.argtypes = [_i32, _i64, _i32, _i32, C.POINTER(_sz)]
_lib.moa_mlp_block.argtypes = [_i32, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, C.c_float, _vp, _vp, _sz, _vp]
_lib.moa_rmsnorm.argtypes = [_i32, _vp, _i64, _i32, _vp, C.c_float, _vp, _vp]
for _n in _SYMBOLS[2:30]:
    getattr(_lib, _n).restype = C.c_int32


class _ProfileRow(C.Structure):
    _fields_ = [("site", C.c_int32), ("kernel", C.c_int32), ("launches", C.c_int64), ("total_ms", C.c_double)]


_lib.moa_profile_enable.argtypes = [_i32, _i32]
_lib.moa_profile_sample_every.argtypes = [_i32]
_lib.moa_profile_collect.argtypes = [C.POINTER(_ProfileRow), _i32, C.POINTER(_i32)]
_lib.moa_profile_kernel_name.restype = C.c_char_p
_lib.moa_profile_kernel_name.argtypes = [_i32]
_lib.moa_profile_site_name.restype = C.c_char_p
_lib.moa_profile_site_name.argtypes = [_i32]
_lib.moa_debug_force_attn_kernel.argtypes = [_i32]
_lib.moa_debug_force_lsa_kernel.argtypes = [_i32]
_lib.moa_probe_read.argtypes = [_vp, _sz, _vp, _vp]
_lib.moa_probe_mfma.argtypes = [_i32, _vp, C.POINTER(_i64), _vp]


def library_path() -> str:
    return str(_LIB_PATH)


def exported_symbols():
    return list(_SYMBOLS)


def status_str(status: int) -> str:
    return _lib.moa_status_str(status).decode()


def last_error() -> str:
    return _lib.moa_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise MoaError(rc, last_error())


def _dev(t, dtype, numel, name):
    """Device pointer of tensor t after checking it can hold what the call touches."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch tensor")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: must be a contiguous CUDA tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, the call touches {numel}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    if not ws.is_cuda or not ws.is_contiguous():
        raise ValueError("ws: must be a contiguous CUDA tensor")
    return C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def workspace_bytes(shape: Shape, B: int, P_cap: int, M: int, T_lsa: int) -> int:
    out = _sz(0)
    _check(_lib.moa_workspace_bytes(C.byref(shape), B, P_cap, M, T_lsa, C.byref(out)))
    return out.value


def tree_build(parent, mask, depth, dev_status=None, stream=None):
    B, M = parent.shape
    W = (M + 63) // 64
    _check(_lib.moa_tree_build(_dev(parent, torch.int32, B * M, "parent"), B, M,
                               _dev(mask, torch.int64, B * M * W, "mask"), _dev(depth, torch.int32, B * M, "depth"),
                               _dev(dev_status, torch.int32, 1, "dev_status"), _stream(stream)))


def tree_accept(parent, tok, tgt, path, n_path, bonus, stream=None):
    B, M = parent.shape
    i32 = torch.int32
    _check(_lib.moa_tree_accept(_dev(parent, i32, B * M, "parent"), _dev(tok, i32, B * M, "tok"),
                                _dev(tgt, i32, B * M, "tgt"), B, M, _dev(path, i32, B * M, "path"),
                                _dev(n_path, i32, B, "n_path"), _dev(bonus, i32, B, "bonus"), _stream(stream)))


def lsa(shape: Shape, hs, wq, wk, wv, wo, out, ws, stream=None):
    dt = _TORCH_DTYPE[shape.dtype]
    T = hs.shape[0]
    L, d_in, dh = shape.n_layers, shape.d_lsa_in, shape.head_dim
    eq, ekv = shape.lsa_q_heads * dh, shape.lsa_kv_heads * dh
    wsp, wsb = _ws(ws)
    _check(_lib.moa_lsa(C.byref(shape), _dev(hs, dt, T * L * d_in, "hs"), T,
                        _dev(wq, dt, eq * d_in, "wq"), _dev(wk, dt, ekv * d_in, "wk"), _dev(wv, dt, ekv * d_in, "wv"),
                        _dev(wo, dt, eq * eq, "wo"), _dev(out, dt, T * eq, "out"), wsp, wsb, _stream(stream)))


def lsa_packed_weight_bytes(shape: Shape) -> int:
    n = _sz(0)
    _check(_lib.moa_lsa_packed_weight_bytes(C.byref(shape), C.byref(n)))
    return int(n.value)


def lsa_pack_weights(shape: Shape, wq, wk, wv, stream=None):
    """Wq / Wk / Wv in the order the one-kernel LSA consumes them (done once, at load time); returns the packed tensor."""
    dt = _TORCH_DTYPE[shape.dtype]
    d_in, dh = shape.d_lsa_in, shape.head_dim
    eq, ekv = shape.lsa_q_heads * dh, shape.lsa_kv_heads * dh
    nbytes = lsa_packed_weight_bytes(shape)
    packed = torch.empty(nbytes // 2, dtype=dt, device=wq.device)
    _check(_lib.moa_lsa_pack_weights(C.byref(shape), _dev(wq, dt, eq * d_in, "wq"), _dev(wk, dt, ekv * d_in, "wk"),
                                     _dev(wv, dt, ekv * d_in, "wv"), _dev(packed, dt, nbytes // 2, "packed"), nbytes,
                                     _stream(stream)))
    return packed


def lsa_packed(shape: Shape, hs, w_packed, wo, out, ws, stream=None):
    dt = _TORCH_DTYPE[shape.dtype]
    T = hs.shape[0]
    L, d_in, dh = shape.n_layers, shape.d_lsa_in, shape.head_dim
    eq = shape.lsa_q_heads * dh
    wsp, wsb = _ws(ws)
    _check(_lib.moa_lsa_packed(C.byref(shape), _dev(hs, dt, T * L * d_in, "hs"), T,
                               _dev(w_packed, dt, lsa_packed_weight_bytes(shape) // 2, "w_packed"),
                               _dev(wo, dt, eq * eq, "wo"), _dev(out, dt, T * eq, "out"), wsp, wsb, _stream(stream)))


def ca_kv_append(shape: Shape, mem_new, tok_off, wk, wv, kc, vc, ca_len, P_cap, dev_status=None, ws=None, stream=None):
    dt = _TORCH_DTYPE[shape.dtype]
    T, d_mem = mem_new.shape
    B = ca_len.shape[0]
    ekv = shape.n_kv_heads * shape.head_dim
    cache = B * ekv * P_cap
    wsp, wsb = _ws(ws)
    _check(_lib.moa_ca_kv_append(C.byref(shape), _dev(mem_new, dt, T * d_mem, "mem_new"), T, d_mem,
                                 _dev(tok_off, torch.int32, B + 1, "tok_off"), B,
                                 _dev(wk, dt, ekv * d_mem, "wk"), _dev(wv, dt, ekv * d_mem, "wv"),
                                 _dev(kc, dt, cache, "kc"), _dev(vc, dt, cache, "vc"),
                                 _dev(ca_len, torch.int32, B, "ca_len"), P_cap,
                                 _dev(dev_status, torch.int32, 1, "dev_status"), wsp, wsb, _stream(stream)))


def cross_attn_draft(shape: Shape, xq, wq, wo, kc, vc, ca_len, P_cap, out, ws, dev_status=None, stream=None):
    dt = _TORCH_DTYPE[shape.dtype]
    B, Mq, d = xq.shape
    if d != shape.d_model:
        raise ValueError("xq: last dimension must be d_model")
    e, ekv = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    cache = B * ekv * P_cap
    wsp, wsb = _ws(ws)
    _check(_lib.moa_cross_attn_draft(C.byref(shape), _dev(xq, dt, B * Mq * d, "xq"), B, Mq,
                                     _dev(wq, dt, e * d, "wq"), _dev(wo, dt, d * e, "wo"),
                                     _dev(kc, dt, cache, "kc"), _dev(vc, dt, cache, "vc"),
                                     _dev(ca_len, torch.int32, B, "ca_len"), P_cap, _dev(out, dt, B * Mq * d, "out"),
                                     _dev(dev_status, torch.int32, 1, "dev_status"), wsp, wsb, _stream(stream)))


def tree_verify_attn(shape: Shape, x, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap, mask, out, k_tree, v_tree,
                     ws, dev_status=None, stream=None):
    dt = _TORCH_DTYPE[shape.dtype]
    B, M, d = x.shape
    if d != shape.d_model:
        raise ValueError("x: last dimension must be d_model")
    e, ekv = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    cache = B * ekv * P_cap
    W = (M + 63) // 64
    wsp, wsb = _ws(ws)
    _check(_lib.moa_tree_verify_attn(C.byref(shape), _dev(x, dt, B * M * d, "x"), B, M,
                                     _dev(wq, dt, e * d, "wq"), _dev(wk, dt, ekv * d, "wk"), _dev(wv, dt, ekv * d, "wv"),
                                     _dev(wo, dt, d * e, "wo"),
                                     _dev(kcache, dt, cache, "kcache"), _dev(vcache, dt, cache, "vcache"),
                                     _dev(prefix_len, torch.int32, B, "prefix_len"), P_cap,
                                     _dev(mask, torch.int64, B * M * W, "mask"), _dev(out, dt, B * M * d, "out"),
                                     _dev(k_tree, dt, B * ekv * M, "k_tree"), _dev(v_tree, dt, B * ekv * M, "v_tree"),
                                     _dev(dev_status, torch.int32, 1, "dev_status"), wsp, wsb, _stream(stream)))


def tree_verify_attn_noalloc(shape: Shape, x, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap, mask, out, k_tree, v_tree,
                             dev_status=None, stream=None):
    """moa_tree_verify_attn without a workspace: the scratch is the library's own fixed device array."""
    dt = _TORCH_DTYPE[shape.dtype]
    B, M, d = x.shape
    if d != shape.d_model:
        raise ValueError("x: last dimension must be d_model")
    e, ekv = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    cache = B * ekv * P_cap
    W = (M + 63) // 64
    _check(_lib.moa_tree_verify_attn_noalloc(
        C.byref(shape), _dev(x, dt, B * M * d, "x"), B, M,
        _dev(wq, dt, e * d, "wq"), _dev(wk, dt, ekv * d, "wk"), _dev(wv, dt, ekv * d, "wv"), _dev(wo, dt, d * e, "wo"),
        _dev(kcache, dt, cache, "kcache"), _dev(vcache, dt, cache, "vcache"),
        _dev(prefix_len, torch.int32, B, "prefix_len"), P_cap,
        _dev(mask, torch.int64, B * M * W, "mask"), _dev(out, dt, B * M * d, "out"),
        _dev(k_tree, dt, B * ekv * M, "k_tree"), _dev(v_tree, dt, B * ekv * M, "v_tree"),
        _dev(dev_status, torch.int32, 1, "dev_status"), _stream(stream)))


def self_attn_draft(shape: Shape, emb, node_begin, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap, mask, out, k_draft, v_draft,
                    ws, dev_status=None, stream=None):
    """Draft Self-Attention layer on the nodes node_begin .. node_begin+Mn-1 (emb [B, Mn, d]) of the tree whose
    mask [B, M, W] is given; k_draft / v_draft [B, Hkv, M, dh] are updated in place."""
    dt = _TORCH_DTYPE[shape.dtype]
    B, Mn, d = emb.shape
    M = mask.shape[1]
    W = (M + 63) // 64
    dh = shape.head_dim
    e, ekv = shape.n_q_heads * dh, shape.n_kv_heads * dh
    cache = B * ekv * P_cap
    wsp, wsb = _ws(ws)
    _check(_lib.moa_self_attn_draft(C.byref(shape), _dev(emb, dt, B * Mn * d, "emb"), B, M, int(node_begin), Mn,
                                    _dev(wq, dt, e * d, "wq"), _dev(wk, dt, ekv * d, "wk"), _dev(wv, dt, ekv * d, "wv"),
                                    _dev(wo, dt, d * e, "wo"),
                                    _dev(kcache, dt, cache, "kcache"), _dev(vcache, dt, cache, "vcache"),
                                    _dev(prefix_len, torch.int32, B, "prefix_len"), P_cap,
                                    _dev(mask, torch.int64, B * M * W, "mask"), _dev(out, dt, B * Mn * d, "out"),
                                    _dev(k_draft, dt, B * ekv * M, "k_draft"), _dev(v_draft, dt, B * ekv * M, "v_draft"),
                                    _dev(dev_status, torch.int32, 1, "dev_status"), wsp, wsb, _stream(stream)))


def tli_workspace_bytes(shape: Shape, cfg: DecoderCfg, B: int, P_cap: int, M: int) -> int:
    out = _sz(0)
    _check(_lib.moa_tli_workspace_bytes(C.byref(shape), C.byref(cfg), B, P_cap, M, C.byref(out)))
    return int(out.value)


def tli_decoder_layer(shape: Shape, cfg: DecoderCfg, x, node_begin, w, kcache, vcache, prefix_len, P_cap, mask, depth, out,
                      k_draft, v_draft, ws, dev_status=None, stream=None):
    """One reused LLM decoder layer on the nodes node_begin .. node_begin+Mn-1 (x [B, Mn, d]); w = dict(g_attn, wq, wk,
    wv, wo, g_mlp, w_gate, w_up, w_down); k_draft / v_draft [B, Hkv, M, dh] are updated in place."""
    dt = _TORCH_DTYPE[shape.dtype]
    B, Mn, d = x.shape
    M = mask.shape[1]
    W = (M + 63) // 64
    dh = shape.head_dim
    e, ekv, dff = shape.n_q_heads * dh, shape.n_kv_heads * dh, cfg.d_ff
    cache = B * ekv * P_cap
    wsp, wsb = _ws(ws)
    _check(_lib.moa_tli_decoder_layer(
        C.byref(shape), C.byref(cfg), _dev(x, dt, B * Mn * d, "x"), B, M, int(node_begin), Mn,
        _dev(w["g_attn"], dt, d, "g_attn"), _dev(w["wq"], dt, e * d, "wq"), _dev(w["wk"], dt, ekv * d, "wk"),
        _dev(w["wv"], dt, ekv * d, "wv"), _dev(w["wo"], dt, d * e, "wo"), _dev(w["g_mlp"], dt, d, "g_mlp"),
        _dev(w["w_gate"], dt, dff * d, "w_gate"), _dev(w["w_up"], dt, dff * d, "w_up"), _dev(w["w_down"], dt, d * dff, "w_down"),
        _dev(kcache, dt, cache, "kcache"), _dev(vcache, dt, cache, "vcache"),
        _dev(prefix_len, torch.int32, B, "prefix_len"), P_cap, _dev(mask, torch.int64, B * M * W, "mask"),
        _dev(depth, torch.int32, B * M, "depth"), _dev(out, dt, B * Mn * d, "out"),
        _dev(k_draft, dt, B * ekv * M, "k_draft"), _dev(v_draft, dt, B * ekv * M, "v_draft"),
        _dev(dev_status, torch.int32, 1, "dev_status"), wsp, wsb, _stream(stream)))


def mlp_block_workspace_bytes(dtype, R, d, d_ff) -> int:
    out = C.c_size_t(0)
    _check(_lib.moa_mlp_block_workspace_bytes(int(dtype), int(R), int(d), int(d_ff), C.byref(out)))
    return int(out.value)


def mlp_block(dtype, x, res, g, w_gate, w_up, w_down, rms_eps, out, ws, stream=None):
    """out = h + W_down(silu(W_gate n) * W_up n), h = x + res (res may be None), n = rmsnorm(h) * g; x [..., d]."""
    dt = _TORCH_DTYPE[dtype]
    d = x.shape[-1]
    R = x.numel() // d
    d_ff = w_gate.shape[0]
    wsp, wsb = _ws(ws)
    _check(_lib.moa_mlp_block(int(dtype), _dev(x, dt, R * d, "x"), _dev(res, dt, R * d, "res"), R, d, d_ff,
                              _dev(g, dt, d, "g"), _dev(w_gate, dt, d_ff * d, "w_gate"), _dev(w_up, dt, d_ff * d, "w_up"),
                              _dev(w_down, dt, d * d_ff, "w_down"), float(rms_eps), _dev(out, dt, R * d, "out"), wsp, wsb,
                              _stream(stream)))


def rmsnorm(dtype, x, g, rms_eps, out, stream=None):
    """out = x / sqrt(mean(x^2) + rms_eps) * g over the last axis."""
    dt = _TORCH_DTYPE[dtype]
    d = x.shape[-1]
    R = x.numel() // d
    _check(_lib.moa_rmsnorm(int(dtype), _dev(x, dt, R * d, "x"), R, d, _dev(g, dt, d, "g"), float(rms_eps),
                            _dev(out, dt, R * d, "out"), _stream(stream)))


def tree_expand_level(level, child_logp, child_tok, cand_logp, cand_tok, cand_parent, frontier, stream=None):
    """One level of the draft-tree construction: child_logp (fp32) / child_tok (int32) [B, F, Bw]; the state tensors
    cand_logp (fp32), cand_tok, cand_parent [B, n_max] and frontier [B, Bw] (int32) are updated in place."""
    B, F, Bw = child_logp.shape
    n_max = cand_logp.shape[1]
    f32, i32 = torch.float32, torch.int32
    _check(_lib.moa_tree_expand_level(int(level), B, Bw, n_max, _dev(child_logp, f32, B * F * Bw, "child_logp"),
                                      _dev(child_tok, i32, B * F * Bw, "child_tok"), _dev(cand_logp, f32, B * n_max, "cand_logp"),
                                      _dev(cand_tok, i32, B * n_max, "cand_tok"), _dev(cand_parent, i32, B * n_max, "cand_parent"),
                                      _dev(frontier, i32, B * Bw, "frontier"), _stream(stream)))


def tree_finalize(n_cand, m, root_tok, cand_logp, cand_tok, cand_parent, parent, tok, node_cand, dev_status=None, stream=None):
    """Keep the m best candidates: parent / tok / node_cand [B, 1+m] (int32) receive the tree, root first."""
    B, n_max = cand_logp.shape
    f32, i32 = torch.float32, torch.int32
    _check(_lib.moa_tree_finalize(B, int(n_cand), n_max, int(m), _dev(root_tok, i32, B, "root_tok"),
                                  _dev(cand_logp, f32, B * n_max, "cand_logp"), _dev(cand_tok, i32, B * n_max, "cand_tok"),
                                  _dev(cand_parent, i32, B * n_max, "cand_parent"), _dev(parent, i32, B * (1 + m), "parent"),
                                  _dev(tok, i32, B * (1 + m), "tok"), _dev(node_cand, i32, B * (1 + m), "node_cand"),
                                  _dev(dev_status, i32, 1, "dev_status"), _stream(stream)))


def topk_workspace_bytes(F: int, V: int, Bw: int) -> int:
    out = _sz(0)
    _check(_lib.moa_topk_workspace_bytes(int(F), int(V), int(Bw), C.byref(out)))
    return int(out.value)


def topk_logprob(logits, Bw, tok, logp, ws, stream=None):
    """The Bw most probable tokens of each row of logits [F, V] (fp32 or bf16) -> tok (int32), logp (fp32) [F, Bw]."""
    F, V = logits.shape
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[logits.dtype]
    wsp, wsb = _ws(ws)
    _check(_lib.moa_topk_logprob(dtype, _dev(logits, logits.dtype, F * V, "logits"), F, V, int(Bw),
                                 _dev(tok, torch.int32, F * Bw, "tok"), _dev(logp, torch.float32, F * Bw, "logp"),
                                 wsp, wsb, _stream(stream)))


def lm_head_workspace_bytes(V: int) -> int:
    out = _sz(0)
    _check(_lib.moa_lm_head_workspace_bytes(int(V), C.byref(out)))
    return int(out.value)


def lm_head_argmax(x, w, tgt, ws, best=None, stream=None):
    """tgt[r] = argmax over the vocabulary of x[r] . w[v] (x [R, d], w [V, d] bf16; tgt int32 [R]; best fp32 [R] or None)."""
    R, d = x.shape
    V = w.shape[0]
    wsp, wsb = _ws(ws)
    _check(_lib.moa_lm_head_argmax(BF16 if x.dtype == torch.bfloat16 else F32, _dev(x, x.dtype, R * d, "x"), R, d,
                                   _dev(w, x.dtype, V * d, "w"), V, _dev(tgt, torch.int32, R, "tgt"),
                                   _dev(best, torch.float32, R, "best"), wsp, wsb, _stream(stream)))


def msg_pack_tree(tok, parent, msg, dev_status=None, stream=None):
    """tok, parent [B, M] int32 -> msg [B, 4 M] uint8 (3-byte token id + 1-byte parent index per node)."""
    B, M = tok.shape
    _check(_lib.moa_msg_pack_tree(_dev(tok, torch.int32, B * M, "tok"), _dev(parent, torch.int32, B * M, "parent"), B, M,
                                  _dev(msg, torch.uint8, 4 * B * M, "msg"), _dev(dev_status, torch.int32, 1, "dev_status"), _stream(stream)))


def msg_unpack_tree(msg, tok, parent, stream=None):
    B, M = tok.shape
    _check(_lib.moa_msg_unpack_tree(_dev(msg, torch.uint8, 4 * B * M, "msg"), B, M, _dev(tok, torch.int32, B * M, "tok"),
                                    _dev(parent, torch.int32, B * M, "parent"), _stream(stream)))


def msg_accept_bytes(A: int, n_vec: int, n: int) -> int:
    out = _sz(0)
    _check(_lib.moa_msg_accept_bytes(int(A), int(n_vec), int(n), C.byref(out)))
    return int(out.value)


def msg_pack_accept(tok, x, msg, dev_status=None, stream=None):
    """tok [A] int32, x [A, n_vec, n] (fp32 or bf16) -> msg (uint8, msg_accept_bytes(A, n_vec, n))."""
    A, n_vec, n = x.shape
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    _check(_lib.moa_msg_pack_accept(dtype, _dev(tok, torch.int32, A, "tok"), _dev(x, x.dtype, A * n_vec * n, "x"), A, n_vec, n,
                                    _dev(msg, torch.uint8, msg_accept_bytes(A, n_vec, n), "msg"),
                                    _dev(dev_status, torch.int32, 1, "dev_status"), _stream(stream)))


def msg_unpack_accept(msg, tok, x, stream=None):
    A, n_vec, n = x.shape
    _check(_lib.moa_msg_unpack_accept(_dev(msg, torch.uint8, msg_accept_bytes(A, n_vec, n), "msg"), A, n_vec, n,
                                      _dev(tok, torch.int32, A, "tok"), _dev(x, torch.float32, A * n_vec * n, "x"), _stream(stream)))


def msg_gzip(msg: bytes) -> bytes:
    """gzip-compress a (host) message, as the server does with the first message of a conversation."""
    bound = _sz(0)
    _check(_lib.moa_msg_gzip_bound(len(msg), C.byref(bound)))
    out = C.create_string_buffer(max(bound.value, 1))
    n = _sz(0)
    _check(_lib.moa_msg_gzip(msg, len(msg), out, bound.value, C.byref(n)))
    return out.raw[: n.value]


def msg_gunzip(gz: bytes, max_bytes: int) -> bytes:
    """The inverse of msg_gzip; max_bytes bounds the size of the message."""
    out = C.create_string_buffer(max(int(max_bytes), 1))
    n = _sz(0)
    _check(_lib.moa_msg_gunzip(gz, len(gz), out, int(max_bytes), C.byref(n)))
    return out.raw[: n.value]


def linear_workspace_bytes(dtype: int, R: int, K: int, N: int) -> int:
    out = _sz(0)
    _check(_lib.moa_linear_workspace_bytes(dtype, R, K, N, C.byref(out)))
    return int(out.value)


def linear(x, w, y, ws=None, stream=None):
    """y [R, N] = x [R, K] @ w [N, K].T (fp32 or bf16, all the same dtype)."""
    R, K = x.shape
    N = w.shape[0]
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    wsp, wsb = _ws(ws)
    _check(_lib.moa_linear(dtype, _dev(x, x.dtype, R * K, "x"), R, K, _dev(w, x.dtype, N * K, "w"), N, _dev(y, x.dtype, R * N, "y"),
                           wsp, wsb, _stream(stream)))


def fold_projection(w_outer, w_inner, out=None, stream=None):
    """out [N, K] = w_outer [N, J] @ w_inner [J, K] (two projections applied one after the other, folded once)."""
    N, J = w_outer.shape
    K = w_inner.shape[1]
    if out is None:
        out = torch.empty((N, K), dtype=w_outer.dtype, device=w_outer.device)
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[w_outer.dtype]
    _check(_lib.moa_fold_projection(dtype, _dev(w_outer, w_outer.dtype, N * J, "w_outer"), _dev(w_inner, w_outer.dtype, J * K, "w_inner"),
                                    N, J, K, _dev(out, w_outer.dtype, N * K, "out"), _stream(stream)))
    return out


def _ptr_array(tensors, dtype, numel, name):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        p = _dev(t, dtype, numel, f"{name}[{i}]")
        arr[i] = None if p is None else p.value
    return arr


def draft_step_plan(shape: Shape, *, parent, mask, depth, lsa_hs, lsa_w, lsa_out, tok_off, ca_w, ca_k, ca_v, ca_len,
               ca_P_cap, ca_xq, ca_out, v_x, v_w, v_kcache, v_vcache, v_out, v_ktree, v_vtree, prefix_len, P_cap,
               tok, tgt, path, n_path, bonus, ws, dev_status=None, schedule=0, sa=None, folded=None, lsa_w_packed=None):
    """Marshal (and size-check) the arguments of moa_draft_step once; the returned plan can be run many times.
    lsa_w = dict(wq, wk, wv, wo); ca_w = dict(wq, wo, wk, wv); v_w = list (one per verified layer) of
    dict(wq, wk, wv, wo); v_* = lists of per-layer tensors.  The plan keeps the tensors alive.
    sa (optional) = dict(shape, emb, w=dict(wq, wk, wv, wo), kcache, vcache, P_cap, k_draft, v_draft, out): the
    Self-Attention layer in front of the cross-attention (ca_xq may then be None).
    folded (optional) = (ca_wk @ lsa_wo, ca_wv @ lsa_wo) from fold_projection: the memory append then shares the LSA
    output projection's launch.
    lsa_w_packed (optional) = lsa_pack_weights(shape, wq, wk, wv) of the same LSA weights."""
    dt, i32 = _TORCH_DTYPE[shape.dtype], torch.int32
    B, M = parent.shape
    Mq = ca_xq.shape[1]
    T = lsa_hs.shape[0]
    W = (M + 63) // 64
    L, d_in, dh, d = shape.n_layers, shape.d_lsa_in, shape.head_dim, shape.d_model
    eq, ekvl = shape.lsa_q_heads * dh, shape.lsa_kv_heads * dh
    e, ekv = shape.n_q_heads * dh, shape.n_kv_heads * dh
    n = len(v_x)
    if not all(len(v) == n for v in (v_w, v_kcache, v_vcache, v_out, v_ktree, v_vtree)):
        raise ValueError("per-layer lists must have the same length")
    a = _StepArgs()
    a.shape = C.pointer(shape)
    a.B, a.M, a.Mq = B, M, Mq
    a.parent = _dev(parent, i32, B * M, "parent")
    a.mask = _dev(mask, torch.int64, B * M * W, "mask")
    a.depth = _dev(depth, i32, B * M, "depth")
    a.lsa_hs = _dev(lsa_hs, dt, T * L * d_in, "lsa_hs")
    a.T_lsa = T
    a.lsa_wq = _dev(lsa_w["wq"], dt, eq * d_in, "lsa wq")
    a.lsa_wk = _dev(lsa_w["wk"], dt, ekvl * d_in, "lsa wk")
    a.lsa_wv = _dev(lsa_w["wv"], dt, ekvl * d_in, "lsa wv")
    a.lsa_wo = _dev(lsa_w["wo"], dt, eq * eq, "lsa wo")
    a.lsa_out = _dev(lsa_out, dt, T * eq, "lsa_out")
    a.tok_off = _dev(tok_off, i32, B + 1, "tok_off")
    a.ca_wk = _dev(ca_w["wk"], dt, ekv * eq, "ca wk")
    a.ca_wv = _dev(ca_w["wv"], dt, ekv * eq, "ca wv")
    a.ca_k = _dev(ca_k, dt, B * ekv * ca_P_cap, "ca_k")
    a.ca_v = _dev(ca_v, dt, B * ekv * ca_P_cap, "ca_v")
    a.ca_len = _dev(ca_len, i32, B, "ca_len")
    a.ca_P_cap = ca_P_cap
    a.ca_xq = None if (sa is not None and ca_xq is None) else _dev(ca_xq, dt, B * Mq * d, "ca_xq")
    a.ca_wq = _dev(ca_w["wq"], dt, e * d, "ca wq")
    a.ca_wo = _dev(ca_w["wo"], dt, d * e, "ca wo")
    a.ca_out = _dev(ca_out, dt, B * Mq * d, "ca_out")
    a.n_verify_layers = n
    keep = [
        _ptr_array(v_x, dt, B * M * d, "v_x"),
        _ptr_array([w["wq"] for w in v_w], dt, e * d, "v wq"), _ptr_array([w["wk"] for w in v_w], dt, ekv * d, "v wk"),
        _ptr_array([w["wv"] for w in v_w], dt, ekv * d, "v wv"), _ptr_array([w["wo"] for w in v_w], dt, d * e, "v wo"),
        _ptr_array(v_kcache, dt, B * ekv * P_cap, "v_kcache"), _ptr_array(v_vcache, dt, B * ekv * P_cap, "v_vcache"),
        _ptr_array(v_out, dt, B * M * d, "v_out"), _ptr_array(v_ktree, dt, B * ekv * M, "v_ktree"),
        _ptr_array(v_vtree, dt, B * ekv * M, "v_vtree"),
    ]
    (a.v_x_host, a.v_wq_host, a.v_wk_host, a.v_wv_host, a.v_wo_host, a.v_kcache_host, a.v_vcache_host, a.v_out_host,
     a.v_ktree_host, a.v_vtree_host) = [C.cast(k, C.POINTER(C.c_void_p)) for k in keep]
    a.prefix_len = _dev(prefix_len, i32, B, "prefix_len")
    a.P_cap = P_cap
    a.tok = _dev(tok, i32, B * M, "tok")
    a.tgt = _dev(tgt, i32, B * M, "tgt")
    a.path = _dev(path, i32, B * M, "path")
    a.n_path = _dev(n_path, i32, B, "n_path")
    a.bonus = _dev(bonus, i32, B, "bonus")
    a.dev_status = _dev(dev_status, i32, 1, "dev_status")
    a.ws, a.ws_bytes = _ws(ws)
    a.schedule = int(schedule)
    if folded is not None:
        a.ca_wk_lsa_wo = _dev(folded[0], dt, ekv * eq, "ca_wk lsa_wo")
        a.ca_wv_lsa_wo = _dev(folded[1], dt, ekv * eq, "ca_wv lsa_wo")
    if lsa_w_packed is not None:
        a.lsa_w_packed = _dev(lsa_w_packed, dt, lsa_packed_weight_bytes(shape) // 2, "lsa_w_packed")
    if sa is not None:
        ssh = sa["shape"]
        ekv_s = ssh.n_kv_heads * dh
        a.sa_shape = C.pointer(ssh)
        a.sa_emb = _dev(sa["emb"], dt, B * M * d, "sa emb")
        a.sa_wq = _dev(sa["w"]["wq"], dt, e * d, "sa wq")
        a.sa_wk = _dev(sa["w"]["wk"], dt, ekv_s * d, "sa wk")
        a.sa_wv = _dev(sa["w"]["wv"], dt, ekv_s * d, "sa wv")
        a.sa_wo = _dev(sa["w"]["wo"], dt, d * e, "sa wo")
        a.sa_P_cap = int(sa["P_cap"])
        a.sa_kcache = _dev(sa["kcache"], dt, B * ekv_s * a.sa_P_cap, "sa kcache")
        a.sa_vcache = _dev(sa["vcache"], dt, B * ekv_s * a.sa_P_cap, "sa vcache")
        a.sa_k_draft = _dev(sa["k_draft"], dt, B * ekv_s * M, "sa k_draft")
        a.sa_v_draft = _dev(sa["v_draft"], dt, B * ekv_s * M, "sa v_draft")
        a.sa_out = _dev(sa["out"], dt, B * M * d, "sa out")
        keep = keep + [ssh]
    tensors = [sa, folded, lsa_w_packed, parent, mask, depth, lsa_hs, lsa_w, lsa_out, tok_off, ca_w, ca_k, ca_v, ca_len, ca_xq, ca_out, v_x, v_w,
               v_kcache, v_vcache, v_out, v_ktree, v_vtree, prefix_len, tok, tgt, path, n_path, bonus, ws, dev_status]
    return StepPlan(a, shape, keep, tensors)


class StepPlan:
    """Pre-marshalled moa_step_args_t.  run() only fills in the stream and calls the library."""

    def __init__(self, args, shape, arrays, tensors):
        self._args, self._shape, self._arrays, self._tensors = args, shape, arrays, tensors
        self._ref = C.byref(args)

    def run(self, stream=None):
        s = torch.cuda.current_stream() if stream is None else stream
        self._args.stream = s.cuda_stream
        rc = _lib.moa_draft_step(self._ref)
        if rc != 0:
            raise MoaError(rc, last_error())


def draft_step(shape: Shape, *, stream=None, **kw):
    """One pass of the whole path (see draft_step_plan for the arguments)."""
    draft_step_plan(shape, **kw).run(stream)



def profile_kernel_id(name: str) -> int:
    """Id of a kernel name as printed by profile_collect (template variants included)."""
    if name in _kernel_ids:
        return _kernel_ids[name]
    raise KeyError(name)


_kernel_ids: dict = {}


def profile_enable(on: bool, only_kernel: str | None = None, every: int = 1):
    """Events around every `every`-th launch (of `only_kernel` only, when given)."""
    _check(_lib.moa_profile_sample_every(every))
    _check(_lib.moa_profile_enable(1 if on else 0, -1 if only_kernel is None else profile_kernel_id(only_kernel)))


ATTN_KERNEL = {"auto": 0, "whole": 1, "split": 2}


def debug_force_attn_kernel(form: str = "auto"):
    """Force one of the two matrix-core forms of the attention core for every later call ("auto" restores the
    choice by shape); a testing aid."""
    _check(_lib.moa_debug_force_attn_kernel(ATTN_KERNEL[form]))


LSA_KERNEL = {"auto": 0, "fused": 1, "separate": 2}


def debug_force_lsa_kernel(form: str = "auto"):
    """Force the three-kernel form of the Layer Self-Attention ("separate") or restore the choice by shape; a testing aid."""
    _check(_lib.moa_debug_force_lsa_kernel(LSA_KERNEL[form]))


def probe_read(buf, scratch4, stream=None):
    """One plain streaming read of the whole tensor (a measurement probe)."""
    _check(_lib.moa_probe_read(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                               C.c_void_p(scratch4.data_ptr()), _stream(stream)))


def probe_mfma(iters: int, scratch4, stream=None) -> int:
    """Register-resident bf16 MFMA loop (a measurement probe); returns the flops it executes."""
    fl = _i64(0)
    _check(_lib.moa_probe_mfma(iters, C.c_void_p(scratch4.data_ptr()), C.byref(fl), _stream(stream)))
    return fl.value


def profile_collect():
    """[(site name, kernel name, launches, total_ms)] since the last collect; waits for the events."""
    rows = (_ProfileRow * 64)()
    n = _i32(0)
    _check(_lib.moa_profile_collect(rows, 64, C.byref(n)))
    out = []
    for r in rows[: n.value]:
        kname = _lib.moa_profile_kernel_name(r.kernel).decode()
        _kernel_ids[kname] = int(r.kernel)
        out.append((_lib.moa_profile_site_name(r.site).decode(), kname, int(r.launches), float(r.total_ms)))
    return out
