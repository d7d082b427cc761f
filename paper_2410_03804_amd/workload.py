"""Device-side buffers for one draft step and the call that runs it through the C ABI.

Only marshalling: numpy inputs (from the seeded generators) become torch CUDA tensors, outputs are
allocated, and `run` hands everything to moa_draft_step.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as moa

_TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
_MDT = {"f32": moa.F32, "bf16": moa.BF16}


def shape_of(cfg) -> moa.Shape:
    return moa.Shape(cfg.L, cfg.d, cfg.H, cfg.Hkv, cfg.dh, cfg.d_lsa_in, cfg.lsa_heads, cfg.Hkv, _MDT[cfg.dtype])


def _dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(_TDT[dtype])
    return t.cuda()


class DeviceStep:
    """All tensors of one step on the GPU.  `n_len_slots` independent copies of the (tiny) cross-attention
    length array let a benchmark run that many steps back to back without resetting anything."""

    def __init__(self, work, n_len_slots: int = 1, ws: torch.Tensor | None = None, fold: bool = True, pack: bool = True):
        cfg = work["cfg"]
        dt = cfg.dtype
        self.cfg, self.shape = cfg, shape_of(cfg)
        B, M = cfg.B, cfg.M
        T = int(work["lsa_hs"].shape[0])
        W = (M + 63) // 64
        tdt = _TDT[dt]
        self.parent, self.tok, self.tgt = _dev(work["parent"]), _dev(work["tok"]), _dev(work["tgt"])
        self.prefix_len, self.tok_off = _dev(work["prefix_len"]), _dev(work["tok_off"])
        self.P_cap, self.ca_P_cap = int(work["P_cap"]), int(work["ca_P_cap"])
        self.mask = torch.zeros((B, M, W), dtype=torch.int64, device="cuda")
        self.depth = torch.zeros((B, M), dtype=torch.int32, device="cuda")
        self.lsa_w = {k: _dev(v, dt) for k, v in work["lsa_w"].items()}
        self.lsa_hs = _dev(work["lsa_hs"], dt)
        self.lsa_out = torch.zeros((T, cfg.d_lsa), dtype=tdt, device="cuda")
        self.ca_w = {k: _dev(v, dt) for k, v in work["ca_w"].items()}
        # one-time fold of the two projections between LSA's heads and the memory's keys / values
        self.folded = (moa.fold_projection(self.ca_w["wk"], self.lsa_w["wo"]),
                       moa.fold_projection(self.ca_w["wv"], self.lsa_w["wo"])) if fold else None
        # one-time rearrangement of the LSA's Wq / Wk / Wv into MFMA-operand order, for shapes that have one
        self.lsa_w_packed = None
        if pack:
            try:
                self.lsa_w_packed = moa.lsa_pack_weights(self.shape, self.lsa_w["wq"], self.lsa_w["wk"], self.lsa_w["wv"])
            except moa.MoaError as e:
                if e.status != -2:              # MOA_ERR_SHAPE: no packed form for this shape; anything else is a failure
                    raise
        self.ca_xq = _dev(work["ca_xq"], dt)
        self.ca_k, self.ca_v = _dev(work["ca_k"], dt), _dev(work["ca_v"], dt)
        self.ca_len0 = _dev(work["ca_len0"])
        self.ca_len = [self.ca_len0.clone() for _ in range(n_len_slots)]
        self.ca_out = torch.zeros((B, M, cfg.d), dtype=tdt, device="cuda")
        self.v_w = [{k: _dev(v, dt) for k, v in lay["w"].items()} for lay in work["layers"]]
        self.v_x = [_dev(lay["x"], dt) for lay in work["layers"]]
        self.v_kcache = [_dev(lay["kcache"], dt) for lay in work["layers"]]
        self.v_vcache = [_dev(lay["vcache"], dt) for lay in work["layers"]]
        n = len(work["layers"])
        self.v_out = [torch.zeros((B, M, cfg.d), dtype=tdt, device="cuda") for _ in range(n)]
        self.v_ktree = [torch.zeros((B, cfg.Hkv, M, cfg.dh), dtype=tdt, device="cuda") for _ in range(n)]
        self.v_vtree = [torch.zeros((B, cfg.Hkv, M, cfg.dh), dtype=tdt, device="cuda") for _ in range(n)]
        self.path = torch.zeros((B, M), dtype=torch.int32, device="cuda")
        self.n_path = torch.zeros((B,), dtype=torch.int32, device="cuda")
        self.bonus = torch.zeros((B,), dtype=torch.int32, device="cuda")
        self.dev_status = torch.zeros((1,), dtype=torch.int32, device="cuda")
        self.sa = None
        if work.get("sa") is not None:            # the Self-Attention layer in front of the cross-attention
            sa = work["sa"]
            hkv_s = sa["w"]["wk"].shape[0] // cfg.dh
            self.sa = dict(shape=moa.Shape(cfg.L, cfg.d, cfg.H, hkv_s, cfg.dh, cfg.d_lsa_in, cfg.lsa_heads, cfg.Hkv, _MDT[dt]),
                           emb=_dev(sa["emb"], dt), w={k: _dev(v, dt) for k, v in sa["w"].items()},
                           kcache=_dev(sa["kcache"], dt), vcache=_dev(sa["vcache"], dt), P_cap=int(sa["kcache"].shape[2]),
                           k_draft=torch.zeros((B, hkv_s, M, cfg.dh), dtype=tdt, device="cuda"),
                           v_draft=torch.zeros((B, hkv_s, M, cfg.dh), dtype=tdt, device="cuda"),
                           out=torch.zeros((B, M, cfg.d), dtype=tdt, device="cuda"))
        if ws is None:
            nbytes = moa.workspace_bytes(self.shape, B, max(self.P_cap, self.ca_P_cap), M, T)
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        self.ws = ws
        self._plans = {}

    def plan(self, len_slot: int = 0, schedule: int = 0):
        key = (len_slot, schedule)
        if key not in self._plans:
            self._plans[key] = moa.draft_step_plan(
                self.shape, parent=self.parent, mask=self.mask, depth=self.depth, lsa_hs=self.lsa_hs, lsa_w=self.lsa_w,
                lsa_out=self.lsa_out, tok_off=self.tok_off, ca_w=self.ca_w, ca_k=self.ca_k, ca_v=self.ca_v,
                ca_len=self.ca_len[len_slot], ca_P_cap=self.ca_P_cap, ca_xq=self.ca_xq, ca_out=self.ca_out, v_x=self.v_x,
                v_w=self.v_w, v_kcache=self.v_kcache, v_vcache=self.v_vcache, v_out=self.v_out, v_ktree=self.v_ktree,
                v_vtree=self.v_vtree, prefix_len=self.prefix_len, P_cap=self.P_cap, tok=self.tok, tgt=self.tgt,
                path=self.path, n_path=self.n_path, bonus=self.bonus, ws=self.ws, dev_status=self.dev_status,
                schedule=schedule, sa=self.sa, folded=self.folded, lsa_w_packed=self.lsa_w_packed)
        return self._plans[key]

    def run(self, len_slot: int = 0, stream=None, schedule: int = 0):
        self.plan(len_slot, schedule).run(stream)
