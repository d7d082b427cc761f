"""Seeded synthetic inputs for the Mixture-of-Attentions draft step.

This module holds NONE of the method's arithmetic: it only draws random tensors,
trees and tokens with the shapes and value distributions of the workloads, so the
CPU oracle and the GPU library can be fed the same realised values.

Recipe (stand-in for the paper's Llama3-8B-Instruct / SpecBench workloads, Sec. 4
"Experiments": trees of at most 62 verified tokens, depth 6):
  * RNG  : numpy Generator(PCG64(20241003 + 1000*config_index + stream)); streams
           0 prefix lengths, 1 trees, 2 weights, 3 LSA inputs, 4 CA queries,
           5 verify inputs, 6 KV caches, 7 tokens.
  * weights ~ N(0, 1/in_features); activations ~ N(0,1), RMS-normalised per row for
    the Llama-shaped configs; KV caches ~ N(0,1).
  * bf16 configs: every tensor is rounded to bf16 (round-to-nearest-even) once, here,
    and both sides consume the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 20241003
S_PREFIX, S_TREE, S_WEIGHT, S_LSA, S_CAQ, S_VERIFY, S_CACHE, S_TOKEN = range(8)
VOCAB = 128256


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    dtype: str          # "f32" | "bf16"
    B: int
    P_min: int          # prefix lengths drawn uniformly in [P_min, P_max]
    P_max: int
    M: int              # tree nodes, root included
    D: int              # maximum node depth
    max_branch: int
    L: int
    d: int
    H: int
    Hkv: int
    dh: int
    d_lsa_in: int       # LSA input width (K||V of one layer = 2*Hkv*dh in the paper)
    rms_norm: bool

    @property
    def E_kv(self):
        return self.Hkv * self.dh

    @property
    def lsa_heads(self):
        return self.d_lsa_in // self.dh

    @property
    def d_lsa(self):
        return self.lsa_heads * self.dh

    @property
    def P_cap(self):
        return self.P_max + self.M


CONFIGS = {
    "C0": Config("C0", 0, "f32", 1, 64, 64, 8, 4, 4, 4, 256, 4, 2, 64, 256, False),
    "C1": Config("C1", 1, "bf16", 1, 1024, 1024, 60, 6, 4, 32, 4096, 32, 8, 128, 2048, True),
    "C2": Config("C2", 2, "bf16", 16, 512, 2048, 64, 8, 4, 32, 4096, 32, 8, 128, 2048, True),
    "C3": Config("C3", 3, "bf16", 4, 4096, 4096, 60, 6, 4, 80, 8192, 64, 8, 128, 2048, True),
    "C4": Config("C4", 4, "bf16", 8, 32768, 32768, 128, 10, 4, 32, 4096, 32, 8, 128, 2048, True),
}


def scaled(cfg: Config, **kw) -> Config:
    """A variant of a config (smaller batch / prefix / width) that keeps its seeds."""
    return replace(cfg, **kw)


def rng_for(cfg: Config, stream: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg.index + stream + 100000 * extra))


# ------------------------------------------------------------------ bf16 helpers

def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  No NaN inputs expected."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64/fp32 values to the storage dtype and return them as fp32 (exact)."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(x32)).reshape(x32.shape)
    raise ValueError(dtype)


# ------------------------------------------------------------------ tensors

def normal(rng, shape, dtype, scale=1.0, rms_norm=False):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    if rms_norm:
        ms = np.mean(np.square(x, dtype=np.float32), axis=-1, keepdims=True)
        x = x / np.sqrt(ms + np.float32(1e-5))
    return quantize(x, dtype)


def weight(rng, out_f, in_f, dtype):
    return normal(rng, (out_f, in_f), dtype, scale=1.0 / np.sqrt(in_f))


def prefix_lengths(cfg: Config) -> np.ndarray:
    rng = rng_for(cfg, S_PREFIX)
    if cfg.P_min == cfg.P_max:
        return np.full((cfg.B,), cfg.P_max, dtype=np.int32)
    return rng.integers(cfg.P_min, cfg.P_max + 1, size=cfg.B).astype(np.int32)


# ------------------------------------------------------------------ trees

def gen_tree(M: int, D: int, max_branch: int, rng) -> np.ndarray:
    """parent[M] with parent[0] = -1 and parent[i] < i; some node has depth exactly D.

    Nodes 1..D form a spine; every further node picks its parent uniformly among the
    nodes of depth < D that still have fewer than max_branch children.  Nodes are then
    relabelled in (depth, creation order) so that parents precede children."""
    if M < 1 or D < 0 or D + 1 > M:
        raise ValueError("need 1 <= D+1 <= M")
    par = [-1]
    dep = [0]
    nch = [0]
    for i in range(1, M):
        if i <= D:
            p = i - 1
        else:
            cand = [j for j in range(i) if dep[j] < D and nch[j] < max_branch]
            if not cand:
                raise ValueError("tree cannot hold M nodes under these limits")
            p = cand[int(rng.integers(0, len(cand)))]
        par.append(p)
        dep.append(dep[p] + 1)
        nch.append(0)
        nch[p] += 1
    order = sorted(range(M), key=lambda j: (dep[j], j))
    new_of = {old: new for new, old in enumerate(order)}
    out = np.empty((M,), dtype=np.int32)
    for new, old in enumerate(order):
        out[new] = -1 if par[old] < 0 else new_of[par[old]]
    return out


def chain_tree(M: int) -> np.ndarray:
    return np.arange(-1, M - 1, dtype=np.int32)


def star_tree(M: int) -> np.ndarray:
    p = np.zeros((M,), dtype=np.int32)
    p[0] = -1
    return p


def full_tree(branch: int, depth: int) -> np.ndarray:
    par = [-1]
    level = [0]
    for _ in range(depth):
        nxt = []
        for p in level:
            for _ in range(branch):
                par.append(p)
                nxt.append(len(par) - 1)
        level = nxt
    return np.asarray(par, dtype=np.int32)


def beam_tree(breadth: int, depth: int, m: int, rng) -> np.ndarray:
    """Topology of an EAGLE-2 style tree (Sec. 2.2): `breadth` children of the root, then
    per level the `breadth` kept branches each offer `breadth` children; of the
    breadth + (depth-1)*breadth^2 candidates, m-1 survive (closed under ancestors) plus
    the root.  Scores are random; only the shape matters here."""
    par = [-1]
    score = [0.0]
    frontier = []
    for _ in range(breadth):
        par.append(0)
        score.append(float(np.log(rng.random())))
        frontier.append(len(par) - 1)
    for _ in range(depth - 1):
        cand = []
        for p in frontier:
            for _ in range(breadth):
                par.append(p)
                score.append(score[p] + float(np.log(rng.random())))
                cand.append(len(par) - 1)
        cand.sort(key=lambda j: -score[j])
        frontier = cand[:breadth]
    n = len(par)
    ranked = sorted(range(1, n), key=lambda j: -score[j])      # joint scores decrease along a path
    keep = {0}
    for j in ranked:
        if len(keep) >= m:
            break
        keep.add(j)                                            # its ancestors rank higher: already kept
    old = sorted(keep)
    new_of = {o: i for i, o in enumerate(old)}
    assert all(par[o] < 0 or par[o] in new_of for o in old)
    return np.asarray([-1 if par[o] < 0 else new_of[par[o]] for o in old], dtype=np.int32)


def trees(cfg: Config) -> np.ndarray:
    rng = rng_for(cfg, S_TREE)
    return np.stack([gen_tree(cfg.M, cfg.D, cfg.max_branch, rng) for _ in range(cfg.B)])


def tokens(cfg: Config, parent: np.ndarray, p_follow: float = 0.8):
    """tok[b,i]: drafted token of node i (siblings distinct); tgt[b,i]: the LLM's greedy token
    after node i -- a child's token with probability p_follow, otherwise a random one."""
    rng = rng_for(cfg, S_TOKEN)
    B, M = parent.shape
    tok = np.empty((B, M), dtype=np.int32)
    tgt = np.empty((B, M), dtype=np.int32)
    for b in range(B):
        kids = [[] for _ in range(M)]
        for i in range(1, M):
            kids[parent[b, i]].append(i)
        tok[b, 0] = rng.integers(0, VOCAB)
        for i in range(M):
            if kids[i]:
                tok[b, kids[i]] = rng.choice(VOCAB, size=len(kids[i]), replace=False)
        for i in range(M):
            if kids[i] and rng.random() < p_follow:
                tgt[b, i] = tok[b, kids[i][int(rng.integers(0, len(kids[i])))]]
            else:
                tgt[b, i] = rng.integers(0, VOCAB)
    return tok, tgt


# ------------------------------------------------------------------ whole workloads

def lsa_weights(cfg: Config):
    rng = rng_for(cfg, S_WEIGHT, extra=1)
    Hl, dh, d_in = cfg.lsa_heads, cfg.dh, cfg.d_lsa_in
    return dict(wq=weight(rng, Hl * dh, d_in, cfg.dtype), wk=weight(rng, cfg.E_kv, d_in, cfg.dtype),
                wv=weight(rng, cfg.E_kv, d_in, cfg.dtype), wo=weight(rng, cfg.d_lsa, Hl * dh, cfg.dtype))


def lsa_inputs(cfg: Config, T: int):
    return normal(rng_for(cfg, S_LSA), (T, cfg.L, cfg.d_lsa_in), cfg.dtype, rms_norm=cfg.rms_norm)


def sa_kv_heads(cfg: Config) -> int:
    """KV heads of the draft Self-Attention layer: its key/value width is half of the LLM's E_kv
    (appendix table: 512 against 1024 at the 8B shape), at the LLM's head_dim."""
    return max(1, cfg.Hkv // 2)


def sa_weights(cfg: Config, variant: int = 0):
    """Self-Attention layer on draft-token embeddings: embedding d, H query heads, sa_kv_heads KV heads."""
    rng = rng_for(cfg, S_WEIGHT, extra=2 + 50 * variant)
    E, ekv = cfg.H * cfg.dh, sa_kv_heads(cfg) * cfg.dh
    return dict(wq=weight(rng, E, cfg.d, cfg.dtype), wk=weight(rng, ekv, cfg.d, cfg.dtype),
                wv=weight(rng, ekv, cfg.d, cfg.dtype), wo=weight(rng, cfg.d, E, cfg.dtype))


def sa_inputs(cfg: Config, variant: int = 0):
    """Token embeddings of the M tree nodes [B, M, d] and the layer's K/V cache of the verified tokens
    [B, sa_kv_heads, P_cap, dh] (N(0,1), like the other caches)."""
    emb = normal(rng_for(cfg, S_CAQ, extra=7 + 50 * variant), (cfg.B, cfg.M, cfg.d), cfg.dtype, rms_norm=cfg.rms_norm)
    rc = rng_for(cfg, S_CACHE, extra=2000 + 50 * variant)
    shape = (cfg.B, sa_kv_heads(cfg), cfg.P_cap, cfg.dh)
    return emb, normal(rc, shape, cfg.dtype), normal(rc, shape, cfg.dtype)


def tli_d_ff(cfg: Config) -> int:
    """MLP width of the LLM's decoder layer: 3.5 d (14336 at the Llama-3-8B shape)."""
    return 7 * cfg.d // 2


def tli_weights(cfg: Config, layer: int = 0):
    """One reused LLM decoder layer: norm gains near 1, attention and gated-MLP weights ~ N(0, 1/in_features)."""
    rng = rng_for(cfg, S_WEIGHT, extra=500 + layer)
    E, ekv, d, dff = cfg.H * cfg.dh, cfg.E_kv, cfg.d, tli_d_ff(cfg)
    gain = lambda: quantize(1.0 + 0.1 * rng.standard_normal(d), cfg.dtype)
    return dict(g_attn=gain(), wq=weight(rng, E, d, cfg.dtype), wk=weight(rng, ekv, d, cfg.dtype),
                wv=weight(rng, ekv, d, cfg.dtype), wo=weight(rng, d, E, cfg.dtype), g_mlp=gain(),
                w_gate=weight(rng, dff, d, cfg.dtype), w_up=weight(rng, dff, d, cfg.dtype),
                w_down=weight(rng, d, dff, cfg.dtype))


def drafter_mlp_sizes(cfg: Config):
    """(stream width, MLP projection size) of the MLPs behind the drafter's three attention layers, in the proportions
    of the appendix architecture table: 6144 after LSA (width 2048), 512 after SA and 7168 after CA (width 4096)."""
    return dict(lsa=(cfg.d_lsa, 3 * cfg.d_lsa), sa=(cfg.d, max(32, cfg.d // 8)), ca=(cfg.d, 7 * cfg.d // 4))


def drafter_mlp_weights(cfg: Config, which: str):
    """Pre-norm gain (near 1) and gated-MLP weights ~ N(0, 1/in_features) of one of the drafter's MLP sub-blocks."""
    d, dff = drafter_mlp_sizes(cfg)[which]
    rng = rng_for(cfg, S_WEIGHT, extra=700 + {"lsa": 0, "sa": 1, "ca": 2}[which])
    return dict(g=quantize(1.0 + 0.1 * rng.standard_normal(d), cfg.dtype), w_gate=weight(rng, dff, d, cfg.dtype),
                w_up=weight(rng, dff, d, cfg.dtype), w_down=weight(rng, d, dff, cfg.dtype))


def drafter_norm_gain(cfg: Config, which: str):
    """Gain of the pre-norm in front of the drafter's SA / CA sub-layer."""
    rng = rng_for(cfg, S_WEIGHT, extra=720 + {"sa": 1, "ca": 2}[which])
    return quantize(1.0 + 0.1 * rng.standard_normal(cfg.d), cfg.dtype)


def ca_weights(cfg: Config):
    rng = rng_for(cfg, S_WEIGHT, extra=2)
    E = cfg.H * cfg.dh
    return dict(wq=weight(rng, E, cfg.d, cfg.dtype), wo=weight(rng, cfg.d, E, cfg.dtype),
                wk=weight(rng, cfg.E_kv, cfg.d_lsa, cfg.dtype), wv=weight(rng, cfg.E_kv, cfg.d_lsa, cfg.dtype))


def ca_queries(cfg: Config, Mq: int):
    return normal(rng_for(cfg, S_CAQ), (cfg.B, Mq, cfg.d), cfg.dtype, rms_norm=cfg.rms_norm)


def verify_weights(cfg: Config, layer: int = 0):
    rng = rng_for(cfg, S_WEIGHT, extra=3 + layer)
    E = cfg.H * cfg.dh
    return dict(wq=weight(rng, E, cfg.d, cfg.dtype), wk=weight(rng, cfg.E_kv, cfg.d, cfg.dtype),
                wv=weight(rng, cfg.E_kv, cfg.d, cfg.dtype), wo=weight(rng, cfg.d, E, cfg.dtype))


def verify_inputs(cfg: Config, layer: int = 0):
    return normal(rng_for(cfg, S_VERIFY, extra=layer), (cfg.B, cfg.M, cfg.d), cfg.dtype, rms_norm=cfg.rms_norm)


def kv_cache(cfg: Config, which: int = 0, P_cap: int | None = None):
    """One K and one V cache [B, Hkv, P_cap, dh] ~ N(0,1).  `which` selects independent draws
    (0 = LLM layer 0, 1 = layer 1, ...; 1000 = stand-alone CA cache)."""
    rng = rng_for(cfg, S_CACHE, extra=which)
    P_cap = cfg.P_cap if P_cap is None else P_cap
    shape = (cfg.B, cfg.Hkv, P_cap, cfg.dh)
    return normal(rng, shape, cfg.dtype), normal(rng, shape, cfg.dtype)


def step_workload(cfg: Config, n_verify_layers: int = 1, variant: int = 0, lsa_tokens="tree", with_sa: bool = False):
    """All inputs of one draft step as numpy arrays (values already rounded to cfg.dtype).

    `lsa_tokens` says how many tokens per sequence are new to the Layer Self-Attention in this step:
    "tree" = M (every token of the last tree, the default), "prefix" = P_b (first cycle: the whole prompt,
    empty memory before), or an integer A (the accepted tokens of the last cycle).  LSA runs on their sum T;
    the cross-attention memory holds P_b minus that many rows before the step and P_b rows after the append.
    `variant` draws an independent set of the large tensors (weights, activations, caches) so a
    benchmark can rotate buffer sets; trees, tokens and lengths stay the same.
    `with_sa` adds the drafter's Self-Attention layer in front of the cross-attention (key "sa": its weights, the
    tree nodes' token embeddings and its K/V cache of the verified tokens); the layer's output then replaces `ca_xq`."""
    v = 50 * variant
    B, M = cfg.B, cfg.M
    parent = trees(cfg)
    tok, tgt = tokens(cfg, parent)
    plen = prefix_lengths(cfg)
    if isinstance(lsa_tokens, str):
        if lsa_tokens not in ("tree", "prefix"):
            raise ValueError(f"lsa_tokens: {lsa_tokens!r}")
        new_tok = np.full(B, M, dtype=np.int64) if lsa_tokens == "tree" else plen.astype(np.int64)
    else:
        new_tok = np.full(B, int(lsa_tokens), dtype=np.int64)
    if np.any(new_tok < 1) or np.any(plen < new_tok):
        raise ValueError("prefix shorter than the tokens that are new to it")
    T = int(new_tok.sum())
    rng_w = rng_for(cfg, S_WEIGHT, extra=1 + v)
    Hl, dh, d_in = cfg.lsa_heads, cfg.dh, cfg.d_lsa_in
    E = cfg.H * dh
    lsa_w = dict(wq=weight(rng_w, Hl * dh, d_in, cfg.dtype), wk=weight(rng_w, cfg.E_kv, d_in, cfg.dtype),
                 wv=weight(rng_w, cfg.E_kv, d_in, cfg.dtype), wo=weight(rng_w, cfg.d_lsa, Hl * dh, cfg.dtype))
    ca_w = dict(wq=weight(rng_w, E, cfg.d, cfg.dtype), wo=weight(rng_w, cfg.d, E, cfg.dtype),
                wk=weight(rng_w, cfg.E_kv, cfg.d_lsa, cfg.dtype), wv=weight(rng_w, cfg.E_kv, cfg.d_lsa, cfg.dtype))
    lsa_hs = normal(rng_for(cfg, S_LSA, extra=v), (T, cfg.L, d_in), cfg.dtype, rms_norm=cfg.rms_norm)
    ca_xq = normal(rng_for(cfg, S_CAQ, extra=v), (B, M, cfg.d), cfg.dtype, rms_norm=cfg.rms_norm)
    ca_P_cap = cfg.P_max + 8
    rng_c = rng_for(cfg, S_CACHE, extra=1000 + v)
    ca_k = normal(rng_c, (B, cfg.Hkv, ca_P_cap, dh), cfg.dtype)
    ca_v = normal(rng_c, (B, cfg.Hkv, ca_P_cap, dh), cfg.dtype)
    layers = []
    for l in range(n_verify_layers):
        rl = rng_for(cfg, S_WEIGHT, extra=3 + l + v)
        w = dict(wq=weight(rl, E, cfg.d, cfg.dtype), wk=weight(rl, cfg.E_kv, cfg.d, cfg.dtype),
                 wv=weight(rl, cfg.E_kv, cfg.d, cfg.dtype), wo=weight(rl, cfg.d, E, cfg.dtype))
        x = normal(rng_for(cfg, S_VERIFY, extra=l + v), (B, M, cfg.d), cfg.dtype, rms_norm=cfg.rms_norm)
        rc = rng_for(cfg, S_CACHE, extra=l + v)
        kc = normal(rc, (B, cfg.Hkv, cfg.P_cap, dh), cfg.dtype)
        vc = normal(rc, (B, cfg.Hkv, cfg.P_cap, dh), cfg.dtype)
        layers.append(dict(w=w, x=x, kcache=kc, vcache=vc))
    sa = None
    if with_sa:
        emb, sk, sv = sa_inputs(cfg, variant)
        sa = dict(w=sa_weights(cfg, variant), emb=emb, kcache=sk, vcache=sv)
    return dict(cfg=cfg, sa=sa, parent=parent, tok=tok, tgt=tgt, prefix_len=plen, P_cap=cfg.P_cap,
                lsa_w=lsa_w, lsa_hs=lsa_hs, tok_off=np.concatenate([[0], np.cumsum(new_tok)]).astype(np.int32),
                ca_w=ca_w, ca_xq=ca_xq, ca_k=ca_k, ca_v=ca_v, ca_len0=(plen - new_tok).astype(np.int32),
                ca_P_cap=ca_P_cap, layers=layers)
