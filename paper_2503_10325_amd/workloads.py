"""Seeded synthetic inputs for the parallel-verification path.

This module only *draws* inputs: shapes, lengths, trees, logits, uniforms and the
drafters' sampled tokens.  It holds none of the verification method's arithmetic
(no attention, no softmax, no accept test, no fusion) so that the CPU oracle and
the HIP path can both be fed from it without sharing any computation.

Everything is numpy on the host.  bf16 tensors are carried as ``uint16`` bit
patterns (numpy has no bf16); fp32 -> bf16 uses round-to-nearest-even.

The five workloads follow the verification-step shapes of the synthetic
benchmark configurations (a Llama-2-7B-shaped linear draft, a Llama-3-8B-shaped
draft tree, a multi-drafter fusion batch, a Llama-70B-shaped ragged serving
batch, plus a tiny case).  They stand in for the prompts and model weights of the
paper's evaluation (Section 6.1), which the path's cost does not depend on.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Optional, Sequence, Tuple

import numpy as np

PAGE_SIZE = 16


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (format handling only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# configuration table
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    """Shape/distribution recipe of one verification batch.

    ctx:    ("fixed", L) | ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi)
    draft:  ("linear", k) | ("linear_uniform", lo, hi) | ("tree", branching, node_cap)
    q_src:  ("independent", sd)       draft logits ~ N(0, sd) independent of target
            ("noise", sd)             draft logits = target row + N(0, sd)
            ("fusion", N, sd_own)     N drafters, logits = shared target row + N(0, sd_own)_n
    """
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx: Tuple
    draft: Tuple
    vocab: int
    target_sd: float
    q_src: Tuple
    temperature: float = 1.0
    page_size: int = PAGE_SIZE

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def d_model(self) -> int:
        """Width of the hidden state the LM head contracts over (heads x head_dim in the Llama family)."""
        return self.n_q_heads * self.head_dim


CONFIGS = {
    "c0_tiny": VerifyConfig("c0_tiny", 1, 8, 8, 64, ("fixed", 256), ("linear", 4),
                            1000, 2.0, ("independent", 2.0)),
    "c1_llama2_7b": VerifyConfig("c1_llama2_7b", 8, 32, 32, 128, ("fixed", 2048), ("linear", 8),
                                 32000, 3.0, ("noise", 1.0)),
    "c2_tree_llama3_8b": VerifyConfig("c2_tree_llama3_8b", 16, 32, 8, 128, ("fixed", 4096),
                                      ("tree", (4, 4, 2, 2), 64), 128256, 3.0, ("noise", 1.0)),
    "c3_fusion": VerifyConfig("c3_fusion", 32, 32, 32, 128, ("uniform", 1024, 4096), ("linear", 6),
                              32000, 3.0, ("fusion", 4, 1.5)),
    "c4_llama70b_serving": VerifyConfig("c4_llama70b_serving", 64, 64, 8, 128,
                                        ("lognormal", 2048, 0.8, 512, 16384),
                                        ("linear_uniform", 2, 10), 128256, 3.0, ("noise", 1.0)),
}
# Secondary data point: c2 with the full 4,4,2,2 tree (4 + 16 + 32 + 64 = 116 nodes) instead of its first 64 nodes.
CONFIGS["c2b_tree116_llama3_8b"] = dataclasses.replace(CONFIGS["c2_tree_llama3_8b"], name="c2b_tree116_llama3_8b",
                                                       draft=("tree", (4, 4, 2, 2), 116))
CONFIG_ORDER = ["c0_tiny", "c1_llama2_7b", "c2_tree_llama3_8b", "c3_fusion", "c4_llama70b_serving"]
SECONDARY = ["c2b_tree116_llama3_8b"]


def scaled(cfg: VerifyConfig, **overrides) -> VerifyConfig:
    """A copy of ``cfg`` with some fields replaced (used for reduced test sizes)."""
    return dataclasses.replace(cfg, **overrides)


def _rng(seed: int, cfg_name: str, tensor: str) -> np.random.Generator:
    """Independent sub-stream per (master seed, config, tensor name)."""
    key = [seed & 0xFFFFFFFF, zlib.crc32(cfg_name.encode()), zlib.crc32(tensor.encode())]
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(key)))


# --------------------------------------------------------------------------
# draft structure
# --------------------------------------------------------------------------
def tree_parents(branching: Sequence[int], node_cap: int) -> np.ndarray:
    """Parent array of the full tree with the given per-depth branching, numbered
    breadth-first and truncated to ``node_cap`` nodes.  -1 = child of the committed
    prefix.  parent[i] < i for every node."""
    parents = []
    frontier = [-1]
    for br in branching:
        nxt = []
        for p in frontier:
            for _ in range(br):
                if len(parents) >= node_cap:
                    break
                parents.append(p)
                nxt.append(len(parents) - 1)
        frontier = nxt
    return np.asarray(parents, dtype=np.int32)


@dataclasses.dataclass
class DraftStructure:
    n: np.ndarray               # [B] nodes per request
    node_offsets: np.ndarray    # [B+1] int32
    parent: Optional[np.ndarray]  # [total] int32 local parent index, or None for linear drafts
    ctx_len: np.ndarray         # [B] int32

    @property
    def total(self) -> int:
        return int(self.node_offsets[-1])

    def local_parent(self, b: int) -> np.ndarray:
        nb = int(self.n[b])
        if self.parent is None:
            return np.arange(-1, nb - 1, dtype=np.int32)
        o = int(self.node_offsets[b])
        return self.parent[o:o + nb]


def make_structure(cfg: VerifyConfig, seed: int = 0) -> DraftStructure:
    B = cfg.batch
    r = _rng(seed, cfg.name, "structure")
    kind = cfg.ctx[0]
    if kind == "fixed":
        ctx = np.full(B, cfg.ctx[1], dtype=np.int64)
    elif kind == "uniform":
        ctx = r.integers(cfg.ctx[1], cfg.ctx[2] + 1, size=B)
    elif kind == "lognormal":
        _, med, sig, lo, hi = cfg.ctx
        ctx = np.clip(np.rint(np.exp(np.log(med) + sig * r.standard_normal(B))), lo, hi).astype(np.int64)
    else:
        raise ValueError(kind)
    dk = cfg.draft[0]
    parent = None
    if dk == "linear":
        n = np.full(B, cfg.draft[1], dtype=np.int64)
    elif dk == "linear_uniform":
        n = r.integers(cfg.draft[1], cfg.draft[2] + 1, size=B)
    elif dk == "tree":
        p = tree_parents(cfg.draft[1], cfg.draft[2])
        n = np.full(B, len(p), dtype=np.int64)
        parent = np.tile(p, B).astype(np.int32)
    else:
        raise ValueError(dk)
    off = np.zeros(B + 1, dtype=np.int32)
    off[1:] = np.cumsum(n)
    return DraftStructure(n.astype(np.int32), off, parent, ctx.astype(np.int32))


# --------------------------------------------------------------------------
# attention inputs
# --------------------------------------------------------------------------
@dataclasses.dataclass
class AttnInputs:
    cfg: VerifyConfig
    st: DraftStructure
    q: np.ndarray            # [total_q, Hq, D] bf16 bits
    k_pool: np.ndarray       # [num_pages, Hkv, page, D] bf16 bits
    v_pool: np.ndarray       # [num_pages, Hkv, page, D] bf16 bits
    block_table: np.ndarray  # [B, max_pages] int32 (unused entries = -1)
    max_pages: int
    num_pages: int


def _normal_bf16(r: np.random.Generator, shape, sd: float = 1.0, chunk: int = 1 << 24) -> np.ndarray:
    """N(0, sd) rounded to bf16 bits, generated in chunks to bound host memory."""
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.uint16)
    for s in range(0, total, chunk):
        e = min(total, s + chunk)
        x = r.standard_normal(e - s, dtype=np.float32)
        if sd != 1.0:
            x *= np.float32(sd)
        out[s:e] = f32_to_bf16_bits(x)
    return out.reshape(shape)


def make_attn_inputs(cfg: VerifyConfig, seed: int = 0, st: Optional[DraftStructure] = None,
                     spare_pages: int = 3) -> AttnInputs:
    """Q/K/V ~ N(0,1) in bf16.  The KV cache of request b holds ctx_len[b] committed
    tokens followed by its n[b] draft tokens (draft j at logical position ctx_len[b]+j);
    logical pages are mapped to pool pages by one random permutation of the pool."""
    st = st or make_structure(cfg, seed)
    B, P = cfg.batch, cfg.page_size
    pages_per_req = (st.ctx_len.astype(np.int64) + st.n + P - 1) // P
    max_pages = int(pages_per_req.max())
    num_pages = int(pages_per_req.sum()) + spare_pages
    perm = _rng(seed, cfg.name, "page_perm").permutation(num_pages).astype(np.int32)
    bt = np.full((B, max_pages), -1, dtype=np.int32)
    o = 0
    for b in range(B):
        c = int(pages_per_req[b])
        bt[b, :c] = perm[o:o + c]
        o += c
    q = _normal_bf16(_rng(seed, cfg.name, "q"), (st.total, cfg.n_q_heads, cfg.head_dim))
    kp = _normal_bf16(_rng(seed, cfg.name, "k_pool"), (num_pages, cfg.n_kv_heads, P, cfg.head_dim))
    vp = _normal_bf16(_rng(seed, cfg.name, "v_pool"), (num_pages, cfg.n_kv_heads, P, cfg.head_dim))
    return AttnInputs(cfg, st, q, kp, vp, bt, max_pages, num_pages)


# --------------------------------------------------------------------------
# acceptance / fusion inputs
# --------------------------------------------------------------------------
@dataclasses.dataclass
class FusionInputs:
    n_drafters: int
    k_max: int
    k_len: np.ndarray        # [B] int32
    conf: np.ndarray         # [B, k_max, N] float32 in [0,1]
    draft_tokens: np.ndarray  # [B, k_max, N] int32
    draft_logits: np.ndarray  # [B*k_max*N, V] bf16 bits


@dataclasses.dataclass
class AcceptInputs:
    cfg: VerifyConfig
    st: DraftStructure
    target_logits: np.ndarray  # [total_nodes + B, V] bf16 bits; request b owns rows node_offsets[b]+b ...
    draft_q: np.ndarray        # [n_q_rows, V] bf16 bits (logits)
    q_row: Optional[np.ndarray]      # [total_nodes] int32 (None when it is to come from fusion)
    draft_tokens: Optional[np.ndarray]  # [total_nodes] int32 (None when it is to come from fusion)
    u_accept: np.ndarray       # [total_nodes] float32 in [0,1), multiples of 2^-24
    u_resample: np.ndarray     # [B] float32 in [0,1)
    fusion: Optional[FusionInputs] = None


def uniforms24(r: np.random.Generator, n: int) -> np.ndarray:
    """fp32 uniforms in [0,1) that are exact multiples of 2^-24."""
    return (r.integers(0, 1 << 24, size=n, dtype=np.int64).astype(np.float32)
            * np.float32(2.0 ** -24))


def _gumbel_argmax(r: np.random.Generator, logits_bits_row: np.ndarray, inv_t: float, draws: int) -> np.ndarray:
    """``draws`` i.i.d. samples from the categorical law with the given logits, by the
    Gumbel-max construction (argmax of logit/T + Gumbel noise), in fp64."""
    z = bf16_bits_to_f32(logits_bits_row).astype(np.float64) * inv_t
    out = np.empty(draws, dtype=np.int32)
    for d in range(draws):
        u = r.random(z.shape[0])
        g = -np.log(-np.log(np.maximum(u, 1e-300)))
        out[d] = int(np.argmax(z + g))
    return out


def make_accept_inputs(cfg: VerifyConfig, seed: int = 0, st: Optional[DraftStructure] = None,
                       draft_equals_target: bool = False, target_logits: Optional[np.ndarray] = None) -> AcceptInputs:
    """Target logits ~ N(0, target_sd) per row; draft rows per ``cfg.q_src``; draft
    tokens are samples of the very draft rows handed to the acceptance step (siblings
    of a tree are i.i.d. draws from their parent's row and share ``q_row``)."""
    st = st or make_structure(cfg, seed)
    B, V = cfg.batch, cfg.vocab
    total = st.total
    inv_t = 1.0 / cfg.temperature
    if target_logits is None:
        tgt = _normal_bf16(_rng(seed, cfg.name, "target_logits"), (total + B, V), cfg.target_sd)
    else:                                   # rows given by the caller (bf16 bits), e.g. an LM-head product
        tgt = np.ascontiguousarray(target_logits, dtype=np.uint16)
        assert tgt.shape == (total + B, V)
    r_tok = _rng(seed, cfg.name, "draft_tokens")
    r_noise = _rng(seed, cfg.name, "draft_noise")
    u_acc = uniforms24(_rng(seed, cfg.name, "u_accept"), total)
    u_res = uniforms24(_rng(seed, cfg.name, "u_resample"), B)

    def noisy(row_bits: np.ndarray, sd: float) -> np.ndarray:
        x = bf16_bits_to_f32(row_bits) + np.float32(sd) * r_noise.standard_normal(V, dtype=np.float32)
        return f32_to_bf16_bits(x)

    if cfg.q_src[0] == "fusion":
        N, sd_own = int(cfg.q_src[1]), float(cfg.q_src[2])
        assert st.parent is None, "fusion workloads use linear drafts"
        k_max = int(st.n.max())
        dl = np.zeros((B * k_max * N, V), dtype=np.uint16)
        toks = np.zeros((B, k_max, N), dtype=np.int32)
        for b in range(B):
            base = int(st.node_offsets[b]) + b
            for i in range(int(st.n[b])):
                for n in range(N):
                    row = (b * k_max + i) * N + n
                    dl[row] = tgt[base + i] if draft_equals_target else noisy(tgt[base + i], sd_own)
                    toks[b, i, n] = _gumbel_argmax(r_tok, dl[row], inv_t, 1)[0]
        conf = _rng(seed, cfg.name, "conf").beta(2.0, 2.0, size=(B, k_max, N)).astype(np.float32)
        fus = FusionInputs(N, k_max, st.n.astype(np.int32), conf, toks, dl)
        return AcceptInputs(cfg, st, tgt, dl, None, None, u_acc, u_res, fus)

    rows = []
    q_row = np.zeros(total, dtype=np.int32)
    toks = np.zeros(total, dtype=np.int32)
    for b in range(B):
        o = int(st.node_offsets[b])
        base = o + b
        par = st.local_parent(b)
        order = []            # distinct parents in order of first appearance
        kids = {}
        for j, p in enumerate(par):
            p = int(p)
            if p not in kids:
                kids[p] = []
                order.append(p)
            kids[p].append(j)
        for p in order:
            trow = tgt[base + 1 + p]      # p = -1 -> local row 0 (after the committed prefix)
            if draft_equals_target:
                qbits = trow.copy()
            elif cfg.q_src[0] == "noise":
                qbits = noisy(trow, float(cfg.q_src[1]))
            elif cfg.q_src[0] == "independent":
                qbits = f32_to_bf16_bits(np.float32(cfg.q_src[1]) * r_noise.standard_normal(V, dtype=np.float32))
            else:
                raise ValueError(cfg.q_src)
            ridx = len(rows)
            rows.append(qbits)
            draws = _gumbel_argmax(r_tok, qbits, inv_t, len(kids[p]))
            for c, x in zip(kids[p], draws):
                q_row[o + c] = ridx
                toks[o + c] = x
    dq = np.stack(rows) if rows else np.zeros((0, V), dtype=np.uint16)
    return AcceptInputs(cfg, st, tgt, dq, q_row, toks, u_acc, u_res, None)


@dataclasses.dataclass
class RoutingInputs:
    """Inputs of the routing-score update: what the drafters proposed, what was accepted, and the
    target model's token-embedding table (synthetic stand-in, N(0,1) rounded to bf16)."""
    k_len: np.ndarray          # [B] int32
    conf: np.ndarray           # [B, k_max, N] float32
    draft_tokens: np.ndarray   # [B, k_max, N] int32
    accept_len: np.ndarray     # [B] int32
    out_tokens: np.ndarray     # [B, k_max + 1] int32
    embedding: np.ndarray      # [V, E] bf16 bits


def make_routing_inputs(batch: int, k_max: int, n_drafters: int, vocab: int, emb_dim: int, seed: int = 0,
                        name: str = "routing", agree: float = 0.5) -> RoutingInputs:
    """Seeded synthetic case: ragged draft lengths, acceptance lengths anywhere in 0..k, accepted
    tokens that a drafter's own token matches with probability `agree`."""
    r = _rng(seed, name, "routing")
    k_len = r.integers(1, k_max + 1, size=batch).astype(np.int32) if k_max > 0 else np.zeros(batch, np.int32)
    accept_len = (r.integers(0, k_max + 1, size=batch) % (k_len + 1)).astype(np.int32)
    conf = r.beta(2.0, 2.0, size=(batch, k_max, n_drafters)).astype(np.float32)
    out_tokens = r.integers(0, vocab, size=(batch, k_max + 1)).astype(np.int32)
    draft_tokens = r.integers(0, vocab, size=(batch, k_max, n_drafters)).astype(np.int32)
    same = r.random((batch, k_max, n_drafters)) < agree
    draft_tokens = np.where(same, out_tokens[:, :k_max, None], draft_tokens).astype(np.int32)
    embedding = _normal_bf16(_rng(seed, name, "embedding"), (vocab, emb_dim))
    return RoutingInputs(k_len, conf, draft_tokens, accept_len, out_tokens, embedding)


@dataclasses.dataclass
class LmHeadInputs:
    hidden: np.ndarray         # [rows, d_model] bf16 bits: final hidden states of the verified positions
    weight: np.ndarray         # [vocab, d_model] bf16 bits: one row per vocabulary entry


def make_lm_head_inputs(rows: int, d_model: int, vocab: int, seed: int = 0, logit_sd: float = 3.0) -> LmHeadInputs:
    """Hidden states ~ N(0, 1) and weights ~ N(0, logit_sd / sqrt(d_model)): the logits then have the
    spread (standard deviation logit_sd) of the acceptance workloads' target rows."""
    name = f"lm_head_{rows}x{d_model}x{vocab}"
    hidden = _normal_bf16(_rng(seed, name, "hidden"), (rows, d_model))
    weight = _normal_bf16(_rng(seed, name, "weight"), (vocab, d_model), logit_sd / float(np.sqrt(d_model)))
    return LmHeadInputs(hidden, weight)


def attention_bytes_flops(cfg: VerifyConfig, st: DraftStructure) -> Tuple[int, int]:
    """Bytes the attention step must move (K and V of every cached position once per KV
    head, Q in, bf16 O out) and its floating-point operation count (QK^T and PV)."""
    n = st.n.astype(np.int64)
    L = st.ctx_len.astype(np.int64) + n
    D = cfg.head_dim
    by = int((2 * cfg.n_kv_heads * L * D * 2 + 2 * n * cfg.n_q_heads * D * 2).sum())
    fl = int((4 * n * cfg.n_q_heads * L * D).sum())
    return by, fl


def accept_bytes_all_rows(cfg: VerifyConfig, ai: AcceptInputs, bytes_per_logit: int = 2) -> int:
    """Bytes one data-parallel pass over every target row and every draft row moves."""
    return int((ai.target_logits.shape[0] + ai.draft_q.shape[0]) * cfg.vocab * bytes_per_logit)
