"""ctypes front end of the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, the smoke check and the
benchmark's cpu_baseline leg; the product package never imports it.  Inputs are
host numpy arrays (bf16 tensors as uint16 bit patterns); results are fp64 / int32
numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPECV_ORACLE_LIB: another build of oracle.c to load instead (the sanitizer build, in its test)
_LIB_PATH = os.environ.get("SPECV_ORACLE_LIB") or os.path.join(_HERE, "liboracle.so")
_lib = None

BF16, F32 = 0, 1
FUSE_ARGMAX, FUSE_MIXTURE = 0, 1
Q_LOGITS, Q_PROBS = 0, 1
TIE_EPS = 1e-6


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (plain C, OpenMP)."""
    src = os.path.join(_HERE, "oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-fopenmp", "-std=c11", "-fno-fast-math",
                               "-shared", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib.oracle_set_threads.restype = None
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _logits(a: np.ndarray):
    if a.dtype == np.uint16:
        return np.ascontiguousarray(a), BF16
    if a.dtype == np.float32:
        return np.ascontiguousarray(a), F32
    raise TypeError(f"logits must be uint16 (bf16 bits) or float32, got {a.dtype}")


def verify_attn(q, k_pool, v_pool, block_table, ctx_len, q_offsets, parent=None, scale=None,
                want_lse=True):
    """q [total_q,Hq,D], pools [pages,Hkv,page,D] (uint16 bf16 bits).  Returns (out f64, lse f64)."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_pool = np.ascontiguousarray(k_pool, dtype=np.uint16)
    v_pool = np.ascontiguousarray(v_pool, dtype=np.uint16)
    total_q, Hq, D = q.shape
    _, Hkv, page, D2 = k_pool.shape
    assert D2 == D and v_pool.shape == k_pool.shape
    block_table = _i32(block_table)
    B, max_pages = block_table.shape
    ctx_len, q_offsets = _i32(ctx_len), _i32(q_offsets)
    assert q_offsets.shape[0] == B + 1 and q_offsets[-1] == total_q
    par = None if parent is None else _i32(parent)
    scale = (1.0 / np.sqrt(D)) if scale is None else float(scale)
    out = np.zeros((total_q, Hq, D), dtype=np.float64)
    lse = np.zeros((total_q, Hq), dtype=np.float64) if want_lse else None
    rc = lib().oracle_verify_attn(
        ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(page),
        ctypes.c_int(max_pages), _p(q), _p(k_pool), _p(v_pool), _p(block_table), _p(ctx_len),
        _p(q_offsets), _p(par), ctypes.c_double(scale), _p(out), _p(lse))
    if rc != 0:
        raise RuntimeError(f"oracle_verify_attn failed: {rc}")
    return out, lse


def fuse_drafts(k_len, conf, draft_tokens, draft_logits=None, temperature=1.0, mode=FUSE_ARGMAX):
    """conf/draft_tokens [B,k_max,N].  Returns dict(fused_token, winner, q_row[, fused_probs])."""
    conf = np.ascontiguousarray(conf, dtype=np.float32)
    draft_tokens = _i32(draft_tokens)
    B, k_max, N = conf.shape
    k_len = _i32(k_len)
    ldt, V, dl = BF16, 0, None
    if draft_logits is not None:
        dl, ldt = _logits(draft_logits)
        V = dl.shape[1]
        assert dl.shape[0] == B * k_max * N
    fused = np.zeros((B, k_max), dtype=np.int32)
    winner = np.zeros((B, k_max), dtype=np.int32)
    q_row = np.zeros((B, k_max), dtype=np.int32)
    probs = np.zeros((B * k_max, V), dtype=np.float64) if mode == FUSE_MIXTURE else None
    rc = lib().oracle_fuse_drafts(
        ctypes.c_int(B), ctypes.c_int(k_max), ctypes.c_int(N), ctypes.c_int(V), _p(k_len), _p(conf),
        _p(draft_tokens), _p(dl), ctypes.c_int(ldt), ctypes.c_double(temperature), ctypes.c_int(mode),
        _p(fused), _p(winner), _p(q_row), _p(probs))
    if rc != 0:
        raise RuntimeError(f"oracle_fuse_drafts failed: {rc}")
    res = dict(fused_token=fused, winner=winner, q_row=q_row)
    if probs is not None:
        res["fused_probs"] = probs
    return res


def accept(node_offsets, parent, draft_tokens, target_logits, draft_q, q_row, u_accept, u_resample,
           temperature=1.0, qkind=Q_LOGITS, out_stride=None, tie_eps=TIE_EPS):
    """Returns dict(accept_len [B], out_tokens [B,out_stride] (-1 padded), stop_node [B],
    ratio [total] (NaN where not visited), near_tie [B])."""
    node_offsets = _i32(node_offsets)
    B = node_offsets.shape[0] - 1
    total = int(node_offsets[-1])
    par = None if parent is None else _i32(parent)
    draft_tokens, q_row = _i32(draft_tokens), _i32(q_row)
    tl, tdt = _logits(target_logits)
    dq, qdt = _logits(draft_q)
    V = tl.shape[1]
    assert tl.shape[0] == total + B and dq.shape[1] == V
    assert draft_tokens.shape[0] == total and q_row.shape[0] == total
    if total:
        assert 0 <= int(q_row.min()) and int(q_row.max()) < dq.shape[0]
        assert 0 <= int(draft_tokens.min()) and int(draft_tokens.max()) < V
    u_accept = np.ascontiguousarray(u_accept, dtype=np.float32)
    u_resample = np.ascontiguousarray(u_resample, dtype=np.float32)
    n = np.diff(node_offsets)
    if out_stride is None:
        out_stride = int(n.max()) + 1 if B else 1
    accept_len = np.zeros(B, dtype=np.int32)
    out_tokens = np.full((B, out_stride), -1, dtype=np.int32)
    stop = np.zeros(B, dtype=np.int32)
    ratio = np.zeros(total, dtype=np.float64)
    tie = np.zeros(B, dtype=np.int32)
    rc = lib().oracle_accept(
        ctypes.c_int(B), ctypes.c_int(V), _p(node_offsets), _p(par), _p(draft_tokens), _p(tl),
        ctypes.c_int(tdt), _p(dq), ctypes.c_int(qdt), ctypes.c_int(qkind), _p(q_row),
        ctypes.c_double(temperature), _p(u_accept), _p(u_resample), _p(accept_len), _p(out_tokens),
        ctypes.c_int(out_stride), _p(stop), _p(ratio), _p(tie), ctypes.c_double(tie_eps))
    if rc != 0:
        raise RuntimeError(f"oracle_accept failed: {rc}")
    return dict(accept_len=accept_len, out_tokens=out_tokens, stop_node=stop, ratio=ratio, near_tie=tie)


def accept_greedy(node_offsets, parent, draft_tokens, target_logits, out_stride=None):
    """Greedy verification.  Returns dict(accept_len [B], out_tokens [B,out_stride] (-1 padded),
    stop_node [B], row_argmax [total + B])."""
    node_offsets = _i32(node_offsets)
    B = node_offsets.shape[0] - 1
    total = int(node_offsets[-1])
    par = None if parent is None else _i32(parent)
    draft_tokens = _i32(draft_tokens)
    tl, tdt = _logits(target_logits)
    V = tl.shape[1]
    assert tl.shape[0] == total + B and draft_tokens.shape[0] == total
    n = np.diff(node_offsets)
    if out_stride is None:
        out_stride = int(n.max()) + 1 if B else 1
    accept_len = np.zeros(B, dtype=np.int32)
    out_tokens = np.full((B, out_stride), -1, dtype=np.int32)
    stop = np.zeros(B, dtype=np.int32)
    arg = np.zeros(total + B, dtype=np.int32)
    rc = lib().oracle_accept_greedy(
        ctypes.c_int(B), ctypes.c_int(V), _p(node_offsets), _p(par), _p(draft_tokens), _p(tl),
        ctypes.c_int(tdt), _p(accept_len), _p(out_tokens), ctypes.c_int(out_stride), _p(stop), _p(arg))
    if rc != 0:
        raise RuntimeError(f"oracle_accept_greedy failed: {rc}")
    return dict(accept_len=accept_len, out_tokens=out_tokens, stop_node=stop, row_argmax=arg)


def routing_scores(k_len, conf, draft_tokens, accept_len, out_tokens, embedding):
    """Routing-score update (Eq. 1-2).  conf, draft_tokens [B, k_max, N]; out_tokens [B, stride];
    embedding [V, E] (bf16 bits or fp32).  Returns scores [B, N] fp64."""
    conf = np.ascontiguousarray(conf, dtype=np.float32)
    B, k_max, N = conf.shape
    draft_tokens = _i32(draft_tokens).reshape(B, k_max, N)
    k_len, accept_len = _i32(k_len), _i32(accept_len)
    out_tokens = _i32(out_tokens)
    emb, edt = _logits(embedding)
    V, E = emb.shape
    assert out_tokens.shape[0] == B
    scores = np.zeros((B, N), dtype=np.float64)
    rc = lib().oracle_routing_scores(
        ctypes.c_int(B), ctypes.c_int(k_max), ctypes.c_int(N), ctypes.c_int(V), ctypes.c_int(E), _p(k_len),
        _p(conf), _p(draft_tokens), _p(accept_len), _p(out_tokens), ctypes.c_int(out_tokens.shape[1]), _p(emb),
        ctypes.c_int(edt), _p(scores))
    if rc != 0:
        raise RuntimeError(f"oracle_routing_scores failed: {rc}")
    return scores


def adaptive_speculation(gamma, gamma_max_total, in_batch=None):
    """Algorithm 2's AdaptiveSpeculation.  Returns (gamma_out [R] int32, total over the batch)."""
    gamma = _i32(gamma)
    mask = None if in_batch is None else _i32(in_batch)
    out = np.zeros_like(gamma)
    fn = lib().oracle_adaptive_speculation
    fn.restype = ctypes.c_longlong
    total = fn(ctypes.c_int(gamma.shape[0]), _p(gamma), _p(mask), ctypes.c_longlong(int(gamma_max_total)), _p(out))
    return out, int(total)


def compact_kv(k_pool, v_pool, block_table, ctx_len, q_offsets, parent, stop_node, page_size=16):
    """Accepted-path compaction.  Pools [num_pages, Hkv, page, D] uint16 are modified IN PLACE.
    Returns new_len [B] = ctx_len + depth of the accepted path."""
    assert k_pool.dtype == np.uint16 and v_pool.dtype == np.uint16 and k_pool.flags["C_CONTIGUOUS"] and v_pool.flags["C_CONTIGUOUS"]
    _, Hkv, page, D = k_pool.shape
    assert page == page_size
    block_table, ctx_len, q_offsets, stop_node = _i32(block_table), _i32(ctx_len), _i32(q_offsets), _i32(stop_node)
    par = None if parent is None else _i32(parent)
    B = ctx_len.shape[0]
    new_len = np.zeros(B, dtype=np.int32)
    rc = lib().oracle_compact_kv(ctypes.c_int(B), ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(page),
                                 ctypes.c_int(block_table.shape[1]), _p(k_pool), _p(v_pool), _p(block_table),
                                 _p(ctx_len), _p(q_offsets), _p(par), _p(stop_node), _p(new_len))
    if rc != 0:
        raise RuntimeError(f"oracle_compact_kv failed: {rc}")
    return new_len


def lm_head(hidden, weight, temperature=1.0, want_exact=False):
    """LM-head projection with row statistics.  hidden [rows, d] and weight [V, d] as bf16 bit
    patterns (uint16).  Returns dict(logits uint16 [rows, V], row_max [rows], row_z [rows],
    exact fp64 [rows, V] when asked for)."""
    hidden = np.ascontiguousarray(hidden, dtype=np.uint16)
    weight = np.ascontiguousarray(weight, dtype=np.uint16)
    rows, d = hidden.shape
    V, d2 = weight.shape
    assert d == d2
    logits = np.zeros((rows, V), dtype=np.uint16)
    exact = np.zeros((rows, V), dtype=np.float64) if want_exact else None
    row_max = np.zeros(rows, dtype=np.float64)
    row_z = np.zeros(rows, dtype=np.float64)
    rc = lib().oracle_lm_head(ctypes.c_int(rows), ctypes.c_int(d), ctypes.c_int(V), _p(hidden), _p(weight),
                              ctypes.c_double(temperature), _p(logits), _p(exact), _p(row_max), _p(row_z))
    if rc != 0:
        raise RuntimeError(f"oracle_lm_head failed: {rc}")
    out = dict(logits=logits, row_max=row_max, row_z=row_z)
    if want_exact:
        out["exact"] = exact
    return out
