"""Thin ctypes binding of libspecverify.so (include/spec_verify.h).

Argument marshalling only: every step of the verification path runs inside the
library's HIP kernels.  PyTorch is used for device memory and the current stream.
There is no CPU fallback; importing works without the library, calling does not.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecverify.so")

SPEC_OK = 0
SPEC_BF16, SPEC_F32 = 0, 1
SPEC_FUSE_ARGMAX, SPEC_FUSE_MIXTURE = 0, 1
SPEC_Q_LOGITS, SPEC_Q_PROBS = 0, 1

EXPORTS = [
    "spec_verify_attn_workspace_size", "spec_verify_attn",
    "spec_fuse_drafts_workspace_size", "spec_fuse_drafts",
    "spec_accept_workspace_size", "spec_accept", "spec_accept_tuned",
    "spec_describe_attn_plan", "spec_describe_accept_plan",
    "spec_accept_noalloc", "spec_accept_noalloc_max_workspace",
    "spec_accept_greedy_workspace_size", "spec_accept_greedy",
    "spec_routing_scores", "spec_adaptive_speculation", "spec_compact_kv",
    "spec_row_stats_size", "spec_lm_head_workspace_size", "spec_lm_head", "spec_accept_prestats",
    "spec_strerror", "spec_abi_version",
]


class SpecAttnDesc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32), ("total_q", ctypes.c_int32),
        ("max_q_per_req", ctypes.c_int32), ("max_pages_per_req", ctypes.c_int32),
        ("total_kv_tokens_hint", ctypes.c_int64), ("scale", ctypes.c_float), ("out_dtype", ctypes.c_int32),
    ]


class SpecAcceptTuning(ctypes.Structure):
    """Explicit launch choices of spec_accept_tuned (0 / negative = the library's choice)."""
    _fields_ = [("path", ctypes.c_int32), ("levels", ctypes.c_int32), ("slices", ctypes.c_int32),
                ("patience", ctypes.c_int32), ("helpers", ctypes.c_int32)]

    def __init__(self, path=0, levels=0, slices=0, patience=-1, helpers=-1):
        super().__init__(path, levels, slices, patience, helpers)


class SpecError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {status} ({strerror(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        L.spec_strerror.restype = ctypes.c_char_p
        L.spec_strerror.argtypes = [i32]
        L.spec_abi_version.restype = i32
        L.spec_verify_attn_workspace_size.restype = sz
        L.spec_verify_attn_workspace_size.argtypes = [ctypes.POINTER(SpecAttnDesc)]
        L.spec_verify_attn.restype = i32
        L.spec_verify_attn.argtypes = [ctypes.POINTER(SpecAttnDesc)] + [vp] * 10 + [sz, vp]
        L.spec_fuse_drafts_workspace_size.restype = sz
        L.spec_fuse_drafts_workspace_size.argtypes = [i32] * 5
        L.spec_fuse_drafts.restype = i32
        L.spec_fuse_drafts.argtypes = [i32] * 4 + [vp] * 4 + [i32, f32, i32] + [vp] * 5 + [sz, vp]
        L.spec_accept_workspace_size.restype = sz
        L.spec_accept_workspace_size.argtypes = [i32] * 4
        L.spec_accept_greedy_workspace_size.restype = sz
        L.spec_accept_greedy_workspace_size.argtypes = [i32] * 3
        L.spec_accept_greedy.restype = i32
        L.spec_accept_greedy.argtypes = [i32] * 4 + [vp] * 4 + [i32, vp, vp, i32, vp, vp, vp, sz, vp]
        L.spec_routing_scores.restype = i32
        L.spec_routing_scores.argtypes = [i32] * 5 + [vp] * 5 + [i32, vp, i32, vp, vp]
        L.spec_adaptive_speculation.restype = i32
        L.spec_adaptive_speculation.argtypes = [i32, vp, vp, ctypes.c_int64, vp, vp, vp]
        L.spec_compact_kv.restype = i32
        L.spec_compact_kv.argtypes = [i32] * 5 + [vp] * 9
        L.spec_accept.restype = i32
        L.spec_accept.argtypes = ([i32] * 5 + [vp] * 4 + [i32, vp, i32, i32, vp, f32] + [vp] * 4 + [i32]
                                  + [vp] * 3 + [sz, vp])
        L.spec_accept_prestats.restype = i32
        L.spec_accept_prestats.argtypes = L.spec_accept.argtypes
        L.spec_accept_tuned.restype = i32
        L.spec_accept_tuned.argtypes = [ctypes.POINTER(SpecAcceptTuning)] + L.spec_accept.argtypes
        L.spec_accept_noalloc.restype = i32
        L.spec_accept_noalloc.argtypes = L.spec_accept.argtypes[:-3] + [vp]
        L.spec_accept_noalloc_max_workspace.restype = sz
        L.spec_accept_noalloc_max_workspace.argtypes = []
        L.spec_describe_attn_plan.restype = i32
        L.spec_describe_attn_plan.argtypes = [ctypes.POINTER(SpecAttnDesc), ctypes.c_char_p, sz]
        L.spec_describe_accept_plan.restype = i32
        L.spec_describe_accept_plan.argtypes = [ctypes.POINTER(SpecAcceptTuning)] + [i32] * 8 + [ctypes.c_char_p, sz]
        L.spec_row_stats_size.restype = sz
        L.spec_row_stats_size.argtypes = [i32, i32]
        L.spec_lm_head_workspace_size.restype = sz
        L.spec_lm_head_workspace_size.argtypes = [i32, i32, i32]
        L.spec_lm_head.restype = i32
        L.spec_lm_head.argtypes = [i32, i32, i32, vp, vp, f32, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().spec_strerror(int(status)).decode()


def _ptr(t) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return SPEC_BF16
    if t.dtype == torch.float32:
        return SPEC_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def make_attn_desc(batch, num_q_heads, num_kv_heads, head_dim, total_q, max_q_per_req, max_pages_per_req,
                   total_kv_tokens_hint=0, scale=0.0, out_dtype=SPEC_BF16, page_size=16) -> SpecAttnDesc:
    return SpecAttnDesc(batch, num_q_heads, num_kv_heads, head_dim, page_size, total_q, max_q_per_req,
                        max_pages_per_req, total_kv_tokens_hint, scale, out_dtype)


def spec_verify_attn_workspace_size(desc: SpecAttnDesc) -> int:
    return int(lib().spec_verify_attn_workspace_size(ctypes.byref(desc)))


def spec_verify_attn(desc: SpecAttnDesc, q, k_pool, v_pool, block_table, ctx_len, q_offsets, parent, out,
                     lse=None, workspace=None, stream=None) -> None:
    """Device tensors: q/k_pool/v_pool bf16, block_table/ctx_len/q_offsets/parent int32, out bf16 or
    fp32, lse fp32 or None, workspace uint8 of at least spec_verify_attn_workspace_size(desc) bytes."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_verify_attn(ctypes.byref(desc), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                _ptr(ctx_len), _ptr(q_offsets), _ptr(parent), _ptr(out), _ptr(lse),
                                _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_verify_attn", rc)


def spec_fuse_drafts_workspace_size(B, k_max, N, V, mode) -> int:
    return int(lib().spec_fuse_drafts_workspace_size(B, k_max, N, V, mode))


def spec_fuse_drafts(k_len, conf, draft_tokens, draft_logits, temperature, mode, fused_token, winner, q_row,
                     fused_probs=None, workspace=None, stream=None, V: Optional[int] = None) -> None:
    """conf/draft_tokens [B,k_max,N]; draft_logits [B*k_max*N, V] or None (ARGMAX)."""
    B, k_max, N = conf.shape
    if draft_logits is not None:
        V = draft_logits.shape[1]
        ldt = _dtype_code(draft_logits)
    else:
        V, ldt = (V or 0), SPEC_BF16
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_fuse_drafts(B, k_max, N, V, _ptr(k_len), _ptr(conf), _ptr(draft_tokens), _ptr(draft_logits),
                                ldt, float(temperature), int(mode), _ptr(fused_token), _ptr(winner), _ptr(q_row),
                                _ptr(fused_probs), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_fuse_drafts", rc)


def spec_accept_workspace_size(B, total_nodes, n_q_rows, V) -> int:
    return int(lib().spec_accept_workspace_size(B, total_nodes, n_q_rows, V))


def spec_accept(B, total_nodes, max_nodes_per_req, node_offsets, parent, draft_tokens, target_logits, draft_q,
                q_kind, q_row, temperature, u_accept, u_resample, accept_len, out_tokens, stop_node=None,
                dbg_ratio=None, workspace=None, stream=None) -> None:
    """target_logits [total_nodes+B, V], draft_q [n_q_rows, V] (bf16 or fp32 device tensors);
    out_tokens [B, out_stride] int32."""
    V = target_logits.shape[1]
    n_q_rows = 0 if draft_q is None else draft_q.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_accept(B, V, total_nodes, n_q_rows, max_nodes_per_req, _ptr(node_offsets), _ptr(parent),
                           _ptr(draft_tokens), _ptr(target_logits), _dtype_code(target_logits), _ptr(draft_q),
                           SPEC_BF16 if draft_q is None else _dtype_code(draft_q), int(q_kind), _ptr(q_row),
                           float(temperature), _ptr(u_accept), _ptr(u_resample), _ptr(accept_len),
                           _ptr(out_tokens), out_tokens.shape[1], _ptr(stop_node), _ptr(dbg_ratio),
                           _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_accept", rc)


def spec_accept_tuned(tuning, B, total_nodes, max_nodes_per_req, node_offsets, parent, draft_tokens, target_logits,
                      draft_q, q_kind, q_row, temperature, u_accept, u_resample, accept_len, out_tokens,
                      stop_node=None, dbg_ratio=None, workspace=None, stream=None) -> None:
    """spec_accept with explicit launch choices (a SpecAcceptTuning or None)."""
    V = target_logits.shape[1]
    n_q_rows = 0 if draft_q is None else draft_q.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_accept_tuned(None if tuning is None else ctypes.byref(tuning), B, V, total_nodes, n_q_rows,
                                 max_nodes_per_req, _ptr(node_offsets), _ptr(parent), _ptr(draft_tokens),
                                 _ptr(target_logits), _dtype_code(target_logits), _ptr(draft_q),
                                 SPEC_BF16 if draft_q is None else _dtype_code(draft_q), int(q_kind), _ptr(q_row),
                                 float(temperature), _ptr(u_accept), _ptr(u_resample), _ptr(accept_len),
                                 _ptr(out_tokens), out_tokens.shape[1], _ptr(stop_node), _ptr(dbg_ratio),
                                 _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_accept_tuned", rc)


def spec_accept_noalloc(B, total_nodes, max_nodes_per_req, node_offsets, parent, draft_tokens, target_logits,
                        draft_q, q_kind, q_row, temperature, u_accept, u_resample, accept_len, out_tokens,
                        stop_node=None, dbg_ratio=None, stream=None) -> None:
    """spec_accept on the library's built-in scratch array: no workspace argument, no allocation."""
    V = target_logits.shape[1]
    n_q_rows = 0 if draft_q is None else draft_q.shape[0]
    rc = lib().spec_accept_noalloc(B, V, total_nodes, n_q_rows, max_nodes_per_req, _ptr(node_offsets), _ptr(parent),
                                   _ptr(draft_tokens), _ptr(target_logits), _dtype_code(target_logits), _ptr(draft_q),
                                   SPEC_BF16 if draft_q is None else _dtype_code(draft_q), int(q_kind), _ptr(q_row),
                                   float(temperature), _ptr(u_accept), _ptr(u_resample), _ptr(accept_len),
                                   _ptr(out_tokens), out_tokens.shape[1], _ptr(stop_node), _ptr(dbg_ratio),
                                   _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_accept_noalloc", rc)


def spec_describe_attn_plan(desc: SpecAttnDesc) -> str:
    buf = ctypes.create_string_buffer(512)
    rc = lib().spec_describe_attn_plan(ctypes.byref(desc), buf, 512)
    if rc != SPEC_OK:
        raise SpecError("spec_describe_attn_plan", rc)
    return buf.value.decode()


def spec_describe_accept_plan(B, V, total_nodes, max_nodes_per_req, is_tree, target_dtype=SPEC_BF16, q_dtype=SPEC_BF16,
                              q_kind=SPEC_Q_LOGITS, tuning=None) -> str:
    buf = ctypes.create_string_buffer(512)
    rc = lib().spec_describe_accept_plan(None if tuning is None else ctypes.byref(tuning), B, V, total_nodes,
                                         max_nodes_per_req, int(bool(is_tree)), target_dtype, q_dtype, q_kind, buf, 512)
    if rc != SPEC_OK:
        raise SpecError("spec_describe_accept_plan", rc)
    return buf.value.decode()


def spec_accept_prestats(B, total_nodes, max_nodes_per_req, node_offsets, parent, draft_tokens, target_logits,
                         draft_q, q_kind, q_row, temperature, u_accept, u_resample, accept_len, out_tokens,
                         stop_node=None, dbg_ratio=None, workspace=None, stream=None) -> None:
    """spec_accept whose workspace already starts with the target rows' statistics (from spec_lm_head)."""
    V = target_logits.shape[1]
    n_q_rows = 0 if draft_q is None else draft_q.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_accept_prestats(B, V, total_nodes, n_q_rows, max_nodes_per_req, _ptr(node_offsets),
                                    _ptr(parent), _ptr(draft_tokens), _ptr(target_logits),
                                    _dtype_code(target_logits), _ptr(draft_q),
                                    SPEC_BF16 if draft_q is None else _dtype_code(draft_q), int(q_kind),
                                    _ptr(q_row), float(temperature), _ptr(u_accept), _ptr(u_resample),
                                    _ptr(accept_len), _ptr(out_tokens), out_tokens.shape[1], _ptr(stop_node),
                                    _ptr(dbg_ratio), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_accept_prestats", rc)


def spec_row_stats_size(rows, V) -> int:
    return int(lib().spec_row_stats_size(rows, V))


def spec_lm_head_workspace_size(rows, d_model, V) -> int:
    return int(lib().spec_lm_head_workspace_size(rows, d_model, V))


def spec_lm_head(hidden, weight, temperature, logits, target_stats, workspace, stream=None) -> None:
    """hidden [rows, d_model], weight [V, d_model], logits [rows, V]: bf16 device tensors; target_stats:
    device tensor of at least spec_row_stats_size(rows, V) bytes (normally the accept workspace)."""
    rows, d_model = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == d_model and tuple(logits.shape) == (rows, V)
    assert target_stats.numel() * target_stats.element_size() >= spec_row_stats_size(rows, V)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_lm_head(rows, d_model, V, _ptr(hidden), _ptr(weight), float(temperature), _ptr(logits),
                            _ptr(target_stats), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_lm_head", rc)


def spec_accept_greedy_workspace_size(B, total_nodes, V) -> int:
    return int(lib().spec_accept_greedy_workspace_size(B, total_nodes, V))


def spec_accept_greedy(B, total_nodes, max_nodes_per_req, node_offsets, parent, draft_tokens, target_logits,
                       accept_len, out_tokens, stop_node=None, row_argmax=None, workspace=None, stream=None) -> None:
    """target_logits [total_nodes+B, V] (bf16 or fp32 device tensor); out_tokens [B, out_stride] int32."""
    V = target_logits.shape[1]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().spec_accept_greedy(B, V, total_nodes, max_nodes_per_req, _ptr(node_offsets), _ptr(parent),
                                  _ptr(draft_tokens), _ptr(target_logits), _dtype_code(target_logits),
                                  _ptr(accept_len), _ptr(out_tokens), out_tokens.shape[1], _ptr(stop_node),
                                  _ptr(row_argmax), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_accept_greedy", rc)


def spec_routing_scores(k_len, conf, draft_tokens, accept_len, out_tokens, embedding, scores, stream=None) -> None:
    """conf, draft_tokens [B, k_max, N]; out_tokens [B, out_stride] int32; embedding [V, E] (bf16 or fp32);
    scores [B, N] fp32 (device tensors)."""
    B, k_max, N = conf.shape
    V, E = embedding.shape
    rc = lib().spec_routing_scores(B, k_max, N, V, E, _ptr(k_len), _ptr(conf), _ptr(draft_tokens), _ptr(accept_len),
                                   _ptr(out_tokens), out_tokens.shape[1], _ptr(embedding), _dtype_code(embedding),
                                   _ptr(scores), _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_routing_scores", rc)


def spec_adaptive_speculation(gamma_in, gamma_max_total, gamma_out, in_batch=None, total_out=None, stream=None) -> None:
    """gamma_in, gamma_out [R] int32, in_batch [R] int32 or None, total_out [1] int64 or None (device tensors)."""
    rc = lib().spec_adaptive_speculation(gamma_in.shape[0], _ptr(gamma_in), _ptr(in_batch), int(gamma_max_total),
                                         _ptr(gamma_out), _ptr(total_out), _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_adaptive_speculation", rc)


def spec_compact_kv(k_pool, v_pool, block_table, ctx_len, q_offsets, parent, stop_node, new_len=None, stream=None) -> None:
    """Pools [num_pages, Hkv, 16, D] bf16 device tensors (modified in place); the rest int32 device tensors."""
    _, Hkv, page, D = k_pool.shape
    rc = lib().spec_compact_kv(ctx_len.shape[0], Hkv, D, page, block_table.shape[1], _ptr(k_pool), _ptr(v_pool),
                               _ptr(block_table), _ptr(ctx_len), _ptr(q_offsets), _ptr(parent), _ptr(stop_node),
                               _ptr(new_len), _stream(stream))
    if rc != SPEC_OK:
        raise SpecError("spec_compact_kv", rc)
