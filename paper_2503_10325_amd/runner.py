"""Device-side staging of a verification batch: uploads host inputs (numpy, bf16 as
uint16 bits) into torch device tensors, owns outputs and workspaces, and calls the
C-ABI entry points through ``binding``.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as sv
from . import workloads as W


def bf16_to_device(bits: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def bf16_to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def _i32(a, device):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


class DeviceAttn:
    """One verify-attention problem resident on the GPU."""

    def __init__(self, a: W.AttnInputs, device="cuda", out_dtype=torch.bfloat16, want_lse=True,
                 kv_hint=None):
        cfg, st = a.cfg, a.st
        self.cfg, self.st = cfg, st
        self.q = bf16_to_device(a.q, device)
        self.k_pool = bf16_to_device(a.k_pool, device)
        self.v_pool = bf16_to_device(a.v_pool, device)
        self.block_table = _i32(a.block_table, device)
        self.ctx_len = _i32(st.ctx_len, device)
        self.q_offsets = _i32(st.node_offsets, device)
        self.parent = None if st.parent is None else _i32(st.parent, device)
        total_q = st.total
        self.out = torch.zeros((total_q, cfg.n_q_heads, cfg.head_dim), dtype=out_dtype, device=device)
        self.lse = torch.zeros((total_q, cfg.n_q_heads), dtype=torch.float32, device=device) if want_lse else None
        hint = int((st.ctx_len.astype(np.int64) + st.n).sum()) if kv_hint is None else int(kv_hint)
        self.desc = sv.make_attn_desc(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, total_q,
                                      int(st.n.max()) if cfg.batch else 0, a.max_pages, hint, 0.0,
                                      sv.SPEC_BF16 if out_dtype == torch.bfloat16 else sv.SPEC_F32)
        ws = sv.spec_verify_attn_workspace_size(self.desc)
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)

    def run(self, stream=None):
        sv.spec_verify_attn(self.desc, self.q, self.k_pool, self.v_pool, self.block_table, self.ctx_len,
                            self.q_offsets, self.parent, self.out, self.lse, self.workspace, stream)
        return self.out


class DeviceFuse:
    def __init__(self, f: W.FusionInputs, V: int, temperature=1.0, mode=sv.SPEC_FUSE_ARGMAX, device="cuda",
                 draft_logits_dev=None):
        B, k_max, N = f.conf.shape
        self.B, self.k_max, self.N, self.V = B, k_max, N, V
        self.mode, self.temperature = mode, temperature
        self.k_len = _i32(f.k_len, device)
        self.conf = torch.from_numpy(np.ascontiguousarray(f.conf, dtype=np.float32)).to(device)
        self.draft_tokens = _i32(f.draft_tokens, device)
        self.draft_logits = draft_logits_dev if draft_logits_dev is not None else (
            bf16_to_device(f.draft_logits, device) if f.draft_logits.dtype == np.uint16
            else torch.from_numpy(f.draft_logits).to(device))
        self.fused_token = torch.zeros((B, k_max), dtype=torch.int32, device=device)
        self.winner = torch.zeros((B, k_max), dtype=torch.int32, device=device)
        self.q_row = torch.zeros((B, k_max), dtype=torch.int32, device=device)
        self.fused_probs = (torch.zeros((B * k_max, V), dtype=torch.float32, device=device)
                            if mode == sv.SPEC_FUSE_MIXTURE else None)
        ws = sv.spec_fuse_drafts_workspace_size(B, k_max, N, V, mode)
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)

    def run(self, stream=None):
        sv.spec_fuse_drafts(self.k_len, self.conf, self.draft_tokens, self.draft_logits, self.temperature,
                            self.mode, self.fused_token, self.winner, self.q_row, self.fused_probs,
                            self.workspace, stream, V=self.V)


class DeviceAccept:
    """One acceptance problem resident on the GPU.  ``draft_tokens``/``q_row`` may be device
    tensors produced by a preceding fusion call (flattened views) instead of host arrays."""

    def __init__(self, st: W.DraftStructure, target_logits, draft_q, q_row, draft_tokens, u_accept, u_resample,
                 temperature=1.0, q_kind=sv.SPEC_Q_LOGITS, device="cuda", want_debug=True):
        self.B = int(st.n.shape[0])
        self.total = st.total
        self.max_nodes = int(st.n.max()) if self.B else 0
        self.temperature, self.q_kind = temperature, q_kind
        self.node_offsets = _i32(st.node_offsets, device)
        self.parent = None if st.parent is None else _i32(st.parent, device)

        def logits_dev(x):
            if isinstance(x, torch.Tensor):
                return x
            return bf16_to_device(x, device) if x.dtype == np.uint16 else torch.from_numpy(np.ascontiguousarray(x)).to(device)

        self.target = logits_dev(target_logits)
        self.draft_q = logits_dev(draft_q)
        self.q_row = q_row if isinstance(q_row, torch.Tensor) else _i32(q_row, device)
        self.draft_tokens = draft_tokens if isinstance(draft_tokens, torch.Tensor) else _i32(draft_tokens, device)
        self.u_accept = torch.from_numpy(np.ascontiguousarray(u_accept, dtype=np.float32)).to(device)
        self.u_resample = torch.from_numpy(np.ascontiguousarray(u_resample, dtype=np.float32)).to(device)
        self.accept_len = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.out_tokens = torch.zeros((self.B, self.max_nodes + 1), dtype=torch.int32, device=device)
        self.stop_node = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.dbg_ratio = torch.zeros(max(self.total, 1), dtype=torch.float32, device=device) if want_debug else None
        self.V = self.target.shape[1]
        ws = sv.spec_accept_workspace_size(self.B, self.total, self.draft_q.shape[0], self.V)
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)

    def run(self, stream=None, tuning=None):
        if tuning is not None:
            sv.spec_accept_tuned(tuning, self.B, self.total, self.max_nodes, self.node_offsets, self.parent,
                                 self.draft_tokens, self.target, self.draft_q, self.q_kind, self.q_row,
                                 self.temperature, self.u_accept, self.u_resample, self.accept_len, self.out_tokens,
                                 self.stop_node, self.dbg_ratio, self.workspace, stream)
            return
        sv.spec_accept(self.B, self.total, self.max_nodes, self.node_offsets, self.parent, self.draft_tokens,
                       self.target, self.draft_q, self.q_kind, self.q_row, self.temperature, self.u_accept,
                       self.u_resample, self.accept_len, self.out_tokens, self.stop_node, self.dbg_ratio,
                       self.workspace, stream)

    def run_prestats(self, stream=None):
        """The workspace already starts with the target rows' statistics (DeviceLmHead wrote them)."""
        sv.spec_accept_prestats(self.B, self.total, self.max_nodes, self.node_offsets, self.parent,
                                self.draft_tokens, self.target, self.draft_q, self.q_kind, self.q_row,
                                self.temperature, self.u_accept, self.u_resample, self.accept_len, self.out_tokens,
                                self.stop_node, self.dbg_ratio, self.workspace, stream)

    def results(self):
        torch.cuda.synchronize()
        return dict(accept_len=self.accept_len.cpu().numpy(), out_tokens=self.out_tokens.cpu().numpy(),
                    stop_node=self.stop_node.cpu().numpy(),
                    ratio=None if self.dbg_ratio is None else self.dbg_ratio.cpu().numpy()[:self.total])


class DeviceLmHead:
    """LM-head inputs resident on the GPU, the logits it produces and the statistics buffer
    (its own, or the head of an acceptance workspace handed in as ``stats``)."""

    def __init__(self, li: W.LmHeadInputs, temperature=1.0, stats=None, device="cuda"):
        self.hidden = bf16_to_device(li.hidden, device)
        self.weight = bf16_to_device(li.weight, device)
        self.rows, self.d_model = li.hidden.shape
        self.V = li.weight.shape[0]
        self.temperature = temperature
        self.logits = torch.empty((self.rows, self.V), dtype=torch.bfloat16, device=device)
        n = max(sv.spec_row_stats_size(self.rows, self.V), 16)
        self.stats = torch.zeros(n, dtype=torch.uint8, device=device) if stats is None else stats
        self.workspace = torch.empty(max(sv.spec_lm_head_workspace_size(self.rows, self.d_model, self.V), 256), dtype=torch.uint8,
                                     device=device)

    def run(self, stream=None):
        sv.spec_lm_head(self.hidden, self.weight, self.temperature, self.logits, self.stats, self.workspace, stream)

    def logits_bits(self):
        torch.cuda.synchronize()
        return self.logits.view(torch.int16).cpu().numpy().view(np.uint16)

    def segment_stats(self):
        """(m [rows, nseg] float32, z [rows, nseg] float64) as the acceptance walk reads them."""
        torch.cuda.synchronize()
        nseg = (self.V + 8191) // 8192
        raw = self.stats[: self.rows * nseg * 16].cpu().numpy()
        rec = raw.view(np.dtype([("m", "<f4"), ("pad", "<f4"), ("z", "<f8")])).reshape(self.rows, nseg)
        return rec["m"].copy(), rec["z"].copy()


class DeviceGreedy:
    """Device copies of the greedy-verification inputs of one batch, its outputs and workspace."""

    def __init__(self, st: W.DraftStructure, target_logits, draft_tokens, device="cuda"):
        self.B = int(st.n.shape[0])
        self.total = st.total
        self.max_nodes = int(st.n.max()) if self.B else 0
        self.node_offsets = _i32(st.node_offsets, device)
        self.parent = None if st.parent is None else _i32(st.parent, device)
        if isinstance(target_logits, torch.Tensor):
            self.target = target_logits
        elif target_logits.dtype == np.uint16:
            self.target = bf16_to_device(target_logits, device)
        else:
            self.target = torch.from_numpy(np.ascontiguousarray(target_logits)).to(device)
        self.draft_tokens = draft_tokens if isinstance(draft_tokens, torch.Tensor) else _i32(draft_tokens, device)
        self.accept_len = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.out_tokens = torch.zeros((self.B, self.max_nodes + 1), dtype=torch.int32, device=device)
        self.stop_node = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.row_argmax = torch.zeros(self.total + self.B, dtype=torch.int32, device=device)
        self.V = self.target.shape[1]
        ws = sv.spec_accept_greedy_workspace_size(self.B, self.total, self.V)
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=device)

    def run(self, stream=None):
        sv.spec_accept_greedy(self.B, self.total, self.max_nodes, self.node_offsets, self.parent, self.draft_tokens,
                              self.target, self.accept_len, self.out_tokens, self.stop_node, self.row_argmax,
                              self.workspace, stream)

    def results(self):
        torch.cuda.synchronize()
        return dict(accept_len=self.accept_len.cpu().numpy(), out_tokens=self.out_tokens.cpu().numpy(),
                    stop_node=self.stop_node.cpu().numpy(), row_argmax=self.row_argmax.cpu().numpy())
