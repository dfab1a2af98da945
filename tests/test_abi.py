"""CPU-only checks of the C-ABI library: it loads, exports every function the header
declares, and rejects bad host-visible arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2503_10325_amd import binding as sv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spec_verify.h")

pytestmark = pytest.mark.skipif(not os.path.exists(sv.LIB_PATH), reason="libspecverify.so not built")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(sv.EXPORTS)
    L = ctypes.CDLL(sv.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sv.lib().spec_abi_version() == 3
    assert sv.strerror(0) == "ok" and "workspace" in sv.strerror(-4)


def test_attn_descriptor_validation_needs_no_gpu():
    L = sv.lib()
    null = ctypes.c_void_p(0)

    def call(desc):
        return L.spec_verify_attn(ctypes.byref(desc), null, null, null, null, null, null, null, null, null,
                                  null, 0, null)

    ok = dict(batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, total_q=8, max_q_per_req=4,
              max_pages_per_req=10)
    assert call(sv.make_attn_desc(**ok)) == -1                                   # NULL tensors
    assert call(sv.make_attn_desc(**{**ok, "num_kv_heads": 3})) == -2            # Hq % Hkv
    assert call(sv.make_attn_desc(**{**ok, "head_dim": 96})) == -3
    assert call(sv.make_attn_desc(**{**ok, "page_size": 32})) == -3
    assert call(sv.make_attn_desc(**{**ok, "max_q_per_req": 129})) == -3
    assert call(sv.make_attn_desc(**{**ok, "batch": -1})) == -2
    assert call(sv.make_attn_desc(**{**ok, "batch": 0})) == 0                    # empty batch: nothing to do
    assert L.spec_verify_attn(None, null, null, null, null, null, null, null, null, null, null, 0, null) == -1
    assert sv.spec_verify_attn_workspace_size(sv.make_attn_desc(**ok)) >= 256
    assert sv.spec_verify_attn_workspace_size(sv.make_attn_desc(**{**ok, "head_dim": 96})) == 0


def test_accept_and_fuse_validation_needs_no_gpu():
    L = sv.lib()
    null = ctypes.c_void_p(0)

    def accept(B=2, V=100, total=4, nq=4, maxn=2, T=1.0, stride=3, tdt=0, qdt=0, qk=0):
        return L.spec_accept(B, V, total, nq, maxn, null, null, null, null, tdt, null, qdt, qk, null, T,
                             null, null, null, null, stride, null, null, null, 0, null)

    assert accept() == -1
    assert accept(V=0) == -2
    assert accept(T=0.0) == -2
    assert accept(maxn=129, stride=130) == -3
    assert accept(stride=2) == -2
    assert accept(tdt=7) == -3
    assert accept(qk=2) == -3
    assert accept(B=0) == 0
    assert sv.spec_accept_workspace_size(2, 4, 4, 100) > 0

    def fuse(B=2, k=3, N=4, V=100, mode=0, T=1.0):
        return L.spec_fuse_drafts(B, k, N, V, null, null, null, null, 0, T, mode, null, null, null, null,
                                  null, 0, null)

    assert fuse() == -1
    assert fuse(N=0) == -2
    assert fuse(mode=5) == -3
    assert fuse(B=0) == 0
    assert sv.spec_fuse_drafts_workspace_size(2, 3, 4, 100, 0) == 0
    assert sv.spec_fuse_drafts_workspace_size(2, 3, 4, 100, 1) > 0


def test_greedy_routing_adaptive_validation_needs_no_gpu():
    L = sv.lib()
    null = ctypes.c_void_p(0)

    def greedy(B=2, V=100, total=4, maxn=2, stride=3, tdt=0):
        return L.spec_accept_greedy(B, V, total, maxn, null, null, null, null, tdt, null, null, stride, null, null,
                                    null, 0, null)

    assert greedy() == -1                      # NULL tensors
    assert greedy(V=0) == -2
    assert greedy(maxn=129, stride=130) == -3
    assert greedy(stride=2) == -2
    assert greedy(tdt=5) == -3
    assert greedy(B=40000, total=40000) == -3  # more rows than one launch takes
    assert greedy(B=0) == 0
    assert sv.spec_accept_greedy_workspace_size(2, 4, 100) >= 256

    def routing(B=2, k=3, N=4, V=100, E=64, stride=4, edt=0):
        return L.spec_routing_scores(B, k, N, V, E, null, null, null, null, null, stride, null, edt, null, null)

    assert routing() == -1
    assert routing(E=0) == -2
    assert routing(k=65) == -3
    assert routing(N=17) == -3
    assert routing(edt=3) == -3
    assert routing(B=0) == 0

    def adaptive(R=4):
        return L.spec_adaptive_speculation(R, null, null, 10, null, null, null)

    assert adaptive() == -1
    assert adaptive(R=-1) == -2
    assert adaptive(R=0) == 0


def test_lm_head_validation_needs_no_gpu():
    L = sv.lib()
    null = ctypes.c_void_p(0)

    def lm(rows=4, d=256, V=100, T=1.0):
        return L.spec_lm_head(rows, d, V, null, null, T, null, null, null, 0, null)

    assert lm() == -1
    assert lm(d=0) == -2
    assert lm(T=0.0) == -2
    assert lm(d=200) == -3                      # contraction length must be a multiple of 128
    assert lm(rows=70000) == -3
    assert lm(rows=0) == 0
    assert sv.spec_row_stats_size(4, 8192) == 4 * 16 and sv.spec_row_stats_size(4, 8193) == 4 * 2 * 16
    assert sv.spec_lm_head_workspace_size(4, 256, 100) >= 4 * 8
    assert sv.spec_lm_head_workspace_size(200, 256, 100) >= 200 * 8 + 224 * 256 * 2      # packed hidden states
    a = L.spec_accept_prestats(2, 100, 4, 4, 2, null, null, null, null, 1, null, 0, 0, null, 1.0,
                               null, null, null, null, 3, null, null, null, 0, null)
    assert a == -3                              # statistics from the LM head describe bf16 logits


def test_tuned_accept_and_plan_descriptions_need_no_gpu():
    L = sv.lib()
    null = ctypes.c_void_p(0)

    def tuned(t, B=2, V=100, total=4, nq=4, maxn=2):
        return L.spec_accept_tuned(None if t is None else ctypes.byref(t), B, V, total, nq, maxn, null, null, null,
                                   null, 0, null, 0, 0, null, 1.0, null, null, null, null, 3, null, null, null, 0, null)

    assert tuned(None) == -1                                    # like spec_accept: NULL tensors
    assert tuned(sv.SpecAcceptTuning(path=5)) == -1             # tensors are checked first ...
    assert tuned(sv.SpecAcceptTuning(path=2), B=0) == 0         # ... and an empty batch is nothing to do
    desc = sv.make_attn_desc(batch=16, num_q_heads=32, num_kv_heads=8, head_dim=128, total_q=1024,
                             max_q_per_req=64, max_pages_per_req=260, total_kv_tokens_hint=16 * 4160)
    text = sv.spec_describe_attn_plan(desc)
    assert "attn_" in text and "chunks" in text
    assert "sliced" in text and "at most 1 per request" in text   # 128 pairs x 256 rows: two workgroups per pair, no context cut
    text = sv.spec_describe_accept_plan(16, 128256, 1024, 64, True)
    assert "accept_cluster_kernel" in text
    text = sv.spec_describe_accept_plan(16, 128256, 1024, 64, True, target_dtype=sv.SPEC_F32)
    assert "row_stats_kernel" in text
    text = sv.spec_describe_accept_plan(16, 128256, 1024, 64, True, tuning=sv.SpecAcceptTuning(path=1))
    assert "row_stats_kernel" in text
    text = sv.spec_describe_accept_plan(8, 32000, 64, 8, False)                 # a small batch of linear drafts
    assert "row_stats_kernel" in text and "accept_linear_kernel" in text
    text = sv.spec_describe_accept_plan(64, 128256, 365, 10, False)             # a large one
    assert "row_stats_prog_kernel" in text and "accept_linear_kernel" in text
