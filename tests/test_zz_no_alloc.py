"""The entry point that allocates nothing (spec_accept_noalloc, through the C ABI): its outputs equal
spec_accept's on the same inputs, on two calls in a row, the second with a smaller input (the built-in
scratch array keeps the first call's contents); oversized problems are rejected."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2503_10325_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def _both(rt, cfg, seed, fp32=False):
    sv = rt.sv
    ai = W.make_accept_inputs(cfg, seed=seed)
    tl, dq = ai.target_logits, ai.draft_q
    if fp32:
        tl, dq = W.bf16_bits_to_f32(tl), W.bf16_bits_to_f32(dq)
    ref = rt.DeviceAccept(ai.st, tl, dq, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature)
    ref.run()
    want = ref.results()
    dev = rt.DeviceAccept(ai.st, tl, dq, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature)
    dev.workspace = None
    for t in (dev.accept_len, dev.out_tokens, dev.stop_node):
        t.fill_(-7)
    sv.spec_accept_noalloc(dev.B, dev.total, dev.max_nodes, dev.node_offsets, dev.parent, dev.draft_tokens,
                           dev.target, dev.draft_q, dev.q_kind, dev.q_row, dev.temperature, dev.u_accept,
                           dev.u_resample, dev.accept_len, dev.out_tokens, dev.stop_node, dev.dbg_ratio)
    got = dev.results()
    for key in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(got[key], want[key]), key
    assert np.array_equal(got["ratio"], want["ratio"], equal_nan=True)
    return want


@pytest.mark.parametrize("fp32", [False, True])
def test_noalloc_matches_spec_accept_twice(rt, fp32):
    """bf16 rows take the cluster kernel (message buffers in the scratch array), fp32 rows the statistics
    pass and the walk (row statistics, descriptors and hand-back slots in the scratch array)."""
    big = W.scaled(W.CONFIGS["c2_tree_llama3_8b"], batch=6, vocab=70000)
    small = W.scaled(W.CONFIGS["c1_llama2_7b"], batch=3, vocab=9000, draft=("linear_uniform", 1, 5))
    a = _both(rt, big, seed=41, fp32=fp32)
    b = _both(rt, small, seed=42, fp32=fp32)
    assert a["accept_len"].shape[0] == 6 and b["accept_len"].shape[0] == 3


def test_noalloc_rejects_what_does_not_fit(rt):
    sv = rt.sv
    L = sv.lib()
    cap = int(L.spec_accept_noalloc_max_workspace())
    assert cap == 4 << 20
    B, V, total = 64, 128256, 60000                      # far more row statistics than 4 MiB hold
    assert sv.spec_accept_workspace_size(B, total, total, V) > cap
    null = ctypes.c_void_p(0)
    rc = L.spec_accept_noalloc(B, V, total, total, 64, null, null, null, null, 0, null, 0, 0, null, 1.0, null, null,
                               null, null, 65, null, null, null)
    assert rc == -4
