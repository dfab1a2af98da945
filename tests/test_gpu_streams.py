"""The library only enqueues work on the stream it is given: calls captured into a HIP graph must
replay to the eager results, every time, and independent problems on two streams must not disturb
each other (each has its own workspace)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import ATTN_TOL, attn_rel_err, compare_accept, oracle_attn

pytestmark = pytest.mark.gpu
C = W.CONFIGS


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def test_graph_replay_matches_eager(rt):
    cfg = W.scaled(C["c4_llama70b_serving"], batch=6, n_q_heads=16, n_kv_heads=2, ctx=("lognormal", 400, 0.8, 20, 2500))
    a = W.make_attn_inputs(cfg, seed=2)
    ai = W.make_accept_inputs(cfg, seed=2, st=a.st)
    attn = rt.DeviceAttn(a)
    acc = rt.DeviceAccept(a.st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample)
    attn.run(); acc.run()                                   # eager: reference results (and one-time set-up)
    torch.cuda.synchronize()
    out0, lse0 = attn.out.clone(), attn.lse.clone()
    res0 = {k: v.copy() for k, v in acc.results().items() if v is not None}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            attn.run(); acc.run()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        attn.out.zero_(); attn.lse.zero_(); acc.accept_len.fill_(-9); acc.out_tokens.fill_(-9)
        attn.workspace.fill_(0xEE)                          # partials of earlier runs must not be needed
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(attn.out, out0) and torch.equal(attn.lse, lse0), rep
        res = acc.results()
        for k, v in res0.items():
            assert np.array_equal(res[k], v, equal_nan=True), (rep, k)
    ref, _ = oracle_attn(a)
    assert attn_rel_err(out0.float().cpu().numpy(), ref) <= ATTN_TOL


def test_two_streams_do_not_interfere(rt):
    cfgs = [W.scaled(C["c2_tree_llama3_8b"], batch=3, n_q_heads=8, n_kv_heads=2, ctx=("fixed", 700), vocab=70000),
            W.scaled(C["c1_llama2_7b"], batch=5, n_q_heads=4, n_kv_heads=4, ctx=("fixed", 900))]
    probs = []
    for i, cfg in enumerate(cfgs):
        a = W.make_attn_inputs(cfg, seed=20 + i)
        ai = W.make_accept_inputs(cfg, seed=20 + i, st=a.st)
        probs.append((a, ai, rt.DeviceAttn(a),
                      rt.DeviceAccept(a.st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept,
                                      ai.u_resample)))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):
        for (a, ai, attn, acc), s in zip(probs, streams):
            attn.run(stream=s)
            acc.run(stream=s)
    torch.cuda.synchronize()
    for a, ai, attn, acc in probs:
        ref, _ = oracle_attn(a)
        assert attn_rel_err(attn.out.float().cpu().numpy(), ref) <= ATTN_TOL
        want = oracle.accept(a.st.node_offsets, a.st.parent, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                             ai.u_accept, ai.u_resample)
        bad, ties, B = compare_accept(acc.results(), want, a.st.n)
        assert not bad
