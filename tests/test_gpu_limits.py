"""GPU parity at the edges of what the library accepts: the largest vocabulary, the longest draft
chain, contexts long enough to hit the chunk-count cap of the work-list launch and the chunk-length
cap of the row-split kernel, and a batch just above the work-list limit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import ATTN_TOL, attn_rel_err, compare_accept, oracle_attn, ratio_err

pytestmark = pytest.mark.gpu
C = W.CONFIGS


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def _attn(rt, cfg, seed, st=None, **kw):
    a = W.make_attn_inputs(cfg, seed=seed, st=st)
    ref, ref_lse = oracle_attn(a)
    dev = rt.DeviceAttn(a, **kw)
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    assert np.isfinite(got).all()
    assert attn_rel_err(got, ref) <= ATTN_TOL
    assert np.abs(dev.lse.cpu().numpy() - ref_lse).max() < 2e-2


def test_attention_long_ragged_contexts_hit_the_chunk_cap(rt):
    # 16 query rows per KV head (four waves per block) and 80 rows (one wave per block, every tile):
    # the second cuts a 30000-token context into the maximum of 16 chunks
    for draft, heads in ((("linear", 2), (8, 1)), (("linear", 10), (8, 1))):
        cfg = W.scaled(C["c4_llama70b_serving"], batch=3, n_q_heads=heads[0], n_kv_heads=heads[1], draft=draft,
                       ctx=("fixed", 100))
        st = W.make_structure(cfg, seed=3)
        st.ctx_len[:] = [100, 30000, 5000]
        _attn(rt, cfg, 3, st=st)


def test_attention_row_split_long_context(rt):
    # 64-node tree x GQA 4 = 256 rows per KV head on a context longer than one row-split chunk may be
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=1, n_q_heads=4, n_kv_heads=1, ctx=("fixed", 40000))
    _attn(rt, cfg, 5)
    _attn(rt, cfg, 5, kv_hint=0)


def test_attention_longest_chain_and_d64(rt):
    cfg = W.scaled(C["c0_tiny"], batch=2, n_q_heads=2, n_kv_heads=1, ctx=("uniform", 0, 300), draft=("linear", 64))
    _attn(rt, cfg, 7)                                       # 128 rows per KV head, head_dim 64, 64 chained drafts


def test_attention_batch_above_the_work_list_limit(rt):
    cfg = W.scaled(C["c4_llama70b_serving"], batch=130, n_q_heads=8, n_kv_heads=1, ctx=("lognormal", 200, 0.8, 10, 900))
    _attn(rt, cfg, 9)                                       # 130 requests: grid-mapped launch although ragged


def test_accept_largest_vocabulary(rt):
    V = 2097152
    cfg = W.scaled(C["c1_llama2_7b"], batch=2, vocab=V, draft=("linear", 2))
    ai = W.make_accept_inputs(cfg, seed=1)
    ref = oracle.accept(ai.st.node_offsets, ai.st.parent, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                        ai.u_accept, ai.u_resample, temperature=cfg.temperature)
    dev = rt.DeviceAccept(ai.st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature)
    dev.run()
    got = dev.results()
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= 1
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    g = rt.DeviceGreedy(ai.st, ai.target_logits, ai.draft_tokens)
    g.run()
    gr = g.results()
    want = oracle.accept_greedy(ai.st.node_offsets, ai.st.parent, ai.draft_tokens, ai.target_logits)
    for key in ("row_argmax", "accept_len", "out_tokens"):
        assert np.array_equal(gr[key], want[key]), key


@pytest.mark.parametrize("shape,path", [("linear", 3), ("linear", 1), ("tree", 1), ("tree", 2)])
def test_accept_clamps_indices_read_from_device_memory(rt, shape, path):
    """Draft tokens, q_row entries and parents live in device memory the host layer cannot check.  Every kernel
    clamps them before it uses them as an index (token to [0, V), q_row to [0, n_q_rows), a parent outside
    [-1, j) to -1), so a corrupt entry changes that request's answer and nothing else: the result equals the
    oracle's on the clamped arrays."""
    from paper_2503_10325_amd import binding as sv
    if shape == "linear":
        cfg = W.scaled(C["c1_llama2_7b"], batch=6, vocab=5000)
    else:
        cfg = W.scaled(C["c2_tree_llama3_8b"], batch=4, vocab=8192, draft=("tree", (3, 2, 2), 17))
    ai = W.make_accept_inputs(cfg, seed=21)
    V, nq = cfg.vocab, ai.draft_q.shape[0]
    rng = np.random.default_rng(5)
    toks, qrow = ai.draft_tokens.copy(), ai.q_row.copy()
    hit = rng.choice(len(toks), size=max(3, len(toks) // 5), replace=False)
    toks[hit[0::3]] = -7
    toks[hit[1::3]] = V + 9
    qrow[hit[2::3]] = nq + 3
    qrow[hit[0]] = -1
    st = ai.st
    parent = None
    if st.parent is not None:
        parent = st.parent.copy()
        local = np.concatenate([np.arange(n) for n in st.n])
        roots = np.flatnonzero(parent == -1)          # children of the prefix: clamping leaves the tree as it was
        bad = rng.choice(roots, size=4, replace=False)
        parent[bad[:2]] = local[bad[:2]] + 1          # not an earlier node
        parent[bad[2:]] = -9
        st = W.DraftStructure(st.n, st.node_offsets, parent, st.ctx_len)
    c_toks, c_qrow = np.clip(toks, 0, V - 1), np.clip(qrow, 0, nq - 1)
    c_parent = None
    if parent is not None:
        local = np.concatenate([np.arange(n) for n in st.n])
        c_parent = np.where((parent < -1) | (parent >= local), -1, parent).astype(np.int32)
    ref = oracle.accept(st.node_offsets, c_parent, c_toks, ai.target_logits, ai.draft_q, c_qrow, ai.u_accept,
                        ai.u_resample, temperature=cfg.temperature)
    dev = rt.DeviceAccept(st, ai.target_logits, ai.draft_q, qrow, toks, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature)
    dev.run(tuning=sv.SpecAcceptTuning(path=path))
    got = dev.results()
    # accepted tokens are reported as given (clamped): compare on the clamped arrays
    bad_req, ties, B = compare_accept(got, ref, st.n)
    assert not bad_req and ties <= 1


def test_accept_vocabulary_above_the_limit_is_refused(rt):
    from paper_2503_10325_amd import binding as sv
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(sv.SpecError):
        sv.spec_accept(1, 1, 1, t, None, t, torch.zeros((2, 2097153), dtype=torch.bfloat16, device="cuda"),
                       torch.zeros((1, 2097153), dtype=torch.bfloat16, device="cuda"), sv.SPEC_Q_LOGITS, t, 1.0,
                       torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda"), t, t.view(1, 8), workspace=t)
