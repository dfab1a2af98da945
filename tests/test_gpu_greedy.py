"""GPU parity of greedy verification (spec_accept_greedy, through the C ABI) against the CPU
oracle: exact integer comparison of acceptance lengths, emitted tokens, stop nodes and the
argmax of every target row; small cases with ties, odd vocabularies, fp32 logits and empty
requests, and the five benchmark workloads at full size."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def greedy_draft_tokens(st, ai):
    """Greedy drafting: sibling number r of a parent proposes the r-th most likely token of the
    parent's draft row (a linear draft proposes each row's argmax)."""
    q = W.bf16_bits_to_f32(ai.draft_q) if ai.draft_q.dtype == np.uint16 else ai.draft_q
    toks = np.zeros(st.total, dtype=np.int32)
    for b in range(len(st.n)):
        o, n = int(st.node_offsets[b]), int(st.n[b])
        rank = {}
        for j in range(n):
            par = j - 1 if st.parent is None else int(st.parent[o + j])
            r = rank.get(par, 0)
            rank[par] = r + 1
            row = q[int(ai.q_row[o + j])]
            top = np.argpartition(-row, min(r + 1, row.shape[0] - 1))[:r + 1]
            toks[o + j] = top[np.argsort(-row[top], kind="stable")][r]
    return toks


def check(rt, st, target_logits, toks):
    ref = oracle.accept_greedy(st.node_offsets, st.parent, toks, target_logits)
    dev = rt.DeviceGreedy(st, target_logits, toks)
    dev.run()
    got = dev.results()
    for key in ("row_argmax", "accept_len", "stop_node", "out_tokens"):
        assert np.array_equal(got[key], ref[key]), key
    return ref


C = W.CONFIGS
CASES = {
    "tiny_full": C["c0_tiny"],
    "linear_v32000": W.scaled(C["c1_llama2_7b"], batch=6),
    "linear_odd_vocab": W.scaled(C["c1_llama2_7b"], batch=9, vocab=1001, draft=("linear_uniform", 1, 7)),
    "tree_v20000": W.scaled(C["c2_tree_llama3_8b"], batch=5, vocab=20000),
    "ragged_big_vocab": W.scaled(C["c4_llama70b_serving"], batch=5),
    # more than 64 nodes per request
    "tree116_v20000": W.scaled(C["c2_tree_llama3_8b"], batch=12, vocab=20000, draft=("tree", (4, 4, 2, 2), 116),
                               q_src=("noise", 0.5)),
    "tree126_deep": W.scaled(C["c2_tree_llama3_8b"], batch=12, vocab=20000, draft=("tree", (2, 2, 2, 2, 2, 2), 126),
                             q_src=("noise", 0.5)),
    "tree128_flat": W.scaled(C["c2_tree_llama3_8b"], batch=6, vocab=3000, draft=("tree", (40, 3), 128)),
    "chain128": W.scaled(C["c1_llama2_7b"], batch=5, vocab=4000, draft=("linear_uniform", 60, 128), q_src=("noise", 0.05)),
}


@pytest.mark.parametrize("name", list(CASES))
def test_greedy_matches_oracle(rt, name):
    cfg = CASES[name]
    ai = W.make_accept_inputs(cfg, seed=4)
    toks = greedy_draft_tokens(ai.st, ai)
    ref = check(rt, ai.st, ai.target_logits, toks)
    print(f"{name}: mean accept_len {ref['accept_len'].mean():.2f}")
    if name != "tiny_full":
        assert ref["accept_len"].max() >= 1            # the case exercises real descents
    if name in ("tree116_v20000", "tree126_deep"):
        assert ref["stop_node"].max() >= 64            # ... into nodes held by the second ballot word


def test_greedy_fp32_logits_ties_and_special_values(rt):
    rng = np.random.default_rng(2)
    B, k, V = 7, 5, 8200                                # two segments, the second ragged
    st = W.make_structure(W.scaled(C["c1_llama2_7b"], batch=B, vocab=V, draft=("linear", k)), seed=0)
    x = np.round(rng.standard_normal((B * (k + 1), V)) * 1.5).astype(np.float32)      # few values: many ties
    x[0] = 0.0
    x[1] = -np.inf
    x[2, :] = -0.0
    x[2, 5000] = 0.0                                    # -0 == +0: index 0 wins
    x[3, 100] = np.nan
    x[4, :8192] = -5.0
    x[4, 8195] = 7.0                                    # maximum in the ragged tail
    toks = rng.integers(0, V, size=B * k).astype(np.int32)
    arg = np.argmax(np.where(np.isnan(x), -np.inf, x), axis=1)
    for b in range(B):                                  # half of the drafts follow the argmax
        for j in range(k):
            if rng.random() < 0.6:
                toks[b * k + j] = arg[b * (k + 1) + j]
    ref = check(rt, st, x, toks)
    assert np.array_equal(ref["row_argmax"], arg)
    check(rt, st, W.f32_to_bf16_bits(x), toks)


def test_greedy_zero_nodes_request(rt):
    cfg = W.scaled(C["c1_llama2_7b"], batch=4, vocab=1000, draft=("linear", 3))
    st = W.make_structure(cfg, seed=1)
    st.n[2] = 0
    st.node_offsets[1:] = np.cumsum(st.n)
    ai = W.make_accept_inputs(cfg, seed=1, st=st)
    check(rt, st, ai.target_logits, greedy_draft_tokens(st, ai))


@pytest.mark.parametrize("name", W.CONFIG_ORDER + W.SECONDARY)
def test_greedy_fullsize(rt, name):
    cfg = W.CONFIGS[name]
    st = W.make_structure(cfg, seed=0)
    ai = W.make_accept_inputs(cfg, seed=0, st=st)
    if ai.fusion is not None:
        rf = oracle.fuse_drafts(ai.fusion.k_len, ai.fusion.conf, ai.fusion.draft_tokens)
        toks = rf["fused_token"].reshape(-1)
    else:
        toks = greedy_draft_tokens(st, ai)
    ref = check(rt, st, ai.target_logits, toks)
    print(f"{name}: mean accept_len {ref['accept_len'].mean():.2f}")
