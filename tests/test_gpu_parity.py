"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on seeded inputs whose sizes span several tiles, chunks and ragged tails."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import ATTN_TOL, attn_rel_err, compare_accept, oracle_attn, ratio_err, visited_pattern_agrees

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()                      # fail loudly when the HIP library is missing
    return runner


C = W.CONFIGS
ATTN_CASES = {
    "tiny_full": C["c0_tiny"],
    "linear_mha_d128": W.scaled(C["c1_llama2_7b"], batch=3, n_q_heads=4, n_kv_heads=4, ctx=("fixed", 333)),
    "linear_multi_chunk": W.scaled(C["c1_llama2_7b"], batch=2, n_q_heads=2, n_kv_heads=2, ctx=("fixed", 1500)),
    "tree64_gqa4": W.scaled(C["c2_tree_llama3_8b"], batch=2, n_q_heads=8, n_kv_heads=2, ctx=("fixed", 210)),
    "tree_small_gqa": W.scaled(C["c2_tree_llama3_8b"], batch=3, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 1, 90),
                               draft=("tree", (3, 2, 2), 17)),
    "ragged_gqa8": W.scaled(C["c4_llama70b_serving"], batch=7, n_q_heads=16, n_kv_heads=2,
                            ctx=("lognormal", 300, 0.8, 17, 1500)),
    # ragged lengths with 16 to 128 query rows per KV head: the work list mixes both attention bodies, and the
    # long requests of either kind are cut into several chunks
    "ragged_rows_mixed": W.scaled(C["c4_llama70b_serving"], batch=6, n_q_heads=16, n_kv_heads=2,
                                  ctx=("lognormal", 2500, 0.9, 30, 9000), draft=("linear_uniform", 2, 16)),
    "d64_gqa2": W.scaled(C["c0_tiny"], batch=3, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 5, 400),
                         draft=("linear_uniform", 1, 9)),
    "d64_rows_mixed": W.scaled(C["c0_tiny"], batch=5, n_q_heads=16, n_kv_heads=2, ctx=("uniform", 5, 3000),
                               draft=("linear_uniform", 2, 14)),
    # more than 64 query nodes per request (two ancestor-mask words): the full 4,4,2,2 tree of Section 6.1's
    # setting (116 nodes), a tree whose last node hangs under node 0, chains of up to 128 tokens, head_dim 64
    "tree116_gqa4": W.scaled(C["c2_tree_llama3_8b"], batch=2, n_q_heads=8, n_kv_heads=2, ctx=("uniform", 100, 700),
                             draft=("tree", (4, 4, 2, 2), 116)),
    "tree128_flat": W.scaled(C["c2_tree_llama3_8b"], batch=2, n_q_heads=2, n_kv_heads=2, ctx=("uniform", 0, 200),
                             draft=("tree", (64, 1), 128)),
    "chain128_multi_chunk": W.scaled(C["c1_llama2_7b"], batch=3, n_q_heads=2, n_kv_heads=1, ctx=("uniform", 40, 5000),
                                     draft=("linear_uniform", 60, 128)),
    "tree100_d64": W.scaled(C["c0_tiny"], batch=3, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 5, 600),
                            draft=("tree", (3, 3, 3, 3), 100)),
    "ctx_zero": W.scaled(C["c1_llama2_7b"], batch=2, n_q_heads=2, n_kv_heads=1, ctx=("fixed", 0), draft=("linear", 5)),
    "page_boundary": W.scaled(C["c1_llama2_7b"], batch=2, n_q_heads=2, n_kv_heads=2, ctx=("fixed", 56), draft=("linear", 8)),
}


@pytest.mark.parametrize("name", list(ATTN_CASES))
def test_attention_matches_oracle(rt, name):
    cfg = ATTN_CASES[name]
    a = W.make_attn_inputs(cfg, seed=11)
    ref, ref_lse = oracle_attn(a)
    dev = rt.DeviceAttn(a)
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    err = attn_rel_err(got, ref)
    assert np.isfinite(got).all()
    assert err <= ATTN_TOL, f"{name}: rel err {err}"
    lse = dev.lse.cpu().numpy()
    assert np.abs(lse - ref_lse).max() < 2e-2, f"{name}: lse err {np.abs(lse - ref_lse).max()}"


@pytest.mark.parametrize("name", ["ragged_gqa8", "ragged_rows_mixed", "d64_rows_mixed", "d64_gqa2", "linear_multi_chunk", "tree_small_gqa",
                                  "chain128_multi_chunk", "tree116_gqa4"])
@pytest.mark.parametrize("hint", ["none", "exact", "small"])
def test_attention_launch_modes(rt, name, hint):
    """The total-token hint only steers how the work is cut (grid-mapped chunks when it is absent or
    says the lengths are uniform, a sorted work list when it says they are ragged): results must
    meet the same bar whatever it says, including a hint far below the truth."""
    cfg = ATTN_CASES[name]
    a = W.make_attn_inputs(cfg, seed=12)
    ref, ref_lse = oracle_attn(a)
    true_total = int((a.st.ctx_len.astype(np.int64) + a.st.n).sum())
    kv_hint = {"none": 0, "exact": true_total, "small": max(1, true_total // 7)}[hint]
    dev = rt.DeviceAttn(a, kv_hint=kv_hint)
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    assert np.isfinite(got).all()
    assert attn_rel_err(got, ref) <= ATTN_TOL
    assert np.abs(dev.lse.cpu().numpy() - ref_lse).max() < 2e-2


@pytest.mark.parametrize("batch,nodes", [(13, 116), (25, 64)])
def test_attention_256_row_workgroups_with_a_context_cut(rt, batch, nodes):
    """Enough (request, KV head, 256-row group) triples that the plan keeps 256-row workgroups (not the sliced
    variant) and still cuts the context in two: the partial-result path of the eight-wave row-split kernel and
    the combine kernel behind it, with one and with two ancestor-mask words per node."""
    from paper_2503_10325_amd import binding as sv
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=batch, ctx=("uniform", 300, 700), draft=("tree", (4, 4, 2, 2), nodes))
    a = W.make_attn_inputs(cfg, seed=17)
    dev = rt.DeviceAttn(a)
    plan = sv.spec_describe_attn_plan(dev.desc)
    assert "256 query rows per workgroup" in plan and "at most 2 per request" in plan, plan
    ref, ref_lse = oracle_attn(a)
    dev.out.fill_(float("nan"))
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    assert np.isfinite(got).all()
    assert attn_rel_err(got, ref) <= ATTN_TOL
    assert np.abs(dev.lse.cpu().numpy() - ref_lse).max() < 2e-2


def test_attention_fp32_output_and_determinism(rt):
    cfg = ATTN_CASES["ragged_gqa8"]
    a = W.make_attn_inputs(cfg, seed=5)
    ref, _ = oracle_attn(a)
    dev = rt.DeviceAttn(a, out_dtype=torch.float32)
    dev.run()
    torch.cuda.synchronize()
    first = dev.out.clone()
    assert attn_rel_err(first.cpu().numpy(), ref) <= ATTN_TOL
    dev.workspace.fill_(0xFF)                     # poisoned workspace must not leak into results
    dev.out.zero_()
    dev.run()
    torch.cuda.synchronize()
    assert torch.equal(first, dev.out)            # bit-identical from run to run


def test_attention_ignores_stale_cache_slots(rt):
    """Slots past ctx+n in the last page and unused pool pages may hold anything (NaN here)."""
    cfg = W.scaled(C["c1_llama2_7b"], batch=3, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 20, 200), draft=("linear", 3))
    a = W.make_attn_inputs(cfg, seed=2)
    ref, _ = oracle_attn(a)
    nan_bits = np.uint16(0x7FC0)
    used = np.zeros(a.num_pages, dtype=bool)
    for b in range(cfg.batch):
        L = int(a.st.ctx_len[b] + a.st.n[b])
        npg = (L + 15) // 16
        used[a.block_table[b, :npg]] = True
        if L % 16:
            pg = a.block_table[b, npg - 1]
            a.k_pool[pg, :, L % 16:, :] = nan_bits
            a.v_pool[pg, :, L % 16:, :] = nan_bits
    a.k_pool[~used] = nan_bits
    a.v_pool[~used] = nan_bits
    dev = rt.DeviceAttn(a)
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    assert np.isfinite(got).all()
    assert attn_rel_err(got, ref) <= ATTN_TOL


def test_attention_empty_request_in_batch(rt):
    cfg = W.scaled(C["c1_llama2_7b"], batch=3, n_q_heads=2, n_kv_heads=2, ctx=("fixed", 100), draft=("linear", 4))
    st = W.make_structure(cfg, seed=1)
    st.n[1] = 0
    st.node_offsets[1:] = np.cumsum(st.n)
    a = W.make_attn_inputs(cfg, seed=1, st=st)
    ref, _ = oracle_attn(a)
    dev = rt.DeviceAttn(a)
    dev.run()
    torch.cuda.synchronize()
    assert attn_rel_err(dev.out.float().cpu().numpy(), ref) <= ATTN_TOL


# --------------------------------------------------------------------------------
ACCEPT_CASES = {
    "tiny_full": (C["c0_tiny"], {}),
    "linear_v32000": (W.scaled(C["c1_llama2_7b"], batch=6), {}),
    "linear_odd_vocab": (W.scaled(C["c1_llama2_7b"], batch=9, vocab=1001, draft=("linear_uniform", 1, 7)), {}),
    "tree_v20000": (W.scaled(C["c2_tree_llama3_8b"], batch=5, vocab=20000), {}),
    "tree_wide": (W.scaled(C["c2_tree_llama3_8b"], batch=12, vocab=3000, draft=("tree", (5, 3), 20),
                           q_src=("noise", 2.0)), {}),
    "ragged_big_vocab": (W.scaled(C["c4_llama70b_serving"], batch=5), {}),
    # more than 64 nodes per request: the full 4,4,2,2 tree (116 nodes), a flat tree whose nodes 64.. are
    # children of low-numbered nodes, a chain of up to 128 tokens
    "tree116_v20000": (W.scaled(C["c2_tree_llama3_8b"], batch=12, vocab=20000, draft=("tree", (4, 4, 2, 2), 116),
                                q_src=("noise", 0.8)), {"deep": True}),
    "tree126_deep": (W.scaled(C["c2_tree_llama3_8b"], batch=12, vocab=20000, draft=("tree", (2, 2, 2, 2, 2, 2), 126),
                              q_src=("noise", 0.5)), {"deep": True}),
    "tree128_flat": (W.scaled(C["c2_tree_llama3_8b"], batch=6, vocab=3000, draft=("tree", (40, 3), 128),
                              q_src=("noise", 2.0)), {}),
    "chain128": (W.scaled(C["c1_llama2_7b"], batch=5, vocab=4000, draft=("linear_uniform", 60, 128),
                          q_src=("noise", 0.05)), {"deep": True}),
    "fp32_logits": (W.scaled(C["c1_llama2_7b"], batch=8, vocab=5000), {"fp32": True}),
    "temperature": (W.scaled(C["c1_llama2_7b"], batch=8, vocab=4096, temperature=0.7), {"fp32": True}),
}


def _run_accept(rt, cfg, ai, fp32=False, q_kind=0, draft_q=None, tuning=None):
    tl, dq = ai.target_logits, (ai.draft_q if draft_q is None else draft_q)
    if fp32:
        tl = W.bf16_bits_to_f32(tl)
        if dq.dtype == np.uint16:
            dq = W.bf16_bits_to_f32(dq)
    ref = oracle.accept(ai.st.node_offsets, ai.st.parent, ai.draft_tokens, tl, dq, ai.q_row, ai.u_accept,
                        ai.u_resample, temperature=cfg.temperature, qkind=q_kind)
    dev = rt.DeviceAccept(ai.st, tl, dq, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature, q_kind=q_kind)
    dev.run(tuning=tuning)
    return dev.results(), ref


def _tuning(**kw):
    from paper_2503_10325_amd import binding as sv
    return sv.SpecAcceptTuning(**kw)


@pytest.mark.parametrize("path", [0, 1, 2, 3])
@pytest.mark.parametrize("name", list(ACCEPT_CASES))
def test_accept_matches_oracle(rt, name, path):
    """path 0: the library's choice; 1: statistics pass over all rows + one walking workgroup per
    request; 2: workgroup clusters that read only the walked rows (bf16 rows; other inputs fall back to 1);
    3: statistics pass + the linear-draft kernel (trees fall back to 1)."""
    cfg, opt = ACCEPT_CASES[name]
    ai = W.make_accept_inputs(cfg, seed=4)
    got, ref = _run_accept(rt, cfg, ai, fp32=opt.get("fp32", False), tuning=_tuning(path=path) if path else None)
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    print(f"{name}: near-ties {ties}/{B}, mean accept_len {ref['accept_len'].mean():.2f}")
    assert not bad, f"{name}: requests {bad} differ outside near-ties"
    assert ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    assert np.array_equal(np.isnan(got["ratio"]), np.isnan(ref["ratio"]))
    if opt.get("deep"):
        assert ref["stop_node"].max() >= 64            # the walk reaches nodes of the second mask word


LINEAR_CASES = {
    # all accepted (draft rows = target rows): the draw comes from the row after the last draft
    "all_accepted": (W.scaled(C["c1_llama2_7b"], batch=5, vocab=9000, q_src=("noise", 0.0)), {}),
    # drafts far from the target: almost every request is rejected at its first node
    "mostly_rejected": (W.scaled(C["c1_llama2_7b"], batch=7, vocab=12345, q_src=("independent", 3.0)), {}),
    # a vocabulary of several units with a ragged last one (odd size: no 16-byte loads), ragged draft lengths
    "units_ragged": (W.scaled(C["c4_llama70b_serving"], batch=9, vocab=20001, draft=("linear_uniform", 1, 12)), {}),
    "one_unit_fp32": (W.scaled(C["c1_llama2_7b"], batch=4, vocab=777), {"fp32": True}),
    "temperature_2": (W.scaled(C["c1_llama2_7b"], batch=6, vocab=8192, temperature=2.0), {}),
}


@pytest.mark.parametrize("name", list(LINEAR_CASES))
def test_accept_linear_kernel_matches_oracle(rt, name):
    """The linear-draft kernel (path 3): every workgroup repeats the scalar tests, one of them - whichever arrives
    last - draws.  Same bar as every other path; and the walk kernel's results on the same inputs are the same
    outside near-ties."""
    cfg, opt = LINEAR_CASES[name]
    ai = W.make_accept_inputs(cfg, seed=9)
    assert ai.st.parent is None
    got, ref = _run_accept(rt, cfg, ai, fp32=opt.get("fp32", False), tuning=_tuning(path=3))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    print(f"{name}: near-ties {ties}/{B}, mean accept_len {ref['accept_len'].mean():.2f}")
    assert not bad, f"{name}: requests {bad} differ outside near-ties"
    assert ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    assert np.array_equal(np.isnan(got["ratio"]), np.isnan(ref["ratio"]))
    assert visited_pattern_agrees(got, ref, ai.st.node_offsets)
    walk, _ = _run_accept(rt, cfg, ai, fp32=opt.get("fp32", False), tuning=_tuning(path=1))
    bad2, _, _ = compare_accept(walk, ref, ai.st.n)
    assert not bad2
    assert np.array_equal(got["stop_node"], walk["stop_node"]) or ties > 0


@pytest.mark.parametrize("name", list(LINEAR_CASES))
def test_accept_statistics_that_stop_at_the_first_rejection(rt, name):
    """Path 4: the statistics pass skips rows behind each request's first rejection (it takes the accept decisions
    itself, with the arithmetic of the linear-draft kernel).  Rows it skips hold whatever the workspace held before
    - the workspace is filled with NaN patterns and with huge values here - and the results must be those of path 3
    bit for bit, and the oracle's outside near-ties."""
    cfg, opt = LINEAR_CASES[name]
    ai = W.make_accept_inputs(cfg, seed=9)
    fp32 = opt.get("fp32", False)
    tl, dq = ai.target_logits, ai.draft_q
    if fp32:
        tl, dq = W.bf16_bits_to_f32(tl), W.bf16_bits_to_f32(dq)
    ref = oracle.accept(ai.st.node_offsets, ai.st.parent, ai.draft_tokens, tl, dq, ai.q_row, ai.u_accept,
                        ai.u_resample, temperature=cfg.temperature)
    outs = {}
    for path, fill in ((3, 0), (4, 0xFF), (4, 0x7B)):
        dev = rt.DeviceAccept(ai.st, tl, dq, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                              temperature=cfg.temperature)
        dev.workspace.fill_(fill)
        dev.run(tuning=_tuning(path=path))
        outs[(path, fill)] = dev.results()
    base = outs[(3, 0)]
    bad, ties, B = compare_accept(base, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    for key, got in outs.items():
        for f in ("accept_len", "out_tokens", "stop_node"):
            assert np.array_equal(got[f], base[f]), (key, f)
        assert np.array_equal(got["ratio"], base["ratio"], equal_nan=True), key


def test_accept_linear_kernel_probability_drafts(rt):
    """Draft rows given as probabilities (SPEC_Q_PROBS) through the linear-draft kernel."""
    cfg = W.scaled(C["c1_llama2_7b"], batch=6, vocab=6000)
    ai = W.make_accept_inputs(cfg, seed=10)
    logits = W.bf16_bits_to_f32(ai.draft_q).astype(np.float64) / cfg.temperature
    probs = np.exp(logits - logits.max(axis=1, keepdims=True))
    probs = (probs / probs.sum(axis=1, keepdims=True)).astype(np.float32)
    got, ref = _run_accept(rt, cfg, ai, fp32=True, q_kind=1, draft_q=probs, tuning=_tuning(path=3))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)


# (levels, slices) of the cluster path; 0 = the library's choice.  Vocabulary 128256 = 16 units of 8192 logits:
# 4 slices of 4 units, 8 of 2, 16 of 1; 70000 = 9 units: 3 slices of 4 (the last with one), 5 of 2, 9 of 1.
CLUSTER_SHAPES = [(0, 0), (1, 4), (2, 4), (4, 4), (1, 8), (3, 8), (1, 16), (2, 16)]


@pytest.mark.parametrize("levels,slices", CLUSTER_SHAPES)
def test_accept_cluster_shapes_tree(rt, levels, slices):
    """Every split of a request over workgroups (window levels x vocabulary slices) reproduces the oracle's
    decisions on tree drafts with a large vocabulary."""
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=6)
    ai = W.make_accept_inputs(cfg, seed=8)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=2, levels=levels, slices=slices))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    assert (got["accept_len"] >= 0).all()
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    assert np.array_equal(np.isnan(got["ratio"]), np.isnan(ref["ratio"])) or ties


@pytest.mark.parametrize("levels,slices,vocab,draft", [
    (9, 2, 32000, ("linear", 8)), (4, 4, 32000, ("linear", 8)), (1, 1, 32000, ("linear_uniform", 1, 7)),
    (5, 3, 70000, ("linear_uniform", 2, 10)), (2, 9, 70000, ("linear_uniform", 2, 10)), (3, 5, 70000, ("linear", 4)),
    (16, 1, 8192, ("linear", 20)), (7, 1, 8200, ("linear", 3)),
])
def test_accept_cluster_shapes_linear(rt, levels, slices, vocab, draft):
    """Linear drafts: windows longer and shorter than the draft, slices that end inside the vocabulary's
    last unit, a slice beyond the vocabulary's end (8200 = one full unit + 8 logits)."""
    cfg = W.scaled(C["c1_llama2_7b"], batch=7, vocab=vocab, draft=draft)
    ai = W.make_accept_inputs(cfg, seed=21)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=2, levels=levels, slices=slices))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6


@pytest.mark.parametrize("levels,slices", [(0, 0), (2, 8), (1, 4)])
def test_accept_cluster_owner_walks_alone(rt, levels, slices):
    """With no patience the first workgroup of every cluster never waits for its peers: it tells them to
    leave and computes every slice's part itself, in the same order (what happens when peers are late because
    other kernels fill the GPU).  Same decisions as the oracle AND bit-identical outputs to the cluster's."""
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=5)
    ai = W.make_accept_inputs(cfg, seed=13)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=2, levels=levels, slices=slices, patience=0))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    full, _ = _run_accept(rt, cfg, ai, tuning=_tuning(path=2, levels=levels, slices=slices))
    for key in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(got[key], full[key]), key
    assert np.array_equal(got["ratio"], full["ratio"], equal_nan=True)


def test_accept_cluster_one_workgroup_per_request(rt):
    """More requests than compute units leave one workgroup per request (the library's choice is then the
    statistics pass; the cluster path is forced here): it computes the slices' parts in turn."""
    cfg = W.scaled(C["c4_llama70b_serving"], batch=300, vocab=40000)
    ai = W.make_accept_inputs(cfg, seed=17)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=2))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)


def test_accept_cluster_back_to_back_calls_share_a_workspace(rt):
    """The message buffers of one call must not leak into the next (they are cleared by a kernel ahead of
    the walk): two different batches through one workspace, twice."""
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=4, vocab=50000)
    a1 = W.make_accept_inputs(cfg, seed=31)
    a2 = W.make_accept_inputs(cfg, seed=32)
    refs = [oracle.accept(a.st.node_offsets, a.st.parent, a.draft_tokens, a.target_logits, a.draft_q, a.q_row,
                          a.u_accept, a.u_resample, temperature=cfg.temperature) for a in (a1, a2)]
    devs = [rt.DeviceAccept(a.st, a.target_logits, a.draft_q, a.q_row, a.draft_tokens, a.u_accept, a.u_resample,
                            temperature=cfg.temperature) for a in (a1, a2)]
    devs[1].workspace = devs[0].workspace
    for _ in range(2):
        for d in devs:
            d.run()
    for a, d, ref in zip((a1, a2), devs, refs):
        bad, ties, B = compare_accept(d.results(), ref, a.st.n)
        assert not bad


@pytest.mark.parametrize("helpers", [0, 1, 2, 3])
def test_accept_helper_workgroups(rt, helpers):
    """Statistics-pass path: large vocabularies split every full pass over helper workgroups; any helper
    count must reproduce the oracle's decisions."""
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=6, vocab=70001 if helpers == 2 else 128256)
    ai = W.make_accept_inputs(cfg, seed=8)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=1, helpers=helpers))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    assert (got["accept_len"] >= 0).all()
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6


def test_accept_master_without_helper_answers(rt):
    """Statistics-pass path: with no patience at all the master never waits for a helper and sums every
    segment itself (what it does when helper workgroups are late because other kernels fill the GPU); late
    answers are ignored."""
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=5)
    ai = W.make_accept_inputs(cfg, seed=13)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=1, helpers=3, patience=0))
    bad, ties, B = compare_accept(got, ref, ai.st.n)
    assert not bad and ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6


def test_accept_draft_equals_target_accepts_all(rt):
    cfg = W.scaled(C["c1_llama2_7b"], batch=5, vocab=8000)
    ai = W.make_accept_inputs(cfg, seed=9, draft_equals_target=True)
    got, ref = _run_accept(rt, cfg, ai)
    assert np.array_equal(got["accept_len"], ai.st.n)
    bad, ties, _ = compare_accept(got, ref, ai.st.n)
    assert not bad


def test_accept_with_probability_rows(rt):
    """Draft rows given as probabilities (as the MIXTURE fusion produces them)."""
    cfg = W.scaled(C["c1_llama2_7b"], batch=6, vocab=2048)
    ai = W.make_accept_inputs(cfg, seed=6)
    z = W.bf16_bits_to_f32(ai.draft_q).astype(np.float64)
    e = np.exp(z - z.max(-1, keepdims=True))
    probs = (e / e.sum(-1, keepdims=True)).astype(np.float32)
    got, ref = _run_accept(rt, cfg, ai, q_kind=1, draft_q=probs)
    bad, ties, _ = compare_accept(got, ref, ai.st.n)
    assert not bad


@pytest.mark.parametrize("path", [0, 1, 2])
def test_accept_sibling_group_takes_its_first_childs_draft_row(rt, path):
    """The children of one node are draws from one draft distribution, the row their first child names (the
    reading the oracle implements).  Later siblings whose q_row entries name other rows change nothing: the
    kernels, like the oracle, use the group's row for q(x) and for the residual."""
    import dataclasses
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=6, vocab=20000, q_src=("noise", 1.5))
    ai = W.make_accept_inputs(cfg, seed=13)
    st = ai.st
    n_q_rows = ai.draft_q.shape[0]
    q_row = ai.q_row.copy()
    seen, changed = set(), 0
    for b in range(cfg.batch):
        o = int(st.node_offsets[b])
        for j in range(int(st.n[b])):
            key = (b, int(st.parent[o + j]))
            if key in seen:                               # not the first child of its parent
                q_row[o + j] = (int(q_row[o + j]) + 1 + 7 * j) % n_q_rows
                changed += 1
            seen.add(key)
    assert changed > 0
    ai2 = dataclasses.replace(ai, q_row=q_row)
    got, ref = _run_accept(rt, cfg, ai2, tuning=_tuning(path=path) if path else None)
    ref0 = oracle.accept(st.node_offsets, st.parent, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                         ai.u_accept, ai.u_resample, temperature=cfg.temperature, qkind=0)
    for k in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(ref[k], ref0[k])            # the oracle ignores the later siblings' entries
    assert (ref["accept_len"] > 0).any() and np.isfinite(ref["ratio"]).sum() > 2 * cfg.batch   # siblings were tried
    bad, ties, B = compare_accept(got, ref, st.n)
    assert not bad, f"requests {bad} differ outside near-ties"
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
    assert np.array_equal(np.isnan(got["ratio"]), np.isnan(ref["ratio"]))


def test_accept_prestats_on_a_tree_the_cluster_kernel_takes(rt):
    """spec_accept_prestats on a shape for which the library picks the cluster kernel: that kernel takes the
    statistics of the walked rows itself, so the statistics region of the workspace is not read (it holds NaN
    patterns here) and the results are those of spec_accept, and the oracle's."""
    from paper_2503_10325_amd import binding as sv
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=4, vocab=65536)
    ai = W.make_accept_inputs(cfg, seed=21)
    assert "accept_cluster_kernel" in sv.spec_describe_accept_plan(cfg.batch, cfg.vocab, ai.st.total, int(ai.st.n.max()), True)
    got, ref = _run_accept(rt, cfg, ai)
    dev = rt.DeviceAccept(ai.st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample,
                          temperature=cfg.temperature)
    dev.workspace.fill_(0xFF)
    dev.run_prestats()
    pre = dev.results()
    for key in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(pre[key], got[key]), key
    bad, _, _ = compare_accept(pre, ref, ai.st.n)
    assert not bad


@pytest.mark.parametrize("path", [0, 1, 3, 4])
def test_accept_zero_nodes_request(rt, path):
    cfg = W.scaled(C["c1_llama2_7b"], batch=4, vocab=1000, draft=("linear", 3))
    st = W.make_structure(cfg, seed=2)
    st.n[2] = 0
    st.node_offsets[1:] = np.cumsum(st.n)
    ai = W.make_accept_inputs(cfg, seed=2, st=st)
    got, ref = _run_accept(rt, cfg, ai, tuning=_tuning(path=path) if path else None)
    bad, ties, _ = compare_accept(got, ref, st.n)
    assert not bad and got["accept_len"][2] == 0


# --------------------------------------------------------------------------------
def test_fusion_argmax_and_mixture_match_oracle(rt):
    from paper_2503_10325_amd import binding as sv
    cfg = W.scaled(C["c3_fusion"], batch=4, vocab=3000)
    ai = W.make_accept_inputs(cfg, seed=8)
    f = ai.fusion
    f.k_len = np.array([6, 5, 6, 1], dtype=np.int32)
    f.conf[0, 2, :] = 0.5                                  # a tie: lowest drafter index wins
    ref = oracle.fuse_drafts(f.k_len, f.conf, f.draft_tokens)
    dev = rt.DeviceFuse(f, cfg.vocab)
    dev.run()
    torch.cuda.synchronize()
    for key, t in (("fused_token", dev.fused_token), ("winner", dev.winner), ("q_row", dev.q_row)):
        assert np.array_equal(t.cpu().numpy(), ref[key]), key
    T = 1.3
    refm = oracle.fuse_drafts(f.k_len, f.conf, f.draft_tokens, f.draft_logits, temperature=T,
                              mode=oracle.FUSE_MIXTURE)
    devm = rt.DeviceFuse(f, cfg.vocab, temperature=T, mode=sv.SPEC_FUSE_MIXTURE)
    devm.run()
    torch.cuda.synchronize()
    assert np.array_equal(devm.q_row.cpu().numpy(), refm["q_row"])
    got = devm.fused_probs.cpu().numpy().astype(np.float64)
    valid = (np.arange(6)[None, :] < f.k_len[:, None]).reshape(-1)
    err = np.abs(got[valid] - refm["fused_probs"][valid]) / (refm["fused_probs"][valid] + 1e-12)
    assert err.max() < 2e-5, err.max()
    assert np.abs(got[valid].sum(-1) - 1).max() < 1e-5


def test_fusion_then_accept_pipeline(rt):
    """Config-3 style: ARGMAX fusion output feeds the acceptance step on the device."""
    cfg = W.scaled(C["c3_fusion"], batch=5, vocab=4000)
    ai = W.make_accept_inputs(cfg, seed=12)
    f = ai.fusion
    rf = oracle.fuse_drafts(f.k_len, f.conf, f.draft_tokens)
    ref = oracle.accept(ai.st.node_offsets, None, rf["fused_token"].reshape(-1), ai.target_logits, f.draft_logits,
                        rf["q_row"].reshape(-1), ai.u_accept, ai.u_resample)
    dev = rt.DeviceFuse(f, cfg.vocab)
    dev.run()
    acc = rt.DeviceAccept(ai.st, ai.target_logits, dev.draft_logits, dev.q_row.view(-1), dev.fused_token.view(-1),
                          ai.u_accept, ai.u_resample)
    acc.run()
    bad, ties, _ = compare_accept(acc.results(), ref, ai.st.n)
    assert not bad
