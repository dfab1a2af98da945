"""GPU parity of the accepted-path KV compaction (spec_compact_kv, through the C ABI): the pools must
equal the oracle's byte for byte, for trees, linear drafts, nothing accepted, both head sizes, and for
stop nodes that come out of the acceptance step itself."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

pytestmark = pytest.mark.gpu
C = W.CONFIGS


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return binding, runner


def run(mods, a, stop, stop_dev=None):
    """``stop``: host stop nodes (the oracle's input); ``stop_dev``: a device tensor the GPU call reads
    instead (stop nodes written by spec_accept) - the oracle never sees a value the GPU produced."""
    sv, runner = mods
    st = a.st
    t = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    k, v = runner.bf16_to_device(a.k_pool, "cuda"), runner.bf16_to_device(a.v_pool, "cuda")
    new_len = torch.full((len(stop),), -5, dtype=torch.int32, device="cuda")
    sv.spec_compact_kv(k, v, t(a.block_table), t(st.ctx_len), t(st.node_offsets), t(st.parent),
                       t(stop) if stop_dev is None else stop_dev, new_len)
    torch.cuda.synchronize()
    k2, v2 = a.k_pool.copy(), a.v_pool.copy()
    want_len = oracle.compact_kv(k2, v2, a.block_table, st.ctx_len, st.node_offsets, st.parent, stop)
    assert np.array_equal(k.view(torch.int16).cpu().numpy().view(np.uint16), k2)
    assert np.array_equal(v.view(torch.int16).cpu().numpy().view(np.uint16), v2)
    assert np.array_equal(new_len.cpu().numpy(), want_len)
    return not np.array_equal(k2, a.k_pool)


@pytest.mark.parametrize("case", ["tree64_d128", "tree116_d128", "tree_small_d64", "linear", "chain128", "none_accepted"])
def test_compaction_matches_oracle(mods, case):
    rng = np.random.default_rng(7)
    if case == "tree64_d128":
        cfg = W.scaled(C["c2_tree_llama3_8b"], batch=5, n_q_heads=8, n_kv_heads=2, ctx=("uniform", 0, 300))
    elif case == "tree116_d128":
        cfg = W.scaled(C["c2_tree_llama3_8b"], batch=4, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 0, 300),
                       draft=("tree", (4, 4, 2, 2), 116))
    elif case == "chain128":
        cfg = W.scaled(C["c1_llama2_7b"], batch=3, n_q_heads=2, n_kv_heads=2, ctx=("uniform", 5, 200), draft=("linear", 128))
    elif case == "tree_small_d64":
        cfg = W.scaled(C["c0_tiny"], batch=6, n_q_heads=4, n_kv_heads=4, ctx=("uniform", 1, 90), draft=("tree", (3, 2, 2), 17))
    else:
        cfg = W.scaled(C["c1_llama2_7b"], batch=4, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 5, 200), draft=("linear", 7))
    a = W.make_attn_inputs(cfg, seed=3)
    stop = np.array([rng.integers(-1, int(k)) for k in a.st.n], dtype=np.int32)
    if case == "none_accepted":
        stop[:] = -1
    if case in ("tree64_d128", "tree116_d128", "chain128"):
        stop[0] = int(a.st.n[0]) - 1                     # a deepest leaf / the whole chain
    moved = run(mods, a, stop)
    assert moved == case.startswith("tree")


def test_compaction_after_acceptance(mods):
    """stop_node as spec_accept writes it, on the tree workload's shape (small batch)."""
    sv, runner = mods
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=4, n_q_heads=8, n_kv_heads=2, ctx=("fixed", 130), vocab=3000)
    a = W.make_attn_inputs(cfg, seed=11)
    ai = W.make_accept_inputs(cfg, seed=11, st=a.st)
    acc = runner.DeviceAccept(a.st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept, ai.u_resample)
    acc.run()
    torch.cuda.synchronize()
    ref = oracle.accept(a.st.node_offsets, a.st.parent, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                        ai.u_accept, ai.u_resample)
    assert not ref["near_tie"].any()                 # seeded case without near-ties: both walks stop at the same nodes
    # the GPU compaction reads the stop nodes spec_accept left on the device, the oracle its own
    run(mods, a, ref["stop_node"].astype(np.int32), stop_dev=acc.stop_node)
