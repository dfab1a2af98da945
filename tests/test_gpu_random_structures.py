"""GPU parity on randomly drawn draft structures: batches that mix empty requests, short drafts and drafts of
up to 128 nodes; trees whose parents lie anywhere below the node, deep narrow trees, heaps, chains; random
contexts.  Attention, stochastic acceptance (every launch path), greedy acceptance and the cache compaction
along the accepted path are each compared with the oracle on the same structure."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import ATTN_TOL, attn_rel_err, compare_accept, oracle_attn, ratio_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return binding, runner


def random_structure(rng, B, n_max, ctx_max, linear):
    n = np.array([rng.choice([0, 1, rng.integers(2, 65), rng.integers(65, n_max + 1), rng.integers(65, n_max + 1)])
                  for _ in range(B)], dtype=np.int64)
    if n.max() <= 64:
        n[0] = n_max
    off = np.zeros(B + 1, dtype=np.int32)
    off[1:] = np.cumsum(n)
    parent = None
    if not linear:
        ps = []
        for b in range(B):
            style = rng.integers(0, 3)
            for i in range(int(n[b])):
                if style == 0:
                    p = rng.integers(-1, i)                            # anywhere below the node
                elif style == 1:
                    p = max(-1, i - 1 - int(rng.integers(0, 4)))       # deep and narrow
                else:
                    p = (i - 1) // 3 - (0 if i > 3 else 1) if i >= 3 else -1      # a ternary heap under three roots
                ps.append(min(int(p), i - 1))
        parent = np.asarray(ps, dtype=np.int32)
    ctx = rng.integers(0, ctx_max + 1, size=B).astype(np.int32)
    return W.DraftStructure(n=n, node_offsets=off, parent=parent, ctx_len=ctx)


SHAPES = [(8, 2, 128), (4, 4, 128), (8, 1, 128), (4, 2, 64), (2, 2, 64)]      # (query heads, KV heads, head_dim)


@pytest.mark.parametrize("seed", [1, 7, 23, 41, 59])
def test_random_structures_match_oracle(mods, seed):
    sv, runner = mods
    rng = np.random.default_rng(seed)
    to_dev = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    for it in range(5):
        linear = it % 3 == 2
        B = int(rng.integers(2, 9))
        hq, hkv, D = SHAPES[(it + seed) % len(SHAPES)]
        V = int(rng.choice([777, 4096, 20000, 33000]))
        cfg = W.scaled(W.CONFIGS["c2_tree_llama3_8b"], name=f"random{seed}_{it}", batch=B, n_q_heads=hq, n_kv_heads=hkv,
                       head_dim=D, vocab=V, q_src=("noise", float(rng.choice([0.2, 0.8, 2.0]))))
        st = random_structure(rng, B, 128, int(rng.choice([60, 700, 5000])), linear)
        case = f"seed {seed} case {it}: B {B} heads {hq}/{hkv} D {D} V {V} linear {linear} n {st.n.tolist()} ctx {st.ctx_len.tolist()}"
        print(case, flush=True)

        a = W.make_attn_inputs(cfg, seed=it, st=st)
        ref, _ = oracle_attn(a)
        for hint in (0, int((st.ctx_len.astype(np.int64) + st.n).sum())):
            dev = runner.DeviceAttn(a, kv_hint=hint)
            dev.out.fill_(float("nan"))
            dev.run()
            torch.cuda.synchronize()
            got = dev.out.float().cpu().numpy()
            assert np.isfinite(got).all(), case
            assert attn_rel_err(got, ref) <= ATTN_TOL, case

        ai = W.make_accept_inputs(cfg, seed=it, st=st)
        want = oracle.accept(st.node_offsets, st.parent, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                             ai.u_accept, ai.u_resample, temperature=cfg.temperature)
        for path in (0, 1, 2, 3):
            acc = runner.DeviceAccept(st, ai.target_logits, ai.draft_q, ai.q_row, ai.draft_tokens, ai.u_accept,
                                      ai.u_resample, temperature=cfg.temperature)
            acc.workspace.fill_(0xEE)
            acc.run(tuning=sv.SpecAcceptTuning(path=path) if path else None)
            res = acc.results()
            bad, _, _ = compare_accept(res, want, st.n)
            assert not bad, f"{case}: path {path}, requests {bad}"
            assert ratio_err(res["ratio"], want["ratio"]) < 5e-6, case

        want_g = oracle.accept_greedy(st.node_offsets, st.parent, ai.draft_tokens, ai.target_logits)
        gr = runner.DeviceGreedy(st, ai.target_logits, ai.draft_tokens)
        gr.run()
        res_g = gr.results()
        for f in ("accept_len", "out_tokens", "stop_node"):
            assert np.array_equal(res_g[f], want_g[f]), f"{case}: greedy {f}"

        # compaction along the oracle's accepted paths (the GPU call never sees a value the GPU produced)
        k, v = runner.bf16_to_device(a.k_pool, "cuda"), runner.bf16_to_device(a.v_pool, "cuda")
        stop = want["stop_node"].astype(np.int32)
        new_len = torch.full((B,), -5, dtype=torch.int32, device="cuda")
        sv.spec_compact_kv(k, v, to_dev(a.block_table), to_dev(st.ctx_len), to_dev(st.node_offsets), to_dev(st.parent),
                           to_dev(stop), new_len)
        torch.cuda.synchronize()
        k2, v2 = a.k_pool.copy(), a.v_pool.copy()
        want_len = oracle.compact_kv(k2, v2, a.block_table, st.ctx_len, st.node_offsets, st.parent, stop)
        assert np.array_equal(k.view(torch.int16).cpu().numpy().view(np.uint16), k2), case
        assert np.array_equal(v.view(torch.int16).cpu().numpy().view(np.uint16), v2), case
        assert np.array_equal(new_len.cpu().numpy(), want_len), case
