"""Pins of the oracle's accepted-path KV compaction.  What fixes it: after compaction, a query that
attends causally over the first ctx + depth cache positions must see exactly what a query restricted
to the context plus the accepted path saw in the original tree layout (checked with the attention
oracle, which has its own pins); linear drafts are left untouched; positions outside the path's
destinations keep their contents; a hand-worked path."""
import numpy as np
import pytest

import oracle
from paper_2503_10325_amd import workloads as W

C = W.CONFIGS


def _case(seed, draft=("tree", (3, 2, 2), 15), batch=4):
    cfg = W.scaled(C["c2_tree_llama3_8b"], batch=batch, n_q_heads=4, n_kv_heads=2, ctx=("uniform", 3, 70), draft=draft)
    a = W.make_attn_inputs(cfg, seed=seed)
    rng = np.random.default_rng(seed)
    stop = np.array([rng.integers(-1, int(k)) for k in a.st.n], dtype=np.int32)
    return cfg, a, stop


def _path(parent, stop):
    p, a = [], int(stop)
    while a >= 0:
        p.append(a)
        a = int(parent[a]) if parent is not None else a - 1
    return p[::-1]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_attention_after_compaction_equals_attention_along_the_path(seed):
    cfg, a, stop = _case(seed)
    st = a.st
    B = cfg.batch
    # one probe query per request: in the tree layout it is a new node hanging below stop_node
    probe_q = W.f32_to_bf16_bits(np.random.default_rng(seed + 50).standard_normal((B, cfg.n_q_heads, cfg.head_dim)).astype(np.float32))
    want = np.zeros((B, cfg.n_q_heads, cfg.head_dim))
    for b in range(B):
        o, n = int(st.node_offsets[b]), int(st.n[b])
        par = st.parent[o:o + n]
        path = _path(par, stop[b])
        # ancestor chain expressed with a linear mask over [ctx, path nodes]: gather those K/V into a scratch cache
        L = int(st.ctx_len[b]) + len(path)
        pos = list(range(int(st.ctx_len[b]))) + [int(st.ctx_len[b]) + j for j in path]
        kp = np.zeros((-(-L // 16) + 1, cfg.n_kv_heads, 16, cfg.head_dim), dtype=np.uint16)
        vp = np.zeros_like(kp)
        for t, src in enumerate(pos):
            pg = a.block_table[b, src // 16]
            kp[t // 16, :, t % 16] = a.k_pool[pg, :, src % 16]
            vp[t // 16, :, t % 16] = a.v_pool[pg, :, src % 16]
        bt = np.arange(kp.shape[0], dtype=np.int32)[None, :]
        # one "draft" query with L - 1 context positions: it sees them plus its own slot L - 1, i.e. exactly
        # the first L cache positions
        out, _ = oracle.verify_attn(probe_q[b:b + 1], kp, vp, bt, np.array([L - 1], np.int32), np.array([0, 1], np.int32), None)
        want[b] = out[0]
    k2, v2 = a.k_pool.copy(), a.v_pool.copy()
    new_len = oracle.compact_kv(k2, v2, a.block_table, st.ctx_len, st.node_offsets, st.parent, stop)
    for b in range(B):
        depth = len(_path(st.parent[int(st.node_offsets[b]):int(st.node_offsets[b]) + int(st.n[b])], stop[b]))
        assert new_len[b] == st.ctx_len[b] + depth
        L = int(new_len[b])
        out, _ = oracle.verify_attn(probe_q[b:b + 1], k2, v2, a.block_table[b:b + 1], np.array([L - 1], np.int32),
                                    np.array([0, 1], np.int32), None)
        assert np.allclose(out[0], want[b], rtol=0, atol=1e-12)


def test_linear_drafts_and_rejected_everything_leave_the_cache_alone():
    cfg, a, stop = _case(3, draft=("linear", 6))
    k2, v2 = a.k_pool.copy(), a.v_pool.copy()
    oracle.compact_kv(k2, v2, a.block_table, a.st.ctx_len, a.st.node_offsets, None, stop)
    assert np.array_equal(k2, a.k_pool) and np.array_equal(v2, a.v_pool)
    cfg, a, stop = _case(4)
    stop[:] = -1
    k2, v2 = a.k_pool.copy(), a.v_pool.copy()
    new_len = oracle.compact_kv(k2, v2, a.block_table, a.st.ctx_len, a.st.node_offsets, a.st.parent, stop)
    assert np.array_equal(k2, a.k_pool) and np.array_equal(new_len, a.st.ctx_len)


def test_hand_worked_path_and_untouched_slots():
    cfg, a, stop = _case(5, batch=1)
    st = a.st
    # tree (3,2,2) breadth-first: nodes 0,1,2 under the prefix; 3,4 under 0; 5,6 under 1; 7,8 under 2; ...
    stop[0] = 8                                            # path: 2 -> 8
    ctx = int(st.ctx_len[0])
    k2, v2 = a.k_pool.copy(), a.v_pool.copy()
    oracle.compact_kv(k2, v2, a.block_table, st.ctx_len, st.node_offsets, st.parent, stop)

    def slot(pool, pos):
        return pool[a.block_table[0, pos // 16], :, pos % 16]

    assert np.array_equal(slot(k2, ctx + 0), slot(a.k_pool, ctx + 2))
    assert np.array_equal(slot(v2, ctx + 1), slot(a.v_pool, ctx + 8))
    changed = [p for p in range(ctx + int(st.n[0])) if not np.array_equal(slot(k2, p), slot(a.k_pool, p))]
    assert set(changed) <= {ctx, ctx + 1}
