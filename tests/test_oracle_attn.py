"""Pins of the oracle's attention against things other than itself: a library SDPA
call on the causal special case, closed forms, and structural invariants
(tree/path equivalence, page-permutation invariance, the log-sum-exp merge identity).
The paper prints no worked numeric example for this step, so numeric parity with
the paper itself is unpinned; these pins fix the definition instead."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_10325_amd import workloads as W


def _rand_bits(rng, shape, sd=1.0):
    return W.f32_to_bf16_bits((sd * rng.standard_normal(shape)).astype(np.float32))


def _identity_cache(rng, B, L_tot, Hkv, D, page=16):
    """Per-request dense K/V [B, L_tot, Hkv, D] laid into a pool with an identity block table."""
    pages = (L_tot + page - 1) // page
    k = _rand_bits(rng, (B, pages * page, Hkv, D))
    v = _rand_bits(rng, (B, pages * page, Hkv, D))
    kp = k.reshape(B, pages, page, Hkv, D).transpose(0, 1, 3, 2, 4).reshape(B * pages, Hkv, page, D).copy()
    vp = v.reshape(B, pages, page, Hkv, D).transpose(0, 1, 3, 2, 4).reshape(B * pages, Hkv, page, D).copy()
    bt = np.arange(B * pages, dtype=np.int32).reshape(B, pages)
    return k, v, kp, vp, bt


def test_causal_case_matches_library_sdpa():
    rng = np.random.default_rng(1)
    B, n, Hq, Hkv, D, ctx = 2, 5, 4, 2, 32, 37
    L = ctx + n
    k, v, kp, vp, bt = _identity_cache(rng, B, L, Hkv, D)
    q = _rand_bits(rng, (B * n, Hq, D))
    qoff = np.arange(B + 1, dtype=np.int32) * n
    out, lse = oracle.verify_attn(q, kp, vp, bt, np.full(B, ctx), qoff)
    G = Hq // Hkv
    qt = torch.from_numpy(W.bf16_bits_to_f32(q).astype(np.float64)).reshape(B, n, Hq, D).permute(0, 2, 1, 3)
    kt = torch.from_numpy(W.bf16_bits_to_f32(k[:, :L]).astype(np.float64)).permute(0, 2, 1, 3).repeat_interleave(G, 1)
    vt = torch.from_numpy(W.bf16_bits_to_f32(v[:, :L]).astype(np.float64)).permute(0, 2, 1, 3).repeat_interleave(G, 1)
    mask = torch.zeros(n, L, dtype=torch.bool)
    for i in range(n):
        mask[i, :ctx + i + 1] = True
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask)
    ref = ref.permute(0, 2, 1, 3).reshape(B * n, Hq, D).numpy()
    assert np.abs(out - ref).max() < 1e-12
    # LSE against a library logsumexp of the same masked scores
    s = torch.einsum("bhid,bhtd->bhit", qt, kt) / np.sqrt(D)
    s = s.masked_fill(~mask, float("-inf"))
    ref_lse = torch.logsumexp(s, -1).permute(0, 2, 1).reshape(B * n, Hq).numpy()
    assert np.abs(lse - ref_lse).max() < 1e-12


def _ancestors(parent, i):
    a = []
    while i >= 0:
        a.append(i)
        i = int(parent[i])
    return a


def test_equal_keys_give_mean_of_allowed_values():
    """If every key is the same vector the softmax is uniform over the allowed set, so
    each output row is the plain mean of the allowed value rows (closed form)."""
    rng = np.random.default_rng(2)
    Hq = Hkv = 2
    D, ctx = 16, 21
    parent = W.tree_parents((3, 2, 2), 14)
    n = len(parent)
    L = ctx + n
    k, v, kp, vp, bt = _identity_cache(rng, 1, L, Hkv, D)
    kp[:] = kp[0, 0, 0][None, None, None, :]
    q = _rand_bits(rng, (n, Hq, D))
    out, _ = oracle.verify_attn(q, kp, vp, bt, [ctx], [0, n], parent)
    vf = W.bf16_bits_to_f32(v[0]).astype(np.float64)   # [L_pad, Hkv, D]
    for i in range(n):
        idx = list(range(ctx)) + [ctx + a for a in _ancestors(parent, i)]
        ref = vf[idx].mean(axis=0)
        assert np.abs(out[i] - ref).max() < 1e-13


def test_tree_node_equals_last_row_of_its_root_path():
    """Tree attention keeps causal dependencies: verifying node j inside the tree gives
    the row obtained by verifying the linear draft made of j's root-to-node path."""
    rng = np.random.default_rng(3)
    Hq, Hkv, D, ctx = 4, 2, 32, 45
    parent = W.tree_parents((2, 2, 2), 14)
    n = len(parent)
    L = ctx + n
    k, v, kp, vp, bt = _identity_cache(rng, 1, L, Hkv, D)
    q = _rand_bits(rng, (n, Hq, D))
    out_tree, lse_tree = oracle.verify_attn(q, kp, vp, bt, [ctx], [0, n], parent)
    for j in range(n):
        path = _ancestors(parent, j)[::-1]
        m = len(path)
        k2, v2 = k.copy(), v.copy()
        for pos, a in enumerate(path):
            k2[0, ctx + pos] = k[0, ctx + a]
            v2[0, ctx + pos] = v[0, ctx + a]
        pages = k2.shape[1] // 16
        kp2 = k2.reshape(1, pages, 16, Hkv, D).transpose(0, 1, 3, 2, 4).reshape(pages, Hkv, 16, D).copy()
        vp2 = v2.reshape(1, pages, 16, Hkv, D).transpose(0, 1, 3, 2, 4).reshape(pages, Hkv, 16, D).copy()
        out_lin, lse_lin = oracle.verify_attn(q[path], kp2, vp2, bt, [ctx], [0, m], None)
        assert np.abs(out_lin[-1] - out_tree[j]).max() < 1e-12
        assert np.abs(lse_lin[-1] - lse_tree[j]).max() < 1e-12


def test_chain_shaped_tree_equals_linear_mask():
    rng = np.random.default_rng(4)
    cfg = W.scaled(W.CONFIGS["c1_llama2_7b"], batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32,
                   ctx=("fixed", 50), draft=("linear", 5), vocab=64)
    a = W.make_attn_inputs(cfg, seed=7)
    chain = np.tile(np.arange(-1, 4, dtype=np.int32), 2)
    o1, l1 = oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets, None)
    o2, l2 = oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets, chain)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_pool_page_permutation_is_invisible():
    cfg = W.scaled(W.CONFIGS["c2_tree_llama3_8b"], batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32,
                   ctx=("fixed", 70), draft=("tree", (2, 2), 6), vocab=64)
    a = W.make_attn_inputs(cfg, seed=5)
    o1, _ = oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets, a.st.parent)
    perm = np.random.default_rng(9).permutation(a.num_pages)
    inv = np.argsort(perm)
    kp2, vp2 = a.k_pool[perm], a.v_pool[perm]          # new page i holds old page perm[i]
    bt2 = np.where(a.block_table >= 0, inv[np.maximum(a.block_table, 0)], -1).astype(np.int32)
    o2, _ = oracle.verify_attn(a.q, kp2, vp2, bt2, a.st.ctx_len, a.st.node_offsets, a.st.parent)
    assert np.array_equal(o1, o2)


def test_single_query_is_plain_decode_attention():
    rng = np.random.default_rng(6)
    Hq = Hkv = 3
    D, ctx = 16, 29
    k, v, kp, vp, bt = _identity_cache(rng, 1, ctx + 1, Hkv, D)
    q = _rand_bits(rng, (1, Hq, D))
    out, lse = oracle.verify_attn(q, kp, vp, bt, [ctx], [0, 1])
    qf = W.bf16_bits_to_f32(q).astype(np.float64)[0]
    kf = W.bf16_bits_to_f32(k[0, :ctx + 1]).astype(np.float64)
    vf = W.bf16_bits_to_f32(v[0, :ctx + 1]).astype(np.float64)
    for h in range(Hq):
        s = kf[:, h] @ qf[h] / np.sqrt(D)
        w = np.exp(s - s.max())
        ref = (w[:, None] * vf[:, h]).sum(0) / w.sum()
        assert np.abs(out[0, h] - ref).max() < 1e-13
        assert abs(lse[0, h] - (s.max() + np.log(w.sum()))) < 1e-12


def test_lse_merge_identity():
    """Attention over A u B equals the merge of attention over A and over B weighted by
    exp(lse): the identity a split-KV implementation relies on."""
    rng = np.random.default_rng(8)
    Hq = Hkv = 2
    D, ctxA, ctxB = 16, 32, 27
    k, v, kp, vp, bt = _identity_cache(rng, 1, ctxA + ctxB + 1, Hkv, D)
    q = _rand_bits(rng, (1, Hq, D))
    # whole: context A+B then the query's own position
    o_all, l_all = oracle.verify_attn(q, kp, vp, bt, [ctxA + ctxB], [0, 1])
    # part A: pages 0..1 (32 tokens) with k=1 whose own K/V is token ctxA-1 of A
    oA, lA = oracle.verify_attn(q, kp, vp, bt, [ctxA - 1], [0, 1])
    # part B: the remaining pages, own token is the true query position
    btB = bt[:, 2:].copy()
    oB, lB = oracle.verify_attn(q, kp, vp, btB, [ctxB], [0, 1])
    wA, wB = np.exp(lA - l_all), np.exp(lB - l_all)
    assert np.abs(wA + wB - 1).max() < 1e-12
    merged = wA[..., None] * oA + wB[..., None] * oB
    assert np.abs(merged - o_all).max() < 1e-12


def test_planted_transpose_would_be_caught():
    """Sanity of the pin itself: swapping K and V pools changes the result by far more
    than the tolerance used above."""
    rng = np.random.default_rng(10)
    k, v, kp, vp, bt = _identity_cache(rng, 1, 40, 1, 16)
    q = _rand_bits(rng, (2, 1, 16))
    o1, _ = oracle.verify_attn(q, kp, vp, bt, [38], [0, 2])
    o2, _ = oracle.verify_attn(q, vp, kp, bt, [38], [0, 2])
    assert np.abs(o1 - o2).max() > 1e-3
