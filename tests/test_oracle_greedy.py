"""Pins of the oracle's greedy verification (Section 6.1: greedy sampling for draft
generation and verification) against things other than itself: a hand-worked example,
numpy's argmax (first maximum) on rows full of ties, a brute-force Python walk over
random trees, and the zero-temperature limit of the already pinned stochastic walk
(one-hot drafts, sharply peaked target)."""
import numpy as np
import pytest

import oracle
from paper_2503_10325_amd import workloads as W


def bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_hand_worked_linear_example():
    # 3 drafts, V = 5.  Rows: after prefix -> argmax 2; after d0 -> 4; after d1 -> 0; after d2 -> 1.
    rows = np.array([[0, 1, 9, 3, 2],
                     [5, 1, 0, 3, 7],
                     [8, 1, 0, 3, 7],
                     [0, 6, 0, 3, 2]], dtype=np.float32)
    off = np.array([0, 3], dtype=np.int32)
    # drafts 2, 4 match; the third (3) does not: emitted = argmax of the row after d1 = 0
    r = oracle.accept_greedy(off, None, np.array([2, 4, 3], dtype=np.int32), bits(rows))
    assert r["accept_len"].tolist() == [2]
    assert r["out_tokens"][0].tolist() == [2, 4, 0, -1]
    assert r["stop_node"].tolist() == [1]
    assert r["row_argmax"].tolist() == [2, 4, 0, 1]
    # all three match: bonus token = argmax of the last row
    r = oracle.accept_greedy(off, None, np.array([2, 4, 0], dtype=np.int32), bits(rows))
    assert r["accept_len"].tolist() == [3] and r["out_tokens"][0].tolist() == [2, 4, 0, 1]
    # first draft wrong: nothing accepted, the prefix row's argmax is emitted
    r = oracle.accept_greedy(off, None, np.array([1, 4, 0], dtype=np.int32), bits(rows))
    assert r["accept_len"].tolist() == [0] and r["out_tokens"][0].tolist() == [2, -1, -1, -1]
    assert r["stop_node"].tolist() == [-1]


def test_hand_worked_tree_example():
    # nodes: 0,1 children of the prefix; 2,3 children of node 1.  Row after prefix -> 3.
    rows = np.zeros((5, 6), dtype=np.float32)
    rows[0, 3] = 1      # prefix      -> 3
    rows[1, 0] = 1      # after node 0 -> 0 (never visited)
    rows[2, 5] = 1      # after node 1 -> 5
    rows[3, 1] = 1      # after node 2
    rows[4, 2] = 1      # after node 3 -> 2
    off = np.array([0, 4], dtype=np.int32)
    par = np.array([-1, -1, 1, 1], dtype=np.int32)
    toks = np.array([4, 3, 0, 5], dtype=np.int32)       # second sibling matches at both levels
    r = oracle.accept_greedy(off, par, toks, bits(rows))
    assert r["accept_len"].tolist() == [2]
    assert r["out_tokens"][0, :3].tolist() == [3, 5, 2]
    assert r["stop_node"].tolist() == [3]


def test_row_argmax_is_first_maximum_with_ties():
    rng = np.random.default_rng(3)
    V, rows = 257, 40
    x = np.round(rng.standard_normal((rows, V)) * 2).astype(np.float32)     # few distinct values: many ties
    x[5] = 0.0                                                               # all equal -> index 0
    x[6, :] = -np.inf
    x[7, 0] = -0.0
    x[7, 1:] = 0.0                                                           # -0 == +0 -> index 0
    off = np.array([0, rows - 1], dtype=np.int32)
    toks = np.zeros(rows - 1, dtype=np.int32)
    for dt in (x, bits(x)):
        r = oracle.accept_greedy(off, None, toks, dt)
        assert np.array_equal(r["row_argmax"], np.argmax(x, axis=1))


def _python_walk(n, parent, toks, arg):
    cur, out = -1, []
    while True:
        g = int(arg[cur + 1])
        nxt = -1
        for c in range(n):
            pc = (c - 1) if parent is None else int(parent[c])
            if pc == cur and int(toks[c]) == g:
                nxt = c
                break
        out.append(g)
        if nxt < 0:
            return len(out) - 1, out, cur
        cur = nxt


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_trees_against_brute_force(seed):
    rng = np.random.default_rng(seed)
    B, V = 12, 7                                   # tiny vocabulary: matches are frequent
    n = rng.integers(0, 14, size=B)
    off = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(off[-1])
    parent = np.concatenate([[rng.integers(-1, j) for j in range(k)] for k in n if k > 0] or [[]]).astype(np.int32)
    toks = rng.integers(0, V, size=total).astype(np.int32)
    logits = bits(rng.standard_normal((total + B, V)))
    r = oracle.accept_greedy(off, parent, toks, logits)
    arg = np.argmax(W.bf16_bits_to_f32(logits), axis=1)
    for b in range(B):
        o, k = int(off[b]), int(n[b])
        depth, out, cur = _python_walk(k, parent[o:o + k], toks[o:o + k], arg[o + b:o + b + k + 1])
        assert r["accept_len"][b] == depth
        assert r["out_tokens"][b, :depth + 1].tolist() == out
        assert np.all(r["out_tokens"][b, depth + 1:] == -1)
        assert r["stop_node"][b] == cur


def test_linear_chain_equals_parent_none():
    rng = np.random.default_rng(9)
    B, k, V = 6, 5, 4
    off = (np.arange(B + 1) * k).astype(np.int32)
    toks = rng.integers(0, V, size=B * k).astype(np.int32)
    logits = bits(rng.standard_normal((B * (k + 1), V)))
    chain = np.tile(np.arange(-1, k - 1), B).astype(np.int32)
    a = oracle.accept_greedy(off, None, toks, logits)
    c = oracle.accept_greedy(off, chain, toks, logits)
    for key in a:
        assert np.array_equal(a[key], c[key]), key


def test_zero_temperature_limit_of_the_stochastic_walk():
    """With one-hot draft distributions (greedy drafting) and a target sharpened by a small
    temperature, the acceptance-rejection walk of Section 2.1 degenerates to the greedy rule on
    a linear draft: p(x)/q(x) is ~1 for the target's argmax and ~e^-20 otherwise; the residual
    and the bonus distribution are one-hot at the argmax.  The stochastic oracle has its own
    pins.  (Sibling drafts are left out: the stochastic sibling rule assumes i.i.d. draws from
    one q, which one-hot rows with different tokens are not.)"""
    rng = np.random.default_rng(5)
    B, V, T, n = 60, 24, 0.05, 6
    off = (np.arange(B + 1) * n).astype(np.int32)
    # target rows: distinct integers (gap >= 1, exact in bf16) in random order
    tl = np.stack([rng.permutation(V).astype(np.float32) for _ in range(B * (n + 1))])
    arg = np.argmax(tl, axis=1)
    toks = rng.integers(0, V, size=B * n).astype(np.int32)
    for b in range(B):                              # make matches likely
        for j in range(n):
            if rng.random() < 0.7:
                toks[b * n + j] = arg[b * (n + 1) + j]
    q = np.zeros((B * n, V), dtype=np.float32)
    q[np.arange(B * n), toks] = 1.0                # node j's own one-hot row
    q_row = np.arange(B * n, dtype=np.int32)
    u_acc = np.clip(W.uniforms24(rng, B * n), 1e-3, 1 - 1e-3).astype(np.float32)
    u_res = np.clip(W.uniforms24(rng, B), 1e-3, 1 - 1e-3).astype(np.float32)
    s = oracle.accept(off, None, toks, bits(tl), q, q_row, u_acc, u_res, temperature=T, qkind=oracle.Q_PROBS)
    g = oracle.accept_greedy(off, None, toks, bits(tl))
    assert g["accept_len"].max() >= 3 and g["accept_len"].min() == 0     # real descents and early stops
    for key in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(s[key], g[key]), key
