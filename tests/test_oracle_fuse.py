"""Pins of the oracle's confidence-based token fusion (Algorithm 1, TokenFusion; Eq. 4):
identity with one drafter, tie-breaking, permutation behaviour, and the MIXTURE
ensemble mode against a library softmax."""
import numpy as np
from scipy.special import softmax

import oracle
from paper_2503_10325_amd import workloads as W


def _inputs(seed=0, B=3, k=4, N=5, V=50):
    rng = np.random.default_rng(seed)
    conf = rng.random((B, k, N)).astype(np.float32)
    toks = rng.integers(0, V, size=(B, k, N)).astype(np.int32)
    logits = W.f32_to_bf16_bits((2 * rng.standard_normal((B * k * N, V))).astype(np.float32))
    k_len = np.array([k, k - 1, 1][:B], dtype=np.int32)
    return conf, toks, logits, k_len


def test_single_drafter_is_identity():
    conf, toks, logits, k_len = _inputs(N=1)
    r = oracle.fuse_drafts(k_len, conf, toks)
    for b in range(conf.shape[0]):
        kk = k_len[b]
        assert np.array_equal(r["fused_token"][b, :kk], toks[b, :kk, 0])
        assert np.all(r["winner"][b, :kk] == 0)
        assert np.array_equal(r["q_row"][b, :kk], b * conf.shape[1] + np.arange(kk))
        assert np.all(r["fused_token"][b, kk:] == -1) and np.all(r["q_row"][b, kk:] == -1)


def test_argmax_picks_highest_confidence_token():
    conf, toks, logits, k_len = _inputs(seed=1)
    B, k, N = conf.shape
    r = oracle.fuse_drafts(k_len, conf, toks)
    w = conf.argmax(-1)                                   # library argmax, first maximum
    for b in range(B):
        for i in range(k_len[b]):
            assert r["winner"][b, i] == w[b, i]
            assert r["fused_token"][b, i] == toks[b, i, w[b, i]]
            assert r["fused_token"][b, i] in toks[b, i]
            assert r["q_row"][b, i] == (b * k + i) * N + w[b, i]


def test_equal_confidences_choose_first_drafter():
    conf, toks, logits, k_len = _inputs(seed=2)
    conf[:] = 0.5
    r = oracle.fuse_drafts(k_len, conf, toks)
    for b in range(conf.shape[0]):
        assert np.all(r["winner"][b, :k_len[b]] == 0)


def test_permuting_drafters_permutes_winner_only():
    conf, toks, logits, k_len = _inputs(seed=3)
    perm = np.array([3, 0, 4, 1, 2])
    r0 = oracle.fuse_drafts(k_len, conf, toks)
    r1 = oracle.fuse_drafts(k_len, conf[..., perm].copy(), toks[..., perm].copy())
    valid = r0["winner"] >= 0
    assert np.array_equal(r0["fused_token"], r1["fused_token"])
    assert np.array_equal(perm[r1["winner"][valid]], r0["winner"][valid])


def test_mixture_against_library_softmax():
    conf, toks, logits, k_len = _inputs(seed=4)
    B, k, N = conf.shape
    V = logits.shape[1]
    T = 1.7
    r = oracle.fuse_drafts(k_len, conf, toks, logits, temperature=T, mode=oracle.FUSE_MIXTURE)
    lf = W.bf16_bits_to_f32(logits).astype(np.float64).reshape(B, k, N, V)
    sm = softmax(lf / T, axis=-1)
    w = conf.astype(np.float64) / conf.astype(np.float64).sum(-1, keepdims=True)
    ref = (w[..., None] * sm).sum(2).reshape(B * k, V)
    for b in range(B):
        for i in range(k):
            row = b * k + i
            if i < k_len[b]:
                assert np.abs(r["fused_probs"][row] - ref[row]).max() < 1e-14
                assert abs(r["fused_probs"][row].sum() - 1) < 1e-12
                assert r["q_row"][b, i] == row
            else:
                assert np.all(r["fused_probs"][row] == 0)


def test_mixture_with_one_hot_confidence_is_the_winners_distribution():
    conf, toks, logits, k_len = _inputs(seed=5)
    B, k, N = conf.shape
    V = logits.shape[1]
    hot = np.random.default_rng(0).integers(0, N, size=(B, k))
    conf[:] = 0
    np.put_along_axis(conf, hot[..., None], 1.0, axis=-1)
    r = oracle.fuse_drafts(k_len, conf, toks, logits, mode=oracle.FUSE_MIXTURE)
    lf = W.bf16_bits_to_f32(logits).astype(np.float64).reshape(B, k, N, V)
    for b in range(B):
        for i in range(k_len[b]):
            assert r["winner"][b, i] == hot[b, i]
            assert np.abs(r["fused_probs"][b * k + i] - softmax(lf[b, i, hot[b, i]])).max() < 1e-14
    # all-zero confidences: uniform weights
    conf[:] = 0
    r = oracle.fuse_drafts(k_len, conf, toks, logits, mode=oracle.FUSE_MIXTURE)
    assert np.abs(r["fused_probs"][0] - softmax(lf[0, 0], axis=-1).mean(0)).max() < 1e-14
