"""Pins of the oracle's LM-head projection (Section 3.1: verification on the target model is
dominated by matrix-matrix products; this is the product that yields the logits o_i) against
things other than itself: a hand-worked case, numpy's fp64 matmul, torch's float->bfloat16
conversion on sums that are exact integers (ties included), and scipy's logsumexp."""
import numpy as np
import torch
from scipy.special import logsumexp

import oracle
from paper_2503_10325_amd import workloads as W


def bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_hand_worked_case():
    h = bits([[1.0, 2.0]])
    w = bits([[3.0, 4.0], [-1.0, 0.5], [0.25, 0.0]])
    r = oracle.lm_head(h, w, temperature=2.0, want_exact=True)
    assert r["exact"].tolist() == [[11.0, 0.0, 0.25]]
    assert W.bf16_bits_to_f32(r["logits"]).tolist() == [[11.0, 0.0, 0.25]]
    assert r["row_max"].tolist() == [11.0]
    assert abs(r["row_z"][0] - (1.0 + np.exp(-11.0 / 2.0) + np.exp(-10.75 / 2.0))) < 1e-15


def test_products_against_numpy_matmul():
    rng = np.random.default_rng(0)
    rows, d, V = 13, 96, 37                      # all different: a transposed operand cannot pass
    h = bits(rng.standard_normal((rows, d)))
    w = bits(rng.standard_normal((V, d)) * 0.1)
    r = oracle.lm_head(h, w, want_exact=True)
    ref = W.bf16_bits_to_f32(h).astype(np.float64) @ W.bf16_bits_to_f32(w).astype(np.float64).T
    assert r["exact"].shape == (rows, V)
    assert np.max(np.abs(r["exact"] - ref)) < 1e-12
    # rounding: the stored logit is one of the two bf16 neighbours and the nearer one
    lg = W.bf16_bits_to_f32(r["logits"]).astype(np.float64)
    assert np.all(np.abs(lg - ref) <= np.abs(ref) * 2.0 ** -8)


def test_rounding_to_bf16_is_nearest_even_like_torch():
    rng = np.random.default_rng(1)
    rows, d, V = 9, 16, 300
    h = rng.integers(-8, 9, size=(rows, d)).astype(np.float32)
    w = rng.integers(-8, 9, size=(V, d)).astype(np.float32)
    # plant exact ties: 257 lies halfway between 256 and 258, 259 between 258 and 260
    h[0, :] = 0.0; h[0, 0] = 1.0
    w[0, 0], w[1, 0], w[2, 0], w[3, 0] = 257.0, 259.0, -257.0, -259.0
    hb, wb = bits(h), bits(w)
    exact = W.bf16_bits_to_f32(hb).astype(np.float64) @ W.bf16_bits_to_f32(wb).astype(np.float64).T
    assert np.all(exact == np.round(exact)) and np.abs(exact).max() < 2 ** 24      # exact in fp32 too
    r = oracle.lm_head(hb, wb)
    want = torch.from_numpy(exact.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(r["logits"], want)
    assert W.bf16_bits_to_f32(r["logits"])[0, :4].tolist() == [256.0, 260.0, -256.0, -260.0]


def test_row_statistics_against_logsumexp():
    rng = np.random.default_rng(2)
    rows, d, V = 7, 64, 1000
    h = bits(rng.standard_normal((rows, d)))
    w = bits(rng.standard_normal((V, d)) * 0.3)
    for T in (1.0, 0.7, 2.5):
        r = oracle.lm_head(h, w, temperature=T)
        lg = W.bf16_bits_to_f32(r["logits"]).astype(np.float64)
        assert np.array_equal(r["row_max"], lg.max(axis=1))
        assert np.allclose(np.log(r["row_z"]) + r["row_max"] / T, logsumexp(lg / T, axis=1), rtol=0, atol=1e-12)


def test_statistics_feed_the_acceptance_softmax():
    """exp((l - max)/T) / row_z is the target probability the acceptance step uses: it must equal the
    softmax of the same logits (scipy) entry by entry."""
    rng = np.random.default_rng(3)
    h = bits(rng.standard_normal((4, 32)))
    w = bits(rng.standard_normal((50, 32)))
    T = 0.9
    r = oracle.lm_head(h, w, temperature=T)
    lg = W.bf16_bits_to_f32(r["logits"]).astype(np.float64)
    p = np.exp((lg - r["row_max"][:, None]) / T) / r["row_z"][:, None]
    from scipy.special import softmax
    assert np.allclose(p, softmax(lg / T, axis=1), rtol=0, atol=1e-15)
