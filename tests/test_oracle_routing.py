"""Pins of the oracle's routing-score update (Section 4.1, Eq. 1 and Eq. 2) against closed forms and
library routines: identical tokens (d = 1), orthogonal one-hot embeddings (d in {0, 1}), 2-D
embeddings at a known angle with c = 1 - cos(angle) (every term is exactly 1/2), the acceptance-length
cut-off, scipy's cosine distance on random rows, scale invariance, and the readings for negative
cosines, zero rows and the 0/0 corners."""
import numpy as np
import pytest
from scipy.spatial.distance import cosine as cosine_distance

import oracle
from paper_2503_10325_amd import workloads as W


def case(B=3, K=4, N=2, V=11, E=8, seed=0):
    rng = np.random.default_rng(seed)
    emb = rng.standard_normal((V, E)).astype(np.float32)
    conf = rng.uniform(0.05, 0.95, size=(B, K, N)).astype(np.float32)
    toks = rng.integers(0, V, size=(B, K, N)).astype(np.int32)
    out = rng.integers(0, V, size=(B, K + 1)).astype(np.int32)
    acc = rng.integers(0, K + 1, size=B).astype(np.int32)
    k_len = np.full(B, K, dtype=np.int32)
    return k_len, conf, toks, acc, out, emb


def test_identical_tokens_give_accept_fraction():
    k_len, conf, toks, acc, out, emb = case()
    for b in range(toks.shape[0]):
        toks[b, :, :] = out[b, :toks.shape[1], None]          # every drafter proposed the accepted token
    m = oracle.routing_scores(k_len, conf, toks, acc, out, emb)
    # d = 1 on accepted positions: c / (c + 0) = 1; d = 0 elsewhere: 0
    assert np.allclose(m, (acc / k_len)[:, None], atol=1e-12)


def test_one_hot_embeddings_count_matches():
    k_len, conf, toks, acc, out, _ = case(V=9, E=9, seed=1)
    emb = np.eye(9, dtype=np.float32)
    m = oracle.routing_scores(k_len, conf, toks, acc, out, emb)
    B, K, N = toks.shape
    for b in range(B):
        for n in range(N):
            hits = sum(1 for i in range(K) if i < acc[b] and toks[b, i, n] == out[b, i])
            assert m[b, n] == pytest.approx(hits / K, abs=1e-12)


def test_known_angle_gives_one_half_per_term():
    # token 0 -> (1, 0); token t -> (cos a_t, sin a_t); with c = 1 - cos a_t the term is
    # c d / (c d + (1-c)(1-d)) = (1-d) d / ((1-d) d + d (1-d)) = 1/2.
    angles = np.array([0.3, 0.7, 1.1, 1.4])
    emb = np.zeros((5, 2), dtype=np.float32)
    emb[0] = (1, 0)
    emb[1:, 0], emb[1:, 1] = np.cos(angles), np.sin(angles)
    K, N = 4, 1
    toks = np.arange(1, 5, dtype=np.int32).reshape(1, K, N)
    d = (emb[1:] @ emb[0]).astype(np.float64) / np.linalg.norm(emb[1:].astype(np.float64), axis=1)
    conf = (1.0 - d).astype(np.float32).reshape(1, K, N)
    out = np.zeros((1, K + 1), dtype=np.int32)
    for L in range(K + 1):
        m = oracle.routing_scores([K], conf, toks, [L], out, emb)
        assert m[0, 0] == pytest.approx(0.5 * L / K, abs=2e-7)      # conf is fp32


def test_matches_scipy_cosine_and_formula_on_random_rows():
    k_len, conf, toks, acc, out, emb = case(B=5, K=6, N=3, V=40, E=33, seed=3)
    k_len[1] = 4
    acc[1] = min(acc[1], 4)
    m = oracle.routing_scores(k_len, conf, toks, acc, out, W.f32_to_bf16_bits(emb))
    e = W.bf16_bits_to_f32(W.f32_to_bf16_bits(emb)).astype(np.float64)
    for b in range(5):
        for n in range(3):
            tot = 0.0
            for i in range(int(k_len[b])):
                d = 0.0
                if i < acc[b]:
                    d = max(0.0, 1.0 - cosine_distance(e[out[b, i]], e[toks[b, i, n]]))
                c = float(conf[b, i, n])
                tot += c * d / (c * d + (1 - c) * (1 - d))
            assert m[b, n] == pytest.approx(tot / k_len[b], rel=1e-12, abs=1e-14)


def test_scale_invariance_and_symmetry_in_c_and_d():
    k_len, conf, toks, acc, out, emb = case(seed=4)
    m1 = oracle.routing_scores(k_len, conf, toks, acc, out, emb)
    scaled = (emb * np.linspace(0.5, 8.0, emb.shape[0], dtype=np.float32)[:, None]).astype(np.float32)
    m2 = oracle.routing_scores(k_len, conf, toks, acc, out, scaled)
    assert np.allclose(m1, m2, atol=1e-6)                  # cosine ignores row norms (fp32 rounding of the scaling)
    # Eq. 2 is symmetric in (c, d): with 2-D unit embeddings, swapping confidence and cosine keeps the term
    a = 0.9
    emb2 = np.array([[1, 0], [np.cos(a), np.sin(a)], [0.25, np.sqrt(1 - 0.25 ** 2)]], dtype=np.float32)
    d1 = float(emb2[1, 0])                                  # cos of token 1 against token 0
    out2 = np.zeros((1, 2), dtype=np.int32)
    x = oracle.routing_scores([1], np.array([[[0.25]]], np.float32), np.array([[[1]]], np.int32), [1], out2, emb2)
    y = oracle.routing_scores([1], np.array([[[d1]]], np.float32), np.array([[[2]]], np.int32), [1], out2, emb2)
    assert x[0, 0] == pytest.approx(y[0, 0], abs=1e-6)


def test_readings_of_the_unspecified_corners():
    emb = np.array([[1, 0], [-1, 0], [0, 0], [0, 1]], dtype=np.float32)
    out = np.zeros((1, 5), dtype=np.int32)                   # accepted token 0 everywhere
    toks = np.array([1, 2, 3, 0], dtype=np.int32).reshape(1, 4, 1)
    conf = np.array([0.6, 0.6, 1.0, 0.0], dtype=np.float32).reshape(1, 4, 1)
    m = oracle.routing_scores([4], conf, toks, [4], out, emb)
    # opposite row: cosine -1 counts as 0; zero row: cosine 0; (c=1, d=0): 0/0 -> 0; (c=0, d=1): 0/0 -> 0
    assert m[0, 0] == 0.0
    assert oracle.routing_scores([0], conf, toks, [0], out, emb)[0, 0] == 0.0      # K = 0
