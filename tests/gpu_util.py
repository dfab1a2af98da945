"""Helpers shared by the GPU parity tests: error metrics and oracle-vs-GPU comparison."""
import numpy as np

import oracle
from paper_2503_10325_amd import workloads as W

ATTN_TOL = 2e-2     # max relative error of attention outputs (bf16 inputs, fp32 accumulation)
TIE_EPS = 1e-6      # |ratio - u| (or |CDF - u|) below which a decision counts as a near-tie


def attn_rel_err(gpu_f32: np.ndarray, ref_f64: np.ndarray) -> float:
    """max |g - r| / max(|r|, 0.05 * rowmax|r|) over all (node, head) rows."""
    ref = np.asarray(ref_f64, dtype=np.float64)
    g = np.asarray(gpu_f32, dtype=np.float64)
    rowmax = np.abs(ref).max(axis=-1, keepdims=True)
    denom = np.maximum(np.abs(ref), 0.05 * rowmax)
    denom = np.where(denom == 0, 1.0, denom)
    return float((np.abs(g - ref) / denom).max())


def oracle_attn(a: W.AttnInputs):
    return oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets,
                              a.st.parent)


def compare_accept(gpu: dict, ref: dict, n: np.ndarray):
    """Bit-exact comparison of acceptance lengths and emitted tokens for every request the
    oracle did not flag as a near-tie.  Returns (n_mismatch_outside_ties, n_ties, n_requests)."""
    B = ref["accept_len"].shape[0]
    bad, ties = [], 0
    for b in range(B):
        if ref["near_tie"][b]:
            ties += 1
            continue
        k = int(ref["accept_len"][b])
        same = (int(gpu["accept_len"][b]) == k and
                np.array_equal(gpu["out_tokens"][b, :k + 1], ref["out_tokens"][b, :k + 1]) and
                int(gpu["stop_node"][b]) == int(ref["stop_node"][b]) and
                np.all(gpu["out_tokens"][b, k + 1:] == -1))
        if not same:
            bad.append(b)
    return bad, ties, B


def visited_pattern_agrees(gpu: dict, ref: dict, node_offsets: np.ndarray) -> bool:
    """The GPU visited (wrote a ratio for) exactly the nodes the oracle visited, in every request
    the oracle did not flag as a near-tie (after a near-tie the two walks may part ways)."""
    for b in range(ref["accept_len"].shape[0]):
        if ref["near_tie"][b]:
            continue
        o, e = int(node_offsets[b]), int(node_offsets[b + 1])
        if not np.array_equal(np.isnan(gpu["ratio"][o:e]), np.isnan(ref["ratio"][o:e])):
            return False
    return True


def ratio_err(gpu_ratio: np.ndarray, ref_ratio: np.ndarray) -> float:
    """Largest relative deviation of the compared ratios on nodes both walks visited (that the
    two visit the same nodes is checked by visited_pattern_agrees)."""
    vis = ~np.isnan(ref_ratio)
    r = ref_ratio[vis]
    g = gpu_ratio[vis].astype(np.float64)
    fin = np.isfinite(r) & (r > 0) & ~np.isnan(g)
    if not fin.any():
        return 0.0
    return float(np.max(np.abs(g[fin] - r[fin]) / r[fin]))
