"""GPU parity of the LM-head projection fused with the row statistics (spec_lm_head, through the
C ABI) against the CPU oracle, and of the acceptance step that starts from those statistics
(spec_accept_prestats) against spec_accept and the oracle's walk on the same logits.

Tolerances.  The kernel accumulates in fp32, the oracle in fp64, both round once to bf16:
  |gpu - exact| <= 2^-8 |exact|  (half a bf16 step)  +  1e-5 * sum_k |h_k w_k|  (fp32 accumulation,
  far above the sqrt(K) 2^-24 growth observed),
and the two roundings may fall on different sides only when the exact value sits within the
accumulation error of a rounding boundary: fewer than 0.5 % of the entries.  Statistics against the
ORACLE's row_max / row_z: with p, p' the softmax of the oracle's and of the kernel's row and
dl_v = l'_v - l_v (non-zero only on those boundary entries), convexity of log-sum-exp gives
  sum_v p_v dl_v / T  <=  LSE' - LSE  <=  sum_v p'_v dl_v / T,
so |LSE' - LSE| <= sum_v max(p_v, p'_v) |dl_v| / T =: lse_bound(row), evaluated from the two logit
arrays the test holds, plus 3e-6 for the kernel's fp32 exp2 and fp32 partial sums (at most 128
terms each; the segment sums are fp64).  The row maximum can differ from the oracle's only if the
largest entries themselves are boundary entries: |M' - M| <= max_v |dl_v|.  As a second, size-free
property the segment statistics are also checked against an fp64 evaluation of the kernel's own
logits (exact maximum, sums to 3e-6)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import compare_accept, ratio_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def merged(m, z, T):
    """Row maximum and row sum of exp((l - max)/T) from per-segment statistics (fp64)."""
    M = m.max(axis=1).astype(np.float64)
    Z = (z * np.exp((m.astype(np.float64) - M[:, None]) / T)).sum(axis=1)
    return M, Z


def lse_bound(got_rows, ref_rows, T):
    """Per-row bound on |LSE(kernel's row) - LSE(oracle's row)| from the two logit arrays (fp64)."""
    d = np.abs(got_rows - ref_rows)
    out = np.zeros(got_rows.shape[0])
    for i in range(got_rows.shape[0]):
        idx = np.nonzero(d[i])[0]
        if idx.size == 0:
            continue
        pg = np.exp((got_rows[i, idx] - got_rows[i].max()) / T) / np.exp((got_rows[i] - got_rows[i].max()) / T).sum()
        pr = np.exp((ref_rows[i, idx] - ref_rows[i].max()) / T) / np.exp((ref_rows[i] - ref_rows[i].max()) / T).sum()
        out[i] = (np.maximum(pg, pr) * d[i, idx]).sum() / T
    return out


def check_row_stats_against_oracle(M, Z, got, ref, rsel, T):
    """Merged (max, log Z) of the kernel's rows `rsel` against the oracle's row_max / row_z.
    `got` holds the kernel's logits of those rows (fp64), `ref` the oracle's result for them."""
    ref_rows = W.bf16_bits_to_f32(ref["logits"]).astype(np.float64)
    dmax = np.abs(got - ref_rows).max(axis=1)
    assert np.all(np.abs(M[rsel] - ref["row_max"]) <= dmax), "row maximum"
    lse_gpu = np.log(Z[rsel]) + M[rsel] / T
    lse_ref = np.log(ref["row_z"]) + ref["row_max"] / T
    bound = lse_bound(got, ref_rows, T) + 3e-6
    excess = np.abs(lse_gpu - lse_ref) - bound
    assert np.all(excess <= 0), f"log-sum-exp: worst excess {excess.max():.3e} (bound up to {bound.max():.3e})"


def check_lm_head(rt, rows, d_model, V, T, seed=0):
    li = W.make_lm_head_inputs(rows, d_model, V, seed=seed)
    ref = oracle.lm_head(li.hidden, li.weight, temperature=T, want_exact=True)
    dev = rt.DeviceLmHead(li, temperature=T)
    dev.logits.fill_(float("nan"))
    dev.run()
    got_bits = dev.logits_bits()
    got = W.bf16_bits_to_f32(got_bits).astype(np.float64)
    assert np.isfinite(got).all()
    absprod = np.abs(W.bf16_bits_to_f32(li.hidden)).astype(np.float64) @ np.abs(W.bf16_bits_to_f32(li.weight)).astype(np.float64).T
    tol = np.abs(ref["exact"]) * 2.0 ** -8 + 1e-5 * absprod
    err = np.abs(got - ref["exact"])
    assert np.all(err <= tol), f"worst excess {np.max(err - tol)}"
    mismatch = np.mean(got_bits != ref["logits"])
    assert mismatch < 5e-3, mismatch
    # statistics: exact maximum of the kernel's own logits, sums against fp64 on the same logits
    m, z = dev.segment_stats()
    nseg = (V + 8191) // 8192
    for s in range(nseg):
        seg = got[:, s * 8192:(s + 1) * 8192]
        assert np.array_equal(m[:, s].astype(np.float64), seg.max(axis=1)), f"segment {s} maximum"
        zr = np.exp((seg - seg.max(axis=1, keepdims=True)) / T).sum(axis=1)
        assert np.max(np.abs(z[:, s] - zr) / zr) < 3e-6, f"segment {s} sum"
    M, Z = merged(m, z, T)
    check_row_stats_against_oracle(M, Z, got, ref, np.arange(rows), T)
    return mismatch


@pytest.mark.parametrize("rows,d_model,V,T", [
    (70, 256, 3000, 1.0),        # ragged row tile, ragged vocabulary block
    (5, 128, 1001, 1.0),         # one slice per half, odd vocabulary (scalar stores)
    (200, 512, 8300, 0.7),       # more than 128 rows: packed hidden states, last wave with one row tile
    (300, 256, 1500, 1.0),       # two row blocks of 256, the second with 44 rows (three waves without rows)
    (128, 1024, 16384, 1.3),     # full tiles everywhere
    (1, 128, 130, 1.0),          # a single row, a second vocabulary block of two entries
])
def test_lm_head_matches_oracle(rt, rows, d_model, V, T):
    mismatch = check_lm_head(rt, rows, d_model, V, T)
    print(f"rows {rows} d {d_model} V {V}: bf16 neighbours chosen differently in {mismatch:.2e} of the entries")


@pytest.mark.parametrize("rows", [127, 128, 129, 255, 256, 257, 511, 512, 513, 520, 544, 545, 600])
def test_lm_head_row_count_boundaries(rt, rows):
    """Row counts around every switch of kernel, prefetch depth and row block (128, 256, 512; a last
    block of up to 32 rows splits the contraction over the waves), with a vocabulary that ends inside
    a tile."""
    check_lm_head(rt, rows, 128, 300, 1.0, seed=rows)


@pytest.mark.parametrize("rows,d_model", [(530, 1024), (1040, 640), (1025, 2048)])
def test_lm_head_split_contraction_tail(rt, rows, d_model):
    """Last row block of 18 / 16 / 1 rows with 16 / 10 / 32 slices: every wave has slices, some waves
    have one more than others, and 4 per wave."""
    check_lm_head(rt, rows, d_model, 700, 0.8, seed=rows + d_model)


def test_lm_head_is_deterministic_and_leaves_neighbours_alone(rt):
    li = W.make_lm_head_inputs(37, 384, 2500, seed=3)
    dev = rt.DeviceLmHead(li)
    guard = torch.full((64,), 7, dtype=torch.uint8, device="cuda")
    dev.run()
    a = dev.logits_bits().copy()
    sa = dev.stats.cpu().numpy().copy()
    dev.logits.zero_()
    dev.run()
    assert np.array_equal(a, dev.logits_bits())
    assert np.array_equal(sa, dev.stats.cpu().numpy())
    assert bool((guard == 7).all())


def pipeline_agrees(got, ref, st, toks, gpu_bits, ref_bits, max_disagree=1):
    """The GPU pipeline (spec_lm_head -> acceptance) against the oracle's (oracle.lm_head ->
    oracle.accept), both fed the same host inputs.  The two sets of logits are bf16 neighbours in
    about one entry in ten thousand; a request none of whose drafted (row, token) logits is such an
    entry must decide exactly as the oracle does (outside the oracle's near-ties), and at most
    ``max_disagree`` requests may contain one."""
    disagree = []
    for b in range(len(st.n)):
        o, n = int(st.node_offsets[b]), int(st.n[b])
        for j in range(n):
            par = j - 1 if st.parent is None else int(st.parent[o + j])
            r = o + b + 1 + par
            if gpu_bits[r, toks[o + j]] != ref_bits[r, toks[o + j]]:
                disagree.append(b)
                break
    bad, ties, B = compare_accept(got, ref, st.n)
    assert set(bad) <= set(disagree), (bad, disagree)
    assert len(disagree) <= max_disagree
    return ties


def test_accept_from_lm_head_statistics(rt):
    """hidden x weight -> logits + statistics (one kernel family), then the walk from those
    statistics.  Reference: the oracle's own pipeline on the same host inputs.  The prestats entry
    must also decide exactly like spec_accept on the same device logits."""
    T = 0.9
    cfg = W.scaled(W.CONFIGS["c1_llama2_7b"], batch=10, vocab=9000, draft=("linear_uniform", 2, 7), temperature=T)
    st = W.make_structure(cfg, seed=1)
    rows = st.total + cfg.batch
    li = W.make_lm_head_inputs(rows, 512, cfg.vocab, seed=1)
    tl = oracle.lm_head(li.hidden, li.weight, temperature=T)["logits"]
    # drafts: node j of request b is drawn from a noisy copy of the target row it will be compared with
    rng = np.random.default_rng(5)
    q = np.zeros((st.total, cfg.vocab), dtype=np.uint16)
    toks = np.zeros(st.total, dtype=np.int32)
    for b in range(cfg.batch):
        o = int(st.node_offsets[b])
        for j in range(int(st.n[b])):
            x = W.bf16_bits_to_f32(tl[o + b + j]) + np.float32(0.7) * rng.standard_normal(cfg.vocab).astype(np.float32)
            q[o + j] = W.f32_to_bf16_bits(x)
            toks[o + j] = int(np.argmax(W.bf16_bits_to_f32(q[o + j]) / T + rng.gumbel(size=cfg.vocab)))
    q_row = np.arange(st.total, dtype=np.int32)
    u_acc = W.uniforms24(rng, st.total)
    u_res = W.uniforms24(rng, cfg.batch)
    ref = oracle.accept(st.node_offsets, None, toks, tl, q, q_row, u_acc, u_res, temperature=T, qkind=0)

    ws = torch.zeros(rt.sv.spec_accept_workspace_size(cfg.batch, st.total, st.total, cfg.vocab), dtype=torch.uint8,
                     device="cuda")
    head = rt.DeviceLmHead(li, temperature=T, stats=ws)
    head.run()
    pre = rt.DeviceAccept(st, head.logits, q, q_row, toks, u_acc, u_res, temperature=T)
    pre.workspace = ws
    pre.run_prestats()
    got_pre = pre.results()
    plain = rt.DeviceAccept(st, head.logits, q, q_row, toks, u_acc, u_res, temperature=T)
    plain.run()
    got_plain = plain.results()

    ties = pipeline_agrees(got_pre, ref, st, toks, head.logits_bits(), tl)
    assert ties <= 2
    assert ref["accept_len"].max() >= 2 and ref["accept_len"].min() < st.n.max()
    # fused statistics against a second pass over the same device logits: same walk
    for key in ("accept_len", "out_tokens", "stop_node"):
        assert np.array_equal(got_pre[key], got_plain[key]), key
    assert ratio_err(got_pre["ratio"], got_plain["ratio"].astype(np.float64)) < 5e-6


def test_accept_prestats_with_probability_rows(rt):
    """Draft rows given as probabilities need no statistics of their own: the prestats entry then
    only clears the walk's exchange words."""
    T = 1.0
    cfg = W.scaled(W.CONFIGS["c1_llama2_7b"], batch=4, vocab=2048, draft=("linear", 3))
    st = W.make_structure(cfg, seed=2)
    rows = st.total + cfg.batch
    li = W.make_lm_head_inputs(rows, 256, cfg.vocab, seed=2)
    tl = oracle.lm_head(li.hidden, li.weight, temperature=T)["logits"]
    rng = np.random.default_rng(6)
    qp = rng.dirichlet(np.full(cfg.vocab, 0.05), size=st.total).astype(np.float32)
    toks = np.array([rng.choice(cfg.vocab, p=qp[j].astype(np.float64) / qp[j].astype(np.float64).sum())
                     for j in range(st.total)], dtype=np.int32)
    q_row = np.arange(st.total, dtype=np.int32)
    u_acc, u_res = W.uniforms24(rng, st.total), W.uniforms24(rng, cfg.batch)
    ref = oracle.accept(st.node_offsets, None, toks, tl, qp, q_row, u_acc, u_res, temperature=T, qkind=1)

    ws = torch.zeros(rt.sv.spec_accept_workspace_size(cfg.batch, st.total, st.total, cfg.vocab), dtype=torch.uint8,
                     device="cuda")
    ws.fill_(0xAB)                                   # stale bytes: everything the walk reads must be rewritten
    head = rt.DeviceLmHead(li, temperature=T, stats=ws)
    head.run()
    dev = rt.DeviceAccept(st, head.logits, qp, q_row, toks, u_acc, u_res, temperature=T, q_kind=1)
    dev.workspace = ws
    dev.run_prestats()
    assert pipeline_agrees(dev.results(), ref, st, toks, head.logits_bits(), tl) <= 1


def own_logits_stats_agree(dev, V, T):
    """Every row's segment statistics against an fp64 evaluation of the kernel's own logits
    (library reductions on the device: a property that holds at any size)."""
    m, z = dev.segment_stats()
    lg = dev.logits.double()
    assert torch.isfinite(lg).all()
    nseg = (V + 8191) // 8192
    for s in range(nseg):
        seg = lg[:, s * 8192:(s + 1) * 8192]
        mx = seg.max(dim=1).values
        zr = torch.exp((seg - mx[:, None]) / T).sum(dim=1)
        assert np.array_equal(m[:, s].astype(np.float64), mx.cpu().numpy()), f"segment {s} maximum"
        assert np.max(np.abs(z[:, s] - zr.cpu().numpy()) / zr.cpu().numpy()) < 3e-6, f"segment {s} sum"
    return m, z


@pytest.mark.parametrize("rows,d_model,V", [
    (72, 4096, 32000),         # c1's target rows on the Llama-2-7B head: the weight-read-bound kernel
    (224, 4096, 32000),        # c3's target rows: the wide kernel with the weights four slices ahead
])
def test_lm_head_full_size_whole_matrix(rt, rows, d_model, V):
    """Benchmark shapes of the 32000-entry heads, in the launch configuration bench.py times: every
    logit and every row's statistics against the oracle."""
    mismatch = check_lm_head(rt, rows, d_model, V, 1.0, seed=7)
    print(f"rows {rows} d {d_model} V {V}: whole matrix, neighbours chosen differently in {mismatch:.2e}")


@pytest.mark.parametrize("rows,d_model,V", [
    (1040, 4096, 128256),      # c2's target rows on the Llama-3-8B head: packed hidden states, 512-row blocks
    (429, 8192, 128256),       # c4's target rows on the Llama-70B head (d_model 8192)
])
def test_lm_head_full_size_rows_and_columns(rt, rows, d_model, V):
    """Benchmark shapes of the 128256-entry heads.  The oracle computes (a) whole rows - the first and
    last row of every 32-row tile border, of every 128-, 256- and 512-row block border and random ones,
    at least 32 - whose logits AND merged statistics are compared with the oracle's, and (b) 512 whole
    vocabulary columns - tile and segment borders, the ragged end, random ones - for ALL rows."""
    T = 1.0
    li = W.make_lm_head_inputs(rows, d_model, V, seed=7)
    dev = rt.DeviceLmHead(li, temperature=T)
    dev.logits.fill_(float("nan"))
    dev.run()
    got_bits = dev.logits_bits()
    rng = np.random.default_rng(11)
    border = [0, 31, 32, 63, 64, 127, 128, 255, 256, 257, 511, 512, 513, 543, 544, 1023, 1024, 1039,
              rows - 33, rows - 32, rows - 17, rows - 16, rows - 2, rows - 1]
    rsel = sorted(set([r for r in border if 0 <= r < rows] + rng.integers(0, rows, size=32).tolist()))
    assert len(rsel) >= 32
    vborder = [0, 1, 31, 32, 127, 128, 8191, 8192, 65535, 65536, V - 257, V - 256, V - 129, V - 128, V - 2, V - 1]
    vsel = sorted(set(vborder + rng.integers(0, V, size=520).tolist()))[:512 + len(vborder)]
    assert len(vsel) >= 512
    hid = W.bf16_bits_to_f32(li.hidden).astype(np.float64)
    wgt_abs_sel = np.abs(W.bf16_bits_to_f32(li.weight[vsel])).astype(np.float64)

    # (a) whole rows: logits and statistics against the oracle
    ref = oracle.lm_head(li.hidden[rsel], li.weight, temperature=T, want_exact=True)
    got = W.bf16_bits_to_f32(got_bits[rsel]).astype(np.float64)
    absprod = np.zeros_like(got)
    habs = np.abs(hid[rsel]).astype(np.float32)
    for v0 in range(0, V, 16384):                       # fp32 is plenty for a tolerance term
        absprod[:, v0:v0 + 16384] = habs @ np.abs(W.bf16_bits_to_f32(li.weight[v0:v0 + 16384])).T
    tol = np.abs(ref["exact"]) * 2.0 ** -8 + 1e-5 * absprod
    assert np.all(np.abs(got - ref["exact"]) <= tol), "whole rows"
    mis_rows = np.mean(got_bits[rsel] != ref["logits"])
    assert mis_rows < 5e-3, mis_rows
    m, z = own_logits_stats_agree(dev, V, T)
    M, Z = merged(m, z, T)
    check_row_stats_against_oracle(M, Z, got, ref, np.array(rsel), T)

    # (b) whole columns for every row
    refc = oracle.lm_head(li.hidden, li.weight[vsel], temperature=T, want_exact=True)
    gotc = W.bf16_bits_to_f32(got_bits[:, vsel]).astype(np.float64)
    tolc = np.abs(refc["exact"]) * 2.0 ** -8 + 1e-5 * (np.abs(hid) @ wgt_abs_sel.T)
    assert np.all(np.abs(gotc - refc["exact"]) <= tolc), "whole columns"
    mis_cols = np.mean(got_bits[:, vsel] != refc["logits"])
    assert mis_cols < 5e-3, mis_cols
    print(f"rows {rows} d {d_model} V {V}: {len(rsel)} whole rows (neighbours {mis_rows:.2e}), "
          f"{len(vsel)} whole columns (neighbours {mis_cols:.2e})")
