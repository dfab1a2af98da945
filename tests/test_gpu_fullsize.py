"""GPU parity at the full sizes of the five benchmark workloads, in the launch
configuration bench.py times (same descriptors, same chunking hint).  Attention is
compared on sampled requests (the oracle recomputes whole requests, all heads, all
draft nodes); acceptance on every request."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

from gpu_util import ATTN_TOL, attn_rel_err, compare_accept, ratio_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding, runner
    binding.lib()
    return runner


def _oracle_attn_subset(a: W.AttnInputs, reqs):
    """Oracle attention of a few whole requests (same pools, their block-table rows)."""
    st = a.st
    off = np.zeros(len(reqs) + 1, dtype=np.int32)
    rows = []
    for i, b in enumerate(reqs):
        o, n = int(st.node_offsets[b]), int(st.n[b])
        rows.append(np.arange(o, o + n))
        off[i + 1] = off[i] + n
    rows = np.concatenate(rows)
    par = None if st.parent is None else st.parent[rows]
    out, lse = oracle.verify_attn(a.q[rows], a.k_pool, a.v_pool, a.block_table[reqs], st.ctx_len[reqs], off, par)
    return rows, out, lse


SAMPLES = {"c0_tiny": None, "c1_llama2_7b": None, "c2_tree_llama3_8b": 2, "c3_fusion": 3, "c4_llama70b_serving": 4}


@pytest.mark.parametrize("name", W.CONFIG_ORDER)
def test_fullsize_attention(rt, name):
    cfg = W.CONFIGS[name]
    a = W.make_attn_inputs(cfg, seed=0)
    dev = rt.DeviceAttn(a)
    dev.run()
    torch.cuda.synchronize()
    got = dev.out.float().cpu().numpy()
    lse = dev.lse.cpu().numpy()
    assert np.isfinite(got).all()
    k = SAMPLES[name]
    if k is None:
        reqs = np.arange(cfg.batch)
    else:
        L = a.st.ctx_len.astype(np.int64) + a.st.n
        pick = {int(np.argmax(L)), int(np.argmin(L)), int(np.argmax(a.st.n))}
        rng = np.random.default_rng(1)
        while len(pick) < k:
            pick.add(int(rng.integers(cfg.batch)))
        reqs = np.array(sorted(pick))[:max(k, 1)]
    rows, ref, ref_lse = _oracle_attn_subset(a, reqs)
    err = attn_rel_err(got[rows], ref)
    print(f"{name}: requests {reqs.tolist()}, rel err {err:.3e}")
    assert err <= ATTN_TOL
    assert np.abs(lse[rows] - ref_lse).max() < 2e-2


@pytest.mark.parametrize("name", W.CONFIG_ORDER)
def test_fullsize_accept(rt, name):
    cfg = W.CONFIGS[name]
    st = W.make_structure(cfg, seed=0)
    ai = W.make_accept_inputs(cfg, seed=0, st=st)
    if ai.fusion is not None:
        f = ai.fusion
        rf = oracle.fuse_drafts(f.k_len, f.conf, f.draft_tokens)
        fd = rt.DeviceFuse(f, cfg.vocab)
        fd.run()
        torch.cuda.synchronize()
        for key, t in (("fused_token", fd.fused_token), ("winner", fd.winner), ("q_row", fd.q_row)):
            assert np.array_equal(t.cpu().numpy(), rf[key]), key
        toks, qrow, dq_host, dq_dev = rf["fused_token"].reshape(-1), rf["q_row"].reshape(-1), f.draft_logits, fd.draft_logits
        dev = rt.DeviceAccept(st, ai.target_logits, dq_dev, fd.q_row.view(-1), fd.fused_token.view(-1), ai.u_accept,
                              ai.u_resample, temperature=cfg.temperature)
    else:
        toks, qrow, dq_host = ai.draft_tokens, ai.q_row, ai.draft_q
        dev = rt.DeviceAccept(st, ai.target_logits, dq_host, qrow, toks, ai.u_accept, ai.u_resample,
                              temperature=cfg.temperature)
    dev.run()
    got = dev.results()
    ref = oracle.accept(st.node_offsets, st.parent, toks, ai.target_logits, dq_host, qrow, ai.u_accept, ai.u_resample,
                        temperature=cfg.temperature)
    bad, ties, B = compare_accept(got, ref, st.n)
    print(f"{name}: near-ties {ties}/{B}, mean accepted {ref['accept_len'].mean():.2f}, "
          f"ratio err {ratio_err(got['ratio'], ref['ratio']):.2e}")
    assert not bad, f"requests {bad} differ outside near-ties"
    assert ties <= max(1, B // 4)
    assert ratio_err(got["ratio"], ref["ratio"]) < 5e-6
