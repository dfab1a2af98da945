"""Regression fixture: the oracle on the tiny configuration reproduces the stored
values (written by tests/golden/make_golden.py from the oracle alone)."""
import json
import os

import numpy as np

import oracle
from paper_2503_10325_amd import workloads as W

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c0_tiny_seed0.json")


def test_oracle_reproduces_stored_tiny_case():
    doc = json.load(open(GOLD))
    cfg = W.CONFIGS[doc["config"]]
    a = W.make_attn_inputs(cfg, seed=doc["seed"])
    ai = W.make_accept_inputs(cfg, seed=doc["seed"], st=a.st)
    assert ai.draft_tokens.tolist() == doc["draft_tokens"]
    out, lse = oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets)
    acc = oracle.accept(a.st.node_offsets, None, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                        ai.u_accept, ai.u_resample, temperature=cfg.temperature)
    assert acc["accept_len"].tolist() == doc["accept_len"]
    assert acc["out_tokens"].tolist() == doc["out_tokens"]
    got = [[float(x) for x in out[i, h, :8]] for i in range(out.shape[0]) for h in (0, 7)]
    assert np.allclose(got, doc["attn_out_first8"], rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, doc["attn_lse"], rtol=1e-12)
