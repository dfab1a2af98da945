"""Writes tests/golden/c0_tiny_seed0.json from the CPU oracle alone (never from the
GPU path).  The paper prints no worked numeric example for the verification step,
so this file is a regression fixture of the oracle on the tiny configuration, not
an independent pin.  Run:  python tests/golden/make_golden.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
from paper_2503_10325_amd import workloads as W  # noqa: E402


def main():
    cfg = W.CONFIGS["c0_tiny"]
    a = W.make_attn_inputs(cfg, seed=0)
    ai = W.make_accept_inputs(cfg, seed=0, st=a.st)
    out, lse = oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets)
    acc = oracle.accept(a.st.node_offsets, None, ai.draft_tokens, ai.target_logits, ai.draft_q, ai.q_row,
                        ai.u_accept, ai.u_resample, temperature=cfg.temperature)
    doc = {
        "config": cfg.name, "seed": 0,
        "draft_tokens": ai.draft_tokens.tolist(),
        "u_accept": [float(x) for x in ai.u_accept], "u_resample": [float(x) for x in ai.u_resample],
        "accept_len": acc["accept_len"].tolist(), "out_tokens": acc["out_tokens"].tolist(),
        "ratio": [None if np.isnan(x) else float(x) for x in acc["ratio"]],
        "attn_out_first8": [[float(x) for x in out[i, h, :8]] for i in range(out.shape[0]) for h in (0, 7)],
        "attn_lse": [[float(x) for x in lse[i]] for i in range(lse.shape[0])],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c0_tiny_seed0.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
