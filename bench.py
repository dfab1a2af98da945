#!/usr/bin/env python3
"""Benchmark of the parallel-verification hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch: spec_verify_attn,
spec_fuse_drafts and spec_accept enqueued on one stream.  Inputs are resident in
HBM before the timed region; several independent copies of every input are rotated
so that no step finds its data in the last-level cache.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "verified draft tokens/sec + achieved HBM GB/s (verify-attn+accept), 1 MI355X"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c1_llama2_7b")
    ap.add_argument("--copies", type=int, default=4, help="independent input copies rotated per step")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MiB (known traffic for counter scaling)")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per step instead of launching every call from the host")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the oracle timing leg")
    ap.add_argument("--fuse", choices=["auto", "always"], default="auto",
                    help="auto: spec_fuse_drafts runs on workloads with several drafters (its only use in the method); "
                         "always: single-drafter workloads also run it with N = 1 (an identity)")
    ap.add_argument("--routing", action="store_true",
                    help="multi-drafter workloads: also run spec_routing_scores (Eq. 1-2) after acceptance, on a "
                         "synthetic [vocab, 4096] bf16 embedding table")
    ap.add_argument("--accept-mode", choices=["sampling", "greedy"], default="sampling",
                    help="sampling: spec_accept (acceptance-rejection with residual resampling, the headline path); "
                         "greedy: spec_accept_greedy (the decoding rule of the paper's experiments)")
    ap.add_argument("--fuse-mode", choices=["argmax", "mixture"], default="argmax",
                    help="multi-drafter workloads: argmax = the paper's confidence rule (Eq. 4, the headline path); "
                         "mixture = confidence-weighted average of the drafters' distributions (Section 2.2), written "
                         "as fp32 probabilities that the acceptance step then reads as its draft rows")
    ap.add_argument("--lm-head", action="store_true",
                    help="also run the projection that produces the target logits (spec_lm_head on synthetic "
                         "[rows, d_model] hidden states and a [vocab, d_model] bf16 weight, d_model = heads x "
                         "head_dim) inside the step; acceptance then starts from its statistics "
                         "(spec_accept_prestats).  Not the headline step: the line gains an lm_head object")
    return ap.parse_args()


def read_traffic(workload):
    """HBM bytes per attention launch derived from rocprofv3 --pmc runs, if recorded."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


class Step:
    """Device state of one input copy and the three calls of one step."""

    def __init__(self, cfg, a, ai, runner, sv, accept_mode="sampling", fuse="auto", routing=False, lm=None,
                 fuse_mode="argmax"):
        import torch
        self.routing = None
        self.head = None
        self.attn = runner.DeviceAttn(a, want_lse=False)
        st = a.st
        if ai.fusion is not None:
            mixture = fuse_mode == "mixture"
            self.fuse = runner.DeviceFuse(ai.fusion, cfg.vocab, temperature=cfg.temperature,
                                          mode=sv.SPEC_FUSE_MIXTURE if mixture else sv.SPEC_FUSE_ARGMAX)
            assert int(st.n.min()) == int(st.n.max()), "fusion output is used as a flat [B*k] view"
            # ARGMAX: the draft rows are the drafters' logits, q_row picks the winner's; MIXTURE: the draft
            # rows are the fused probabilities the fusion call writes (row b*k+i for node i of request b)
            self.accept = runner.DeviceAccept(st, ai.target_logits,
                                              self.fuse.fused_probs if mixture else self.fuse.draft_logits,
                                              self.fuse.q_row.view(-1), self.fuse.fused_token.view(-1),
                                              ai.u_accept, ai.u_resample, temperature=cfg.temperature,
                                              q_kind=sv.SPEC_Q_PROBS if mixture else sv.SPEC_Q_LOGITS,
                                              want_debug=False)
        else:
            # single drafter: token fusion has nothing to fuse.  With --fuse always it still runs with
            # N = 1 (an identity) and, for linear drafts of uniform length, feeds the acceptance step.
            B, k_max = cfg.batch, int(st.n.max())
            self.fuse = None
            uniform = False
            if fuse == "always":
                from paper_2503_10325_amd import workloads as W
                conf = np.ones((B, k_max, 1), dtype=np.float32)
                toks = np.zeros((B, k_max, 1), dtype=np.int32)
                for b in range(B):
                    o, k = int(st.node_offsets[b]), int(st.n[b])
                    toks[b, :k, 0] = ai.draft_tokens[o:o + k]
                f = W.FusionInputs(1, k_max, st.n.astype(np.int32), conf, toks, None)
                self.fuse = runner.DeviceFuse(f, cfg.vocab, temperature=cfg.temperature,
                                              draft_logits_dev=torch.empty(0, device="cuda"))
                self.fuse.draft_logits = None
                # Only for linear drafts of uniform length are the fused [B, k] outputs the flat node
                # arrays (node j's draft row is row j).  Tree nodes index their parent's draft row, so
                # tree and ragged workloads keep the generator's q_row / tokens.
                uniform = st.parent is None and int(st.n.min()) == int(st.n.max())
            self.accept = runner.DeviceAccept(st, ai.target_logits, ai.draft_q,
                                              self.fuse.q_row.view(-1) if uniform else ai.q_row,
                                              self.fuse.fused_token.view(-1) if uniform else ai.draft_tokens,
                                              ai.u_accept, ai.u_resample, temperature=cfg.temperature,
                                              want_debug=False)
        if routing and ai.fusion is not None and accept_mode == "sampling":
            from paper_2503_10325_amd import workloads as W
            f = ai.fusion
            emb = runner.bf16_to_device(W._normal_bf16(W._rng(0, cfg.name, "embedding"), (cfg.vocab, 4096)), "cuda")
            t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
            scores = torch.zeros((cfg.batch, f.n_drafters), dtype=torch.float32, device="cuda")
            args = (t(f.k_len), t(f.conf), t(f.draft_tokens), self.accept.accept_len, self.accept.out_tokens, emb, scores)
            self.routing = lambda: sv.spec_routing_scores(*args)
        if accept_mode == "greedy":
            # same target rows and draft tokens, no draft distributions or uniforms
            self.accept = runner.DeviceGreedy(st, self.accept.target, self.accept.draft_tokens)
        if lm is not None:
            # the target rows come from the projection (written into the tensor the acceptance step
            # reads), their statistics go to the head of the acceptance workspace
            sampling = accept_mode == "sampling"
            self.head = runner.DeviceLmHead(lm, temperature=cfg.temperature,
                                            stats=self.accept.workspace if sampling else None)
            self.head.logits = self.accept.target
            if sampling:
                self.accept.run = self.accept.run_prestats

    def run(self):
        self.attn.run()
        if self.head is not None:
            self.head.run()
        if self.fuse is not None:
            self.fuse.run()
        self.accept.run()
        if self.routing is not None:
            self.routing()


def cpu_baseline(cfg, a, ai, budget_s, accept_mode="sampling", lm=None, fuse_mode="argmax"):
    """The oracle, as it stands, timed on the host cores over whole batches of the workload."""
    import oracle
    reps, t_total = 0, 0.0
    tokens = int(a.st.total)
    lm_note, lm_s = "", 0.0
    if lm is not None:
        # the projection is timed once on a few rows and scaled to all of them (it is linear in rows)
        rows = lm.hidden.shape[0]
        r = min(rows, 4)
        t0 = time.perf_counter()
        oracle.lm_head(lm.hidden[:r], lm.weight, temperature=cfg.temperature)
        lm_s = (time.perf_counter() - t0) * rows / r
        lm_note = f"; plus the projection, timed on {r} of {rows} rows and scaled: {lm_s:.2f} s per pass"
    def one_pass():
        oracle.verify_attn(a.q, a.k_pool, a.v_pool, a.block_table, a.st.ctx_len, a.st.node_offsets,
                           a.st.parent, want_lse=False)
        qkind = oracle.Q_LOGITS
        if ai.fusion is not None and fuse_mode == "mixture":
            rf = oracle.fuse_drafts(ai.fusion.k_len, ai.fusion.conf, ai.fusion.draft_tokens, ai.fusion.draft_logits,
                                    temperature=cfg.temperature, mode=oracle.FUSE_MIXTURE)
            toks, qrow, dq = rf["fused_token"].reshape(-1), rf["q_row"].reshape(-1), rf["fused_probs"].astype(np.float32)
            qkind = oracle.Q_PROBS
        elif ai.fusion is not None:
            rf = oracle.fuse_drafts(ai.fusion.k_len, ai.fusion.conf, ai.fusion.draft_tokens)
            toks, qrow, dq = rf["fused_token"].reshape(-1), rf["q_row"].reshape(-1), ai.fusion.draft_logits
        else:
            toks, qrow, dq = ai.draft_tokens, ai.q_row, ai.draft_q
        if accept_mode == "greedy":
            oracle.accept_greedy(a.st.node_offsets, a.st.parent, toks, ai.target_logits)
        else:
            oracle.accept(a.st.node_offsets, a.st.parent, toks, ai.target_logits, dq, qrow, ai.u_accept,
                          ai.u_resample, temperature=cfg.temperature, qkind=qkind)

    while reps < 1 or (t_total < budget_s and reps < 1000):
        t0 = time.perf_counter()
        one_pass()
        t_total += time.perf_counter() - t0
        reps += 1
    threads = oracle.num_threads()
    out = dict(value=tokens * reps / (t_total + reps * lm_s), unit="tokens/s", cores=threads, kind="oracle",
               sample=f"{reps} pass(es) over the full {cfg.name} batch ({tokens} draft tokens each), "
                      f"{t_total:.2f} s of oracle time" + lm_note)
    # one more pass on a single thread where that stays within a few seconds (not the LM-head product)
    if lm is None and threads > 1 and t_total / reps * threads < 8.0:
        oracle.set_threads(1)
        t0 = time.perf_counter()
        one_pass()
        out["single_thread_value"] = tokens / (time.perf_counter() - t0)
        oracle.set_threads(threads)
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2503_10325_amd import binding as sv
    from paper_2503_10325_amd import runner
    from paper_2503_10325_amd import workloads as W
    sv.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    cfg = W.CONFIGS[args.workload]
    a = W.make_attn_inputs(cfg, seed=args.seed)
    lm = None
    if args.lm_head:
        # Target rows = the projection of synthetic hidden states, evaluated here on the host (fp32
        # accumulation, rounded to bf16) so that drafts and the CPU baseline see logits that do not come
        # from the GPU; the GPU recomputes them every step.
        rows = int(a.st.total) + cfg.batch
        lm = W.make_lm_head_inputs(rows, cfg.d_model, cfg.vocab, seed=args.seed, logit_sd=cfg.target_sd)
        hf = torch.from_numpy(W.bf16_bits_to_f32(lm.hidden))
        wf = torch.from_numpy(W.bf16_bits_to_f32(lm.weight))
        host_logits = (hf @ wf.t()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        del hf, wf
        ai = W.make_accept_inputs(cfg, seed=args.seed, st=a.st, target_logits=host_logits)
    else:
        ai = W.make_accept_inputs(cfg, seed=args.seed, st=a.st)
    copies = [Step(cfg, a, ai, runner, sv, args.accept_mode, args.fuse, args.routing, lm, args.fuse_mode)
              for _ in range(max(1, args.copies))]
    torch.cuda.synchronize()

    for i in range(args.warmup):
        copies[i % len(copies)].run()
    torch.cuda.synchronize()

    # Optionally capture each copy's step once into a HIP graph and replay the graphs in the
    # timed region (on this machine the eager launches already keep the GPU queue full).
    graphs = None
    if args.graph:
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in copies:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    c.run()
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        for g in graphs:                    # one untimed replay each
            g.replay()
        torch.cuda.synchronize()

    t0 = time.perf_counter()
    if graphs is None:
        for i in range(args.steps):
            copies[i % len(copies)].run()
    else:
        for i in range(args.steps):
            graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # Duration of the dominant kernel: the attention entry point alone, one launch per input copy
    # in rotation, each bracketed by HIP events on the launch stream.
    n_ev = max(20, min(args.steps, 200))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    torch.cuda.synchronize()
    for i in range(n_ev):
        c = copies[i % len(copies)]
        ev[i][0].record()
        c.attn.run()
        ev[i][1].record()
    torch.cuda.synchronize()
    attn_ms = np.array([e0.elapsed_time(e1) for e0, e1 in ev])
    attn_s = float(attn_ms.mean()) * 1e-3
    lm_obj = None
    if lm is not None:
        for i in range(n_ev):
            c = copies[i % len(copies)]
            ev[i][0].record()
            c.head.run()
            ev[i][1].record()
        torch.cuda.synchronize()
        lm_s = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e-3
        rows = lm.hidden.shape[0]
        w_bytes = cfg.vocab * cfg.d_model * 2
        lm_bytes = w_bytes + rows * cfg.d_model * 2 + rows * cfg.vocab * 2       # weight + hidden read, logits written
        lm_flops = 2.0 * rows * cfg.d_model * cfg.vocab
        mfma_time, hbm_time = lm_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12), lm_bytes / (HBM_PEAK_GBS * 1e9)
        bound = "hbm" if hbm_time >= mfma_time else "mfma"
        ach = lm_bytes / lm_s / 1e9 if bound == "hbm" else lm_flops / lm_s / 1e12
        peak = HBM_PEAK_GBS if bound == "hbm" else MFMA_BF16_PEAK_TFLOPS
        lm_kernel = ("lm_head_kernel (up to 128 rows: weight matrix read once)" if rows <= 128 else
                     "lm_pack_hidden_kernel + lm_head_wide_kernel (512 rows per workgroup)")
        lm_obj = {"kernel": f"spec_lm_head: {lm_kernel} + lm_stats_merge_kernel; duration is the whole call",
                  "rows": rows, "d_model": cfg.d_model, "vocab": cfg.vocab, "launch_us_mean": lm_s * 1e6,
                  "roofline": {"bound": bound, "achieved": ach, "peak": peak,
                               "unit": "GB/s" if bound == "hbm" else "TFLOP/s", "frac": ach / peak,
                               "traffic": read_traffic("lm_head_c1") if cfg.name == "c1_llama2_7b" else None,
                               "algorithmic_bytes": lm_bytes, "flops": lm_flops}}
    if args.calibration_copy_mb > 0:
        # a plain copy kernel of known size: reads N MiB and writes N MiB
        src = torch.empty(args.calibration_copy_mb << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    tokens = int(a.st.total)
    attn_bytes, attn_flops = W.attention_bytes_flops(cfg, a.st)
    # draft rows the statistics pass reads: with several drafters only the rows a fused token was drawn from
    n_logit_rows = ai.target_logits.shape[0] + (int(a.st.total) if ai.fusion else ai.draft_q.shape[0])
    if args.accept_mode == "greedy":
        n_logit_rows = ai.target_logits.shape[0]          # no draft distributions are read
    accept_bytes = n_logit_rows * cfg.vocab * 2
    if ai.fusion is not None and args.fuse_mode == "mixture" and args.accept_mode == "sampling":
        # the drafters' rows are streamed twice by the fusion call (statistics, weighted sum), the fused fp32
        # rows are written once and read once by the acceptance statistics
        n_fused = ai.fusion.conf.shape[0] * ai.fusion.conf.shape[1]
        accept_bytes = (ai.target_logits.shape[0] * 2 + ai.fusion.draft_logits.shape[0] * 2 * 2 + n_fused * 4 * 2) * cfg.vocab
    # the attention kernel the library's plan picks for this shape (all query rows that share a KV head)
    max_rows = int(a.st.n.max()) * (cfg.n_q_heads // cfg.n_kv_heads)
    total_tok = int((a.st.ctx_len.astype(np.int64) + a.st.n).sum())
    ragged = cfg.batch <= 128 and total_tok * 100 < 85 * cfg.batch * a.max_pages * 16     # the library's own rule
    if max_rows > 128:
        attn_kernel = f"attn_rows_kernel<{cfg.head_dim},8> (row-split, 8 waves share each K/V tile)"
    elif ragged:
        attn_kernel = (f"attn_stream_list_kernel<{cfg.head_dim}> (token-split body, device-built work list sorted by "
                       f"length, 2 persistent workgroups per CU)")
    else:
        attn_kernel = f"attn_stream_kernel<{cfg.head_dim}> (token-split, one workgroup per request x KV head x context chunk)"
    achieved = attn_bytes / attn_s / 1e9
    out = {
        "metric": METRIC,
        "value": tokens * args.steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "launch_mode": "eager" if graphs is None else "hip_graph_replay",
        "accept_mode": args.accept_mode,
        "fuse_mode": args.fuse_mode if ai.fusion is not None else None,
        "calls_per_step": ["spec_verify_attn"] + (["spec_lm_head"] if lm is not None else []) +
                          (["spec_fuse_drafts"] if copies[0].fuse is not None else []) +
                          [("spec_accept_prestats" if lm is not None else "spec_accept")
                           if args.accept_mode == "sampling" else "spec_accept_greedy"] +
                          (["spec_routing_scores"] if copies[0].routing is not None else []),
        "config": {"workload": cfg.name, "batch": cfg.batch, "draft_tokens_per_step": tokens,
                   "q_heads": cfg.n_q_heads, "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim,
                   "context": str(cfg.ctx), "draft": str(cfg.draft), "vocab": cfg.vocab,
                   "input_copies_rotated": len(copies)},
        "step_hbm_gbs": (attn_bytes + accept_bytes) / (elapsed / args.steps) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "spec_verify_attn: " + attn_kernel + "; duration is the whole call, incl. the chunk-combine kernel where the context is split",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_traffic(cfg.name), "algorithmic_bytes": attn_bytes,
                     "launch_us_mean": attn_s * 1e6, "launch_us_p10": float(np.percentile(attn_ms, 10)) * 1e3,
                     "launch_us_p90": float(np.percentile(attn_ms, 90)) * 1e3,
                     "mfma_tflops": attn_flops / attn_s / 1e12},
    }
    if lm_obj is not None:
        out["lm_head"] = lm_obj
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, a, ai, args.cpu_seconds, args.accept_mode, lm, args.fuse_mode)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
