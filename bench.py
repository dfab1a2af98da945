#!/usr/bin/env python3
"""Benchmark of the parallel-verification hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch: spec_verify_attn,
spec_fuse_drafts (workloads with several drafters) and spec_accept enqueued on one
stream.  Inputs are resident in HBM before the timed region; several independent
copies of every input are rotated so that no step finds its data in the last-level
cache.  Prints ONE JSON line: the headline workload (the largest single-GPU
configuration, c4_llama70b_serving) at the top level, and one entry per measured
workload in `workloads`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--also a,b,c|none]
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
HEADLINE = "c4_llama70b_serving"
OTHERS = "c1_llama2_7b,c2_tree_llama3_8b,c3_fusion,c2b_tree116_llama3_8b"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE, help="the workload of the top-level fields")
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads measured in the same run and reported in `workloads` "
                         f"(default: {OTHERS} when --workload is the headline workload, else none)")
    ap.add_argument("--copies", type=int, default=4, help="independent input copies rotated per step")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MiB (known traffic for counter scaling)")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per step instead of launching every call from the host")
    ap.add_argument("--cpu-seconds", type=float, default=20.0,
                    help="budget of the oracle timing leg, split evenly over the measured workloads")
    ap.add_argument("--min-event-steps", type=int, default=100,
                    help="steps of the separate event-timed loop the per-step median/p10/p90 come from")
    ap.add_argument("--fuse", choices=["auto", "always"], default="auto",
                    help="auto: spec_fuse_drafts runs on workloads with several drafters (its only use in the method); "
                         "always: single-drafter workloads also run it with N = 1 (an identity)")
    ap.add_argument("--routing", action="store_true",
                    help="multi-drafter workloads: also run spec_routing_scores (Eq. 1-2) after acceptance, on a "
                         "synthetic [vocab, 4096] bf16 embedding table")
    ap.add_argument("--accept-mode", choices=["sampling", "greedy"], default="sampling",
                    help="sampling: spec_accept (acceptance-rejection with residual resampling, the headline path); "
                         "greedy: spec_accept_greedy (the decoding rule of the paper's experiments)")
    ap.add_argument("--accept-path", type=int, default=0, choices=[0, 1, 2, 3, 4],
                    help="0: the library's choice; 1: statistics pass over all rows + walk; 2: workgroup clusters; 3: statistics pass + linear-draft kernel; 4: the same, statistics up to each first rejection")
    ap.add_argument("--fuse-mode", choices=["argmax", "mixture"], default="argmax",
                    help="multi-drafter workloads: argmax = the paper's confidence rule (Eq. 4, the headline path); "
                         "mixture = confidence-weighted average of the drafters' distributions (Section 2.2), written "
                         "as fp32 probabilities that the acceptance step then reads as its draft rows")
    ap.add_argument("--lm-head", action="store_true",
                    help="also run the projection that produces the target logits (spec_lm_head on synthetic "
                         "[rows, d_model] hidden states and a [vocab, d_model] bf16 weight, d_model = heads x "
                         "head_dim) inside the step; acceptance then starts from its statistics "
                         "(spec_accept_prestats).  Not the headline step: the entry gains an lm_head object")
    return ap.parse_args()


def read_traffic(key):
    """HBM bytes per launch derived from rocprofv3 --pmc runs, if recorded under profiles/."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{key}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


class Step:
    """Device state of one input copy and the calls of one step."""

    def __init__(self, cfg, a, ai, runner, sv, args, lm=None, want_debug=False):
        import torch
        accept_mode, fuse, routing, fuse_mode = args.accept_mode, args.fuse, args.routing, args.fuse_mode
        self.routing = None
        self.head = None
        self.tuning = sv.SpecAcceptTuning(path=args.accept_path) if args.accept_path else None
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
                                              want_debug=want_debug)
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
                                              want_debug=want_debug)
        if routing and ai.fusion is not None and accept_mode == "sampling":
            from paper_2503_10325_amd import workloads as W
            f = ai.fusion
            emb = runner.bf16_to_device(W._normal_bf16(W._rng(0, cfg.name, "embedding"), (cfg.vocab, 4096)), "cuda")
            t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
            scores = torch.zeros((cfg.batch, f.n_drafters), dtype=torch.float32, device="cuda")
            rargs = (t(f.k_len), t(f.conf), t(f.draft_tokens), self.accept.accept_len, self.accept.out_tokens, emb, scores)
            self.routing = lambda: sv.spec_routing_scores(*rargs)
        self.sampling = accept_mode == "sampling"
        if accept_mode == "greedy":
            # same target rows and draft tokens, no draft distributions or uniforms
            self.accept = runner.DeviceGreedy(st, self.accept.target, self.accept.draft_tokens)
        self.prestats = False
        if lm is not None:
            # the target rows come from the projection (written into the tensor the acceptance step
            # reads), their statistics go to the head of the acceptance workspace
            self.head = runner.DeviceLmHead(lm, temperature=cfg.temperature,
                                            stats=self.accept.workspace if self.sampling else None)
            self.head.logits = self.accept.target
            self.prestats = self.sampling

    def run_accept(self):
        if self.prestats:
            self.accept.run_prestats()
        elif self.sampling:
            self.accept.run(tuning=self.tuning)
        else:
            self.accept.run()

    def run(self):
        self.attn.run()
        if self.head is not None:
            self.head.run()
        if self.fuse is not None:
            self.fuse.run()
        self.run_accept()
        if self.routing is not None:
            self.routing()


def cpu_baseline(cfg, a, ai, budget_s, accept_mode="sampling", lm=None, fuse_mode="argmax"):
    """The oracle, as it stands, timed on the host cores over whole batches of the workload.
    Also returns the oracle's count of near-ties (decisions within 1e-6 of the uniform)."""
    import oracle
    reps, t_total = 0, 0.0
    tokens = int(a.st.total)
    lm_note, lm_s = "", 0.0
    near = {"n": None}
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
            r = oracle.accept(a.st.node_offsets, a.st.parent, toks, ai.target_logits, dq, qrow, ai.u_accept,
                              ai.u_resample, temperature=cfg.temperature, qkind=qkind)
            near["n"] = int(np.count_nonzero(r["near_tie"]))

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
    if lm is None and threads > 1 and t_total / reps * threads < 4.0:
        oracle.set_threads(1)
        t0 = time.perf_counter()
        one_pass()
        out["single_thread_value"] = tokens / (time.perf_counter() - t0)
        oracle.set_threads(threads)
    return out, near["n"]


def accept_min_rows(st, ratio, accept_len, stop_node):
    """Logit rows the walked paths need (the algorithmic minimum of the acceptance step): for every node
    the walk stood on, its target row and - if it tested a child - the draft row of its children, read
    once; one further read of that row pair for every rejection (the residual's mass).  Derived from the
    library's own outputs: `ratio` is not NaN exactly on the nodes whose token was tested."""
    rows = 0
    for b in range(len(st.n)):
        o, n = int(st.node_offsets[b]), int(st.n[b])
        par = np.arange(-1, n - 1) if st.parent is None else st.parent[o:o + n]
        tested = ~np.isnan(ratio[o:o + n])
        path = set()
        c = int(stop_node[b])
        while c >= 0:
            path.add(c)
            c = int(par[c])
        stood = [-1] + sorted(path)
        rows += len(stood)                                        # target rows
        rows += sum(1 for c in stood if np.any(tested & (par == c)))     # draft rows
        rejected = int(tested.sum()) - len(path)
        rows += 2 * rejected
    return rows


def event_times_us(torch, fn, n, copies):
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    torch.cuda.synchronize()
    for i in range(n):
        ev[i][0].record()
        fn(copies[i % len(copies)])
        ev[i][1].record()
    torch.cuda.synchronize()
    return np.array([e0.elapsed_time(e1) for e0, e1 in ev]) * 1e3


def pct(x):
    return {"median": float(np.median(x)), "p10": float(np.percentile(x, 10)), "p90": float(np.percentile(x, 90)),
            "mean": float(np.mean(x))}


def measure(name, args, cpu_seconds):
    """Builds the inputs of one workload, times K steps, and returns its report entry."""
    import torch
    from paper_2503_10325_amd import binding as sv
    from paper_2503_10325_amd import runner
    from paper_2503_10325_amd import workloads as W
    cfg = W.CONFIGS[name]
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
    copies = [Step(cfg, a, ai, runner, sv, args, lm) for _ in range(max(1, args.copies))]
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

    # ---- the timed region: exactly K steps ----
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

    # ---- separate event-timed loops: per-step distribution, and each call of the step on its own ----
    n_ev = max(args.min_event_steps, min(args.steps, 400))
    step_us = event_times_us(torch, lambda c: c.run(), n_ev, copies)
    attn_us = event_times_us(torch, lambda c: c.attn.run(), n_ev, copies)
    accept_us = event_times_us(torch, lambda c: c.run_accept(), n_ev, copies)
    attn_s = float(attn_us.mean()) * 1e-6
    accept_s = float(accept_us.mean()) * 1e-6

    lm_obj = None
    if lm is not None:
        lm_us = event_times_us(torch, lambda c: c.head.run(), n_ev, copies)
        lm_s = float(lm_us.mean()) * 1e-6
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

    # ---- what the step produced (the library's own outputs of copy 0) ----
    tokens = int(a.st.total)
    c0 = copies[0]
    if args.accept_mode == "sampling":          # one untimed step that also writes the tested ratios
        c0.accept.dbg_ratio = torch.zeros(max(tokens, 1), dtype=torch.float32, device="cuda")
    c0.run()
    res = c0.accept.results()
    accepted_per_step = int(res["accept_len"].sum()) + cfg.batch          # accepted drafts + one emitted token each
    attn_bytes, attn_flops = W.attention_bytes_flops(cfg, a.st)
    n_draft_rows_read = int(a.st.total) if ai.fusion else ai.draft_q.shape[0]
    all_rows = ai.target_logits.shape[0] + (0 if args.accept_mode == "greedy" else n_draft_rows_read)
    all_rows_bytes = all_rows * cfg.vocab * 2
    if args.accept_mode == "sampling" and res.get("ratio") is not None:
        min_rows = accept_min_rows(a.st, res["ratio"], res["accept_len"], res["stop_node"])
    else:
        min_rows = all_rows                                                # greedy verification reads every target row
    min_bytes = min_rows * cfg.vocab * (4 if (ai.fusion is not None and args.fuse_mode == "mixture") else 2)
    if ai.fusion is not None and args.fuse_mode == "mixture" and args.accept_mode == "sampling":
        # the drafters' rows are streamed twice by the fusion call (statistics, weighted sum), the fused fp32
        # rows are written once and read once by the acceptance statistics
        n_fused = ai.fusion.conf.shape[0] * ai.fusion.conf.shape[1]
        all_rows_bytes = (ai.target_logits.shape[0] * 2 + ai.fusion.draft_logits.shape[0] * 2 * 2 + n_fused * 4 * 2) * cfg.vocab

    attn_plan = sv.spec_describe_attn_plan(c0.attn.desc)
    if args.accept_mode == "greedy":
        accept_plan = "row_argmax_kernel + greedy_walk_kernel"
    elif lm is not None:
        # (spec_accept_prestats: what the library would pick for spec_accept, minus the target rows' statistics;
        # the kernel that reads only the walked rows of a tree takes its statistics itself)
        plain = sv.spec_describe_accept_plan(cfg.batch, cfg.vocab, int(a.st.total), int(a.st.n.max()), a.st.parent is not None,
                                             q_kind=c0.accept.q_kind, q_dtype=sv._dtype_code(c0.accept.draft_q))
        if "accept_cluster_kernel" in plain:
            accept_plan = plain + " (statistics from spec_lm_head not needed)"
        else:
            accept_plan = ("row_stats_kernel (draft rows only) + " +
                           ("accept_linear_kernel" if a.st.parent is None else "accept_walk_kernel") +
                           ", target statistics from spec_lm_head")
    else:
        accept_plan = sv.spec_describe_accept_plan(cfg.batch, cfg.vocab, int(a.st.total), int(a.st.n.max()), a.st.parent is not None,
                                                   q_kind=c0.accept.q_kind, q_dtype=sv._dtype_code(c0.accept.draft_q),
                                                   tuning=c0.tuning)
    step_s = elapsed / args.steps
    attn_ach = attn_bytes / attn_s / 1e9
    # the bound is the larger of the two times the call would need at the published peaks (many query rows per
    # KV head put the contraction above the ridge of 312 flop/B)
    attn_mfma_bound = attn_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) > attn_bytes / (HBM_PEAK_GBS * 1e9)
    attn_roofline = {"bound": "mfma" if attn_mfma_bound else "hbm",
                     "kernel": "spec_verify_attn: " + attn_plan + "; duration is the whole call, incl. "
                               "the chunk-combine kernel where the context is split",
                     "achieved": attn_flops / attn_s / 1e12 if attn_mfma_bound else attn_ach,
                     "peak": MFMA_BF16_PEAK_TFLOPS if attn_mfma_bound else HBM_PEAK_GBS,
                     "unit": "TFLOP/s" if attn_mfma_bound else "GB/s",
                     "frac": attn_flops / attn_s / 1e12 / MFMA_BF16_PEAK_TFLOPS if attn_mfma_bound else attn_ach / HBM_PEAK_GBS,
                     "traffic": read_traffic(cfg.name), "algorithmic_bytes": attn_bytes, "algorithmic_flops": attn_flops,
                     "hbm_gbs": attn_ach, "launch_us": pct(attn_us), "mfma_tflops": attn_flops / attn_s / 1e12}
    acc_ach = min_bytes / accept_s / 1e9
    entry = {
        "workload": cfg.name,
        "batch": cfg.batch, "draft_tokens_per_step": tokens,
        "q_heads": cfg.n_q_heads, "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim,
        "context": str(cfg.ctx), "draft": str(cfg.draft), "vocab": cfg.vocab,
        "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_s * 1e3,
        "tokens_per_s": tokens / step_s,
        "accepted_tokens_per_step": accepted_per_step,
        "accepted_tokens_per_s": accepted_per_step / step_s,
        "step_us": pct(step_us), "step_us_samples": int(n_ev),
        "calls_per_step": ["spec_verify_attn"] + (["spec_lm_head"] if lm is not None else []) +
                          (["spec_fuse_drafts"] if c0.fuse is not None else []) +
                          [("spec_accept_prestats" if lm is not None else "spec_accept")
                           if args.accept_mode == "sampling" else "spec_accept_greedy"] +
                          (["spec_routing_scores"] if c0.routing is not None else []),
        # algorithmic bytes of the step (attention: K/V once per KV head + Q + O; acceptance: the rows the walked
        # paths need) over the step's wall time
        "step_hbm_gbs": (attn_bytes + min_bytes) / step_s / 1e9,
        "step_hbm_frac": (attn_bytes + min_bytes) / step_s / 1e9 / HBM_PEAK_GBS,
        # the same with every target row and every referenced draft row counted once (what an all-rows pass moves)
        "step_hbm_gbs_all_rows": (attn_bytes + all_rows_bytes) / step_s / 1e9,
        "roofline": attn_roofline,
        "accept_roofline": {"bound": "hbm", "kernel": ("spec_accept: " if args.accept_mode == "sampling" else
                                                       "spec_accept_greedy: ") + accept_plan + "; duration is the whole call",
                            "achieved": acc_ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": acc_ach / HBM_PEAK_GBS,
                            "traffic": read_traffic("accept_" + cfg.name),
                            "algorithmic_bytes": min_bytes, "algorithmic_rows": int(min_rows),
                            "all_rows_bytes": all_rows_bytes, "all_rows": int(all_rows),
                            "launch_us": pct(accept_us)},
        "near_ties": None,
    }
    if lm_obj is not None:
        entry["lm_head"] = lm_obj
    if args.calibration_copy_mb > 0:
        # a plain copy kernel of known size: reads N MiB and writes N MiB
        src = torch.empty(args.calibration_copy_mb << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    del copies, c0, graphs
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        entry["cpu_baseline"], entry["near_ties"] = cpu_baseline(cfg, a, ai, cpu_seconds, args.accept_mode, lm,
                                                                 args.fuse_mode)
    return entry


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2503_10325_amd import binding as sv
    sv.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    also = args.also
    if also is None:
        also = OTHERS if args.workload == HEADLINE else "none"
    names = [args.workload] + [n for n in also.split(",") if n and n != "none" and n != args.workload]
    share = args.cpu_seconds / len(names)
    entries = [measure(n, args, share) for n in names]
    head = entries[0]
    out = {
        "metric": METRIC,
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "launch_mode": "hip_graph_replay" if args.graph else "eager",
        "accept_mode": args.accept_mode,
        "fuse_mode": args.fuse_mode,
        "config": {"workload": head["workload"], "batch": head["batch"],
                   "draft_tokens_per_step": head["draft_tokens_per_step"], "q_heads": head["q_heads"],
                   "kv_heads": head["kv_heads"], "head_dim": head["head_dim"], "context": head["context"],
                   "draft": head["draft"], "vocab": head["vocab"], "input_copies_rotated": max(1, args.copies)},
        "accepted_tokens_per_s": head["accepted_tokens_per_s"],
        "near_ties": head["near_ties"],
        "step_us": head["step_us"],
        "step_hbm_gbs": head["step_hbm_gbs"],
        "step_hbm_frac": head["step_hbm_frac"],
        "roofline": head["roofline"],
        "accept_roofline": head["accept_roofline"],
    }
    if "lm_head" in head:
        out["lm_head"] = head["lm_head"]
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    out["workloads"] = entries
    print(json.dumps(out))


if __name__ == "__main__":
    main()
