#!/usr/bin/env python3
"""Benchmark of the Global Resolution verifier on one MI355X.

One "step" = the whole hot path over one batch of synthetic input already resident in HBM: streaming support
selection, per-row solve, verification of every row -- one gr_solve_verify call (the workgroup that solved a row
verifies it in the same launch; gr_solve_logits_verify with --logits); --two-calls times gr_solve (gr_solve_logits)
followed by gr_verify instead.  Default workload: the large-vocabulary configuration (B=256 rows, V=128256,
n=8 drafts, top-k 128).

The timed region: K steps on ONE stream, one batch at a time, between two device synchronisations, with HIP
events around every step and around every kernel launch; `value` = B K / wall time of that region, the
median step duration is reported beside it (`step_events`).  A second region deals the same K steps
round-robin to --streams handles on their own HIP streams and input copies (several batches in flight);
it is reported under `pipelined` and is not the headline.

Prints ONE JSON line: solves/s, ms per step, the roofline of the dominant kernel (durations from
HIP events recorded around every launch of the timed region) and the CPU checker timed on a
bounded sample of the same rows.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP64_PEAK_TFLOPS = 78.6        # MI355X published vector fp64 rate (256 CUs x 64 lanes x 2 flop x 2.4 GHz)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs) on the default
# workload, scaled by what the same counters read for the device copy of 8 V B bytes that this script runs itself
# (profiles/hbm_traffic_large_vocab.md).  Only valid for that workload at the default tau.
MEASURED_TRAFFIC_BYTES = {"select_kernel": 266583000, "solve_kernel": 41623000, "verify_kernel": 636000}


def _oracle_row(job):
    """One row through the CPU checker (a worker of the all-cores leg; also the single-thread leg's body)."""
    from oracle import gr_oracle as G
    p, q, n, k, tol, drafts, u = job
    sol = G.solve_row(p, q, n, k, tol=tol)
    G.verify_row(sol, p, drafts, u)
    return 1


def _worker_init():
    try:                                       # one thread per worker: the rows are the parallel axis
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass


def cpu_baseline(wl, tol, budget_s=10.0):
    """The CPU checker as it stands on the first rows of the same batch: single thread, then the same rows
    farmed over the host cores the box gives this job (plain row-level multiprocessing; call it before the
    GPU is initialised: the workers are forked)."""
    import multiprocessing as mp
    jobs = [(wl.p[b], wl.q[b], wl.n, wl.k, tol, wl.drafts[b], wl.uniforms[b]) for b in range(wl.B)]
    t0 = time.perf_counter(); rows = 0
    while rows < wl.B and time.perf_counter() - t0 < budget_s:
        _oracle_row(jobs[rows]); rows += 1
    dt = time.perf_counter() - t0
    single = rows / dt
    cores = max(1, min(16, os.cpu_count() or 1))
    sample = min(wl.B, max(cores, int(single * budget_s * cores * 0.8)))
    t1 = time.perf_counter()
    with mp.get_context("fork").Pool(cores, initializer=_worker_init) as pool:
        done = sum(pool.imap_unordered(_oracle_row, jobs[:sample], chunksize=1))
    dt_all = time.perf_counter() - t1
    return {"value": single, "unit": "solves/s", "cores": 1, "kind": "oracle",
            "sample": f"first {rows} rows of the same batch, {dt:.1f} s, single thread",
            "all_cores": {"value": done / dt_all, "unit": "solves/s", "cores": cores, "kind": "oracle",
                          "sample": f"first {done} rows of the same batch over {cores} worker processes, {dt_all:.1f} s "
                                    f"(pool start-up included)"}}


def bench_sweep(args):
    """Side measurement: gr_accept_sweep (alpha* over a grid of top-k sizes and draft counts) on the
    large-vocabulary batch.  One step = one call = one streaming pass over p and q plus the per-row grid."""
    import numpy as np
    import torch
    from paper_2511_15898_amd import binding as gr, workloads as W
    wl = W.large_vocab()
    ks, ns = [8, 16, 32, 64, 128, 256], list(range(1, 11))
    if args.sweep_to_v:
        ks = [10, 100, 1000, 10000, 100000, 0]          # the study's grid: powers of ten up to the whole vocabulary (0)
    dev = torch.device("cuda:0")
    p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
    acc = torch.empty((wl.B, len(ks), len(ns)), dtype=torch.float32, device=dev)
    st = torch.empty(wl.B, dtype=torch.int32, device=dev)
    h = gr.gr_create(wl.B, wl.V, max_k=0 if args.sweep_to_v else gr.GR_MAX_SUPPORT)
    for _ in range(args.warmup):
        gr.gr_accept_sweep(h, p, q, ks, ns, acc, st)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)   # the calls run on torch's current stream
    t0 = time.perf_counter(); e0.record()
    for _ in range(args.steps):
        gr.gr_accept_sweep(h, p, q, ks, ns, acc, st)
    e1.record(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    call_ms = e0.elapsed_time(e1) / args.steps
    gr.gr_destroy(h)
    algo_bytes = 8.0 * wl.V * wl.B
    achieved = algo_bytes / (call_ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import gr_oracle as G
        c0 = time.perf_counter(); rows = 0
        while rows < wl.B and time.perf_counter() - c0 < 10.0:
            G.acceptance_sweep(wl.p[rows], wl.q[rows], ks, ns); rows += 1
            if args.sweep_to_v:
                break                                   # the checker orders 128256 tokens per k: one row is the sample
        cdt = time.perf_counter() - c0
        cpu = {"value": rows / cdt, "unit": "rows/s", "cores": 1, "kind": "oracle",
               "sample": f"first {rows} rows of the same batch, {cdt:.1f} s, single thread"}
    print(json.dumps({
        "metric": "acceptance-sweep rows/sec", "value": wl.B * args.steps / dt, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"sweep on {wl.name}: B={wl.B} rows x V={wl.V} vocab, top-k in {ks}, drafts in {ns}",
                   "B": wl.B, "V": wl.V, "ks": ks, "ns": ns, "cells_per_row": len(ks) * len(ns)},
        "status_histogram": [int(x) for x in np.bincount(st.cpu().numpy(), minlength=4)],
        "roofline": {"bound": "hbm", "kernel": ("full_order + full_sweep_rank + full_sweep_scan kernels" if args.sweep_to_v else "select_kernel + sweep_kernel") + " (one gr_accept_sweep call)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "call_ms": call_ms},
        "cpu_baseline": cpu,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--tol", type=float, default=1e-4, help="the paper's error threshold tau")
    ap.add_argument("--workload", default="large", choices=["large", "llm", "small", "stress", "stress_full", "sweep"],
                    help="large = the configuration the metric is quoted on; the others are side measurements")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events")
    ap.add_argument("--event-stride", type=int, default=4,
                    help="record the per-kernel HIP events on every N-th step of the timed region (five event records per "
                         "step cost about 8 %% of a step here); the per-step events are recorded on every step")
    ap.add_argument("--logits", action="store_true",
                    help="side measurement: feed the same rows as float32 logits and temperatures to gr_solve_logits "
                         "(workloads large / llm / small); the drafts of the probability rows are kept")
    ap.add_argument("--sweep-to-v", action="store_true",
                    help="workload sweep: run the top-k sizes up to the whole vocabulary (HBM-resident ordering)")
    ap.add_argument("--tail-mass", type=float, default=0.0,
                    help="nucleus cut of the draft (gr_config.tail_mass) for workloads without a top-k; 0: none")
    ap.add_argument("--two-calls", action="store_true",
                    help="time gr_solve followed by gr_verify (two launches after the selection pass) instead of gr_solve_verify")
    ap.add_argument("--streams", type=int, default=3,
                    help="handles / HIP streams the steps of the second timed region are dealt to (1: skip that region); "
                         "three of them plus the default stream fill the four hardware queues of a process")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="run one 256 MiB device-to-device copy first (reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; rows are independent and would shard across GPUs "
                 "without any exchange, but no multi-GPU figure is produced.  Use --gpus 1.")

    if args.workload == "sweep":
        return bench_sweep(args)

    import numpy as np
    import torch
    from paper_2511_15898_amd import binding as gr, workloads as W

    if args.logits and args.workload not in ("large", "llm", "small"):
        sys.exit("bench.py: --logits goes with the workloads large, llm and small")
    if args.logits:
        wl = {"large": W.large_vocab, "llm": W.llm_shaped, "small": W.small}[args.workload](keep_logits=True)
    else:
        wl = {"large": W.large_vocab, "llm": W.llm_shaped, "small": W.small, "stress": W.stress,
              "stress_full": lambda: W.stress(k=0)}[args.workload]()     # stress_full: no top-k, the support is the whole row
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, args.tol)      # before the GPU is touched: it forks workers
    dev = torch.device("cuda:0")
    p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
    d = torch.from_numpy(wl.drafts).to(dev); u = torch.from_numpy(wl.uniforms).to(dev)
    acc = torch.empty(wl.B, dtype=torch.float32, device=dev); st = torch.empty(wl.B, dtype=torch.int32, device=dev)
    tok = torch.empty(wl.B, dtype=torch.int32, device=dev); ok = torch.empty(wl.B, dtype=torch.uint8, device=dev)
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n, flags=0 if args.no_events else gr.GR_FLAG_PROFILE, tail_mass=args.tail_mass)

    if args.logits:
        # the float32 logits stand in for p and q (never written as probabilities); a draft that the logits' top-k
        # does not hold (float32 ties of q) gives token -1 for that row and changes no timing
        p = torch.from_numpy(wl.meta["target_logits"]).to(dev); q = torch.from_numpy(wl.meta["draft_logits"]).to(dev)
        temps = torch.from_numpy(wl.meta["temps"].astype(np.float32)).to(dev)

    fused = not args.two_calls

    def step():
        if fused and args.logits:
            gr.gr_solve_logits_verify(h, p, q, temps, wl.n, wl.k, args.tol, d, u, acc, st, tok, ok)
            return
        if fused:
            gr.gr_solve_verify(h, p, q, wl.n, wl.k, args.tol, d, u, acc, st, tok, ok)
            return
        if args.logits:
            gr.gr_solve_logits(h, p, q, temps, wl.n, wl.k, args.tol, acc, st)
        else:
            gr.gr_solve(h, p, q, wl.n, wl.k, args.tol, acc, st)
        gr.gr_verify(h, d, u, tok, ok)

    if args.pmc_copy:
        src = torch.ones(1 << 26, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if not args.no_events:
        gr.gr_profile_read(h)                      # drop the warm-up events
        gr.gr_profile_stride(h, max(1, args.event_stride))
    # HIP events around every step on the stream the kernels are launched on (torch's current stream)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)] if not args.no_events else None
    t0 = time.perf_counter()
    for i in range(args.steps):
        if marks:
            marks[i].record()
        step()
    if marks:
        marks[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)) if marks else None
    prof = None if args.no_events else gr.gr_profile_read(h)
    stats = gr.gr_solve_stats(h, wl.B, dev)
    torch.cuda.synchronize()
    status = st.cpu().numpy(); iters = stats["evaluations"].cpu().numpy()
    node_tokens = float(stats["node_tokens"].sum().item())
    gr.gr_destroy(h)
    single_dt = dt
    step_events = None
    if step_ms:
        med = step_ms[len(step_ms) // 2]
        step_events = {"launches": len(step_ms), "median_ms": med, "mean_ms": sum(step_ms) / len(step_ms), "min_ms": step_ms[0],
                       "max_ms": step_ms[-1], "solves_per_s_at_median": wl.B / (med * 1e-3)}

    # second region: the same K steps dealt to several handles, each on its own stream
    ns = max(1, min(args.streams, 8))
    pipelined = None
    if ns > 1:
        hs = [gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n, tail_mass=args.tail_mass) for _ in range(ns)]
        ss = [torch.cuda.Stream() for _ in range(ns)]
        outs = [(torch.empty_like(acc), torch.empty_like(st), torch.empty_like(tok), torch.empty_like(ok)) for _ in range(ns)]
        ins = [(p, q)] + [(p.clone(), q.clone()) for _ in range(ns - 1)]      # every stream reads its own copy of the batch

        def pstep(i):
            j = i % ns
            a, s_, t_, o_ = outs[j]
            if fused and args.logits:
                gr.gr_solve_logits_verify(hs[j], ins[j][0], ins[j][1], temps, wl.n, wl.k, args.tol, d, u, a, s_, t_, o_, stream=ss[j])
                return
            if fused:
                gr.gr_solve_verify(hs[j], ins[j][0], ins[j][1], wl.n, wl.k, args.tol, d, u, a, s_, t_, o_, stream=ss[j])
                return
            if args.logits:
                gr.gr_solve_logits(hs[j], ins[j][0], ins[j][1], temps, wl.n, wl.k, args.tol, a, s_, stream=ss[j])
            else:
                gr.gr_solve(hs[j], ins[j][0], ins[j][1], wl.n, wl.k, args.tol, a, s_, stream=ss[j])
            gr.gr_verify(hs[j], d, u, t_, o_, stream=ss[j])

        for i in range(max(args.warmup, 2 * ns)):
            pstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            pstep(i)
        torch.cuda.synchronize()
        pdt = time.perf_counter() - t0
        same = all(torch.equal(tok, o[2]) and torch.equal(acc, o[0]) for o in outs)
        for hh in hs:
            gr.gr_destroy(hh)
        del ins
        if not same:
            sys.exit("bench.py: the pipelined region gave different results than the single-stream region")
        pipelined = {"streams": ns, "value": wl.B * args.steps / pdt, "unit": "solves/s", "ms_per_step": pdt / args.steps * 1e3,
                     "step_hbm_frac": 8.0 * wl.V * wl.B / (pdt / args.steps) / 1e9 / HBM_PEAK_GBS,
                     "note": "the same K steps dealt round-robin to independent handles, each on its own HIP stream with its own "
                             "copy of the inputs: several batches in flight, not the one-batch step of the headline"}
    dt = single_dt

    # what a plain device copy of the same number of bytes reaches on this machine (read + write counted)
    nbytes = 8 * wl.V * wl.B
    src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev); dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        dst.copy_(src)
    e1.record(); torch.cuda.synchronize()
    copy_gbs = 2.0 * nbytes / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e9
    del src, dst

    ms_per_step = dt / args.steps * 1e3
    algo_bytes = 8.0 * wl.V * wl.B                 # one read of the p row and of the q row per solve
    roofline = None
    if prof and prof["steps"]:
        k_eff = wl.V if (wl.k <= 0 or wl.k >= wl.V) else wl.k
        hbm_path = k_eff > 256                         # support kept in HBM: other kernels behind the same three events
        first, second = (("full_order+full_scan+full_trunc kernels", "full_programs_kernel") if hbm_path
                         else ("select_kernel", "solve_kernel"))
        kernels = {first: prof["select_ms"], second: prof["solve_ms"]}
        if not (fused and not hbm_path):               # one launch solves and verifies: no verify kernel of its own
            kernels["verify_kernel"] = prof["verify_ms"]
        dom = max(kernels, key=kernels.get)
        if dom == first:
            achieved = algo_bytes / (kernels[dom] * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": achieved / HBM_PEAK_GBS, "traffic": None}
        elif dom == second:
            # algorithmic arithmetic of the solve: 4 n^2 flops per (evaluator call, quadrature node, active token)
            flops = 4.0 * wl.n * wl.n * node_tokens
            achieved = flops / (kernels[dom] * 1e-3) / 1e12
            roofline = {"bound": "alu", "kernel": dom, "achieved": achieved, "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / FP64_PEAK_TFLOPS, "traffic": None,
                        "algorithmic_flops_per_launch": flops, "node_tokens_per_launch": node_tokens}
        else:
            roofline = {"bound": "hbm", "kernel": dom, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": None, "traffic": None}
        if args.workload == "large" and abs(args.tol - 1e-4) < 1e-12:
            roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get(dom)
            if fused and dom == "solve_kernel":        # the launch that also verifies the rows moves the verify kernel's bytes too
                roofline["traffic"] += MEASURED_TRAFFIC_BYTES["verify_kernel"]
            roofline["traffic_all_kernels"] = MEASURED_TRAFFIC_BYTES or None
        roofline["region"] = "the timed region: one stream, one batch at a time (launch durations from HIP events)"
        roofline["kernel_ms"] = {k: round(v, 5) for k, v in kernels.items()}
        roofline["events_steps"] = prof["steps"]
        roofline["events_every"] = max(1, args.event_stride)
        roofline["select_hbm_frac"] = algo_bytes / (kernels[first] * 1e-3) / 1e9 / HBM_PEAK_GBS
        roofline["step_hbm_frac"] = algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
        if step_events:
            roofline["step_hbm_frac_median"] = algo_bytes / (step_events["median_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
        roofline["device_copy_GBs"] = copy_gbs
        roofline["select_vs_device_copy"] = algo_bytes / (kernels[first] * 1e-3) / 1e9 / copy_gbs
    out = {
        "metric": "verifier solves/sec",
        "value": wl.B * args.steps / dt,
        "unit": "solves/s",
        "us_per_solve": dt / (wl.B * args.steps) * 1e6,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} rows x V={wl.V} vocab, n={wl.n} drafts, top-k={wl.k}, tau={args.tol:g}",
                   "B": wl.B, "V": wl.V, "n": wl.n, "k": wl.k, "tau": args.tol, "tail_mass": args.tail_mass, "rows_given_as": "logits" if args.logits else "probabilities", "streams": 1,
                   "calls_per_step": ("gr_solve_logits_verify" if args.logits else "gr_solve_verify") if fused
                                     else ("gr_solve_logits" if args.logits else "gr_solve") + " + gr_verify"},
        "step_events": step_events,
        "pipelined": pipelined,
        "status_histogram": [int(x) for x in np.bincount(status, minlength=4)],
        "solver_evaluations_mean": float(iters.mean()), "solver_evaluations_max": int(iters.max()),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
