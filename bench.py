#!/usr/bin/env python3
"""Benchmark of the stage step: one step = forward+backward of the whole stage
(every kernel of the hot path) on one synthetic micro-batch resident in HBM.

Prints ONE JSON line.  `value` = samples/s of the whole job on one MI355X.
`roofline` is for the kernel class that dominates the step (the NT-form GEMM
that runs the forward and input-gradient contractions), timed with HIP events
on the stream the kernels run on.  `cpu_baseline` times the CPU oracle on a
bounded sample of the same workload on this machine's host cores.
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

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_FP32_TFLOPS = 157.3      # vector fp32 (fp32 debug mode runs on the vector ALUs)
# Bytes per launch of the dominant kernel that cross the L2 towards memory (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000,
# the factors a 256 MiB device copy gives), from the rocprofv3 --pmc runs summarised in
# profiles/c2_step_hbm_traffic_pmc.md and profiles/c5_step_hbm_traffic_pmc.md.
MEASURED_TRAFFIC_BYTES = {("C2", "keep-all"): 80.3e6, ("C5", "seed7-mixed"): 2096.3e6}
# Average duration of an NT-form GEMM launch in the rocprofv3 kernel traces (profiles/*_step_kernel_trace.md).
ROCPROF_NT_LAUNCH_US = {
    ("C2", "keep-all"): {"us": 29.20, "hip_events_same_run_us": 33.47},
    ("C5", "keep-all"): {"us": 972.79, "hip_events_same_run_us": 976.13},
    ("C5", "seed7-mixed"): {
        "us": 1840.00, "hip_events_same_run_us": 1838.37,
        "note": "under the profiler this plan's device-to-host copies run as shader blit kernels beside the GEMMs and "
                "slow them; the trace and the HIP events of that profiled run agree with each other, and the keep-all "
                "trace (no copies: 972.79 us by rocprofv3, 976.13 us by HIP events in that run) shows the same kernels undisturbed"},
}


def cpu_baseline(cfg, weights, x, dy, budget_s=25.0, mem=None):
    """The oracle as it stands (fp64 numpy) on a bounded sample of the workload: the first layer of the stage on
    the first sample of the micro-batch; if one layer on the whole micro-batch fits the time budget it is run on
    that, and if the whole stage fits, on that; otherwise on as many samples of one layer as about 20 s hold.  The
    time is scaled to the whole step: every layer costs the same, and no operator mixes samples, so the cost is
    linear in both."""
    import numpy as np
    from oracle import stage as O

    def run(n_layers, n_samples):
        rows = n_samples * cfg.seq
        if cfg.mem_seq > 0:
            from oracle import decoder as Dc
            st = Dc.DecoderStage(n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.mem_seq, n_samples,
                                 cfg.causal, cfg.gelu, cfg.ln_eps, p_attn=cfg.p_attn, p_hidden=cfg.p_hidden, norm=cfg.norm)
            t0 = time.perf_counter()
            Dc.decoder_step(st, weights[:n_layers], x[:rows], mem[:n_samples * cfg.mem_seq], dy[:rows], dtype=np.float64)
            return time.perf_counter() - t0
        st = O.Stage(n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, n_samples, cfg.norm_style,
                     cfg.causal, cfg.gelu, cfg.ln_eps, p_attn=cfg.p_attn, p_hidden=cfg.p_hidden, norm=cfg.norm)
        t0 = time.perf_counter()
        O.stage_step(st, weights[:n_layers], x[:rows], dy[:rows], dtype=np.float64)
        return time.perf_counter() - t0

    L, B = cfg.n_layers, cfg.micro_batch
    dt = run(1, 1)
    layers, samples = 1, 1
    if dt * B <= budget_s:
        dt, samples = run(1, B), B
        if dt * L <= budget_s:
            dt, layers = run(L, B), L
    else:
        # as many samples of one layer as about 20 s hold (a divisor of the micro-batch, so the scaling is whole)
        fit = max(n for n in range(1, B + 1) if B % n == 0 and dt * n <= max(20.0, dt))
        if fit > 1:
            dt, samples = run(1, fit), fit
    step_s = dt * (L / layers) * (B / samples)
    sample = (f"{layers} of {L} layers on {samples} of {B} samples (fp64 numpy), "
              f"time scaled by {L // layers} x {B // samples}" if (layers, samples) != (L, B)
              else f"the whole step: all {L} layers on the full micro-batch (fp64 numpy)")
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": cfg.micro_batch / step_s, "unit": "samples/s", "cores": int(cores),
            "kind": "oracle", "seconds": round(dt, 3), "sample": sample}


def partition_and_measure(args, cfg, run):
    """The partition search in front of the path: node times and link speed measured on `run`'s handle, a chain
    of --chain-layers layers cut into --partition stages under --budget-gb a device, then every stage of the
    result (and of the equal-layers split, for comparison) timed in its own steady state on this one GPU."""
    import dataclasses
    import synthetic as syn
    from paper_2505_05856_amd import binding as B
    from paper_2505_05856_amd.harness import StageRunner, steady_state_ms, to_binding_config
    ell, n = args.partition, args.chain_layers
    cm = B.stage_measure_cost_model(run.stage, run.x, run.dy, run.y, run.dx, run.g, steps=3)
    one = dataclasses.replace(cfg, n_layers=1)
    _, rep1 = B.plan_validate(to_binding_config(one), syn.plan_keep_all(one))
    fixed_per_layer = rep1["weight_bytes"] + rep1["grad_bytes"]
    fixed_per_stage = rep1["fixed_bytes"] - fixed_per_layer
    budget = int(args.budget_gb * 1e9)
    chain = dataclasses.replace(cfg, n_layers=n)
    t_search = time.perf_counter()
    code, part = B.partition(to_binding_config(chain), cm, ell, budget, fixed_per_layer, fixed_per_stage,
                             flags=B.MEMOPT_VALIDATE, raise_on_error=False)
    t_search = time.perf_counter() - t_search      # host time of the whole search (Section 5.3 reports under 1 s for its models)
    measured = {}

    def measure(n_layers, inflight, plan=None):
        """Steady state of one stage: under `plan` (the search's), else under the plan dp_plan_generate makes
        for that many layers alone."""
        key = (n_layers, inflight, plan is None)
        if key not in measured:
            c = dataclasses.replace(cfg, n_layers=n_layers)
            w = syn.make_weights(c)
            x, dy = syn.make_activations(c)
            r = StageRunner(c, w, x, dy, mem=syn.make_memory(c) if c.mem_seq > 0 else None)
            predicted = None
            if plan is None:
                scode, plan, mrep = B.plan_generate(r.bcfg, cm, budget, inflight=inflight, flags=B.MEMOPT_VALIDATE,
                                                    raise_on_error=False)
                predicted = round((mrep["base_ns"] + mrep["moo_ns"]) / 1e6, 3)
            else:
                scode, _ = B.plan_validate(r.bcfg, plan, budget_bytes=budget, inflight=inflight, raise_on_error=False)
            if scode != 0:
                measured[key] = {"fits": False}
            else:
                _, vrep = B.plan_validate(r.bcfg, plan, budget_bytes=budget, inflight=inflight)
                ms = steady_state_ms(r, plan, inflight, budget, 2, max(3, args.steps // 4))
                measured[key] = {"fits": True, "measured_ms": round(ms, 3),
                                 "held_bytes": inflight * vrep["peak_bytes"]}
                if predicted is not None:
                    measured[key]["predicted_ms"] = predicted
            r.close()
        return measured[key]

    out = {"stages": ell, "chain_layers": n, "budget_bytes": budget, "feasible": part["feasible"],
           "rho_cb": part["rho_cb"], "rho_mb": part["rho_mb"], "memopt_runs": part["n_memopt"],
           "positions_visited": part["n_positions"], "search_seconds": round(t_search, 4), "cost_model": cm.as_dict()}
    if part["feasible"]:
        out["cuts"] = part["cuts"]
        out["predicted_ms"] = round(part["time_ns"] / 1e6, 3)
        out["per_stage"] = [dict(layers=s["n_layers"], inflight=s["inflight"], model_ms=round(s["time_ns"] / 1e6, 3),
                                 **measure(s["n_layers"], s["inflight"], s["plan"])) for s in part["stages"]]
        fits = [s for s in out["per_stage"] if s["fits"]]
        if len(fits) == ell:
            out["measured_ms"] = max(s["measured_ms"] for s in fits)
            out["pipeline_samples_per_s"] = round(cfg.micro_batch / (out["measured_ms"] * 1e-3), 3)
    # what equal layer counts would give under the same budget
    if n % ell == 0:
        eq = [measure(n // ell, ell - x) for x in range(ell)]
        out["equal_layers"] = {"per_stage": eq,
                               "measured_ms": max(s["measured_ms"] for s in eq) if all(s["fits"] for s in eq) else None}
    return out


PLAN_MAKERS = {
    "keep-all": lambda syn: syn.plan_keep_all,
    "all-recompute": lambda syn: syn.plan_all_recompute,
    "all-swap": lambda syn: syn.plan_all_swap,
    "recompute-attention": lambda syn: syn.plan_recompute_attention,
    "swap-fc1-recompute-ln-gelu": lambda syn: syn.plan_swap_ffn_recompute_norm_gelu,
    "seed7-mixed": lambda syn: (lambda c: syn.plan_seeded(c, 7)),
    "memopt": lambda syn: syn.plan_keep_all,
}


def workload_text(name, cfg):
    return (f"{name}: {cfg.n_layers} {cfg.norm_style}-LN layers, hidden {cfg.hidden}, {cfg.n_heads} heads, "
            f"ffn {cfg.ffn}, seq {cfg.seq}, micro-batch {cfg.micro_batch}, "
            f"{'causal' if cfg.causal else 'full'} attention"
            + (f", cross-attention over a memory of {cfg.mem_seq}" if cfg.mem_seq > 0 else "")
            + (f", dropout {cfg.p_attn}" if cfg.p_attn > 0 else ""))


def time_steps(run, plan, budget, warmup, steps):
    """EXACTLY `steps` steps between two device synchronisations (wall clock), with HIP events on the launch
    stream at the step boundaries (the paper times its iterations the same way, Appendix C.1)."""
    import torch
    for _ in range(warmup):
        run.step(plan, budget)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        run.step(plan, budget)
        marks[i + 1].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    events = {"mean": round(sum(per_step) / len(per_step), 4), "median": round(per_step[len(per_step) // 2], 4),
              "min": round(per_step[0], 4), "max": round(per_step[-1], 4)} if per_step else None
    return ms, events


def op_times_and_roofline(run, cfg, name, plan_name, plan, budget, k):
    """The same steps again with every launch bracketed by HIP events on the launch stream: per-class times and
    the roofline of the dominant class, the NT-form GEMM (forward and input-gradient contractions)."""
    from paper_2505_05856_amd import binding as B
    B.stage_set_profiling(run.stage, True)
    for _ in range(k):
        run.step(plan, budget)
    times = B.stage_op_times(run.stage)
    flops = B.stage_op_flops(run.stage)
    B.stage_set_profiling(run.stage, False)
    op_ms = {n: round(v[0] / k, 4) for n, v in times.items()}
    nt_ms = (times["gemm_fwd"][0] + times["gemm_dgrad"][0]) / k
    nt_launches = (times["gemm_fwd"][1] + times["gemm_dgrad"][1]) / k
    # algorithmic work (2*M*N*K) of exactly the launches that were timed: the step's own forward and
    # input-gradient GEMMs plus the forward ones a plan replays
    nt_flops = (flops["gemm_fwd"] + flops["gemm_dgrad"]) / k
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    achieved = nt_flops / (nt_ms * 1e-3) / 1e12
    roof = {"kernel": "gemm_nt (forward + input-gradient GEMMs)", "bound": "mfma" if cfg.dtype == "bf16" else "alu",
            "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
            "avg_launch_us": round(nt_ms * 1e3 / max(nt_launches, 1), 2),
            "avg_launch_us_source": "HIP event pairs recorded around every launch on the launch stream (event overhead "
                                    "included; the rocprofv3 kernel trace of the same command gives avg_launch_us_rocprof)",
            "avg_launch_us_rocprof": ROCPROF_NT_LAUNCH_US.get((name, plan_name)),
            "launches_per_step": nt_launches,
            "traffic": MEASURED_TRAFFIC_BYTES.get((name, plan_name))}
    return op_ms, roof


def swap_overlap(run, plan, budget, ms, stats, steps):
    """(compute only + copies only - step) / min(compute only, copies only): compute only = the same plan with
    every SWAP turned into KEEP; copies only = the plan's swap bytes out, then back in, through pinned memory."""
    import numpy as np
    import torch
    import synthetic as syn
    kept = np.where(plan == syn.SWAP, syn.KEEP, plan).astype(np.uint8)
    for _ in range(2):
        run.step(kept, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run.step(kept, 0)
    torch.cuda.synchronize()
    t_comp = (time.perf_counter() - t0) * 1e3 / steps
    nslots = max(1, int((plan == syn.SWAP).sum()))
    piece = stats["d2h_bytes"] // nslots
    dev = torch.empty(piece, dtype=torch.uint8, device="cuda:0")
    host = torch.empty(piece * nslots, dtype=torch.uint8).pin_memory()

    def copies():
        for i in range(nslots):
            host[i * piece:(i + 1) * piece].copy_(dev, non_blocking=True)
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(nslots):
            dev.copy_(host[i * piece:(i + 1) * piece], non_blocking=True)
        torch.cuda.synchronize()
        return a
    copies()
    t0 = time.perf_counter(); mid = copies(); t1 = time.perf_counter()
    t_out, t_in = (mid - t0) * 1e3, (t1 - mid) * 1e3
    t_copy = t_out + t_in
    ov = (t_comp + t_copy - ms) / min(t_comp, t_copy)
    del dev, host
    return {"step_ms": round(ms, 3), "compute_only_ms": round(t_comp, 3), "copy_only_ms": round(t_copy, 3),
            "d2h_GBps": round(stats["d2h_bytes"] / t_out / 1e6, 2), "h2d_GBps": round(stats["h2d_bytes"] / t_in / 1e6, 2),
            "overlap_frac": round(max(0.0, min(1.0, ov)), 4),
            "definition": "(compute_only + copy_only - step) / min(compute_only, copy_only), clipped to [0,1]",
            # measured inside the library, from HIP events on the copy streams and around the compute stream's waits
            "in_library": {"d2h_busy_ms": round(stats["d2h_busy_ms"], 3), "h2d_busy_ms": round(stats["h2d_busy_ms"], 3),
                           "compute_waited_for_swaps_ms": round(stats["swap_wait_ms"], 3),
                           "replay_ms": round(stats["replay_ms"], 3)}}


def measure(run, name, cfg, plan_name, plan, budget, warmup, steps, op_times=True, overlap=False):
    """One workload under one plan: `steps` timed steps, then per-class times, statistics, overlap."""
    from paper_2505_05856_amd import binding as B
    _, rep = B.plan_validate(run.bcfg, plan, budget_bytes=budget)
    _, tight = B.plan_validate(run.bcfg, plan, budget_bytes=0)   # no budget: the tightest arena policy
    ms, events = time_steps(run, plan, budget, warmup, steps)
    op_ms = roof = None
    if op_times:
        op_ms, roof = op_times_and_roofline(run, cfg, name, plan_name, plan, budget, max(1, min(steps, 10)))
    stats = run.step(plan, budget, want_stats=True)
    tf = cfg.model_flops() / (ms * 1e-3) / 1e12
    out = {"workload": workload_text(name, cfg), "plan": plan_name, "budget_bytes": budget,
           "validator_peak_bytes": rep["peak_bytes"], "arena_peak_bytes": rep["arena_peak_bytes"],
           "min_feasible_budget_bytes": tight["peak_bytes"], "fallback_launches": rep["n_fallback_launches"],
           "ms_per_step": round(ms, 4), "samples_per_s": round(cfg.micro_batch / (ms * 1e-3), 3),
           "model_tflops": round(tf, 2), "mfma_peak_frac": round(tf / PEAK_BF16_TFLOPS, 4),
           "step_ms_by_hip_events": events, "fwd_ms": round(stats["fwd_ms"], 4), "bwd_ms": round(stats["bwd_ms"], 4),
           "swap_bytes": {"d2h": stats["d2h_bytes"], "h2d": stats["h2d_bytes"]},
           "replayed_ops": stats["n_replayed_ops"], "replay_ms": round(stats["replay_ms"], 3),
           "kernel_launches": stats["n_kernel_launches"], "op_ms": op_ms, "roofline": roof}
    if overlap and stats["d2h_bytes"] > 0:
        out["swap_overlap"] = swap_overlap(run, plan, budget, ms, stats, steps)
    return out, stats, rep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None,
                    help="workload name from synthetic.CONFIGS; default: the largest workload under its budget (C5, "
                         "its seeded plan, 64 GB) as the headline, with C2, C3, C4 and C5 keep-all under per_config")
    ap.add_argument("--plan", default=None, help="plan name (default: the config's own); 'memopt' generates one")
    ap.add_argument("--budget-frac", type=float, default=0.5,
                    help="with --plan memopt: budget as a fraction of the way from the all-recompute to the all-KEEP peak")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-op-times", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="default run: the headline workload only")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the plan with its SWAP slots kept (compute only) and its copies alone "
                         "(always on for the headline of the default run)")
    ap.add_argument("--inflight", type=int, default=0,
                    help="also time the steady state of a one-forward-one-backward schedule with this many "
                         "micro-batches between forward and backward (dp_stage_forward / dp_stage_backward)")
    ap.add_argument("--partition", type=int, default=0,
                    help="also cut a chain of --chain-layers layers of this shape into this many pipeline stages "
                         "(dp_partition, cost model measured here) and time every stage of the result")
    ap.add_argument("--chain-layers", type=int, default=24)
    ap.add_argument("--budget-gb", type=float, default=0.0, help="with --partition: device memory per stage (0 = no limit)")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the measurement of what the matrix cores sustain with nothing else in the way, on zeros "
                         "and on this workload's own weights and activations (the clock under load depends on the data)")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate on the attention probabilities and after the projection and FC2 (default: none)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 4 times (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import synthetic as syn
    from paper_2505_05856_amd import binding as B
    from paper_2505_05856_amd.harness import StageRunner

    B.lib()   # fails loudly if the HIP library is not built
    default_run = args.config is None
    name = args.config or "C5"
    cfg = syn.CONFIGS[name]
    if args.dropout > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, p_attn=args.dropout, p_hidden=args.dropout)
    plan_name, mk = syn.PLANS[name][0]
    if args.plan:
        plan_name, mk = args.plan, PLAN_MAKERS[args.plan](syn)
    plan = mk(cfg)
    budget = syn.BUDGETS.get(name, 0)
    weights = syn.make_weights(cfg)
    x, dy = syn.make_activations(cfg)
    mem = syn.make_memory(cfg) if cfg.mem_seq > 0 else None
    run = StageRunner(cfg, weights, x, dy, mem=mem)
    memopt = None
    if plan_name == "memopt":
        # the plan generator in front of the path: cost model measured here, plan for the budget, prediction
        cm = B.stage_measure_cost_model(run.stage, run.x, run.dy, run.y, run.dx, run.g, steps=3)
        _, hi = B.plan_validate(run.bcfg, syn.plan_keep_all(cfg))
        _, lo = B.plan_validate(run.bcfg, syn.plan_all_recompute(cfg))
        budget = int(lo["peak_bytes"] + args.budget_frac * (hi["peak_bytes"] - lo["peak_bytes"]))
        _, plan, mrep = B.plan_generate(run.bcfg, cm, budget, flags=B.MEMOPT_VALIDATE)
        memopt = {"cost_model": cm.as_dict(), "budget_frac": args.budget_frac,
                  "base_ms": mrep["base_ns"] / 1e6, "model_moo_ms": mrep["moo_ns"] / 1e6,
                  "predicted_ms": mrep["exact_step_ns"] / 1e6,
                  "free_swaps": mrep["n_free_swaps"], "paid_swaps": mrep["n_paid_swaps"],
                  "recomputed": mrep["n_recomputed"], "refine_rounds": mrep["refine_rounds"]}
    if args.copy_calibration:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head, stats, rep = measure(run, name, cfg, plan_name, plan, budget, args.warmup, args.steps,
                               op_times=not args.no_op_times, overlap=args.overlap or default_run)
    ms = head["ms_per_step"]

    schedule = None
    if args.inflight > 0:
        # steady state of the schedule: backward of the oldest micro-batch, then the forward of the next into
        # the slot it left; the budget covers every micro-batch in flight
        from paper_2505_05856_amd.harness import steady_state_ms
        k = args.inflight
        sms = steady_state_ms(run, plan, k, k * budget, args.warmup, args.steps)
        schedule = {"inflight": k, "ms_per_micro_batch": round(sms, 4),
                    "samples_per_s": round(cfg.micro_batch / (sms * 1e-3), 3),
                    "budget_bytes": k * budget, "device_bytes_held": k * rep["arena_peak_bytes"],
                    "vs_fused_step": round(ms / sms, 4)}

    probe = None
    if not args.no_mfma_probe and cfg.dtype == "bf16":
        probe = {}
        for tag, t in (("zeros", torch.zeros(1 << 20, dtype=torch.bfloat16, device="cuda:0")),
                       ("weights", run.w[0]["w_fc1"]), ("activations", run.x),
                       ("random_bits", torch.randint(-2 ** 15, 2 ** 15, (1 << 20,), dtype=torch.int16,
                                                     device="cuda:0").view(torch.bfloat16))):
            tf, mhz = B.probe_mfma(t, 40000)
            probe[tag] = {"tflops": round(tf, 1), "shader_mhz": round(mhz)}
    partition = None
    if args.partition > 0:
        partition = partition_and_measure(args, cfg, run)

    # the other workloads of the metric, each under its own plan and budget, in the same JSON line
    per_config = None
    if default_run and not args.no_per_config:
        per_config = {}
        keep, _, _ = measure(run, name, cfg, "keep-all", syn.plan_keep_all(cfg), budget, 2, max(3, args.steps // 2),
                             op_times=not args.no_op_times)
        per_config["C5 keep-all"] = keep
    run.close()
    del run
    if per_config is not None:
        shared_w = {}
        for other in ("C2", "C3", "C4"):
            ocfg = syn.CONFIGS[other]
            oname, omk = syn.PLANS[other][0]
            key = (ocfg.n_layers, ocfg.hidden, ocfg.ffn, ocfg.n_heads)
            if key not in shared_w:     # C4 is C3's stage at a larger micro-batch: the same seeded weights
                shared_w[key] = syn.make_weights(ocfg)
            ox, ody = syn.make_activations(ocfg)
            orun = StageRunner(ocfg, shared_w[key], ox, ody)
            swaps = other == "C4"
            res, _, _ = measure(orun, other, ocfg, oname, omk(ocfg), syn.BUDGETS.get(other, 0), 3,
                                args.steps if not swaps else max(3, args.steps // 2),
                                op_times=not args.no_op_times, overlap=swaps)
            per_config[other] = res
            orun.close()
            del orun, ox, ody
            torch.cuda.empty_cache()

    out = {
        "metric": "stage fwd+bwd samples/sec + MFMA util % at fixed memory budget",
        "value": head["samples_per_s"], "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "plan": plan_name, "budget_bytes": budget,
                   "validator_peak_bytes": head["validator_peak_bytes"], "arena_peak_bytes": head["arena_peak_bytes"],
                   "min_feasible_budget_bytes": head["min_feasible_budget_bytes"],
                   "fallback_launches": head["fallback_launches"]},
        "model_tflops": head["model_tflops"], "mfma_peak_frac": head["mfma_peak_frac"],
        "step_ms_by_hip_events": head["step_ms_by_hip_events"],
        "fwd_ms": head["fwd_ms"], "bwd_ms": head["bwd_ms"], "swap_bytes": head["swap_bytes"],
        "replayed_ops": head["replayed_ops"], "replay_ms": head["replay_ms"], "kernel_launches": head["kernel_launches"],
        "op_ms": head["op_ms"], "roofline": head["roofline"],
    }
    roof = head["roofline"]
    if "swap_overlap" in head:
        out["swap_overlap"] = head["swap_overlap"]
    if per_config is not None:
        out["per_config"] = per_config
    if schedule is not None:
        out["schedule"] = schedule
    if partition is not None:
        out["partition"] = partition
    if probe is not None:
        out["mfma_issue_probe"] = probe
        if roof is not None and roof["bound"] == "mfma":
            roof["frac_of_issue_rate_on_activations"] = round(roof["achieved"] / probe["activations"]["tflops"], 4)
    if memopt is not None:
        memopt["measured_ms"] = round(ms, 4)
        out["memopt"] = memopt
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, weights, x, dy, mem=mem)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
