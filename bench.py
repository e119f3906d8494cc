#!/usr/bin/env python3
"""Benchmark of the RegTop-k round on one MI355X.

A step is one whole round (accumulate, score, exact top-k, compaction + error
update, aggregation) for all N workers on fresh synthetic gradients that are
already resident in HBM.  Default workload: N = 16, d = 25.6M, k = 1 % of d,
mu = 1 (the "large CNN-sized" configuration, 20 rounds from a zero error
state): rounds 0..W-1 are the warm-up, rounds W..W+K-1 are timed.  Prints ONE
JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--mu MU] [--k K] [--grad-dtype f32|bf16]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak


def algorithmic_bytes(N, d, k, g_bytes=4):
    """Bytes one round must move: read eps, read g, write eps; dense aggregate;
    index/value lists written, read back for the aggregate and for the next
    round's scores, plus the gathered previous aggregate."""
    return (8 + g_bytes) * N * d + 4 * d + 28 * N * k


def measured_traffic(workload, mode):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE (two runs, scaled by what the same counters read for the
    1 GiB reference copy), read from the committed summary of that profile -- not
    measured by this run.  None if there is no summary for the workload."""
    name = {"regtopk": "regtopk_round_%s_hbm_traffic.txt", "global": "regtopk_global_round_%s_hbm_traffic.txt"}[mode] % workload
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.strip().startswith("dominant kernel traffic per launch:"):
                return int(line.split(":")[1].split()[0]), "profiles/" + name
    except (OSError, ValueError):
        pass
    return None, None


def cpu_baseline(cfg, wl, rounds=3, workers=None, bf16=False, variant=(0, 0), glob=False, exponent=1.0):
    """The oracle, unchanged, single-threaded, on a bounded sample: the first
    `workers` rows of the same workload for `rounds` rounds."""
    workers = cfg.N if workers is None else workers
    import numpy as np
    import torch
    from oracle import oracle as orc
    o = orc.Oracle(workers, cfg.d, cfg.k, cfg.mu)
    o.set_score_variant(*variant)
    if exponent != 1.0:
        o.set_prior_exponent(exponent)
    agg = None
    elapsed = 0.0
    for t in range(rounds):
        g = wl.grads(t)[:workers].contiguous()
        if bf16:
            g = g.to(torch.bfloat16).float()
        g = g.cpu().numpy()
        t0 = time.perf_counter()
        _, _, agg = o.step_global(g) if glob else o.step(g, agg)
        elapsed += time.perf_counter() - t0
    o.close()
    entries = workers * cfg.d * rounds
    return {
        "value": entries / elapsed, "unit": "gradient entries/s", "cores": 1, "kind": "oracle",
        "sample": "first %d of %d workers, d=%d, k=%d, rounds 0..%d (%.1f s)" % (
            workers, cfg.N, cfg.d, cfg.k, rounds - 1, elapsed),
    }


def time_extras(torch, binding, r, agg, N, d, reps=20):
    """The two small kernels around the round, outside the timed region: the
    mask-overlap count (reads the N mask rows: N*d/8 bytes) and the SGD update
    of a d-vector (12 bytes per entry), timed with events on the current stream."""
    theta = torch.zeros(d, dtype=torch.float32, device=agg.device)
    g = agg.clone()
    res = {}
    for name, fn, nbytes in (("mask_overlap", lambda: r.mask_overlap(), N * d / 8.0),
                             ("sgd_update", lambda: binding.sgd_update(theta, g, 1e-2), 12.0 * d)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        res[name] = {"ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9, "bytes": nbytes}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_cnn")
    ap.add_argument("--mu", type=float, default=None)
    ap.add_argument("--k", type=int, default=None, help="entries kept per worker, if not the workload's own")
    ap.add_argument("--grad-dtype", choices=["f32", "bf16"], default="f32",
                    help="storage type of the local gradients (bf16: widened exactly, arithmetic stays f32)")
    ap.add_argument("--prior-roots", type=int, default=0, help="score variant: prior |a|^(2^-m)")
    ap.add_argument("--prior-exponent", type=float, default=1.0, help="score variant: prior |a|^y with a general 0 < y <= 1")
    ap.add_argument("--likelihood", type=int, default=0, help="score variant: 0 tanh, 1 clipped linear, 2 erf")
    ap.add_argument("--mode", choices=["regtopk", "global"], default="regtopk",
                    help="global: the genie-aided global Top-k baseline instead of the RegTop-k round")
    ap.add_argument("--force-dense", action="store_true",
                    help="never speculate: every round takes the dense selection (the cost of a failed speculation)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--max-buffers", type=int, default=24,
                    help="rounds of gradients kept resident in HBM (cycled if steps+warmup is larger)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (all N workers are a batch dimension on it); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_05633_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    if args.workload not in workloads.CONFIGS or workloads.CONFIGS[args.workload].kind == "linreg":
        print("bench.py: --workload must be one of %s (the closed-loop linear regression is a parity case, "
              "see tests/ and paper_2501_05633_amd.demo)" % ", ".join(
                  n for n, c in workloads.CONFIGS.items() if c.kind != "linreg"), file=sys.stderr)
        sys.exit(2)
    cfg = workloads.CONFIGS[args.workload]
    if args.mu is not None:
        cfg = workloads.scaled(cfg, d=cfg.d, k=cfg.k, mu=args.mu)
    if args.k is not None:
        cfg = workloads.scaled(cfg, d=cfg.d, k=args.k)
    N, d, k = cfg.N, cfg.d, cfg.k
    wl = workloads.Workload(cfg, dev)

    n_buf = min(args.warmup + args.steps, args.max_buffers)
    grads = [wl.grads(t) for t in range(n_buf)]
    g_bytes = 4
    if args.grad_dtype == "bf16":
        grads = [g.to(torch.bfloat16).contiguous() for g in grads]
        g_bytes = 2
    torch.cuda.synchronize()

    # one plain copy of known size (256 Mi floats: 1 GiB read, 1 GiB written): the
    # reference dispatch for scaling hardware traffic counters when profiling
    ref = torch.empty(2, 1 << 28, dtype=torch.float32, device=dev)
    binding.copy_f32(ref[1], ref[0])
    torch.cuda.synchronize()
    del ref

    r = binding.RegTopk(N, d, k, cfg.mu, device=dev)
    r.set_option(binding.OPT_PROFILE, 1)
    r.set_option(binding.OPT_FORCE_DENSE, 1 if args.force_dense else 0)
    r.set_option(binding.OPT_PRIOR_ROOTS, args.prior_roots)
    r.set_option(binding.OPT_LIKELIHOOD, args.likelihood)
    if args.prior_exponent != 1.0:
        r.set_option(binding.OPT_PRIOR_EXPONENT, args.prior_exponent)
    agg = None
    dense_rounds = 0
    glob = args.mode == "global"
    for t in range(args.warmup):
        _, _, agg = r.step_global(grads[t % n_buf]) if glob else r.step(grads[t % n_buf], agg)
    torch.cuda.synchronize()
    warm = [x[3] for x in r.timings(64)] if args.warmup else []     # whole-round event times of the warm-up rounds
    # The timed region records only the two events of the dominant kernel (profile level 2; they travel
    # with the kernel's own dispatch): an event recorded between two kernels keeps the second from
    # starting back to back (about 4 us each), and those of the full stage breakdown would add some
    # 10 us to every timed round.
    r.set_option(binding.OPT_PROFILE, 2)

    t0 = time.perf_counter()
    for i in range(args.steps):
        t = args.warmup + i
        _, _, agg = r.step_global(grads[t % n_buf]) if glob else r.step(grads[t % n_buf], agg)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sweep_ms = sum(x[0] for x in r.timings(64)) / args.steps
    st = r.stats()
    dense_rounds = sum(w["used_dense"] for w in st)
    cands = [w["n_candidates"] for w in st]

    # stage breakdown: as many rounds again, after the timed region, with all stage events
    r.set_option(binding.OPT_PROFILE, 1)
    for i in range(args.steps):
        t = args.warmup + args.steps + i
        _, _, agg = r.step_global(grads[t % n_buf]) if glob else r.step(grads[t % n_buf], agg)
    torch.cuda.synchronize()
    stage = r.timings(64)
    select_ms = sum(x[1] for x in stage) / len(stage)
    tail_ms = sum(x[2] for x in stage) / len(stage)
    round_ms_events = sum(x[3] for x in stage) / len(stage)

    # every fully instrumented round of the run by its own HIP events (round 0 has no history; the first
    # rounds are slower while the k-th score still moves fast): round 0, and median / min / max of the others
    all_rounds = warm + [x[3] for x in stage]
    later = sorted(all_rounds[1:]) if len(all_rounds) > 1 else sorted(all_rounds)
    round_ms = {"round0": all_rounds[0] if args.warmup and len(warm) == args.warmup else None,
                "median_later_rounds": later[len(later) // 2], "min": later[0], "max": later[-1],
                "rounds": len(all_rounds)}
    entries = N * d
    value = entries / (ms_per_step * 1e-3)
    sweep_bytes = (8 + g_bytes) * N * d           # read eps, read g, write eps
    if glob:
        sweep_bytes += 4 * d                      # the accumulation also writes the unsparsified aggregate
    traffic, traffic_src = (None, None)
    if args.grad_dtype == "f32" and args.prior_roots == 0 and args.prior_exponent == 1.0 and args.likelihood == 0 \
            and not args.force_dense and args.k is None:
        traffic, traffic_src = measured_traffic(cfg.name, args.mode)
    achieved = sweep_bytes / (sweep_ms * 1e-3) / 1e9
    b_alg = algorithmic_bytes(N, d, k, g_bytes)
    out = {
        "metric": "gradient entries/sec per RegTop-k round (N*d)",
        "value": value, "unit": "gradient entries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d workers, d=%d, k=%d, mu=%g, per-layer scales, %s entries, "
                               "30%% shared component" % (cfg.name, N, d, k, cfg.mu, cfg.marginal),
                   "N": N, "d": d, "k": k, "mu": cfg.mu, "rounds_resident": n_buf,
                   "grad_dtype": args.grad_dtype, "prior_roots": args.prior_roots, "prior_exponent": args.prior_exponent, "likelihood": args.likelihood, "mode": args.mode, "force_dense": args.force_dense},
        "hbm_frac_round": b_alg / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes_per_round": b_alg,
        "stage_ms": {"sweep": sweep_ms, "select": select_ms, "compact_aggregate": tail_ms,
                     "round_events": round_ms_events,
                     "source": "sweep: the timed rounds; the others: as many rounds after the timed region, "
                               "recorded with all stage events (about 10 us more per round)"},
        "round_ms_by_events": round_ms,
        "dense_fallback_workers_last_round": dense_rounds,
        "candidates_last_round": cands,
        "roofline": {"bound": "hbm", "kernel": "k_global_accum" if glob else "k_accum_emit_vec", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": sweep_bytes, "avg_launch_ms": sweep_ms,
                     "traffic": traffic, "traffic_source": traffic_src},
    }
    out["extras"] = time_extras(torch, binding, r, agg, N, d)
    r.close()
    del grads
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl, bf16=args.grad_dtype == "bf16",
                                           variant=(args.prior_roots, args.likelihood), glob=glob,
                                           exponent=args.prior_exponent)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
