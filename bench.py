#!/usr/bin/env python3
"""Benchmark of the verify-and-select stage on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic logits already resident in
HBM, through the C ABI: by default one speckv_step call (row statistics of both sides in one
launch, signals + accept + controller in one launch, two resample launches); with
--path three_calls the same step as speckv_signals + speckv_verify + speckv_select_gamma (seven
launches, identical results).  The default workload is the headline configuration: B=256,
gamma=8, V=128256, bf16, Zipf-shaped logits.

Prints one JSON line: throughput in verified sequence-steps/s, the HBM roofline of the dominant
kernel (row statistics) from HIP events stamped on sampled launches inside the timed steps, and the
CPU oracle timed on the host cores over the same batch.  The step's outputs are checked against
the oracle before anything is reported.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0  # MI355X published peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed steps first; the GPU needs ~100 steps (25 ms) of this load to reach steady clocks")
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--path", default="one_call", choices=["one_call", "three_calls"])
    ap.add_argument("--B", type=int, default=None, help="override the batch size (not the headline number)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the plain copy kernel on 1 GiB (reference for the profiler's byte counters)")
    ap.add_argument("--opt", action="append", default=[], help="name=value launch option, repeatable")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; sequences shard across GPUs with no exchange, "
              "so N GPUs would run N independent copies of this benchmark. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads
    import paper_2605_02888_amd as pkg
    from paper_2605_02888_amd.runner import StepRunner

    dev = "cuda:0"
    torch.cuda.set_device(0)
    over = {} if args.B is None else {"B": args.B}
    cfg = workloads.config(args.workload, **over)
    gamma = None
    if args.workload == "C4":
        gamma = torch.full((cfg.B,), 4, dtype=torch.int32)
    inp = workloads.make_step(cfg, device=dev, gamma=gamma)
    E = 4 if cfg.dtype == "f32" else 2
    n_draft_rows = int(inp.draft.shape[0])
    n_target_rows = int(inp.target.shape[0])

    sk = pkg.SpecKV(device=0)
    for kv in args.opt:
        k, v = kv.split("=")
        sk.set_option(k, int(v))
    # the optional argmax output of speckv_signals is not one of the paper's signals: not requested
    runner = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, device=dev,
                        with_argmax=False)
    batch = runner.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
    seed = cfg.seed

    def three_calls(i):
        runner.step(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, seed, i)

    def one_call(i):
        runner.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, seed, i)

    step, other = (one_call, three_calls) if args.path == "one_call" else (three_calls, one_call)
    # the single-launch statistics kernel exists for the default launch shape only
    paired = args.path == "one_call" and all(
        sk.get_option(k) in v for k, v in (("stats_threads", (256, 512)), ("stats_unroll", (2,)),
                                           ("stats_pipeline", (1,)), ("stats_nontemporal", (1,))))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; every 20th launch of the row-statistics kernels carries a
    # start/stop event pair stamped with the dispatch's own times (a stamped kernel is followed by
    # a gap of 4-6 us, so stamping every launch would cost about 6 % of the step) ------------------
    sk.set_option("profile_every", 20)
    sk.profile(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sk.profile(0)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = cfg.B / (ms_per_step * 1e-3)
    n_d, ms_d = sk.profile_read("row_stats_draft")
    n_t, ms_t = sk.profile_read("row_stats_target")
    n_p, ms_p = sk.profile_read("row_stats_pair")

    # the same K steps without any event, to show what the instrumentation costs
    sk.set_option("profile_every", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_plain = (time.perf_counter() - t0) * 1e3 / args.steps

    # the other way to issue the same step, for comparison
    for i in range(min(args.warmup, 50)):
        other(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        other(i)
    torch.cuda.synchronize()
    ms_other = (time.perf_counter() - t0) * 1e3 / args.steps

    # every kernel class once more, for the breakdown
    sk.profile(2)
    for i in range(min(args.steps, 50)):
        step(i)
    torch.cuda.synchronize()
    sk.profile(0)
    breakdown = {}
    for k in ("row_stats_pair", "step_tail", "step_epilogue", "row_stats_draft", "signals_finalize", "row_stats_target",
              "verify_tail", "accept", "resample_mass", "resample_pick", "select_gamma"):
        n, ms = sk.profile_read(k)
        if n:
            breakdown[k] = round(ms / n * 1e3, 2)  # microseconds per launch

    # ---- roofline of the dominant kernel: the row statistics ------------------------------------
    bytes_t = n_target_rows * cfg.V * E          # algorithmic: every target logit read once
    bytes_d = n_draft_rows * cfg.V * E

    def traffic_of(key):
        # measured with rocprofv3 --pmc in separate runs (a profiler cannot be attached from in here)
        tpath = os.path.join(ROOT, "profiles", f"row_stats_{args.workload.lower()}_traffic.txt")
        if os.path.exists(tpath) and args.B is None and not args.opt:
            for line in open(tpath):
                if line.startswith(key + " "):
                    return int(line.split()[1])
        return None

    def roof(kernel, nbytes, n, ms):
        avg = ms / max(n, 1) * 1e-3
        ach = nbytes / avg / 1e9 if n else 0.0
        return {"kernel": kernel, "achieved": round(ach, 1), "frac": round(ach / HBM_PEAK_GBS, 4),
                "bytes_per_launch": nbytes, "avg_launch_us": round(avg * 1e6, 2), "launches": n}

    if paired:
        r = roof("row_stats_pair", bytes_d + bytes_t, n_p, ms_p)
        roofline = {"bound": "hbm", "kernel": r["kernel"], "achieved": r["achieved"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": r["frac"], "traffic": traffic_of("row_stats_pair_bytes_per_launch"),
                    "bytes_per_launch": r["bytes_per_launch"], "avg_launch_us": r["avg_launch_us"],
                    "launches": r["launches"]}
    else:
        r = roof("row_stats_target", bytes_t, n_t, ms_t)
        rd = roof("row_stats_draft", bytes_d, n_d, ms_d)
        roofline = {"bound": "hbm", "kernel": r["kernel"], "achieved": r["achieved"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": r["frac"], "traffic": traffic_of("row_stats_target_bytes_per_launch"),
                    "bytes_per_launch": r["bytes_per_launch"], "avg_launch_us": r["avg_launch_us"],
                    "launches": r["launches"],
                    "row_stats_draft": {k: rd[k] for k in ("achieved", "frac", "bytes_per_launch", "avg_launch_us",
                                                           "launches")}}
    # whole-step bytes: every logit once, plus position n of both sides a second time (upper bound)
    step_bytes = bytes_t + bytes_d
    extra = {
        "step_logit_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "ms_per_step_without_events": round(ms_plain, 4),
        "path": args.path,
        "ms_per_step_" + ("three_calls" if args.path == "one_call" else "one_call"): round(ms_other, 4),
        "value_" + ("three_calls" if args.path == "one_call" else "one_call"): round(cfg.B / (ms_other * 1e-3), 1),
        "kernel_us": breakdown,
    }

    if not args.no_probe:
        # bare streaming read of the target logits: what a plain 16-byte-per-lane stream reaches here
        sink = torch.zeros(1, dtype=torch.int64, device=dev)
        nbytes = (inp.target.numel() * E) // 16 * 16
        for _ in range(3):
            sk.probe_read(inp.target, nbytes, sink)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 20
        for _ in range(reps):
            sk.probe_read(inp.target, nbytes, sink)
        torch.cuda.synchronize()
        extra["probe_read_GBps"] = round(nbytes * reps / (time.perf_counter() - t0) / 1e9, 1)

    # the same step with the accept rule as the paper words it (top-1 match): no resample pass
    for i in range(30):
        runner.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, seed, i, greedy=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(200):
        runner.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, seed, i, greedy=True)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / 200 * 1e6
    extra["greedy_step"] = {"us": round(us, 2), "sequence_steps_per_s": round(cfg.B / us * 1e6, 1)}

    # the step before the path: proposing the draft tokens on the device (all draft rows at once)
    tok_out = torch.zeros(n_draft_rows, dtype=torch.int32, device=dev)
    for i in range(20):
        sk.sample_draft(batch, inp.draft, runner.dtype, seed, i, 0, tok_out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(100):
        sk.sample_draft(batch, inp.draft, runner.dtype, seed, i, 0, tok_out)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / 100 * 1e6
    extra["sample_draft"] = {"rows": n_draft_rows, "us": round(us, 2), "GBps": round(bytes_d / us / 1e3, 1)}

    if args.calibrate:
        n = 1 << 30
        src = torch.zeros(n, dtype=torch.uint8, device=dev)
        dst = torch.empty(n, dtype=torch.uint8, device=dev)
        for _ in range(5):
            sk.probe_copy(dst, src, n)
        torch.cuda.synchronize()
        extra["calibrate_copy_bytes"] = n

    # ---- parity of this very step against the oracle, and the oracle's own speed -----------------
    step(0)
    gpu = runner.results(n_draft_rows)
    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        from parity import compare, oracle_step
        cores = min(16, os.cpu_count() or 1)
        oracle.set_threads(cores)
        # bounded sample: at most the first 256 sequences of the batch (the whole headline batch)
        nb = min(cfg.B, 256)
        sub = inp
        if nb < cfg.B:
            g = inp.gamma_host()
            rd = int(g[:nb].sum())
            sub = workloads.StepInputs(cfg=workloads.config(args.workload, B=nb), gamma=None if inp.gamma is None else inp.gamma[:nb],
                                       row_off=None if inp.row_off is None else inp.row_off[:nb + 1],
                                       draft=inp.draft[:rd], target=inp.target[:rd + nb],
                                       draft_tokens=inp.draft_tokens[:rd], comp=inp.comp[:nb], mlp=inp.mlp)
        t0 = time.perf_counter()
        ref = oracle_step(sub, seed, 0)
        dt = time.perf_counter() - t0
        rd = int(sub.draft.shape[0])
        gsub = {k: (v[:rd] if k in ("H", "conf", "argmax") else v[:nb]) for k, v in gpu.items()}
        problems, counts = compare(gsub, ref, check_argmax=False)
        parity = {"ok": not problems, **counts}
        cpu_baseline = {"value": round(nb / dt, 2), "unit": "sequence-steps/s", "cores": cores, "kind": "oracle",
                        "sample": f"first {nb} sequences of the same batch, one step, {dt:.1f} s wall",
                        "mean_accept_rate": round(float(ref['ver']['accept_rate'].mean()), 3)}
        # the same oracle on one thread, on a smaller sample (uniform batches only)
        n1 = min(nb, 16)
        if inp.gamma is None and n1 > 0:
            g = cfg.gamma
            one = workloads.StepInputs(cfg=workloads.config(args.workload, B=n1), gamma=None, row_off=None,
                                       draft=inp.draft[:n1 * g], target=inp.target[:n1 * (g + 1)],
                                       draft_tokens=inp.draft_tokens[:n1 * g], comp=inp.comp[:n1], mlp=inp.mlp)
            oracle.set_threads(1)
            t0 = time.perf_counter()
            oracle_step(one, seed, 0)
            cpu_baseline["single_thread_value"] = round(n1 / (time.perf_counter() - t0), 2)
            cpu_baseline["single_thread_sample"] = f"first {n1} sequences"
            oracle.set_threads(cores)
        if problems:
            print("PARITY FAILURE:\n" + "\n".join(problems[:20]), file=sys.stderr)

    out = {
        "metric": "verified sequence-steps/sec and achieved HBM GB/s (% of peak), B=256 \u03b3=8 V=128k",
        "value": round(value, 1), "unit": "sequence-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} gamma={'ragged' if inp.gamma is not None else cfg.gamma} "
                               f"V={cfg.V} {cfg.dtype} logits, {cfg.law}-shaped, seed {cfg.seed}",
                   "logits_dtype": cfg.dtype, "draft_rows": n_draft_rows, "target_rows": n_target_rows,
                   "launch": {k: sk.get_option(k) for k in ("stats_threads", "stats_unroll", "stats_target_wgs",
                                                            "stats_max_split", "stats_pipeline", "stats_nontemporal",
                                                            "step_tail")}},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity, **extra,
    }
    print(json.dumps(out))
    return 0 if (parity is None or parity["ok"]) else 1


if __name__ == "__main__":
    sys.exit(main())
