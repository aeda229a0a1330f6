#!/usr/bin/env python3
"""Benchmark of the verify-and-select stage on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic logits already resident in
HBM, through the C ABI: by default one speckv_step call = two launches (row statistics of the draft
and the target rows in one, then one workgroup per sequence for signals, accept scan, controller,
residual masses and token pick); with --path three_calls the same step as speckv_signals +
speckv_verify + speckv_select_gamma (five launches, identical results).  The default workload is
the headline configuration: B=256, gamma=8, V=128256, bf16, Zipf-shaped logits.

Prints one JSON line: throughput in verified sequence-steps/s over exactly --steps steps, the HBM
roofline of the dominant kernel (row statistics) from HIP events stamped on sampled launches inside
those steps, the distribution of the step time, the bytes the method must move per step and the
rate they amount to, and the CPU oracle timed on the host cores over the same batch.  The step's
outputs are checked against the oracle before anything is reported.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0  # MI355X published peak
STEADY_STEPS = 300     # steps of this load after which the GPU's clocks have settled (about 100 are needed)


def kernel_sources_digest():
    """sha256 over the library's sources: the traffic figures under profiles/ name the digest they were
    measured at, and are reported only while it still matches."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2605_02888_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--path", default="one_call", choices=["one_call", "three_calls"])
    ap.add_argument("--B", type=int, default=None, help="override the batch size (not the headline number)")
    ap.add_argument("--V", type=int, default=None, help="override the vocabulary size (not the headline number)")
    ap.add_argument("--seed-offset", type=int, default=0, help="added to the workload's seed (reruns on other draws)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the probe, the other path, greedy and proposal timings")
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
    if args.V is not None:
        over["V"] = args.V
    cfg = workloads.config(args.workload, **over)
    cfg.seed += args.seed_offset
    gamma = None
    if args.workload == "C4":
        gamma = torch.full((cfg.B,), 4, dtype=torch.int32)   # the configuration's first step (Fixed-4)
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

    # the library creates its pool of timing events on the first speckv_profile call (tens of ms during
    # which the GPU would sit idle and drop its clocks): done here, before anything is timed
    sk.profile(1)
    for i in range(4):   # and the runtime's first stamped launches are slow (lazy set-up): taken here, untimed
        step(i)
    torch.cuda.synchronize()
    sk.profile(0)
    # untimed: a pre-roll that brings the clocks to their steady state when the warm-up asked for is
    # too short for that, then the warm-up itself
    preroll = max(0, STEADY_STEPS - args.warmup)
    for i in range(preroll + args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps.  A few launches of the row-statistics kernel carry a
    # start/stop event pair stamped with the dispatch's own times (a stamped kernel is followed by
    # a gap of 4-6 us, so stamping every launch would cost about 6 % of the step): every 20th, or
    # more often when K is small, so that at least 10 launches are sampled ---------------------------
    every = max(1, min(20, args.steps // 10))
    sk.set_option("profile_every", every)
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
    sk.set_option("profile_every", 1)

    # ---- distribution of the step time: the same K steps again, without stamped launches, an event
    # on the stream after every group of steps (at least 20 groups) -----------------------------------
    group = max(1, args.steps // 50)
    n_groups = args.steps // group
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_groups + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for gi in range(n_groups):
        for i in range(group):
            step(gi * group + i)
        marks[gi + 1].record()
    torch.cuda.synchronize()
    ms_plain = (time.perf_counter() - t0) * 1e3 / (n_groups * group)
    per = np.array([marks[k].elapsed_time(marks[k + 1]) / group for k in range(n_groups)]) * 1e3   # us per step
    dist = {"group_steps": group, "groups": n_groups, "median": round(float(np.median(per)), 2),
            "p10": round(float(np.percentile(per, 10)), 2), "p90": round(float(np.percentile(per, 90)), 2),
            "min": round(float(per.min()), 2), "max": round(float(per.max()), 2)}

    # ---- bytes the method must move in one step (every logit once, and position n of the target row
    # and, after a rejection, of the draft row a second time), from this step's accepted lengths ------
    step(0)
    gpu = runner.results(n_draft_rows)
    g_host = inp.gamma_host()
    bytes_t = n_target_rows * cfg.V * E
    bytes_d = n_draft_rows * cfg.V * E
    reread = int((1 + (gpu["n_accepted"] < g_host)).sum()) * cfg.V * E
    alg_bytes = bytes_t + bytes_d + reread

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
    def traffic_of(key):
        # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (a profiler cannot be
        # attached from in here): taken from profiles/ while the library's sources are the ones measured
        tpath = os.path.join(ROOT, "profiles", f"row_stats_{args.workload.lower()}_traffic.txt")
        if not os.path.exists(tpath) or args.B is not None or args.V is not None or args.opt or args.seed_offset:
            return None
        vals = dict(line.split()[:2] for line in open(tpath) if line.strip() and not line.startswith("#"))
        if vals.get("kernel_sources_digest") != kernel_sources_digest():
            return None
        return int(vals[key]) if key in vals else None

    def roof(kernel, nbytes, n, ms):
        avg = ms / max(n, 1) * 1e-3
        ach = nbytes / avg / 1e9 if n else 0.0
        return {"kernel": kernel, "achieved": round(ach, 1), "frac": round(ach / HBM_PEAK_GBS, 4),
                "bytes_per_launch": nbytes, "avg_launch_us": round(avg * 1e6, 2), "launches": n}

    if paired:
        r = roof("row_stats_pair", bytes_d + bytes_t, n_p, ms_p)
        roofline = {"bound": "hbm", "kernel": r["kernel"], "achieved": r["achieved"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": r["frac"], "traffic": traffic_of("row_stats_pair_bytes_per_launch"),
                    "traffic_source": "profiles/ (rocprofv3 counters of an earlier run of the same sources), not this run",
                    "bytes_per_launch": r["bytes_per_launch"], "avg_launch_us": r["avg_launch_us"],
                    "launches": r["launches"]}
    else:
        r = roof("row_stats_target", bytes_t, n_t, ms_t)
        rd = roof("row_stats_draft", bytes_d, n_d, ms_d)
        roofline = {"bound": "hbm", "kernel": r["kernel"], "achieved": r["achieved"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": r["frac"], "traffic": traffic_of("row_stats_target_bytes_per_launch"),
                    "traffic_source": "profiles/ (rocprofv3 counters of an earlier run of the same sources), not this run",
                    "bytes_per_launch": r["bytes_per_launch"], "avg_launch_us": r["avg_launch_us"],
                    "launches": r["launches"],
                    "row_stats_draft": {k: rd[k] for k in ("achieved", "frac", "bytes_per_launch", "avg_launch_us",
                                                           "launches")}}
    sec = ms_per_step * 1e-3
    extra = {
        # every logit once (the statistics pass) over the step time
        "step_logit_GBps": round((bytes_t + bytes_d) / sec / 1e9, 1),
        "step_frac_of_peak": round((bytes_t + bytes_d) / sec / 1e9 / HBM_PEAK_GBS, 4),
        # all bytes the method must move: the statistics pass plus the second read of position n
        "step_algorithmic_bytes": alg_bytes,
        "step_reread_bytes": reread,
        "step_algorithmic_GBps": round(alg_bytes / sec / 1e9, 1),
        "step_algorithmic_frac_of_peak": round(alg_bytes / sec / 1e9 / HBM_PEAK_GBS, 4),
        "step_us": dist,
        "preroll_steps": preroll,
        "profile_every": every,
        "ms_per_step_without_events": round(ms_plain, 4),
        "path": args.path,
        "kernel_us": breakdown,
    }

    if not args.no_extras:
        # the other way to issue the same step, for comparison
        for i in range(50):
            other(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            other(i)
        torch.cuda.synchronize()
        ms_other = (time.perf_counter() - t0) * 1e3 / args.steps
        name = "three_calls" if args.path == "one_call" else "one_call"
        extra["ms_per_step_" + name] = round(ms_other, 4)
        extra["value_" + name] = round(cfg.B / (ms_other * 1e-3), 1)

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

        # configurations whose logits fit the memory-side cache: single steps between events, warm
        # (the same buffers again) and cold (after 512 MB of other memory were written).  Everything
        # is queued ahead without host synchronisation, and the warm case queues a small fill in
        # place of the large one, so that both measure a step that starts behind another kernel.
        if bytes_t + bytes_d < 200e6:
            flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
            spacer = torch.empty(4096, dtype=torch.uint8, device=dev)
            res = {}
            for label, filler in (("warm", spacer), ("cold", flush)):
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(40)]
                for i, (a, b) in enumerate(ev):
                    filler.fill_(i & 0xff)
                    a.record()
                    step(i)
                    b.record()
                torch.cuda.synchronize()
                ts = np.array([a.elapsed_time(b) * 1e3 for a, b in ev[5:]])
                res[label] = {"median_us": round(float(np.median(ts)), 2), "p10": round(float(np.percentile(ts, 10)), 2),
                              "p90": round(float(np.percentile(ts, 90)), 2)}
            extra["single_step_between_events"] = res
            del flush

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
        excused = counts["excused_accept"] + counts["excused_cdf"] + counts["excused_gamma"] + counts["excused_mass"]
        # more than one excused sequence in thirty-two would itself be a finding
        parity = {"ok": not problems and excused <= max(1, nb // 32) and not counts["accept_outside_relative_band"],
                  **counts}
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
        "metric": "verified sequence-steps/sec and achieved HBM GB/s (% of peak), B=256 γ=8 V=128k",
        "value": round(value, 1), "unit": "sequence-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} gamma={'ragged' if inp.gamma is not None else cfg.gamma} "
                               f"V={cfg.V} {cfg.dtype} logits, {cfg.law}-shaped, seed {cfg.seed}",
                   "logits_dtype": cfg.dtype, "draft_rows": n_draft_rows, "target_rows": n_target_rows,
                   "launch": {k: sk.get_option(k) for k in ("stats_threads", "stats_unroll", "stats_target_wgs",
                                                            "stats_max_split", "stats_pipeline", "stats_nontemporal",
                                                            "stats_wgs_per_cu", "step_tail")}},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity, **extra,
    }
    print(json.dumps(out))
    return 0 if (parity is None or parity["ok"]) else 1


if __name__ == "__main__":
    sys.exit(main())
