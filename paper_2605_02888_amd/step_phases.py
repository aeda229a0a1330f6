"""Where the time inside the two launches of speckv_step goes, from the per-workgroup clock
readings that speckv_trace records (measurement helper; the library's results are not affected).

    python -m paper_2605_02888_amd.step_phases [--workload C3] [--steps 20] [--opt name=value ...]

Prints, in microseconds and over all traced steps: the time between successive marks of the tail
launch per sequence (entry ... token stored), when its workgroups start and
end relative to the first one, the lifetime of the statistics workgroups, how long the statistics
launch takes to drain (last exit minus the exit of the workgroup at the 90th percentile), and the
gap between the last exit of the statistics launch and the first entry of the tail launch.
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def pct(a, qs=(10, 50, 90, 100)):
    a = np.asarray(a, dtype=np.float64)
    return "  ".join(f"p{q}={np.percentile(a, q):7.2f}" for q in qs) + f"  mean={a.mean():7.2f}"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--B", type=int, default=None)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--opt", action="append", default=[])
    args = ap.parse_args()

    import torch
    import workloads
    import paper_2605_02888_amd as pkg
    from paper_2605_02888_amd.runner import StepRunner

    dev = "cuda:0"
    cfg = workloads.config(args.workload, **({} if args.B is None else {"B": args.B}))
    gamma = torch.full((cfg.B,), 4, dtype=torch.int32) if args.workload == "C4" else None
    inp = workloads.make_step(cfg, device=dev, gamma=gamma)
    sk = pkg.SpecKV(device=0)
    for kv in args.opt:
        k, v = kv.split("=")
        sk.set_option(k, int(v))
    r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, device=dev,
                   with_argmax=False)
    batch = r.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
    khz = 100000  # the constant-rate clock of this GPU family; replaced below by what the runtime reports
    try:
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        v = ctypes.c_int()
        # hipDeviceAttributeWallClockRate = 10017 (hip_runtime_api.h)
        if hip.hipDeviceGetAttribute(ctypes.byref(v), 10017, 0) == 0 and v.value > 0:
            khz = v.value
    except OSError:
        pass
    tick_us = 1e3 / khz
    S = 32  # clock readings per sequence in the tail launch
    words = S * cfg.B + 2 * 70000
    buf = torch.zeros(words, dtype=torch.int64, device=dev)
    for i in range(args.warmup):
        r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, cfg.seed, i)
    torch.cuda.synchronize()
    sk.trace(buf)
    marks = ["entry", "statistics merged, token logits gathered", "accept scan done", "descriptor visible (barrier)",
             "own share of the residual masses done", "all masses done (barrier)", "chunk holding the threshold found",
             "that chunk re-read and summed", "prefix exchanged (barrier)", "token found (barrier)", "token stored"]
    rec = {k: [] for k in ("wave_first", "wave_last", "tail_wg", "tail_start", "tail_end", "stats_wg", "stats_start", "stats_drain", "gap",
                           "stats_span", "tail_span", "n0_mass", "nx_mass")}
    delta = [[] for _ in marks]
    for i in range(args.steps):
        buf.zero_()
        r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, cfg.seed, i)
        torch.cuda.synchronize()
        h = buf.cpu().numpy().astype(np.float64) * tick_us
        tail = h[:S * cfg.B].reshape(cfg.B, S)
        st = h[S * cfg.B:].reshape(-1, 2)
        st = st[(st[:, 0] > 0) & (st[:, 1] > 0)]
        n_acc = r.n_accepted.cpu().numpy()
        t0 = tail[:, 0].min()
        last = len(marks) - 1
        for k in range(1, len(marks)):
            delta[k] += list(tail[:, k] - tail[:, k - 1])
        wv = tail[:, 16:32]
        wv = np.where(wv > 0, wv, np.nan)
        rec["wave_first"] += list(np.nanmin(wv, axis=1) - tail[:, 3])
        rec["wave_last"] += list(np.nanmax(wv, axis=1) - tail[:, 3])
        rec["tail_wg"] += list(tail[:, last] - tail[:, 0])
        rec["tail_start"] += list(tail[:, 0] - t0)
        rec["tail_end"] += list(tail[:, last] - t0)
        rec["tail_span"].append(tail[:, last].max() - t0)
        rec["n0_mass"] += list((tail[:, 5] - tail[:, 3])[n_acc == 0])
        rec["nx_mass"] += list((tail[:, 5] - tail[:, 3])[n_acc != 0])
        if len(st):
            s0 = st[:, 0].min()
            rec["stats_wg"] += list(st[:, 1] - st[:, 0])
            rec["stats_start"] += list(st[:, 0] - s0)
            rec["stats_span"].append(st[:, 1].max() - s0)
            rec["stats_drain"].append(st[:, 1].max() - np.percentile(st[:, 1], 90))
            rec["gap"].append(t0 - st[:, 1].max())
    sk.trace(None)
    print(f"workload {cfg.name} B={cfg.B} V={cfg.V} {cfg.dtype}; {args.steps} traced steps; clock {khz} kHz "
          f"({tick_us * 1e3:.0f} ns per tick); options {args.opt}")
    print(f"sequences with n = 0 in the last step: {int((n_acc == 0).sum())} of {cfg.B}")
    print("tail launch, thread 0 of each workgroup, time since the previous mark (us):")
    for k in range(1, len(marks)):
        print(f"  -> {marks[k]:<46}{pct(delta[k])}")
    names = {"wave_first": "tail: descriptor visible -> first wave out of chunks",
             "wave_last": "tail: descriptor visible -> last wave out of chunks", "tail_wg": "tail: workgroup lifetime", "tail_start": "tail: entry after first entry",
             "tail_end": "tail: exit after first entry", "tail_span": "tail: first entry -> last exit (per step)",
             "n0_mass": "tail: residual masses, n = 0", "nx_mass": "tail: residual masses, n > 0",
             "stats_wg": "statistics: workgroup lifetime", "stats_start": "statistics: entry after first entry",
             "stats_span": "statistics: first entry -> last exit (per step)",
             "stats_drain": "statistics: last exit - p90 exit (per step)",
             "gap": "last statistics exit -> first tail entry (per step)"}
    for k, label in names.items():
        if rec[k]:
            print(f"{label:<52}{pct(rec[k])}")
    sk.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
