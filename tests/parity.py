"""Comparison of the HIP path's outputs with the CPU oracle's, shared by the GPU tests, the smoke
check and the benchmark.

Rules.  Discrete outputs (accepted length, emitted tokens, chosen gamma, argmax, flags) must be
identical, except that a row may differ in accepted length when the oracle's accept margin
min_i |u_i q_i(t_i) - p_i(t_i)| is below 1e-6, in the emitted token when the oracle's CDF margin is
below 1e-6, in the chosen gamma when the oracle's best-minus-second score gap is below
2e-5 * max(1, |score|), and in the fall-back flag and the emitted token when the oracle's residual
mass is below 1e-6 (whether a residual that small is exactly zero is decided by rounding: there
the two distributions agree to 1e-6 and either draw is as good).  Such rows are counted as
excused; any other difference is a failure.
Floating outputs (entropy, confidence, aggregates, acceptance rate) must satisfy
|gpu - ref| <= 1e-4 |ref| + 1e-6; the controller's scores |gpu - ref| <= 1e-4 |ref| + 1e-5: a
score is a product plus one (Eq. 1) and may cancel to nearly zero, while its error is set by the
size of the terms -- the signals reach the network rounded to binary32 (6e-8 relative) and a wide
network on [x, gamma] sums dozens of terms of size 1 to 10.
"""
import numpy as np

import oracle
from workloads import stored_bits

RTOL, ATOL = 1e-4, 1e-6
ATOL_SCORE = 1e-5
MARGIN = 1e-6


def oracle_step(inp, seed, step=0, mode="pos0", seq_base=0, gamma_max=None):
    """Run the whole oracle on one StepInputs (host copies of the same bytes)."""
    cfg = inp.cfg
    gamma = inp.gamma_host()
    d, t = stored_bits(inp.draft), stored_bits(inp.target)
    tok = inp.draft_tokens.cpu().numpy()
    gm = cfg.gamma_max if gamma_max is None else gamma_max
    sig = oracle.signals(d, cfg.dtype, cfg.B, cfg.V, gamma=gamma)
    ver = oracle.verify(d, t, cfg.dtype, cfg.B, cfg.V, tok, seed, step=step, gamma=gamma, gamma_max=gm,
                        seq_base=seq_base)
    sel = oracle.select_gamma(inp.mlp, mode, sig["H"], sig["conf"], sig["agg"], sig["row_off"],
                              inp.comp.cpu().numpy())
    return dict(sig=sig, ver=ver, sel=sel)


def _close(name, got, ref, problems, atol=ATOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bad = ~(np.abs(got - ref) <= RTOL * np.abs(ref) + atol)
    bad &= ~(np.isnan(got) & np.isnan(ref))
    if bad.any():
        i = np.argwhere(bad)[0]
        problems.append(f"{name}: {bad.sum()} values out of tolerance, first at {tuple(i)}: "
                        f"gpu={got[tuple(i)]!r} ref={ref[tuple(i)]!r}")


def compare(gpu, ref, check_flags=True, check_argmax=True):
    """-> (problems: list[str], counts: dict).  Empty problems means parity holds."""
    sig, ver, sel = ref["sig"], ref["ver"], ref["sel"]
    problems = []
    B = ver["n_accepted"].shape[0]
    clean = (ver["row_flags"] & oracle.FLAG_NONFINITE) == 0   # outputs of flagged rows are unspecified
    row_clean = np.repeat(clean, sig["gamma"])
    _close("H", gpu["H"][row_clean], sig["H"][row_clean], problems)
    _close("conf", gpu["conf"][row_clean], sig["conf"][row_clean], problems)
    _close("agg", gpu["agg"][clean], sig["agg"][clean], problems)
    if check_argmax and not (gpu["argmax"][row_clean] == sig["argmax"][row_clean]).all():
        problems.append("argmax differs")
    tiny_mass = ver["resid_mass"] < MARGIN   # there the fall-back decision hangs on rounding
    gflags = gpu["row_flags"].astype(np.uint32)
    flag_diff = gflags != ver["row_flags"]
    flag_diff &= ~(tiny_mass & ((gflags ^ ver["row_flags"]) == oracle.FLAG_FALLBACK))
    if check_flags and flag_diff.any():
        bad = np.flatnonzero(flag_diff)
        problems.append(f"row_flags differ at rows {bad[:8]}: gpu={gpu['row_flags'][bad[:8]]} "
                        f"ref={ver['row_flags'][bad[:8]]}")
    counts = dict(rows=int(B), excused_accept=0, excused_cdf=0, excused_gamma=0, excused_mass=0, mismatch=0)
    for b in range(B):
        if not clean[b]:
            W = gpu["tokens"].shape[1]
            n = gpu["n_accepted"][b]
            if not (0 <= n <= sig["gamma"][b] and gpu["num_tokens"][b] == n + 1 and 0 <= gpu["tokens"][b, n] < 2**31):
                problems.append(f"row {b} (non-finite input): outputs out of range")
            continue
        ng, nr = int(gpu["n_accepted"][b]), int(ver["n_accepted"][b])
        if ng != nr:
            if ver["marg_acc"][b] < MARGIN:
                counts["excused_accept"] += 1
            else:
                counts["mismatch"] += 1
                problems.append(f"row {b}: n_accepted gpu={ng} ref={nr} margin={ver['marg_acc'][b]:.3e}")
            continue
        if gpu["num_tokens"][b] != ng + 1:
            problems.append(f"row {b}: num_tokens {gpu['num_tokens'][b]} != n+1")
        if not (gpu["tokens"][b, :ng] == ver["tokens"][b, :ng]).all() or \
                not (gpu["tokens"][b, ng + 1:] == -1).all():
            counts["mismatch"] += 1
            problems.append(f"row {b}: accepted prefix / padding differs")
            continue
        if gpu["tokens"][b, ng] != ver["tokens"][b, ng]:
            if tiny_mass[b] and 0 <= gpu["tokens"][b, ng] < 2**31:
                counts["excused_mass"] += 1
            elif ver["marg_cdf"][b] < MARGIN:
                counts["excused_cdf"] += 1
            else:
                counts["mismatch"] += 1
                problems.append(f"row {b}: emitted token gpu={gpu['tokens'][b, ng]} ref={ver['tokens'][b, ng]} "
                                f"cdf margin={ver['marg_cdf'][b]:.3e}")
    same_n = clean & (gpu["n_accepted"] == ver["n_accepted"])
    _close("accept_rate", gpu["accept_rate"][same_n], ver["accept_rate"][same_n], problems)
    _close("scores", gpu["scores"][clean], sel["scores"][clean], problems, atol=ATOL_SCORE)
    dg = clean & (gpu["gamma_next"] != sel["gamma_next"])
    for b in np.flatnonzero(dg):
        if sel["gap"][b] < 2 * ATOL_SCORE * max(1.0, np.abs(sel["scores"][b]).max()):
            counts["excused_gamma"] += 1
        else:
            counts["mismatch"] += 1
            problems.append(f"row {b}: gamma_next gpu={gpu['gamma_next'][b]} ref={sel['gamma_next'][b]} "
                            f"gap={sel['gap'][b]:.3e}")
    return problems, counts
