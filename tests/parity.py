"""Comparison of the HIP path's outputs with the CPU oracle's, shared by the GPU tests, the smoke
check and the benchmark.

Rules.  Discrete outputs (accepted length, emitted tokens, chosen gamma, argmax, flags) must be
identical, except that a row may differ
  * in the accepted length when the oracle's accept margin min_i |u_i q_i(t_i) - p_i(t_i)| < 1e-6
    (an absolute band, which is loose for tokens of small probability: such a row is also counted as
    accept_outside_relative_band when no tested position has |u q - p| < 2^-18 max(u q, p); that
    count must be zero),
  * in the emitted token when the oracle's CDF margin is below 1e-6,
  * in the chosen gamma when the oracle's best-minus-second score gap is below the sum of the
    absolute floors of the score tolerance of those two candidates (each side's two scores may be
    off by that much, which is what it takes to swap them),
  * in the fall-back flag and the emitted token when the oracle's residual mass lies within 2.5e-7
    of the fall-back threshold of 1e-6 (both sides fall back below the threshold; which side of it
    a mass that close lies on is decided by rounding).
Such rows are counted as excused, each class on its own; any other difference is a failure, and
callers bound the counts (assert_parity).
Floating outputs (entropy, confidence, aggregates, acceptance rate) must satisfy
|gpu - ref| <= 1e-4 |ref| + 1e-6.  The controller's scores: |gpu - ref| <= 1e-4 |ref| + floor_k.
The controller's inputs cross the ABI as binary32, so the oracle's controller is fed the oracle's
own signals rounded to binary32; what is left between the two sides is the GPU's error in a signal
(observed up to 7.5e-7 in an entropy near 10 bits, i.e. one binary32 step) times the network's gain.
floor_k = 1e-6 * max(1, G_k) with
G_k = Gamma_k * sum_h |W2[k,h]| * sum_{i in signals} |W1[h,i]| (no hidden layer: Gamma_k * sum_i |W2[k,i]|):
ReLU is 1-Lipschitz, so a change of 1e-6 in each signal input -- the absolute floor of the signal
tolerance itself -- moves score_k by at most 1e-6 * G_k, and a score is a product plus one (Eq. 1)
that can cancel to nearly zero, where the relative term gives no room.
"""
import numpy as np

import oracle
from workloads import stored_bits

RTOL, ATOL = 1e-4, 1e-6
ATOL_SCORE = 1e-6
MARGIN = 1e-6
MASS_BAND = 2.5e-7
REL_BAND = 2.0 ** -18   # the tighter, relative band of the accept test
GAMMAS = np.array([2.0, 4.0, 6.0, 8.0])


def _f32(a):
    """Round to binary32 and widen again: the values a float* argument of the ABI can carry."""
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def score_floor(mlp, mode):
    """Absolute floor of the score tolerance per candidate, shape [4] (see the module docstring)."""
    base = np.full(4, ATOL_SCORE)
    if mlp is None:
        return base
    W1 = mlp.get("W1")
    n_hidden = 0 if W1 is None else int(np.asarray(W1).shape[0])
    n_sig = 2 if mode == "pos0" else 4
    W2 = np.abs(np.asarray(mlp["W2"], dtype=np.float64))
    if n_hidden:
        per_hidden = np.abs(np.asarray(W1, dtype=np.float64))[:, :n_sig].sum(axis=1)
        gain = W2 @ per_hidden
    else:
        gain = W2[:, :n_sig].sum(axis=1)
    gain = np.broadcast_to(gain, (4,)) * GAMMAS
    return ATOL_SCORE * np.maximum(1.0, gain)


def oracle_step(inp, seed, step=0, mode="pos0", seq_base=0, gamma_max=None):
    """Run the whole oracle on one StepInputs (host copies of the same bytes)."""
    cfg = inp.cfg
    gamma = inp.gamma_host()
    d, t = stored_bits(inp.draft), stored_bits(inp.target)
    tok = inp.draft_tokens.cpu().numpy()
    gm = cfg.gamma_max if gamma_max is None else gamma_max
    sig = oracle.signals(d, cfg.dtype, cfg.B, cfg.V, gamma=gamma)
    ver = oracle.verify(d, t, cfg.dtype, cfg.B, cfg.V, tok, seed, step=step, gamma=gamma, gamma_max=gm,
                        seq_base=seq_base, debug=True)
    # the controller's inputs are float* in the ABI: the oracle's controller reads its own signals as binary32
    sel = oracle.select_gamma(inp.mlp, mode, _f32(sig["H"]), _f32(sig["conf"]), _f32(sig["agg"]), sig["row_off"],
                              inp.comp.cpu().numpy())
    return dict(sig=sig, ver=ver, sel=sel, V=cfg.V, mlp=inp.mlp, mode=mode)


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
    V = ref.get("V")
    problems = []
    B = ver["n_accepted"].shape[0]
    clean = (ver["row_flags"] & oracle.FLAG_NONFINITE) == 0   # outputs of flagged rows are unspecified
    row_clean = np.repeat(clean, sig["gamma"])
    _close("H", gpu["H"][row_clean], sig["H"][row_clean], problems)
    _close("conf", gpu["conf"][row_clean], sig["conf"][row_clean], problems)
    _close("agg", gpu["agg"][clean], sig["agg"][clean], problems)
    if check_argmax and not (gpu["argmax"][row_clean] == sig["argmax"][row_clean]).all():
        problems.append("argmax differs")
    # a residual mass this close to the fall-back threshold may land on either side of it
    edge_mass = np.abs(ver["resid_mass"] - oracle.RESID_FLOOR) < MASS_BAND
    gflags = gpu["row_flags"].astype(np.uint32)
    flag_diff = gflags != ver["row_flags"]
    flag_diff &= ~(edge_mass & ((gflags ^ ver["row_flags"]) == oracle.FLAG_FALLBACK))
    if check_flags and flag_diff.any():
        bad = np.flatnonzero(flag_diff)
        problems.append(f"row_flags differ at rows {bad[:8]}: gpu={gpu['row_flags'][bad[:8]]} "
                        f"ref={ver['row_flags'][bad[:8]]}")
    counts = dict(rows=int(B), excused_accept=0, excused_cdf=0, excused_gamma=0, excused_mass=0, mismatch=0,
                  accept_outside_relative_band=0)
    hi = 2**31 if V is None else V
    for b in range(B):
        if not clean[b]:
            n = gpu["n_accepted"][b]
            if not (0 <= n <= sig["gamma"][b] and gpu["num_tokens"][b] == n + 1 and 0 <= gpu["tokens"][b, n] < hi):
                problems.append(f"row {b} (non-finite input): outputs out of range")
            continue
        ng, nr = int(gpu["n_accepted"][b]), int(ver["n_accepted"][b])
        if ng != nr:
            if ver["marg_acc"][b] < MARGIN:
                counts["excused_accept"] += 1
                if "dbg" in ver:   # (u_i, q_i(t_i), p_i(t_i)) of the positions the oracle tested
                    u, q, pp = (ver["dbg"][b, :, k] for k in range(3))
                    tested = ~np.isnan(u)
                    lhs = u[tested] * q[tested]
                    close = np.abs(lhs - pp[tested]) < REL_BAND * np.maximum(lhs, pp[tested])
                    if not close.any():
                        counts["accept_outside_relative_band"] += 1
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
            if edge_mass[b] and 0 <= gpu["tokens"][b, ng] < hi:
                counts["excused_mass"] += 1
            elif ver["marg_cdf"][b] < MARGIN:
                counts["excused_cdf"] += 1
            else:
                counts["mismatch"] += 1
                problems.append(f"row {b}: emitted token gpu={gpu['tokens'][b, ng]} ref={ver['tokens'][b, ng]} "
                                f"cdf margin={ver['marg_cdf'][b]:.3e}")
    same_n = clean & (gpu["n_accepted"] == ver["n_accepted"])
    _close("accept_rate", gpu["accept_rate"][same_n], ver["accept_rate"][same_n], problems)
    floor = score_floor(ref.get("mlp"), ref.get("mode", "pos0"))
    _close("scores", gpu["scores"][clean], sel["scores"][clean], problems, atol=floor[None, :])
    dg = clean & (gpu["gamma_next"] != sel["gamma_next"])
    for b in np.flatnonzero(dg):
        order = np.argsort(-sel["scores"][b], kind="stable")   # the oracle's best and second candidate
        if sel["gap"][b] < floor[order[0]] + floor[order[1]]:
            counts["excused_gamma"] += 1
        else:
            counts["mismatch"] += 1
            problems.append(f"row {b}: gamma_next gpu={gpu['gamma_next'][b]} ref={sel['gamma_next'][b]} "
                            f"gap={sel['gap'][b]:.3e}")
    return problems, counts


def default_caps(rows):
    """Most excused rows a comparison over `rows` sequences may show before it counts as a failure:
    margins of 1e-6 are hit by about one sequence in a few hundred on the benchmark workloads."""
    few = max(1, rows // 32)
    return dict(excused_accept=few, excused_cdf=few, excused_gamma=max(1, rows // 64), excused_mass=0,
                accept_outside_relative_band=0)


def assert_parity(gpu, ref, caps=None, what="", **kw):
    """compare() must report no problem and no more excused rows than `caps` allows (per class)."""
    problems, counts = compare(gpu, ref, **kw)
    assert not problems, (what, problems[:10])
    limit = default_caps(counts["rows"])
    limit.update(caps or {})
    for k, cap in limit.items():
        assert counts[k] <= cap, (what, k, counts)
    return counts
