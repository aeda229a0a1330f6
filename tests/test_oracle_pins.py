"""Pins for the CPU oracle: every oracle routine is checked against something other than
itself -- published known answers, closed forms, library routines (scipy / numpy / torch),
exhaustive enumeration on tiny vocabularies and Monte-Carlo laws with stated error bars.

Run with:  python -m pytest tests -m "not gpu"
"""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import oracle

LN2 = np.log(2.0)


# --------------------------------------------------------------------------- helpers
def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _tile(rows, B):
    """rows [k, V] -> [B*k, V]: every sequence sees the same logits."""
    rows = _f32(rows)
    return np.ascontiguousarray(np.broadcast_to(rows[None], (B,) + rows.shape).reshape(-1, rows.shape[1]))


def _softmax64(x):
    return scipy.special.softmax(np.asarray(x, dtype=np.float64), axis=-1)


def _sample_tokens(q, B, rng):
    """tokens [B, gamma] with column i drawn from q[i] (test-side input preparation)."""
    cols = [rng.choice(q.shape[1], size=B, p=q[i]) for i in range(q.shape[0])]
    return np.stack(cols, axis=1).astype(np.int32)


# --------------------------------------------------------------------------- Philox
def test_philox_known_answers(golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(t, 16) for t in line.split()]
            out = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in out] == w[6:10]
            n += 1
    assert n == 3


def test_uniform_construction_and_counter_layout():
    # u_i must be (word0 >> 8) * 2^-24 of block (seq_base+b, i, step, 0) under key (seed lo, seed hi).
    B, g, V = 5, 3, 4
    seed, step, base = 0x1234567890ABCDEF, 7, 1000
    x = np.zeros((B * g, V), dtype=np.float32)          # p == q: every position is tested
    t = np.zeros((B * (g + 1), V), dtype=np.float32)
    tok = np.zeros(B * g, dtype=np.int32)
    out = oracle.verify(x, t, "f32", B, V, tok, seed, step=step, gamma_uniform=g, seq_base=base,
                        debug=True)
    for b in range(B):
        for i in range(g):
            w = oracle.philox4x32_10([base + b, i, step, 0], [seed & 0xFFFFFFFF, seed >> 32])
            assert out["dbg"][b, i, 0] == (int(w[0]) >> 8) * 2.0 ** -24


def test_accept_uniforms_are_uniform():
    B = 200_000
    x = np.zeros((B, 2), dtype=np.float32)
    t = np.zeros((2 * B, 2), dtype=np.float32)
    out = oracle.verify(x, t, "f32", B, 2, np.zeros(B, dtype=np.int32), seed=99, gamma_uniform=1,
                        debug=True)
    u = out["dbg"][:, 0, 0]
    assert u.min() >= 0.0 and u.max() < 1.0
    assert scipy.stats.kstest(u, "uniform").pvalue > 1e-3


# --------------------------------------------------------------------------- dtype decode
def test_half_and_bfloat_decode_match_torch_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    as_i16 = torch.from_numpy(bits.view(np.int16))
    for name, tdt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        want = as_i16.view(tdt).to(torch.float64).numpy()
        got = oracle.load_logits(bits, name)
        same = (got == want) | (np.isnan(got) & np.isnan(want))
        assert same.all(), name
        assert (np.signbit(got) == np.signbit(want))[~np.isnan(want)].all()


# --------------------------------------------------------------------------- softmax / entropy / confidence
@pytest.mark.parametrize("V", [2, 32000, 128256])
def test_uniform_row_has_log2V_bits_and_conf_1_over_V(V):
    x = np.full(V, 3.25, dtype=np.float32)
    p, H, c, am, bad = oracle.row_softmax(x, "f32", 0, V)
    assert abs(H - np.log2(V)) < 1e-9
    assert abs(c - 1.0 / V) < 1e-15
    assert am == 0 and not bad
    assert abs(p.sum() - 1.0) < 1e-12


def test_two_equal_maxima_rest_masked_is_one_bit():
    x = np.full(1000, -np.inf, dtype=np.float32)
    x[17] = x[400] = 2.5
    p, H, c, am, bad = oracle.row_softmax(x, "f32", 0, 1000)
    assert H == 1.0 and c == 0.5 and am == 17 and not bad
    assert p[17] == 0.5 and p[400] == 0.5 and p.sum() == 1.0


def test_two_level_row_closed_form():
    V, k, a = 5000, 7, 4.0
    x = np.zeros(V, dtype=np.float32)
    x[100:100 + k] = a
    Z = k * np.exp(a) + (V - k)
    ph, pl = np.exp(a) / Z, 1.0 / Z
    H_want = -(k * ph * np.log2(ph) + (V - k) * pl * np.log2(pl))
    _, H, c, am, _ = oracle.row_softmax(x, "f32", 0, V)
    assert abs(H - H_want) < 1e-10 and abs(c - ph) < 1e-15 and am == 100


def test_shift_invariance_and_row_indexing():
    rng = np.random.default_rng(1)
    x = _f32(3 * rng.standard_normal((3, 777)))
    y = x.copy()
    y[1] += 8.0  # exact in binary32 for these magnitudes? compare against the shifted row's own softmax
    _, H0, c0, a0, _ = oracle.row_softmax(x, "f32", 1, 777)
    _, H1, c1, a1, _ = oracle.row_softmax(y, "f32", 1, 777)
    # the shift is applied in float32 so compare loosely; argmax must not move
    assert abs(H0 - H1) < 1e-4 and abs(c0 - c1) < 1e-6 and a0 == a1
    # row 2 of the buffer really is row 2
    p2, *_ = oracle.row_softmax(x, "f32", 2, 777)
    np.testing.assert_allclose(p2, _softmax64(x[2]), rtol=1e-12, atol=0)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_softmax_entropy_against_scipy(dtype):
    rng = np.random.default_rng(7)
    V, rows = 4099, 6
    x32 = torch.from_numpy(_f32(3 * rng.standard_normal((rows, V))))
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    stored = x32.to(tdt)
    x64 = stored.to(torch.float64).numpy()
    bits = stored.numpy() if dtype == "f32" else stored.view(torch.int16).numpy().view(np.uint16)
    for r in range(rows):
        p, H, c, am, bad = oracle.row_softmax(bits, dtype, r, V)
        want = _softmax64(x64[r])
        np.testing.assert_allclose(p, want, rtol=1e-12, atol=1e-300)
        assert abs(H - scipy.stats.entropy(want, base=2)) < 1e-10
        assert abs(c - want.max()) < 1e-15
        assert am == int(np.argmax(x64[r])) and not bad


def test_signals_aggregates_and_ragged_layout():
    rng = np.random.default_rng(3)
    V = 257
    gamma = np.array([2, 8, 1, 4], dtype=np.int32)
    rows = int(gamma.sum())
    x = _f32(2 * rng.standard_normal((rows, V)))
    s = oracle.signals(x, "f32", 4, V, gamma=gamma)
    off = np.concatenate([[0], np.cumsum(gamma)])
    P = _softmax64(x)
    H = scipy.stats.entropy(P, base=2, axis=1)
    C = P.max(axis=1)
    np.testing.assert_allclose(s["H"], H, atol=1e-11)
    np.testing.assert_allclose(s["conf"], C, atol=1e-15)
    assert (s["argmax"] == x.argmax(axis=1)).all()
    for b in range(4):
        sl = slice(off[b], off[b + 1])
        np.testing.assert_allclose(s["agg"][b], [H[sl].mean(), C[sl].mean(), H[sl].max(), C[sl].min()],
                                   atol=1e-11)
        assert s["agg"][b, 3] <= s["agg"][b, 1] and s["agg"][b, 0] <= s["agg"][b, 2]


def test_nonfinite_rows_are_reported():
    x = np.zeros(10, dtype=np.float32)
    assert not oracle.row_softmax(x, "f32", 0, 10)[4]
    x[3] = np.nan
    assert oracle.row_softmax(x, "f32", 0, 10)[4]
    x[3] = np.inf
    assert oracle.row_softmax(x, "f32", 0, 10)[4]
    x[3] = -np.inf
    assert not oracle.row_softmax(x, "f32", 0, 10)[4]


# --------------------------------------------------------------------------- accept / reject
@pytest.mark.parametrize("seed", [0, 1, 2**63 + 5])
def test_identical_distributions_accept_every_draft(seed):
    rng = np.random.default_rng(11)
    B, g, V = 64, 8, 50
    d = _f32(3 * rng.standard_normal((B * g, V)))
    t = np.zeros((B * (g + 1), V), dtype=np.float32)
    for b in range(B):
        t[b * (g + 1): b * (g + 1) + g] = d[b * g:(b + 1) * g]
    tok = rng.integers(0, V, size=B * g).astype(np.int32)
    out = oracle.verify(d, t, "f32", B, V, tok, seed, gamma_uniform=g)
    assert (out["n_accepted"] == g).all() and (out["num_tokens"] == g + 1).all()
    assert (out["accept_rate"] == 1.0).all()
    assert (out["tokens"][:, :g] == tok.reshape(B, g)).all()
    assert ((out["tokens"][:, g] >= 0) & (out["tokens"][:, g] < V)).all()


def test_disjoint_supports_reject_at_once_and_emit_from_target_support():
    B, g, V = 200, 4, 10
    NEG = -np.inf
    drow = np.full(V, NEG, dtype=np.float32); drow[:5] = 0.0
    trow = np.full(V, NEG, dtype=np.float32); trow[5:] = np.arange(5)
    d = _tile(np.stack([drow] * g), B)
    t = _tile(np.stack([trow] * (g + 1)), B)
    tok = np.random.default_rng(5).integers(0, 5, size=B * g).astype(np.int32)
    out = oracle.verify(d, t, "f32", B, V, tok, seed=3, gamma_uniform=g, gamma_max=8)
    assert (out["n_accepted"] == 0).all() and (out["num_tokens"] == 1).all()
    assert (out["tokens"][:, 0] >= 5).all()
    assert (out["tokens"][:, 1:] == -1).all() and out["tokens"].shape == (B, 9)
    assert (out["row_flags"] == 0).all()


def test_accept_boundaries_strict_inequality():
    # q(t) = 0 < p(t): always accepted.  p(t) = 0: never accepted, even if q(t) = 0 too.
    V = 4
    NEG = -np.inf
    d = _f32([[0.0, 0.0, NEG, NEG]])
    t = _f32([[0.0, NEG, 0.0, NEG], [0.0, 0.0, 0.0, 0.0]])
    B = 500
    D, T = _tile(d, B), _tile(t, B)
    for tok_id, want in ((2, 1), (1, 0), (3, 0)):
        tok = np.full(B, tok_id, dtype=np.int32)
        out = oracle.verify(D, T, "f32", B, V, tok, seed=8, gamma_uniform=1)
        assert (out["n_accepted"] == want).all(), tok_id


def test_per_position_acceptance_probability_is_sum_of_min():
    rng = np.random.default_rng(21)
    B, V = 200_000, 6
    d = _f32(rng.standard_normal((1, V)))
    t = _f32(np.stack([d[0] + rng.standard_normal(V), rng.standard_normal(V)]))
    q, p = _softmax64(d), _softmax64(t)
    tok = _sample_tokens(q, B, rng).reshape(-1)
    out = oracle.verify(_tile(d, B), _tile(t, B), "f32", B, V, tok, seed=77, gamma_uniform=1)
    alpha = np.minimum(p[0], q[0]).sum()
    got = out["n_accepted"].mean()
    assert abs(got - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / B)


@pytest.mark.parametrize("g", [2, 4, 6, 8])
@pytest.mark.parametrize("alpha", [0.5, 0.7, 0.9])
def test_expected_tokens_per_step_geometric_law(g, alpha):
    # V = 2, q = (1/2, 1/2), p = (1/2 + delta, 1/2 - delta): acceptance is i.i.d. with rate
    # alpha = 1 - delta, so E[tokens per step] = (1 - alpha^(g+1)) / (1 - alpha).
    B = 120_000
    delta = 1.0 - alpha
    d = _f32([[0.0, 0.0]] * g)
    lt = np.log([0.5 + delta, 0.5 - delta]) if delta < 0.5 else np.array([0.0, -np.inf])
    t = _f32([lt] * (g + 1))
    rng = np.random.default_rng(1000 * g + int(alpha * 10))
    tok = rng.integers(0, 2, size=B * g).astype(np.int32)
    out = oracle.verify(_tile(d, B), _tile(t, B), "f32", B, 2, tok, seed=4242 + g, gamma_uniform=g)
    k = np.arange(g + 1)
    pmf = np.where(k < g, alpha ** k * (1 - alpha), alpha ** g)
    mean = ((k + 1) * pmf).sum()
    assert abs(mean - (1 - alpha ** (g + 1)) / (1 - alpha)) < 1e-12
    var = (((k + 1) - mean) ** 2 * pmf).sum()
    assert abs(out["num_tokens"].mean() - mean) < 4 * np.sqrt(var / B)
    assert (out["num_tokens"] == out["n_accepted"] + 1).all()
    np.testing.assert_array_equal(out["accept_rate"], out["n_accepted"] / g)


# --------------------------------------------------------------------------- residual / inverse CDF
def test_residual_hand_example():
    p = np.array([0.5, 0.1, 0.3, 0.1])
    q = np.array([0.2, 0.4, 0.1, 0.3])
    r, R = oracle.residual(p, q)
    np.testing.assert_allclose(r, [0.3, 0.0, 0.2, 0.0], atol=1e-16)
    assert abs(R - 0.5) < 1e-16
    # tau just below / above the first positive block; zero-mass tokens are never chosen
    assert oracle.inverse_cdf(r, 0.0)[0] == 0
    assert oracle.inverse_cdf(r, 0.29)[0] == 0
    assert oracle.inverse_cdf(r, 0.31)[0] == 2
    assert oracle.inverse_cdf(r, r[0])[0] == 2           # strict: C_v > tau
    assert oracle.inverse_cdf(r, 10.0)[0] == 2           # rounding fallback: last positive entry
    rb, Rb = oracle.residual(p, None)
    np.testing.assert_array_equal(rb, p)
    assert abs(Rb - 1.0) < 1e-15


def test_residual_mass_identity_and_searchsorted_cross_check():
    rng = np.random.default_rng(31)
    for V in (3, 17, 1000):
        p = _softmax64(2 * rng.standard_normal(V))
        q = _softmax64(2 * rng.standard_normal(V))
        r, R = oracle.residual(p, q)
        assert abs(R - (1.0 - np.minimum(p, q).sum())) < 1e-12
        C = np.cumsum(r)
        for tau in rng.uniform(0, R, size=200):
            y, margin = oracle.inverse_cdf(r, tau)
            assert y == int(np.searchsorted(C, tau, side="right"))
            lo = C[y - 1] if y > 0 else 0.0
            assert abs(margin - min(tau - lo, C[y] - tau)) < 1e-15


def test_resample_uniform_is_word1_of_block_n():
    # One rejected position (disjoint supports): the emitted token must be the inverse CDF of
    # word1 * 2^-32 of block (b, n=0, step, 0) over the residual (= p here).
    V, B = 8, 300
    NEG = -np.inf
    d = _f32([[0, 0, 0, 0, NEG, NEG, NEG, NEG]])
    trow = np.array([NEG, NEG, NEG, NEG, 0.3, -0.2, 1.0, 0.1])
    t = _f32([trow, np.zeros(V)])
    seed, step = 555, 3
    out = oracle.verify(_tile(d, B), _tile(t, B), "f32", B, V, np.zeros(B, dtype=np.int32), seed,
                        step=step, gamma_uniform=1)
    p = _softmax64(_f32(trow))
    C = np.cumsum(p)
    for b in range(B):
        w = oracle.philox4x32_10([b, 0, step, 0], [seed & 0xFFFFFFFF, seed >> 32])
        tau = int(w[1]) * 2.0 ** -32 * C[-1]
        if np.min(np.abs(C - tau)) > 1e-12:
            assert out["tokens"][b, 0] == int(np.searchsorted(C, tau, side="right"))


# --------------------------------------------------------------------------- losslessness
def test_losslessness_by_enumeration_from_oracle_arrays():
    # P(first emitted token = y) = min(p,q)(y) + (1 - sum min(p,q)) r(y)/R  must equal p(y).
    rng = np.random.default_rng(41)
    for V in (2, 3, 6):
        for _ in range(20):
            xd = _f32(2 * rng.standard_normal((1, V)))
            xt = _f32(2 * rng.standard_normal((1, V)))
            q = oracle.row_softmax(xd, "f32", 0, V)[0]
            p = oracle.row_softmax(xt, "f32", 0, V)[0]
            r, R = oracle.residual(p, q)
            acc = np.array([q[v] * min(1.0, p[v] / q[v]) for v in range(V)])
            dist = acc + (1.0 - acc.sum()) * r / R
            np.testing.assert_allclose(dist, p, atol=1e-12)


def test_emitted_tokens_follow_target_distribution_chi_square():
    # Fixed rows at every position; slot j of the emitted tokens, when it exists, must be
    # distributed as p_j (j < gamma: accepted draft or correction; j = gamma: bonus).
    rng = np.random.default_rng(51)
    B, g, V = 400_000, 3, 5
    xd = _f32(1.5 * rng.standard_normal((g, V)))
    xt = _f32(np.concatenate([xd + 0.8 * rng.standard_normal((g, V)), rng.standard_normal((1, V))]))
    q, p = _softmax64(xd), _softmax64(xt)
    tok = _sample_tokens(q, B, rng).reshape(-1)
    out = oracle.verify(_tile(xd, B), _tile(xt, B), "f32", B, V, tok, seed=2024, gamma_uniform=g)
    for j in range(g + 1):
        have = out["num_tokens"] > j
        obs = np.bincount(out["tokens"][have, j], minlength=V).astype(float)
        exp = p[j] * have.sum()
        pval = scipy.stats.chisquare(obs, exp).pvalue
        assert pval > 1e-3, (j, pval)
    # exhaustive law of the accepted-prefix length: P(n >= j) = prod_{i<j} sum_v min(p_i, q_i)
    a = np.minimum(p[:g], q).sum(axis=1)
    for j in range(1, g + 1):
        want = np.prod(a[:j])
        got = (out["n_accepted"] >= j).mean()
        assert abs(got - want) < 4 * np.sqrt(want * (1 - want) / B)


def test_joint_law_of_first_two_slots_exhaustive():
    # gamma = 2, V = 3: the emitted pair (slot0, slot1) must have law p_0(a) * p_1(b) whenever
    # slot 1 exists given slot 0 was an accepted draft or not -- enumerate all 9 pairs.
    rng = np.random.default_rng(61)
    B, g, V = 400_000, 2, 3
    xd = _f32(rng.standard_normal((g, V)))
    xt = _f32(rng.standard_normal((g + 1, V)))
    q, p = _softmax64(xd), _softmax64(xt)
    tok = _sample_tokens(q, B, rng).reshape(-1)
    out = oracle.verify(_tile(xd, B), _tile(xt, B), "f32", B, V, tok, seed=909, gamma_uniform=g)
    # P(slot0 = a accepted) = min(p0, q0)(a); then slot 1 ~ p_1 -> P(pair a,b) = min(p0,q0)(a) p1(b)
    have2 = out["num_tokens"] >= 2
    obs = np.zeros((V, V))
    np.add.at(obs, (out["tokens"][have2, 0], out["tokens"][have2, 1]), 1.0)
    exp = np.outer(np.minimum(p[0], q[0]), p[1]) * B
    pval = scipy.stats.chisquare(obs.ravel(), exp.ravel() * obs.sum() / exp.sum()).pvalue
    assert pval > 1e-3
    assert abs(have2.mean() - np.minimum(p[0], q[0]).sum()) < 4 * np.sqrt(0.25 / B)


# --------------------------------------------------------------------------- flags, layout, placement
def test_bad_token_is_flagged_and_rejected_there():
    B, g, V = 3, 4, 6
    x = np.zeros((B * g, V), dtype=np.float32)
    t = np.zeros((B * (g + 1), V), dtype=np.float32)
    tok = np.zeros(B * g, dtype=np.int32)
    tok[1 * g + 2] = V          # sequence 1, position 2
    tok[2 * g + 0] = -1         # sequence 2, position 0
    out = oracle.verify(x, t, "f32", B, V, tok, seed=1, gamma_uniform=g)
    assert list(out["n_accepted"]) == [4, 2, 0]
    assert list(out["row_flags"] & oracle.FLAG_BAD_TOKEN) == [0, 2, 2]
    # p == q and the bad token has probability 0 on both sides: residual mass is 0 -> fallback to p_n
    assert list(out["row_flags"] & oracle.FLAG_FALLBACK) == [0, 4, 4]
    assert ((out["tokens"][np.arange(B), out["n_accepted"]] >= 0)).all()


def test_nonfinite_flag_covers_rows_after_the_first_rejection():
    B, g, V = 1, 3, 4
    NEG = -np.inf
    d = _f32([[0, 0, NEG, NEG]] * g)
    t = _f32([[NEG, NEG, 0, 0]] * (g + 1))
    t[g, 1] = np.nan            # bonus row, never reached by the accept loop
    out = oracle.verify(d, t, "f32", B, V, np.zeros(g, dtype=np.int32), seed=0, gamma_uniform=g)
    assert out["n_accepted"][0] == 0 and out["row_flags"][0] & oracle.FLAG_NONFINITE


def test_ragged_batch_equals_each_sequence_alone():
    rng = np.random.default_rng(71)
    V = 97
    gamma = np.array([2, 8, 4, 6], dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(gamma)])
    rows = int(off[-1])
    d = _f32(2 * rng.standard_normal((rows, V)))
    t = np.zeros((rows + 4, V), dtype=np.float32)
    for b in range(4):
        g = gamma[b]
        t[off[b] + b: off[b] + b + g] = d[off[b]:off[b] + g] + _f32(0.7 * rng.standard_normal((g, V)))
        t[off[b] + b + g] = _f32(rng.standard_normal(V))
    tok = np.array([rng.choice(V, p=_softmax64(d[r])) for r in range(rows)], dtype=np.int32)
    full = oracle.verify(d, t, "f32", 4, V, tok, seed=5, step=2, gamma=gamma, gamma_max=8)
    for b in range(4):
        g = int(gamma[b])
        one = oracle.verify(d[off[b]:off[b] + g], t[off[b] + b:off[b] + b + g + 1], "f32", 1, V,
                            tok[off[b]:off[b] + g], seed=5, step=2, gamma_uniform=g, gamma_max=8,
                            seq_base=b)
        assert one["n_accepted"][0] == full["n_accepted"][b]
        assert (one["tokens"][0] == full["tokens"][b]).all()


def test_residual_mass_is_reported_before_the_fallback():
    # R = sum max(0, p - q) = total-variation distance.  Two-token rows with p = (0.75, 0.25),
    # q = (0.25, 0.75): a drafted token 1 is rejected unless u < 1/3, and then R = 0.5.
    d = np.log(np.array([[0.25, 0.75]], dtype=np.float64)).astype(np.float32)
    t = np.log(np.array([[0.75, 0.25], [0.5, 0.5]], dtype=np.float64)).astype(np.float32)
    hits = 0
    for seed in range(40):
        out = oracle.verify(d, t, "f32", 1, 2, np.array([1], np.int32), seed=seed, gamma_uniform=1)
        if out["n_accepted"][0] == 0:
            hits += 1
            np.testing.assert_allclose(out["resid_mass"][0], 0.5, rtol=1e-6)
            assert out["tokens"][0, 0] == 0 and not out["row_flags"][0] & oracle.FLAG_FALLBACK
        else:
            np.testing.assert_allclose(out["resid_mass"][0], 1.0, rtol=1e-12)   # bonus row: all of p
    assert hits > 10
    # identical rows and an unusable token: rejected with R = 0 exactly, fall-back to p
    out = oracle.verify(d, np.concatenate([d, t[1:]]), "f32", 1, 2, np.array([7], np.int32), seed=1, gamma_uniform=1)
    assert out["resid_mass"][0] == 0.0 and out["row_flags"][0] == (oracle.FLAG_BAD_TOKEN | oracle.FLAG_FALLBACK)


def test_fallback_threshold_on_the_residual_mass():
    # Two-token rows whose total-variation distance R = |delta| sits just below and just above the
    # floor of 1e-6, with an unusable drafted token so that position 0 is rejected whatever u is.
    # Below the floor the token is the inverse CDF of p_0 at u' and the flag is set; above it the
    # residual is the point mass on token 0 (p_0(0) > q_0(0)), whatever u' is.
    q = np.array([0.5, 0.5])
    for delta, falls_back in ((4e-7, True), (9.9e-7, True), (1.01e-6, False), (3e-6, False), (0.0, True)):
        p = np.array([0.5 + delta, 0.5 - delta])
        d = np.log(q)[None, :].astype(np.float64)
        t = np.stack([np.log(p), np.log([0.5, 0.5])]).astype(np.float64)
        # binary32 logits realise delta to about 2e-8 (checked through the reported mass), which
        # leaves every case on its side of the floor
        d32, t32 = d.astype(np.float32), t.astype(np.float32)
        seen = set()
        for seed in range(60):
            out = oracle.verify(d32, t32, "f32", 1, 2, np.array([9], np.int32), seed=seed, gamma_uniform=1)
            R = out["resid_mass"][0]
            assert out["n_accepted"][0] == 0 and out["row_flags"][0] & oracle.FLAG_BAD_TOKEN
            fb = bool(out["row_flags"][0] & oracle.FLAG_FALLBACK)
            assert abs(R - delta) < 5e-8
            assert fb == (R < oracle.RESID_FLOOR) == falls_back
            w = oracle.philox4x32_10([0, 0, 0, 0], [seed, 0])
            u2 = float(w[1]) * 2.0 ** -32
            prow, _, _, _, _ = oracle.row_softmax(t32, "f32", 0, 2)
            if fb:
                want = int(np.searchsorted(np.cumsum(prow), u2 * prow.sum(), side="right"))
            else:
                want = 0
            assert out["tokens"][0, 0] == min(want, 1)
            seen.add(int(out["tokens"][0, 0]))
        if falls_back:
            assert seen == {0, 1}              # a draw from p_0 reaches both tokens


# --------------------------------------------------------------------------- controller
def _zero_mlp(n_in, b2, n_hidden=16):
    return {"W1": np.zeros((n_hidden, n_in), np.float32), "b1": np.zeros(n_hidden, np.float32),
            "W2": np.zeros((4, n_hidden), np.float32), "b2": np.asarray(b2, np.float32)}


def test_controller_known_argmax_and_eq1_scaling():
    H = np.array([1.0, 2.0]); c = np.array([0.5, 0.25]); agg = np.zeros((2, 4))
    off = np.array([0, 1, 2]); comp = np.array([0, 2], np.uint8)
    # predicted rates (0.9, 0.5, 0.4, 0.35) -> scores (2.8, 3.0, 3.4, 3.8): gamma 8 wins although
    # gamma 2 has the largest rate, which is what Eq. 1's multiplication by gamma must do
    out = oracle.select_gamma(_zero_mlp(5, [0.9, 0.5, 0.4, 0.35]), "pos0", H, c, agg, off, comp)
    np.testing.assert_allclose(out["scores"][0], [2.8, 3.0, 3.4, 3.8], rtol=1e-6)
    assert list(out["gamma_next"]) == [8, 8]
    np.testing.assert_allclose(out["gap"], 0.4, rtol=1e-5)
    # rates (0.5, 0.25, 1/6, 0.125) give equal scores of 2: lowest gamma wins the tie
    out = oracle.select_gamma(_zero_mlp(5, [0.5, 0.25, 0.0, 0.125]), "pos0", H, c, agg, off, comp)
    assert list(out["gamma_next"]) == [2, 2]
    out = oracle.select_gamma(_zero_mlp(5, [0.0, 0.3, 0.0, 0.0]), "pos0", H, c, agg, off, comp)
    assert list(out["gamma_next"]) == [4, 4]


@pytest.mark.parametrize("mode,n_in", [("pos0", 5), ("agg4", 7)])
def test_controller_against_numpy_one_liner(mode, n_in):
    rng = np.random.default_rng(81)
    B = 200
    gamma = rng.choice([2, 4, 6, 8], size=B)
    off = np.concatenate([[0], np.cumsum(gamma)])
    H = rng.uniform(0, 12, size=off[-1]); c = rng.uniform(0, 1, size=off[-1])
    agg = rng.uniform(0, 5, size=(B, 4)); comp = rng.integers(0, 3, size=B).astype(np.uint8)
    mlp = {"W1": _f32(0.5 * rng.standard_normal((16, n_in))), "b1": _f32(0.5 * rng.standard_normal(16)),
           "W2": _f32(0.5 * rng.standard_normal((4, 16))), "b2": _f32(0.5 * rng.standard_normal(4))}
    out = oracle.select_gamma(mlp, mode, H, c, agg, off, comp)
    onehot = np.eye(3)[comp]
    sig = np.stack([H[off[:-1]], c[off[:-1]]], axis=1) if mode == "pos0" else agg
    X = np.concatenate([sig, onehot], axis=1)
    hid = np.maximum(0.0, X @ mlp["W1"].astype(np.float64).T + mlp["b1"])
    sc = (hid @ mlp["W2"].astype(np.float64).T + mlp["b2"]) * np.array([2, 4, 6, 8]) + 1.0
    np.testing.assert_allclose(out["scores"], sc, rtol=1e-12, atol=1e-12)
    assert (out["gamma_next"] == np.array([2, 4, 6, 8])[sc.argmax(axis=1)]).all()
    assert set(np.unique(out["gamma_next"])) <= {2, 4, 6, 8}


def test_relu_is_applied():
    # hidden unit 0 gets pre-activation -1 (must be clipped to 0), unit 1 gets +1
    mlp = _zero_mlp(5, [0, 0, 0, 0], n_hidden=2)
    mlp["b1"][:] = [-1.0, 1.0]
    mlp["W2"][0] = [5.0, 0.25]
    out = oracle.select_gamma(mlp, "pos0", np.zeros(1), np.zeros(1), np.zeros((1, 4)),
                              np.array([0, 1]), np.zeros(1, np.uint8))
    np.testing.assert_allclose(out["scores"][0], [0.25 * 2 + 1, 1, 1, 1])


def _controller_inputs(rng, B):
    gamma = rng.choice([2, 4, 6, 8], size=B)
    off = np.concatenate([[0], np.cumsum(gamma)])
    H = rng.uniform(0, 12, size=off[-1]); c = rng.uniform(0, 1, size=off[-1])
    agg = rng.uniform(0, 5, size=(B, 4)); comp = rng.integers(0, 3, size=B).astype(np.uint8)
    return off, H, c, agg, comp


def _context(mode, off, H, c, agg, comp):
    sig = np.stack([H[off[:-1]], c[off[:-1]]], axis=1) if mode == "pos0" else agg
    return np.concatenate([sig, np.eye(3)[comp]], axis=1)


def test_scalar_predictor_closed_form_optimum():
    # Section 4.3 writes the predictor as f(x, gamma).  A linear f = a - b*gamma (no hidden layer,
    # only the gamma weight and the bias set) gives score(gamma) = (a - b*gamma)*gamma + 1, a parabola
    # with its maximum at a/(2b): the chosen candidate is the one nearest to it.
    off, H, c, agg, comp = _controller_inputs(np.random.default_rng(5), 3)
    for a, bb, want in ((0.9, 0.25, 2), (2.0, 0.25, 4), (3.1, 0.25, 6), (0.9, 0.05, 8), (0.5, -0.1, 8)):
        W2 = np.zeros((1, 6), np.float32); W2[0, 5] = -bb
        mlp = {"form": 1, "W1": None, "b1": None, "W2": W2, "b2": np.array([a], np.float32)}
        out = oracle.select_gamma(mlp, "pos0", H, c, agg, off, comp)
        assert list(out["gamma_next"]) == [want] * 3, (a, bb)
        g = np.array([2, 4, 6, 8.0])
        np.testing.assert_allclose(out["scores"][0], (np.float32(a) - np.float32(bb) * g) * g + 1, rtol=1e-12)


@pytest.mark.parametrize("mode,n_in", [("pos0", 5), ("agg4", 7)])
@pytest.mark.parametrize("n_hidden", [0, 16, 32])
def test_scalar_predictor_against_numpy(mode, n_in, n_hidden):
    # f([x, gamma]) evaluated once per candidate: Ridge (no hidden layer) and the MLP sizes of Table 3
    rng = np.random.default_rng(100 + n_hidden)
    off, H, c, agg, comp = _controller_inputs(rng, 150)
    X = _context(mode, off, H, c, agg, comp)
    W2 = _f32(0.5 * rng.standard_normal((1, n_hidden if n_hidden else n_in + 1)))
    b2 = _f32(0.5 * rng.standard_normal(1))
    W1 = _f32(0.5 * rng.standard_normal((n_hidden, n_in + 1))) if n_hidden else None
    b1 = _f32(0.5 * rng.standard_normal(n_hidden)) if n_hidden else None
    out = oracle.select_gamma({"form": 1, "W1": W1, "b1": b1, "W2": W2, "b2": b2}, mode, H, c, agg, off, comp)
    sc = np.zeros((150, 4))
    for j, g in enumerate((2, 4, 6, 8)):
        Xg = np.concatenate([X, np.full((150, 1), float(g))], axis=1)
        if n_hidden:
            f = np.maximum(0.0, Xg @ W1.astype(np.float64).T + b1) @ W2.astype(np.float64)[0] + b2[0]
        else:
            f = Xg @ W2.astype(np.float64)[0] + b2[0]
        sc[:, j] = f * g + 1.0
    np.testing.assert_allclose(out["scores"], sc, rtol=1e-12, atol=1e-12)
    assert (out["gamma_next"] == np.array([2, 4, 6, 8])[sc.argmax(axis=1)]).all()


def test_linear_four_output_predictor_against_numpy():
    rng = np.random.default_rng(77)
    off, H, c, agg, comp = _controller_inputs(rng, 100)
    X = _context("agg4", off, H, c, agg, comp)
    W2 = _f32(0.5 * rng.standard_normal((4, 7))); b2 = _f32(0.5 * rng.standard_normal(4))
    out = oracle.select_gamma({"form": 0, "W1": None, "b1": None, "W2": W2, "b2": b2}, "agg4", H, c, agg, off, comp)
    sc = (X @ W2.astype(np.float64).T + b2) * np.array([2, 4, 6, 8]) + 1.0
    np.testing.assert_allclose(out["scores"], sc, rtol=1e-12, atol=1e-12)


def test_scalar_form_equals_its_unrolled_four_output_network():
    # f([x, gamma_j]) for the four fixed candidates is a four-output network with four copies of
    # the hidden layer, the gamma column folded into each copy's bias: both forms must agree.
    rng = np.random.default_rng(31)
    off, H, c, agg, comp = _controller_inputs(rng, 120)
    nh = 8
    W1 = _f32(0.5 * rng.standard_normal((nh, 6))); b1 = _f32(0.5 * rng.standard_normal(nh))
    W2 = _f32(0.5 * rng.standard_normal((1, nh))); b2 = _f32(0.5 * rng.standard_normal(1))
    # keep the folded biases exactly representable: gamma weights and biases are multiples of 2^-8
    W1[:, 5] = np.round(W1[:, 5] * 256) / 256; b1 = _f32(np.round(b1 * 256) / 256)
    a = oracle.select_gamma({"form": 1, "W1": W1, "b1": b1, "W2": W2, "b2": b2}, "pos0", H, c, agg, off, comp)
    W1v = np.concatenate([W1[:, :5]] * 4); b1v = np.concatenate([b1 + W1[:, 5] * g for g in (2, 4, 6, 8)])
    W2v = np.zeros((4, 4 * nh), np.float32)
    for j in range(4):
        W2v[j, j * nh:(j + 1) * nh] = W2[0]
    b = oracle.select_gamma({"form": 0, "W1": _f32(W1v), "b1": _f32(b1v), "W2": W2v, "b2": np.repeat(b2, 4)},
                            "pos0", H, c, agg, off, comp)
    np.testing.assert_allclose(a["scores"], b["scores"], rtol=1e-12, atol=1e-12)
    assert (a["gamma_next"] == b["gamma_next"]).all()


def test_controller_rejects_mismatched_shapes():
    off, H, c, agg, comp = _controller_inputs(np.random.default_rng(1), 2)
    with pytest.raises(ValueError):
        oracle.select_gamma({"form": 1, "W1": None, "b1": None, "W2": np.zeros((1, 5), np.float32),
                             "b2": np.zeros(1, np.float32)}, "pos0", H, c, agg, off, comp)
    with pytest.raises(ValueError):
        oracle.select_gamma({"form": 0, "W1": np.zeros((4, 6), np.float32), "b1": np.zeros(4, np.float32),
                             "W2": np.zeros((4, 4), np.float32), "b2": np.zeros(4, np.float32)},
                            "pos0", H, c, agg, off, comp)


# --------------------------------------------------------------------------- draft-side proposal
def _sample_u(seed, seq, pos, step):
    w = oracle.philox4x32_10([seq, pos, step, 1], [seed & 0xffffffff, seed >> 32])
    return float(w[0]) * 2.0 ** -32


def test_draft_sampling_uniform_row_is_floor_of_u_times_v():
    # all logits equal, V a power of two: the CDF steps are exact, so the token is floor(u * V)
    V, B, g = 64, 40, 3
    d = np.zeros((B * g, V), np.float32)
    out = oracle.sample_draft(d, "f32", B, V, seed=(7 << 32) | 9, step=5, gamma_uniform=g, seq_base=100, pos0=2)
    for b in range(B):
        for i in range(g):
            u = _sample_u((7 << 32) | 9, 100 + b, 2 + i, 5)
            assert out["tokens"][b * g + i] == int(np.floor(u * V))
    np.testing.assert_allclose(out["prob"], 1.0 / V, rtol=1e-15)
    assert (out["flags"] == 0).all()


def test_draft_sampling_against_numpy_searchsorted():
    # the definition with library routines: cumulative sum and a right-sided search
    import scipy.special
    rng = np.random.default_rng(12)
    V, B, g = 257, 30, 4
    d = (2.0 * rng.standard_normal((B * g, V))).astype(np.float32)
    d[3, 10:200] = -np.inf                       # a masked block never comes out
    out = oracle.sample_draft(d, "f32", B, V, seed=99, step=1, gamma_uniform=g)
    q = scipy.special.softmax(d.astype(np.float64), axis=1)
    for r in range(B * g):
        b, i = divmod(r, g)
        u = _sample_u(99, b, i, 1)
        C = np.cumsum(q[r])
        want = int(np.searchsorted(C, u * C[-1], side="right"))
        if out["margin"][r] > 1e-12:             # away from a CDF edge the two summations agree
            assert out["tokens"][r] == want
        np.testing.assert_allclose(out["prob"][r], q[r, out["tokens"][r]], rtol=1e-12)
    assert not (10 <= out["tokens"][3] < 200)


def test_draft_sampling_follows_q_and_is_independent_of_verification_draws():
    # chi-square: the same row for many sequences; the tokens must be distributed as q
    import scipy.special
    import scipy.stats
    rng = np.random.default_rng(3)
    V, B = 6, 60000
    x = (1.2 * rng.standard_normal(V)).astype(np.float32)
    out = oracle.sample_draft(np.tile(x, (B, 1)), "f32", B, V, seed=2024, step=0, gamma_uniform=1)
    q = scipy.special.softmax(x.astype(np.float64))
    obs = np.bincount(out["tokens"], minlength=V).astype(float)
    assert scipy.stats.chisquare(obs, q * B).pvalue > 1e-3
    # the proposal uniform and the accept uniform of the same (sequence, position, step) are
    # different Philox blocks: over many sequences they are uncorrelated
    ua = np.array([float(oracle.philox4x32_10([b, 0, 0, 0], [2024, 0])[0] >> 8) * 2.0 ** -24 for b in range(4000)])
    us = np.array([_sample_u(2024, b, 0, 0) for b in range(4000)])
    assert abs(np.corrcoef(ua, us)[0, 1]) < 0.06


def test_draft_sampling_special_rows_and_sharding():
    V = 50
    d = np.full((4, V), -np.inf, np.float32)
    d[0, 17] = 3.0                               # one finite logit: always that token
    d[1, :] = 0.0; d[1, 5] = np.nan              # NaN: flagged
    d[2, :] = 1.0; d[2, 9] = np.inf              # +inf: flagged
    #  row 3: no finite logit: flagged
    out = oracle.sample_draft(d, "f32", 4, V, seed=1, gamma_uniform=1)
    assert out["tokens"][0] == 17 and out["prob"][0] == 1.0 and out["flags"][0] == 0
    assert (out["flags"][1:] & oracle.FLAG_NONFINITE).all()
    assert ((out["tokens"] >= 0) & (out["tokens"] < V)).all()
    # a sequence drawn alone with its global index gives the same token as inside the batch
    rng = np.random.default_rng(8)
    x = rng.standard_normal((12, V)).astype(np.float32)
    full = oracle.sample_draft(x, "f32", 6, V, seed=5, step=3, gamma_uniform=2)
    for b in range(6):
        one = oracle.sample_draft(x[2 * b:2 * b + 2], "f32", 1, V, seed=5, step=3, gamma_uniform=2, seq_base=b)
        assert (one["tokens"] == full["tokens"][2 * b:2 * b + 2]).all()
    # ragged batches address rows through the offsets; pos0 shifts the position word
    rag = oracle.sample_draft(x[:7], "f32", 3, V, seed=5, step=3, gamma=np.array([2, 4, 1], np.int32))
    assert (rag["tokens"][:2] == full["tokens"][:2]).all()
    shifted = oracle.sample_draft(x[1:2], "f32", 1, V, seed=5, step=3, gamma_uniform=1, pos0=1)
    assert shifted["tokens"][0] == full["tokens"][1]


# --------------------------------------------------------------------------- greedy verification
def test_greedy_hand_example_and_layout():
    # target top-1 per position: 3, 1, 4, 0 (bonus).  Drafted 3, 1, 2 -> two accepts, then the
    # target's own prediction 4 replaces the third draft.
    V = 5
    t = np.full((4, V), -1.0, dtype=np.float32)
    for i, a in enumerate([3, 1, 4, 0]):
        t[i, a] = 2.0
    out = oracle.verify_greedy(t, "f32", 1, V, np.array([3, 1, 2], dtype=np.int32), gamma_uniform=3, gamma_max=8)
    assert out["n_accepted"][0] == 2 and out["num_tokens"][0] == 3
    assert list(out["tokens"][0]) == [3, 1, 4, -1, -1, -1, -1, -1, -1]
    assert out["accept_rate"][0] == 2 / 3
    # every draft right: the extra token is the top prediction of the bonus row
    out = oracle.verify_greedy(t, "f32", 1, V, np.array([3, 1, 4], dtype=np.int32), gamma_uniform=3)
    assert out["n_accepted"][0] == 3 and list(out["tokens"][0]) == [3, 1, 4, 0]
    # first draft wrong
    out = oracle.verify_greedy(t, "f32", 1, V, np.array([0, 1, 4], dtype=np.int32), gamma_uniform=3)
    assert out["n_accepted"][0] == 0 and list(out["tokens"][0]) == [3, -1, -1, -1]


def test_greedy_against_numpy_argmax_with_ties_and_ragged_rows():
    rng = np.random.default_rng(91)
    V = 41
    gamma = np.array([2, 8, 1, 4, 6], dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(gamma)])
    B = len(gamma)
    t = np.round(2 * rng.standard_normal((off[-1] + B, V))).astype(np.float32)  # rounded: many ties
    top = t.argmax(axis=1)                                                       # numpy: first maximum
    tok = np.zeros(off[-1], dtype=np.int32)
    for b in range(B):
        for i in range(gamma[b]):
            right = rng.random() < 0.7
            tok[off[b] + i] = top[off[b] + b + i] if right else (top[off[b] + b + i] + 1) % V
    out = oracle.verify_greedy(t, "f32", B, V, tok, gamma=gamma, gamma_max=8)
    for b in range(B):
        n = 0
        while n < gamma[b] and tok[off[b] + n] == top[off[b] + b + n]:
            n += 1
        assert out["n_accepted"][b] == n
        assert out["tokens"][b, n] == top[off[b] + b + n]
        assert (out["tokens"][b, :n] == tok[off[b]:off[b] + n]).all() and (out["tokens"][b, n + 1:] == -1).all()


def test_greedy_equals_sampling_when_targets_are_one_hot():
    # With one-hot target rows the lossless sampling rule degenerates to the greedy rule: a draft is
    # accepted iff it is the target's only possible token, and the residual / bonus draw can only
    # return that token.  Two independent code paths of the oracle must agree.
    rng = np.random.default_rng(93)
    B, g, V = 300, 4, 12
    d = _f32(rng.standard_normal((B * g, V)))
    t = np.full((B * (g + 1), V), -np.inf, dtype=np.float32)
    hot = rng.integers(0, V, size=B * (g + 1))
    t[np.arange(B * (g + 1)), hot] = 0.0
    tok = np.zeros(B * g, dtype=np.int32)
    for b in range(B):
        for i in range(g):
            h = hot[b * (g + 1) + i]
            tok[b * g + i] = h if rng.random() < 0.75 else (h + 1) % V
    a = oracle.verify_greedy(t, "f32", B, V, tok, gamma_uniform=g)
    s = oracle.verify(d, t, "f32", B, V, tok, seed=17, gamma_uniform=g)
    assert (a["n_accepted"] == s["n_accepted"]).all()
    assert (a["tokens"] == s["tokens"]).all()
    assert a["n_accepted"].min() == 0 and a["n_accepted"].max() == g


def test_greedy_flags():
    V = 6
    t = np.zeros((4, V), dtype=np.float32)
    t[1, 2] = np.nan
    out = oracle.verify_greedy(t, "f32", 1, V, np.array([0, 9, 0], dtype=np.int32), gamma_uniform=3)
    assert out["row_flags"][0] == (oracle.FLAG_NONFINITE | oracle.FLAG_BAD_TOKEN)
