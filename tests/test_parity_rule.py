"""The rule of comparison (tests/parity.py) applied to planted differences, on the CPU: the "GPU"
side here is the oracle's own result with one thing changed, so each class of excuse, and each
class of failure, is seen to be counted as what it is."""
import copy

import numpy as np
import pytest

import workloads
from parity import MARGIN, REL_BAND, assert_parity, compare, oracle_step


@pytest.fixture(scope="module")
def case():
    cfg = workloads.config("C2", B=6, V=50)
    inp = workloads.make_step(cfg, device="cpu")
    ref = oracle_step(inp, 5, 0)
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    gpu = dict(H=f32(ref["sig"]["H"]), conf=f32(ref["sig"]["conf"]), agg=f32(ref["sig"]["agg"]),
               argmax=ref["sig"]["argmax"].copy(), row_flags=ref["ver"]["row_flags"].copy(),
               n_accepted=ref["ver"]["n_accepted"].copy(), num_tokens=ref["ver"]["num_tokens"].copy(),
               tokens=ref["ver"]["tokens"].copy(), accept_rate=f32(ref["ver"]["accept_rate"]),
               scores=f32(ref["sel"]["scores"]), gamma_next=ref["sel"]["gamma_next"].copy())
    return gpu, ref


def fresh(case):
    return copy.deepcopy(case[0]), copy.deepcopy(case[1])


def test_identical_results_pass_with_nothing_excused(case):
    gpu, ref = fresh(case)
    counts = assert_parity(gpu, ref)
    assert all(v == 0 for k, v in counts.items() if k != "rows")


def shorten(gpu, b):
    """The other side stopped one position earlier in sequence b."""
    n = int(gpu["n_accepted"][b]) - 1
    gpu["n_accepted"][b] = n
    gpu["num_tokens"][b] = n + 1
    gpu["tokens"][b, n + 1:] = -1
    gpu["accept_rate"][b] = n / 4.0


def test_accept_difference_is_excused_only_inside_the_margin(case):
    gpu, ref = fresh(case)
    b = int(np.argmax(ref["ver"]["n_accepted"] >= 2))
    shorten(gpu, b)
    problems, counts = compare(gpu, ref)       # the oracle's margin of this row is far above 1e-6
    assert counts["mismatch"] == 1 and counts["excused_accept"] == 0 and problems
    ref["ver"]["marg_acc"][b] = 0.5 * MARGIN   # a decision at rounding level: excused and counted
    u, q, p = ref["ver"]["dbg"][b, 1]
    ref["ver"]["dbg"][b, 1] = (u, q, u * q * (1 + 0.5 * REL_BAND))
    problems, counts = compare(gpu, ref)
    assert not problems and counts["excused_accept"] == 1 and counts["accept_outside_relative_band"] == 0
    assert_parity(gpu, ref)


def test_absolute_margin_on_a_tiny_probability_is_reported_by_the_relative_band(case):
    gpu, ref = fresh(case)
    b = int(np.argmax(ref["ver"]["n_accepted"] >= 2))
    shorten(gpu, b)
    ref["ver"]["marg_acc"][b] = 1e-9           # |u q - p| = 1e-9 < 1e-6, but p is twice u q
    for i in range(ref["ver"]["dbg"].shape[1]):
        if not np.isnan(ref["ver"]["dbg"][b, i, 0]):
            ref["ver"]["dbg"][b, i] = (0.5, 2e-9, 2e-9)
    problems, counts = compare(gpu, ref)
    assert not problems and counts["excused_accept"] == 1 and counts["accept_outside_relative_band"] == 1
    with pytest.raises(AssertionError):
        assert_parity(gpu, ref)


def test_emitted_token_difference_needs_a_cdf_margin(case):
    gpu, ref = fresh(case)
    b = 0
    n = int(gpu["n_accepted"][b])
    gpu["tokens"][b, n] = (gpu["tokens"][b, n] + 1) % 50
    problems, counts = compare(gpu, ref)
    assert counts["mismatch"] == 1 and problems
    ref["ver"]["marg_cdf"][b] = 0.5 * MARGIN
    problems, counts = compare(gpu, ref)
    assert not problems and counts["excused_cdf"] == 1


def test_float_outputs_and_flags_are_not_excusable(case):
    gpu, ref = fresh(case)
    gpu["H"][3] *= 1.001
    assert any(p.startswith("H:") for p in compare(gpu, ref)[0])
    gpu, ref = fresh(case)
    gpu["row_flags"][2] |= 2
    assert any("row_flags" in p for p in compare(gpu, ref)[0])
    gpu, ref = fresh(case)
    gpu["scores"][1, 2] += 1e-3
    assert any(p.startswith("scores") for p in compare(gpu, ref)[0])
    gpu, ref = fresh(case)
    gpu["argmax"][0] += 1
    assert "argmax differs" in compare(gpu, ref)[0]


def test_gamma_difference_needs_a_score_gap_at_rounding_level(case):
    gpu, ref = fresh(case)
    b = 4
    gpu["gamma_next"][b] = 2 if ref["sel"]["gamma_next"][b] != 2 else 4
    ref["sel"]["gap"][b] = 1.0                  # far above any score tolerance: a plain mismatch
    problems, counts = compare(gpu, ref)
    assert counts["mismatch"] == 1 and problems
    ref["sel"]["gap"][b] = 1e-9
    problems, counts = compare(gpu, ref)
    assert not problems and counts["excused_gamma"] == 1


def test_too_many_excused_rows_fail(case):
    gpu, ref = fresh(case)
    for b in (0, 1):
        n = int(gpu["n_accepted"][b])
        gpu["tokens"][b, n] = (gpu["tokens"][b, n] + 1) % 50
        ref["ver"]["marg_cdf"][b] = 0.5 * MARGIN
    problems, counts = compare(gpu, ref)
    assert not problems and counts["excused_cdf"] == 2
    with pytest.raises(AssertionError):
        assert_parity(gpu, ref)                # at most max(1, rows // 32) = 1 row may be excused
