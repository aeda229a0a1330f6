"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on identical bytes."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import config, make_step

from parity import assert_parity, compare, oracle_step

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def sk():
    import paper_2605_02888_amd as pkg
    h = pkg.SpecKV(device=0)
    yield h
    h.close()


def run_gpu(sk, inp, seed, step=0, mode="pos0", seq_base=0, one_call=False):
    from paper_2605_02888_amd.runner import StepRunner
    cfg = inp.cfg
    r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, mode=mode,
                   device=DEV, seq_base=seq_base)
    batch = r.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
    call = r.step_one_call if one_call else r.step
    call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, seed, step)
    return r.results(inp.draft.shape[0]), r


def check(sk, inp, seed, step=0, mode="pos0", max_excused=None):
    gpu, _ = run_gpu(sk, inp, seed, step, mode)
    ref = oracle_step(inp, seed, step, mode)
    counts = assert_parity(gpu, ref, what=inp.cfg.name)
    print(inp.cfg.name, counts, flush=True)
    if max_excused is not None:
        assert counts["excused_accept"] + counts["excused_cdf"] + counts["excused_gamma"] <= max_excused
    return gpu, ref, counts


SMALL = [
    ("C1", {}),
    ("C2", {}),
    ("C3", {"B": 8}),
    ("C5", {"B": 24}),
]


@pytest.mark.parametrize("name,over", SMALL, ids=[s[0] for s in SMALL])
def test_small_configs_match_oracle(sk, name, over):
    cfg = config(name, **over)
    print("case", name, over, flush=True)
    inp = make_step(cfg, device=DEV)
    check(sk, inp, seed=cfg.seed)


@pytest.mark.parametrize("mode", ["pos0", "agg4"])
def test_feature_modes(sk, mode):
    cfg = config("C2", B=32, V=4099)
    inp = make_step(cfg, device=DEV)
    inp.mlp = workloads.make_mlp(cfg.seed, n_in=5 if mode == "pos0" else 7)
    check(sk, inp, seed=11, mode=mode)


@pytest.mark.parametrize("one_call", [False, True], ids=["three-calls", "one-call"])
@pytest.mark.parametrize("form,n_hidden,mode", [(1, 16, "pos0"), (1, 32, "agg4"), (1, 0, "pos0"), (0, 0, "agg4"),
                                                (0, 32, "pos0"), (1, 64, "agg4"), (0, 1, "pos0")],
                         ids=["scalar-16", "scalar-32-agg4", "ridge", "linear-4out-agg4", "vector-32", "scalar-64-agg4",
                              "vector-1"])
def test_controller_shapes(sk, form, n_hidden, mode, one_call):
    # The predictor of Section 4.3 as one output of [x, gamma] evaluated per candidate, with the
    # hidden sizes of Table 3 and without a hidden layer (Ridge), beside the four-output form.
    cfg = config("C2", B=48, V=3001)
    inp = make_step(cfg, device=DEV)
    inp.mlp = workloads.make_mlp(cfg.seed + n_hidden, n_in=5 if mode == "pos0" else 7, n_hidden=n_hidden, form=form)
    gpu, _ = run_gpu(sk, inp, seed=19, mode=mode, one_call=one_call)
    ref = oracle_step(inp, 19, 0, mode)
    assert_parity(gpu, ref, caps=dict(excused_gamma=1))
    assert np.ptp(gpu["scores"], axis=0).min() > 0     # the scores really depend on the signals


def test_ragged_chained_steps_c4_shape(sk):
    # C4's shape at reduced B: fp16, V = 151936, per-row gamma in {2,4,6,8} chosen by the controller
    # from the previous step's signals; step 0 uses gamma = 4 everywhere.
    cfg = config("C4", B=12)
    gamma = torch.full((cfg.B,), 4, dtype=torch.int32)
    for step in range(3):
        print("C4 chained step", step, gamma.tolist(), flush=True)
        inp = make_step(cfg, device=DEV, step=step, gamma=gamma)
        gpu, ref, _ = check(sk, inp, seed=cfg.seed, step=step)
        assert set(np.unique(gpu["gamma_next"])) <= {2, 4, 6, 8}
        gamma = torch.as_tensor(ref["sel"]["gamma_next"], dtype=torch.int32)


def test_row_offsets_kernel(sk):
    for B in (1, 5, 1024, 5000):
        g = torch.randint(1, 9, (B,), dtype=torch.int32, device=DEV)
        off = torch.empty(B + 1, dtype=torch.int64, device=DEV)
        sk.row_offsets(g, B, off)
        torch.cuda.synchronize()
        want = np.concatenate([[0], np.cumsum(g.cpu().numpy().astype(np.int64))])
        assert (off.cpu().numpy() == want).all()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("V", [1, 2, 7, 100, 4099, 8192, 40001])
def test_odd_vocabulary_sizes_and_misaligned_rows(sk, dtype, V):
    cfg = config("C2", B=6, V=V, dtype=dtype, gamma=3)
    print("case", dtype, V, flush=True)
    inp = make_step(cfg, device=DEV)
    check(sk, inp, seed=5)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_vocabulary_beyond_64_chunks_of_4096(sk, dtype):
    # V > 262144: the resample pass works with 64 longer chunks, the pick walks runs that no longer
    # fit its registers, and the proposal kernel sweeps each chunk twice from memory.
    cfg = config("C2", B=3, V=300001, dtype=dtype, gamma=2)
    inp = make_step(cfg, device=DEV)
    for one_call in (False, True):
        gpu, _ = run_gpu(sk, inp, seed=23, one_call=one_call)
        assert_parity(gpu, oracle_step(inp, 23))
    smp = _run_sample(sk, inp, seed=23)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), dtype, cfg.B, cfg.V, 23, gamma_uniform=2)
    _compare_sample(smp, ref)


def test_ragged_extremes(sk):
    cfg = config("C2", B=5, V=3001, dtype="f16", gamma_max=16)
    gamma = torch.tensor([1, 16, 2, 9, 1], dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=gamma)
    check(sk, inp, seed=9)


def test_gamma_outside_its_range_is_clamped_and_flagged(sk):
    # gamma[b] is device data that the host cannot check.  A value outside [1, gamma_max] is clamped
    # on the device, so the accepted length stays inside the token row and every sequence gets its
    # descriptor; the sequence is flagged.  The rows are packed for the clamped lengths here, so every
    # access stays inside the buffers and the results equal those of the in-range batch.
    import dataclasses
    import paper_2605_02888_amd as pkg
    cfg = config("C2", B=5, V=3001, dtype="bf16", gamma_max=8)
    good = torch.tensor([8, 1, 4, 2, 8], dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=good)
    claimed = torch.tensor([12, 0, 4, 2, 1 << 20], dtype=torch.int32, device=DEV)
    ref = oracle_step(inp, 29, 1)
    for one_call in (False, True):
        gpu, _ = run_gpu(sk, dataclasses.replace(inp, gamma=claimed), seed=29, step=1, one_call=one_call)
        assert list(gpu["row_flags"] & pkg.FLAG_BAD_GAMMA) == [8, 8, 0, 0, 8]
        gpu["row_flags"] = gpu["row_flags"] & ~np.int32(pkg.FLAG_BAD_GAMMA)
        assert_parity(gpu, ref)
    tok = _greedy_inputs(inp, 0.8, seed=5)
    gpu = _run_greedy(sk, dataclasses.replace(inp, gamma=claimed), tok)
    want = oracle.verify_greedy(workloads.stored_bits(inp.target), cfg.dtype, cfg.B, cfg.V, tok.cpu().numpy(),
                                gamma=inp.gamma_host(), gamma_max=cfg.gamma_max)
    assert list(gpu["row_flags"] & pkg.FLAG_BAD_GAMMA) == [8, 8, 0, 0, 8]
    for k in ("n_accepted", "tokens", "num_tokens"):
        assert (gpu[k] == want[k]).all(), k


def _edit(inp, fn):
    """Apply fn(draft32, target32, tokens) on host copies and store back in the stored dtype."""
    d = inp.draft.float().cpu()
    t = inp.target.float().cpu()
    tok = inp.draft_tokens.cpu()
    fn(d, t, tok)
    inp.draft = d.to(inp.draft.dtype).to(DEV)
    inp.target = t.to(inp.target.dtype).to(DEV)
    inp.draft_tokens = tok.to(DEV)
    return inp


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_masked_spiked_and_constant_rows(sk, dtype):
    cfg = config("C2", B=8, V=20000, dtype=dtype, gamma=4)
    inp = make_step(cfg, device=DEV)
    G = cfg.gamma

    def fn(d, t, tok):
        d[0 * G + 1, 100:15000] = -float("inf")          # masked block, also the first tiles of many lanes
        t[0 * (G + 1) + 1, 100:15000] = -float("inf")
        d[1 * G + 0, :] = 0.0                               # constant row: H = log2 V, argmax = 0
        d[2 * G + 2, :] = 0.0
        d[2 * G + 2, 17000] = 200.0                         # late spike far above the lane references
        t[2 * (G + 1) + 2, 19999] = 150.0
        d[3 * G + 0, :] = -30000.0                          # very negative everywhere
        t[4 * (G + 1) + 0, :] = -float("inf")
        t[4 * (G + 1) + 0, 7] = 1.0                         # one-hot target
        d[5 * G + 3, 5] = d[5 * G + 3, 9000] = 50.0         # tie for the maximum: lowest index wins
        tok[1 * G + 0] = 123
    inp = _edit(inp, fn)
    check(sk, inp, seed=3)


def test_flags(sk):
    cfg = config("C2", B=6, V=5000, dtype="f32", gamma=3)
    inp = make_step(cfg, device=DEV)
    G = cfg.gamma

    def fn(d, t, tok):
        d[0 * G + 1, 77] = float("nan")
        t[1 * (G + 1) + 3, 4000] = float("inf")
        tok[2 * G + 1] = cfg.V
        tok[3 * G + 0] = -5
        t[4 * (G + 1):4 * (G + 1) + G] = d[4 * G:5 * G]   # p == q, then a bad token: residual mass 0
        tok[4 * G + 2] = cfg.V + 10
        d[5 * G + 2, :] = -float("inf")                     # a row with no finite logit
    inp = _edit(inp, fn)
    gpu, ref, _ = check(sk, inp, seed=21)
    f = gpu["row_flags"]
    assert f[0] & 1 and f[1] & 1 and f[5] & 1
    assert f[2] & 2 and f[3] & 2 and f[4] & 2 and f[4] & 4
    assert gpu["n_accepted"][3] == 0 and gpu["n_accepted"][4] == 2


def test_residual_mass_at_rounding_level(sk):
    # A rejection where p and q agree mathematically but not bit for bit (V = 1; rows that differ by
    # a constant shift): the oracle's residual mass is 0 or 1e-16, the GPU's is rounding noise of
    # 1e-7.  Both lie below the fall-back threshold of 1e-6, so both sides draw from p and set the
    # flag: nothing is excused.
    cfg = config("C2", B=6, V=1, dtype="f16", gamma=2)
    inp = make_step(cfg, device=DEV)

    def bad_token(d, t, tok):
        tok[2 * 2 + 0] = 5
        tok[5 * 2 + 1] = -1
    inp = _edit(inp, bad_token)
    for one_call in (False, True):
        gpu, _ = run_gpu(sk, inp, seed=3, one_call=one_call)
        assert_parity(gpu, oracle_step(inp, 3))
        assert (gpu["tokens"][np.arange(6), gpu["n_accepted"]] == 0).all()
    cfg = config("C2", B=4, V=3000, dtype="f32", gamma=3)
    inp = make_step(cfg, device=DEV)

    def shifted(d, t, tok):
        t[1 * 4:1 * 4 + 3] = d[1 * 3:2 * 3] + 1.5      # same distribution, other logits
        tok[1 * 3 + 1] = cfg.V                          # rejected there
    inp = _edit(inp, shifted)
    gpu, _ = run_gpu(sk, inp, seed=4)
    ref = oracle_step(inp, 4)
    assert ref["ver"]["resid_mass"][1] < 1e-6 and gpu["n_accepted"][1] == 1
    assert_parity(gpu, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_nan_inside_a_masked_region_is_still_flagged(sk, dtype):
    # A NaN surrounded by -inf: the waves (or chunks) that meet it see nothing finite, so their
    # reference stays at -inf; the NaN must survive the merge with the parts that did see data.
    cfg = config("C2", B=4, V=70001, dtype=dtype, gamma=2)
    inp = make_step(cfg, device=DEV)

    def fn(d, t, tok):
        d[0 * 2 + 1, 100:60000] = -float("inf"); d[0 * 2 + 1, 30001] = float("nan")
        t[1 * 3 + 0, 5000:69000] = -float("inf"); t[1 * 3 + 0, 47111] = float("nan")
        t[2 * 3 + 2, 64:] = -float("inf"); t[2 * 3 + 2, 70000] = float("nan")
        d[3 * 2 + 0, 100:60000] = -float("inf")            # masked only: not flagged
    inp = _edit(inp, fn)
    for one_call in (False, True):
        gpu, _ = run_gpu(sk, inp, seed=2, one_call=one_call)
        assert_parity(gpu, oracle_step(inp, 2))
        assert list(gpu["row_flags"] & 1) == [1, 1, 1, 0]
    smp = _run_sample(sk, inp, seed=2)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), dtype, cfg.B, cfg.V, 2, gamma_uniform=2)
    _compare_sample(smp, ref)
    assert smp["flags"][1] == 1 and smp["flags"][6] == 0 and not (100 <= smp["tokens"][6] < 60000)


OPTION_NAMES = ("stats_threads", "stats_unroll", "stats_target_wgs", "stats_max_split", "stats_pipeline",
                "stats_nontemporal", "step_tail", "stats_wgs_per_cu")


@pytest.mark.parametrize("opts", [
    (128, 2, 1, 1, 1, 1, 1, 4), (128, 4, 4096, 16, 0, 0, 0, 0), (256, 2, 65536, 64, 1, 1, 0, 2), (256, 4, 16384, 16, 1, 0, 1, 16),
    (256, 2, 1, 1, 0, 1, 1, 4), (512, 2, 2048, 3, 1, 1, 1, 3), (512, 4, 65536, 1024, 0, 1, 0, 0), (512, 4, 16384, 16, 1, 1, 1, 2),
    (128, 4, 300, 7, 1, 0, 1, 8), (256, 2, 16384, 16, 1, 1, 0, 0),
], ids=lambda o: "-".join(map(str, o)))
def test_launch_shapes_give_same_answers(sk, opts):
    cfg = config("C3", B=3, V=70001)
    inp = make_step(cfg, device=DEV)
    saved = {k: sk.get_option(k) for k in OPTION_NAMES}
    try:
        for k, v in zip(OPTION_NAMES, opts):
            sk.set_option(k, v)
        check(sk, inp, seed=77)
    finally:
        for k, v in saved.items():
            sk.set_option(k, v)


@pytest.mark.parametrize("step_tail", [0, 1])
def test_tail_kernel_and_separate_kernels_agree_bit_for_bit(sk, step_tail):
    # One workgroup per sequence for accept scan + resample must give exactly what the separate
    # accept / mass / pick kernels give, also on ragged batches, twice in a row.
    cfg = config("C4", B=40, V=9000)
    gamma = torch.tensor([2, 4, 6, 8, 1] * 8, dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=gamma)
    saved = sk.get_option("step_tail")
    try:
        sk.set_option("step_tail", step_tail)
        a, _ = run_gpu(sk, inp, seed=5)
        b, _ = run_gpu(sk, inp, seed=5)
        sk.set_option("step_tail", 1 - step_tail)
        c, _ = run_gpu(sk, inp, seed=5)
    finally:
        sk.set_option("step_tail", saved)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes() == c[k].tobytes(), k
    assert_parity(a, oracle_step(inp, 5))


def test_sharding_by_sequence_is_placement_invariant(sk):
    # Random numbers are keyed by the global sequence index: the second half of a batch run as its
    # own batch with seq_base set gives the same rows.
    cfg = config("C2", B=16, V=2000)
    inp = make_step(cfg, device=DEV)
    full, _ = run_gpu(sk, inp, seed=13, step=4)
    G = cfg.gamma
    half = workloads.StepInputs(cfg=config("C2", B=8, V=2000), gamma=None, row_off=None,
                                draft=inp.draft[8 * G:].contiguous(), target=inp.target[8 * (G + 1):].contiguous(),
                                draft_tokens=inp.draft_tokens[8 * G:].contiguous(), comp=inp.comp[8:].contiguous(),
                                mlp=inp.mlp)
    part, _ = run_gpu(sk, half, seed=13, step=4, seq_base=8)
    for k in ("n_accepted", "tokens", "num_tokens", "gamma_next"):
        assert (part[k] == full[k][8:]).all(), k


def test_gpu_emitted_tokens_follow_target_distribution(sk):
    # Losslessness on the GPU itself: with fixed rows, slot j of the emitted tokens, when present,
    # is distributed as p_j (chi-square over >= 1e6 sequences, tiny vocabulary).
    import scipy.special
    import scipy.stats
    rng = np.random.default_rng(2)
    B, g, V = 1_000_000, 3, 5
    xd = (1.5 * rng.standard_normal((g, V))).astype(np.float32)
    xt = np.concatenate([xd + 0.8 * rng.standard_normal((g, V)), rng.standard_normal((1, V))]).astype(np.float32)
    q = scipy.special.softmax(xd.astype(np.float64), axis=1)
    p = scipy.special.softmax(xt.astype(np.float64), axis=1)
    tok = np.stack([rng.choice(V, size=B, p=q[i]) for i in range(g)], axis=1).astype(np.int32)
    cfg = config("C1", B=B, V=V, gamma=g, gamma_max=g)
    inp = workloads.StepInputs(
        cfg=cfg, gamma=None, row_off=None,
        draft=torch.from_numpy(xd).to(DEV).repeat(B, 1), target=torch.from_numpy(xt).to(DEV).repeat(B, 1),
        draft_tokens=torch.from_numpy(tok.reshape(-1)).to(DEV), comp=torch.zeros(B, dtype=torch.uint8, device=DEV),
        mlp=workloads.make_mlp(1))
    gpu, _ = run_gpu(sk, inp, seed=31337)
    for j in range(g + 1):
        have = gpu["num_tokens"] > j
        obs = np.bincount(gpu["tokens"][have, j], minlength=V).astype(float)
        pval = scipy.stats.chisquare(obs, p[j] * have.sum()).pvalue
        assert pval > 1e-3, (j, pval)
    a = np.minimum(p[:g], q).sum(axis=1)
    for j in range(1, g + 1):
        want = np.prod(a[:j])
        assert abs((gpu["n_accepted"] >= j).mean() - want) < 4 * np.sqrt(want * (1 - want) / B)


def test_deterministic_rerun(sk):
    cfg = config("C3", B=4, V=50000)
    inp = make_step(cfg, device=DEV)
    a, _ = run_gpu(sk, inp, seed=1)
    b, _ = run_gpu(sk, inp, seed=1)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k


def test_full_size_headline_config_matches_oracle(sk):
    # B = 256, gamma = 8, V = 128256, bf16, Zipf-shaped: the benchmark's workload and launch
    # configuration, every sequence checked against the oracle.
    cfg = config("C3")
    inp = make_step(cfg, device=DEV)
    oracle.set_threads(16)
    gpu, ref, counts = check(sk, inp, seed=cfg.seed)
    rate = ref["ver"]["n_accepted"].mean() / cfg.gamma
    print("C3 mean acceptance rate", rate, counts, flush=True)
    assert counts["excused_accept"] + counts["excused_cdf"] <= 8


ONE_CALL_CASES = [
    ("C1", {}, None, "pos0", None),
    ("C2", {}, None, "agg4", None),
    ("C3", {"B": 8}, None, "pos0", None),
    ("C4", {"B": 40, "V": 9000}, [2, 4, 6, 8, 1] * 8, "pos0", None),
    ("C5", {"B": 24}, None, "pos0", None),
    # a launch shape the single-launch statistics kernel is not built for: one launch per side
    ("C3", {"B": 3, "V": 70001}, None, "pos0", {"stats_threads": 512, "stats_unroll": 4}),
    ("C2", {"B": 6, "V": 1, "gamma": 3}, None, "pos0", None),
    # signals + accept + controller in one launch, then the two resample launches
    ("C2", {}, None, "pos0", {"step_tail": 0}),
    ("C4", {"B": 40, "V": 9000}, [2, 4, 6, 8, 1] * 8, "agg4", {"step_tail": 0}),
    ("C5", {"B": 300, "V": 3001}, None, "pos0", None),   # more sequences than compute units
    ("C5", {"B": 600, "V": 3001}, None, "pos0", None),   # enough sequences for the 512-thread tail
    ("C3", {"B": 5, "V": 70001}, None, "pos0", {"stats_threads": 512}),   # single-launch statistics, 512 threads
]


@pytest.mark.parametrize("name,over,gamma,mode,opts", ONE_CALL_CASES,
                         ids=["C1", "C2-agg4", "C3", "C4-ragged", "C5-misaligned", "C3-other-shape", "V1", "C2-four-launches",
                              "C4-ragged-four-launches", "C5-many-sequences", "C5-512-thread-tail", "C3-512-thread-statistics"])
def test_one_call_step_equals_three_calls_bit_for_bit(sk, name, over, gamma, mode, opts):
    # speckv_step (row statistics of both sides in one launch, then one workgroup per sequence for
    # everything else) must return exactly what speckv_signals + speckv_verify + speckv_select_gamma return.
    cfg = config(name, **over)
    g = None if gamma is None else torch.tensor(gamma, dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=g)
    if mode == "agg4":
        inp.mlp = workloads.make_mlp(cfg.seed, n_in=7)
    saved = {k: sk.get_option(k) for k in (opts or {})}
    try:
        for k, v in (opts or {}).items():
            sk.set_option(k, v)
        a, _ = run_gpu(sk, inp, seed=17, step=2, mode=mode, one_call=True)
        b, _ = run_gpu(sk, inp, seed=17, step=2, mode=mode, one_call=False)
    finally:
        for k, v in saved.items():
            sk.set_option(k, v)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k
    assert_parity(a, oracle_step(inp, 17, 2, mode))


@pytest.mark.parametrize("name,over,gamma", [("C2", {"B": 24}, None), ("C3", {"B": 6}, None),
                                             ("C4", {"B": 10, "V": 30011}, [2, 8, 4, 6, 1, 8, 3, 5, 7, 2]),
                                             ("C5", {"B": 12}, None), ("C1", {"V": 9}, None)],
                         ids=["C2", "C3", "C4-ragged", "C5-misaligned", "V9"])
def test_one_call_step_without_the_argmax_output(sk, name, over, gamma):
    # A caller who does not ask for the argmax of the draft rows gets the variant of the statistics
    # launch that carries no position in its hot loop: every other output must be bit-equal to what
    # the call with the argmax returns, and match the oracle.
    from paper_2605_02888_amd.runner import StepRunner
    cfg = config(name, **over)
    g = None if gamma is None else torch.tensor(gamma, dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=g)
    a, _ = run_gpu(sk, inp, seed=23, step=1, one_call=True)
    r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, device=DEV,
                   with_argmax=False)
    batch = r.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
    r.argmax.fill_(-7)
    r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, 23, 1)
    b = r.results(inp.draft.shape[0])
    assert (b["argmax"] == -7).all()   # not requested: not written
    for k in a:
        if k != "argmax":
            assert a[k].tobytes() == b[k].tobytes(), k
    assert_parity(b, oracle_step(inp, 23, 1), check_argmax=False)


def test_one_call_step_flags_and_masked_rows(sk):
    cfg = config("C2", B=6, V=5000, dtype="f32", gamma=3)
    inp = make_step(cfg, device=DEV)
    G = cfg.gamma

    def fn(d, t, tok):
        d[0 * G + 1, 77] = float("nan")
        t[1 * (G + 1) + 3, 4000] = float("inf")
        tok[2 * G + 1] = cfg.V
        t[4 * (G + 1):4 * (G + 1) + G] = d[4 * G:5 * G]
        tok[4 * G + 2] = cfg.V + 10
        d[5 * G + 2, :] = -float("inf")
        d[3 * G + 1, 100:4000] = -float("inf")
    inp = _edit(inp, fn)
    a, _ = run_gpu(sk, inp, seed=21, one_call=True)
    b, _ = run_gpu(sk, inp, seed=21, one_call=False)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k
    assert_parity(a, oracle_step(inp, 21))


def test_one_call_step_full_size_headline_config(sk):
    # the benchmark's default path: B = 256, gamma = 8, V = 128256, bf16 through speckv_step
    cfg = config("C3")
    inp = make_step(cfg, device=DEV)
    oracle.set_threads(16)
    a, _ = run_gpu(sk, inp, seed=cfg.seed, one_call=True)
    b, _ = run_gpu(sk, inp, seed=cfg.seed, one_call=False)
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k
    counts = assert_parity(a, oracle_step(inp, cfg.seed))
    print("C3 one call", counts, flush=True)
    assert counts["excused_accept"] + counts["excused_cdf"] <= 8


def _oracle_in_chunks(inp, seed, step, mode="pos0", chunk=128):
    """The oracle on every sequence of a large batch, a slice of sequences at a time (bounds the host
    copies of the logits); each slice runs with its first global index as seq_base, so its random
    numbers are those of the full batch.  Returns what oracle_step returns, concatenated."""
    cfg = inp.cfg
    g = inp.gamma_host()
    off = np.concatenate([[0], np.cumsum(g)]).astype(np.int64)
    parts = []
    for b0 in range(0, cfg.B, chunk):
        b1 = min(cfg.B, b0 + chunk)
        sub = workloads.StepInputs(
            cfg=config(cfg.name, B=b1 - b0, V=cfg.V, dtype=cfg.dtype, gamma=cfg.gamma, gamma_max=cfg.gamma_max),
            gamma=torch.as_tensor(g[b0:b1], dtype=torch.int32), row_off=None,
            draft=inp.draft[off[b0]:off[b1]], target=inp.target[off[b0] + b0:off[b1] + b1],
            draft_tokens=inp.draft_tokens[off[b0]:off[b1]], comp=inp.comp[b0:b1], mlp=inp.mlp)
        parts.append(oracle_step(sub, seed, step, mode, seq_base=b0))
    cat = lambda grp, k: np.concatenate([p[grp][k] for p in parts])
    sig = {k: cat("sig", k) for k in ("H", "conf", "argmax", "agg", "gamma")}
    sig["row_off"] = off
    ver = {k: cat("ver", k) for k in ("n_accepted", "tokens", "num_tokens", "accept_rate", "row_flags", "marg_acc",
                                      "marg_cdf", "resid_mass", "dbg")}
    sel = {k: cat("sel", k) for k in ("gamma_next", "scores", "gap")}
    return dict(sig=sig, ver=ver, sel=sel, V=cfg.V, mlp=inp.mlp, mode=mode)


def test_full_size_c5_every_sequence_against_oracle(sk):
    # B = 4096, gamma = 8, V = 50257, fp32 (14 GB of logits, rows misaligned to 16 bytes, peaked rows
    # with entropies down to 1e-4 bits), in the launch configuration bench.py times: every sequence
    # is recomputed by the oracle.
    cfg = config("C5")
    inp = make_step(cfg, device=DEV)
    gpu, _ = run_gpu(sk, inp, seed=cfg.seed, one_call=True)
    oracle.set_threads(16)
    ref = _oracle_in_chunks(inp, cfg.seed, 0, chunk=256)
    counts = assert_parity(gpu, ref, what="C5")
    print("C5 all sequences", counts, "mean acceptance rate", gpu["n_accepted"].mean() / 8, flush=True)
    assert (gpu["row_flags"] == 0).all()


def test_full_size_c4_three_chained_steps_on_the_device(sk):
    # B = 1024, V = 151936, fp16, ragged gamma: step 0 runs at gamma = 4 for every sequence (the
    # paper's Fixed-4 default, Section 4.4); steps 1 and 2 run at the gamma the controller chose in
    # the step before (Section 4.3).  The chain stays on the device: the gamma_next tensor a step
    # wrote is the next step's gamma, and speckv_row_offsets turns it into the packing.  The harness
    # only draws and packs the logits (for which it takes the oracle's gamma_next, required below
    # to equal the device's).  Every step, every sequence is compared with the oracle.
    from paper_2605_02888_amd.runner import StepRunner
    cfg = config("C4")
    B = cfg.B
    oracle.set_threads(16)
    r = StepRunner(sk, B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], workloads.make_mlp(cfg.seed),
                   device=DEV)
    gamma_dev = torch.full((B,), 4, dtype=torch.int32, device=DEV)
    row_off = torch.empty(B + 1, dtype=torch.int64, device=DEV)
    gamma_host = torch.full((B,), 4, dtype=torch.int32)
    for step in range(3):
        print("C4 full size, chained step", step, "gamma histogram", np.bincount(gamma_host.numpy(), minlength=9)[[2, 4, 6, 8]],
              flush=True)
        inp = make_step(cfg, device=DEV, step=step, gamma=gamma_host)
        sk.row_offsets(gamma_dev, B, row_off)
        batch = r.batch(gamma=gamma_dev, row_off=row_off)
        r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, cfg.seed, step)
        gpu = r.results(inp.draft.shape[0])
        assert (row_off.cpu().numpy() == inp.row_off.cpu().numpy()).all()
        ref = _oracle_in_chunks(inp, cfg.seed, step, chunk=128)
        counts = assert_parity(gpu, ref, caps=dict(excused_gamma=0), what=f"C4 step {step}")
        print("C4 step", step, counts, flush=True)
        assert (gpu["gamma_next"] == ref["sel"]["gamma_next"]).all()
        # the device's own decision feeds the next step
        gamma_dev = r.gamma_next.clone()
        gamma_host = torch.as_tensor(ref["sel"]["gamma_next"], dtype=torch.int32)
        del inp


def test_full_size_c4_mixed_lengths_every_sequence_against_oracle(sk):
    # The seeded controller of this configuration settles on one length for every sequence, so the
    # chain above packs equal lengths through the ragged interface.  Here: the same shape with
    # lengths drawn from {2, 4, 6, 8} per sequence (packed rows, device row offsets), one step,
    # every sequence against the oracle.
    cfg = config("C4")
    gamma = torch.as_tensor(np.random.default_rng(4).choice([2, 4, 6, 8], size=cfg.B), dtype=torch.int32)
    inp = make_step(cfg, device=DEV, step=1, gamma=gamma)
    gpu, _ = run_gpu(sk, inp, seed=cfg.seed, step=1, one_call=True)
    oracle.set_threads(16)
    counts = assert_parity(gpu, _oracle_in_chunks(inp, cfg.seed, 1, chunk=128), what="C4 mixed")
    print("C4 mixed lengths", counts, flush=True)
    assert (gpu["row_flags"] == 0).all()


def _greedy_inputs(inp, match_prob, seed):
    """Drafted tokens that equal the target's top prediction with probability match_prob (test-side
    input preparation with torch.argmax; everything else comes from the workload generator)."""
    g = inp.gamma_host()
    off = np.concatenate([[0], np.cumsum(g)])
    t_rows = np.concatenate([np.arange(off[b] + b, off[b] + b + g[b]) for b in range(len(g))])
    top = torch.argmax(inp.target[torch.as_tensor(t_rows, device=inp.target.device)].float(), dim=1).to(torch.int32)
    rng = torch.Generator(device="cpu").manual_seed(seed)
    keep = (torch.rand(top.shape[0], generator=rng) < match_prob).to(top.device)
    other = torch.randint(0, inp.cfg.V, top.shape, generator=rng, dtype=torch.int32).to(top.device)
    return torch.where(keep, top, other).contiguous()


def _run_greedy(sk, inp, tok):
    import paper_2605_02888_amd as pkg
    cfg = inp.cfg
    B, W = cfg.B, cfg.gamma_max + 1
    ws = torch.empty(pkg.workspace_bytes(B, cfg.gamma_max), dtype=torch.uint8, device=DEV)
    out = dict(n_accepted=torch.zeros(B, dtype=torch.int32, device=DEV), tokens=torch.zeros(B, W, dtype=torch.int32, device=DEV),
               num_tokens=torch.zeros(B, dtype=torch.int32, device=DEV), accept_rate=torch.zeros(B, dtype=torch.float32, device=DEV),
               row_flags=torch.zeros(B, dtype=torch.int32, device=DEV))
    batch = pkg.Batch(B=B, V=cfg.V, gamma_max=cfg.gamma_max, gamma_uniform=cfg.gamma if inp.gamma is None else 0,
                      gamma=inp.gamma, row_off=inp.row_off)
    sk.verify_greedy(batch, inp.target, pkg.binding.TORCH_TO_DTYPE[inp.target.dtype], tok, ws, out["n_accepted"],
                     out["tokens"], out["num_tokens"], out["accept_rate"], out["row_flags"])
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


@pytest.mark.parametrize("name,over,ragged", [("C1", {}, False), ("C2", {}, False), ("C3", {"B": 16}, False),
                                               ("C4", {"B": 24}, True), ("C5", {"B": 40}, False)],
                         ids=["C1", "C2", "C3", "C4-ragged", "C5"])
def test_greedy_verification_matches_oracle_exactly(sk, name, over, ragged):
    # The paper's own accept rule (target top-1 must equal the drafted token): integer work only,
    # so every output must be identical to the oracle's.
    cfg = config(name, **over)
    gamma = torch.as_tensor(np.random.default_rng(8).choice([1, 2, 4, 6, 8], size=cfg.B), dtype=torch.int32) if ragged else None
    inp = make_step(cfg, device=DEV, gamma=gamma)
    tok = _greedy_inputs(inp, 0.8, seed=5)
    gpu = _run_greedy(sk, inp, tok)
    ref = oracle.verify_greedy(workloads.stored_bits(inp.target), cfg.dtype, cfg.B, cfg.V, tok.cpu().numpy(),
                               gamma=inp.gamma_host(), gamma_max=cfg.gamma_max)
    for k in ("n_accepted", "tokens", "num_tokens"):
        assert (gpu[k] == ref[k]).all(), k
    assert (gpu["row_flags"].astype(np.uint32) == ref["row_flags"]).all()
    np.testing.assert_allclose(gpu["accept_rate"], ref["accept_rate"], rtol=1e-6)
    if cfg.B >= 8:
        assert ref["n_accepted"].max() > 0   # the test really exercises accepted prefixes


@pytest.mark.parametrize("name,over,ragged,mode", [("C2", {}, False, "pos0"), ("C3", {"B": 16}, False, "agg4"),
                                                    ("C4", {"B": 24}, True, "pos0"), ("C5", {"B": 40}, False, "pos0"),
                                                    ("C3", {"B": 5, "V": 70001}, False, "pos0")],
                         ids=["C2", "C3-agg4", "C4-ragged", "C5", "C3-odd-V"])
def test_greedy_step_in_one_call_equals_the_three_calls(sk, name, over, ragged, mode):
    # speckv_step with greedy = 1: signals + top-1 match + controller in two launches, against
    # speckv_signals + speckv_verify_greedy + speckv_select_gamma (bit for bit) and the oracle.
    from paper_2605_02888_amd.runner import StepRunner
    cfg = config(name, **over)
    gamma = torch.as_tensor(np.random.default_rng(8).choice([1, 2, 4, 6, 8], size=cfg.B), dtype=torch.int32) if ragged else None
    inp = make_step(cfg, device=DEV, gamma=gamma)
    if mode == "agg4":
        inp.mlp = workloads.make_mlp(cfg.seed, n_in=7)
    inp.draft_tokens = _greedy_inputs(inp, 0.8, seed=5)
    outs = []
    for one_call in (True, False):
        r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, mode=mode, device=DEV)
        for t in (r.tokens, r.n_accepted, r.num_tokens, r.row_flags, r.gamma_next):
            t.fill_(-9)
        batch = r.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
        if one_call:
            r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, 0, 0, greedy=True)
        else:
            r.step_greedy(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp)
        outs.append(r.results(inp.draft.shape[0]))
    a, b = outs
    for k in a:
        assert a[k].tobytes() == b[k].tobytes(), k
    ref = oracle.verify_greedy(workloads.stored_bits(inp.target), cfg.dtype, cfg.B, cfg.V, inp.draft_tokens.cpu().numpy(),
                               gamma=inp.gamma_host(), gamma_max=cfg.gamma_max)
    for k in ("n_accepted", "tokens", "num_tokens"):
        assert (a[k] == ref[k]).all(), k
    assert (a["row_flags"].astype(np.uint32) == ref["row_flags"]).all()
    sig = oracle.signals(workloads.stored_bits(inp.draft), cfg.dtype, cfg.B, cfg.V, gamma=inp.gamma_host())
    sel = oracle.select_gamma(inp.mlp, mode, sig["H"], sig["conf"], sig["agg"], sig["row_off"], inp.comp.cpu().numpy())
    np.testing.assert_allclose(a["H"], sig["H"], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(a["conf"], sig["conf"], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(a["agg"], sig["agg"], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(a["scores"], sel["scores"], rtol=1e-4, atol=1e-5)
    far = sel["gap"] > 2e-5 * np.maximum(1.0, np.abs(sel["scores"]).max(axis=1))
    assert (a["gamma_next"][far] == sel["gamma_next"][far]).all()
    if cfg.B >= 8:
        assert ref["n_accepted"].max() > 0


def test_greedy_ties_and_flags(sk):
    cfg = config("C2", B=4, V=3000, dtype="bf16", gamma=3)
    inp = make_step(cfg, device=DEV)
    G = cfg.gamma

    def fn(d, t, tok):
        t[0 * (G + 1) + 0, :] = 1.0                       # all equal: top prediction is index 0
        t[0 * (G + 1) + 1, 100] = t[0 * (G + 1) + 1, 2000] = 99.0   # tie: lowest index wins
        t[1 * (G + 1) + 2, 5] = float("nan")
        tok[0 * G + 0] = 0
        tok[0 * G + 1] = 100
        tok[2 * G + 0] = cfg.V + 3
    inp = _edit(inp, fn)
    gpu = _run_greedy(sk, inp, inp.draft_tokens)
    ref = oracle.verify_greedy(workloads.stored_bits(inp.target), cfg.dtype, cfg.B, cfg.V, inp.draft_tokens.cpu().numpy(),
                               gamma_uniform=G, gamma_max=cfg.gamma_max)
    assert gpu["n_accepted"][0] >= 2 and gpu["row_flags"][1] & 1 and gpu["row_flags"][2] & 2
    ok = (ref["row_flags"] & 1) == 0
    for k in ("n_accepted", "tokens", "num_tokens"):
        assert (gpu[k][ok] == ref[k][ok]).all(), k
    assert (gpu["row_flags"].astype(np.uint32) == ref["row_flags"]).all()


# --------------------------------------------------------------------------- draft-side proposal
def _run_sample(sk, inp, seed, step=0, pos0=0, seq_base=0):
    import paper_2605_02888_amd as pkg
    cfg = inp.cfg
    rows = inp.draft.shape[0]
    out = dict(tokens=torch.full((rows,), -7, dtype=torch.int32, device=DEV),
               prob=torch.zeros(rows, dtype=torch.float32, device=DEV),
               flags=torch.full((rows,), 99, dtype=torch.int32, device=DEV))
    batch = pkg.Batch(B=cfg.B, V=cfg.V, gamma_max=cfg.gamma_max, gamma_uniform=cfg.gamma if inp.gamma is None else 0,
                      gamma=inp.gamma, row_off=inp.row_off, seq_base=seq_base)
    sk.sample_draft(batch, inp.draft, pkg.binding.TORCH_TO_DTYPE[inp.draft.dtype], seed, step, pos0, out["tokens"],
                    out["prob"], out["flags"])
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def _compare_sample(gpu, ref):
    """Tokens equal except where the oracle's CDF margin is below 1e-6; probabilities to 1e-4."""
    clean = (ref["flags"] & oracle.FLAG_NONFINITE) == 0
    assert (gpu["flags"].astype(np.uint32) == ref["flags"]).all()
    diff = (gpu["tokens"] != ref["tokens"]) & clean
    excused = diff & (ref["margin"] < 1e-6)
    assert not (diff & ~excused).any(), np.flatnonzero(diff & ~excused)[:10]
    same = clean & ~diff
    np.testing.assert_allclose(gpu["prob"][same], ref["prob"][same], rtol=1e-4, atol=1e-9)
    return int(excused.sum())


@pytest.mark.parametrize("name,over,ragged", [("C1", {}, False), ("C2", {}, False), ("C3", {"B": 8}, False),
                                               ("C4", {"B": 24}, True), ("C5", {"B": 24}, False)],
                         ids=["C1", "C2", "C3", "C4-ragged", "C5-misaligned"])
def test_draft_sampling_matches_oracle(sk, name, over, ragged):
    cfg = config(name, **over)
    gamma = torch.as_tensor(np.random.default_rng(8).choice([1, 2, 4, 6, 8], size=cfg.B), dtype=torch.int32) if ragged else None
    inp = make_step(cfg, device=DEV, gamma=gamma)
    gpu = _run_sample(sk, inp, seed=cfg.seed, step=3, pos0=1, seq_base=1000)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), cfg.dtype, cfg.B, cfg.V, cfg.seed, step=3,
                              gamma=inp.gamma_host(), seq_base=1000, pos0=1)
    excused = _compare_sample(gpu, ref)
    print(name, "rows", len(ref["tokens"]), "excused", excused, flush=True)
    assert excused <= 1


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("V", [1, 2, 7, 100, 4099, 8192, 40001])
def test_draft_sampling_odd_vocabularies(sk, dtype, V):
    cfg = config("C2", B=6, V=V, dtype=dtype, gamma=3)
    inp = make_step(cfg, device=DEV)
    gpu = _run_sample(sk, inp, seed=5)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), dtype, cfg.B, V, 5, gamma_uniform=3)
    _compare_sample(gpu, ref)


def test_draft_sampling_masked_spiked_and_flagged_rows(sk):
    cfg = config("C2", B=8, V=20000, dtype="f32", gamma=1)
    inp = make_step(cfg, device=DEV)

    def fn(d, t, tok):
        d[0, 100:15000] = -float("inf")
        d[1, :] = 0.0
        d[2, :] = 0.0; d[2, 17000] = 200.0        # one chunk far above the others
        d[3, :] = -30000.0
        d[4, :] = -float("inf"); d[4, 7] = 1.0    # a single finite logit
        d[5, 77] = float("nan")
        d[6, 4000] = float("inf")
        d[7, :] = -float("inf")
    inp = _edit(inp, fn)
    gpu = _run_sample(sk, inp, seed=3)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), "f32", 8, cfg.V, 3, gamma_uniform=1)
    _compare_sample(gpu, ref)
    assert gpu["tokens"][2] == 17000 and gpu["tokens"][4] == 7
    assert not (100 <= gpu["tokens"][0] < 15000)
    assert (gpu["flags"][5:] == 1).all() and (gpu["flags"][:5] == 0).all()
    assert ((gpu["tokens"] >= 0) & (gpu["tokens"] < cfg.V)).all()


def test_draft_sampling_follows_q_on_the_gpu(sk):
    # chi-square over 400k rows that all hold the same logits, tiny vocabulary
    import scipy.special
    import scipy.stats
    rng = np.random.default_rng(4)
    B, V = 400_000, 7
    x = (1.3 * rng.standard_normal(V)).astype(np.float32)
    cfg = config("C1", B=B, V=V, gamma=1, gamma_max=1)
    inp = workloads.StepInputs(cfg=cfg, gamma=None, row_off=None, draft=torch.from_numpy(x).to(DEV).repeat(B, 1),
                               target=None, draft_tokens=None, comp=None, mlp=None)
    gpu = _run_sample(sk, inp, seed=77)
    q = scipy.special.softmax(x.astype(np.float64))
    obs = np.bincount(gpu["tokens"], minlength=V).astype(float)
    assert scipy.stats.chisquare(obs, q * B).pvalue > 1e-3
    np.testing.assert_allclose(gpu["prob"], q[gpu["tokens"]], rtol=1e-5)


def test_sampled_tokens_feed_the_step(sk):
    # propose on the device, then verify the proposal: the whole chain stays on the GPU and the
    # verified step still matches the oracle run on the same proposed tokens
    cfg = config("C2", B=32)
    inp = make_step(cfg, device=DEV)
    gpu_s = _run_sample(sk, inp, seed=cfg.seed, step=0)
    inp.draft_tokens = torch.from_numpy(gpu_s["tokens"]).to(DEV)
    check(sk, inp, seed=cfg.seed)


def test_draft_sampling_full_size_headline_rows(sk):
    # all 2048 draft rows of the benchmark workload (V = 128256, bf16)
    cfg = config("C3")
    inp = make_step(cfg, device=DEV)
    gpu = _run_sample(sk, inp, seed=cfg.seed)
    oracle.set_threads(16)
    ref = oracle.sample_draft(workloads.stored_bits(inp.draft), cfg.dtype, cfg.B, cfg.V, cfg.seed, gamma_uniform=cfg.gamma)
    excused = _compare_sample(gpu, ref)
    print("C3 sampling excused", excused, flush=True)
    assert excused <= 4


def test_step_can_be_captured_in_a_hip_graph_and_replayed(sk):
    # speckv_step only launches kernels on the caller's stream (no allocation, no host
    # synchronisation, no memset), so a caller may capture it once and replay it: every replay must
    # return what the eager call returns on the data then in the buffers.
    from paper_2605_02888_amd.runner import StepRunner
    cfg = config("C2", B=16, V=5000)
    inp = make_step(cfg, device=DEV)
    r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, device=DEV)
    batch = r.batch(gamma_uniform=cfg.gamma)
    args = (batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, 41, 6)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r.step_one_call(*args)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r.step_one_call(*args)
    outputs = ("H", "conf", "argmax", "agg", "n_accepted", "tokens", "num_tokens", "accept_rate", "row_flags",
               "gamma_next", "scores")
    for rep in range(3):
        other = make_step(cfg, device=DEV, step=rep + 1)      # new contents, same buffers
        inp.draft.copy_(other.draft); inp.target.copy_(other.target)
        inp.draft_tokens.copy_(other.draft_tokens)
        r.step_one_call(*args)
        eager = r.results(inp.draft.shape[0])
        for k in outputs:
            getattr(r, k).fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        replayed = r.results(inp.draft.shape[0])
        for k in eager:
            assert eager[k].tobytes() == replayed[k].tobytes(), (rep, k)
    assert_parity(replayed, oracle_step(inp, 41, 6))


# --------------------------------------------------------------------------- stray writes
_GUARD = 64  # elements of margin on each side of every output


def _guarded(t, fill):
    """A tensor of t's shape and dtype inside a larger buffer whose margins hold `fill`."""
    big = torch.full((t.numel() + 2 * _GUARD,), fill, dtype=t.dtype, device=t.device)
    return big, big[_GUARD:_GUARD + t.numel()].view(t.shape)


def _add_canaries(r):
    """Move every output tensor and the workspace of a StepRunner into guarded buffers; returns a
    function that checks, on the host after a call, that no margin was written."""
    bigs = {}
    for k, fill in (("H", -7.5), ("conf", -7.5), ("argmax", -77), ("agg", -7.5), ("n_accepted", -77), ("tokens", -77),
                    ("num_tokens", -77), ("accept_rate", -7.5), ("row_flags", -77), ("gamma_next", -77), ("scores", -7.5),
                    ("ws", 0xA5)):
        bigs[k], view = _guarded(getattr(r, k), fill)
        setattr(r, k, view)

    def check(what):
        torch.cuda.synchronize()
        for k, big in bigs.items():
            n = big.numel() - 2 * _GUARD
            lo, hi = big[:_GUARD].cpu(), big[_GUARD + n:].cpu()
            assert (lo == lo[0]).all() and (hi == lo[0]).all(), (what, k, "a margin was overwritten")
    return check


@pytest.mark.parametrize("name,over,gamma", [
    ("C4", {"B": 37, "V": 9001}, [2, 4, 6, 8, 1] * 7 + [8, 3]),          # ragged, packed rows
    ("C5", {"B": 24}, None),                                              # rows misaligned to 16 bytes
    ("C2", {"B": 6, "V": 1, "gamma": 3}, None),                           # one-token vocabulary
    ("C2", {"B": 5, "V": 3001, "dtype": "f16", "gamma_max": 16}, [1, 16, 2, 9, 16]),   # longest speculation
    ("C3", {"B": 3, "V": 70001}, None),                                   # ragged tail of the last chunk
], ids=["ragged", "misaligned", "V1", "gamma16", "odd-V"])
def test_no_write_lands_outside_the_outputs_or_the_workspace(sk, name, over, gamma):
    # Every output and the workspace sit between sentinel-filled margins; the margins are read back on
    # the host after each way of issuing a step and after the proposal kernel.
    from paper_2605_02888_amd.runner import StepRunner
    import paper_2605_02888_amd as pkg
    cfg = config(name, **over)
    g = None if gamma is None else torch.tensor(gamma, dtype=torch.int32)
    inp = make_step(cfg, device=DEV, gamma=g)
    ref = oracle_step(inp, 31, 2)
    r = StepRunner(sk, cfg.B, cfg.V, cfg.gamma_max, workloads.TORCH_DTYPES[cfg.dtype], inp.mlp, device=DEV)
    check = _add_canaries(r)
    batch = r.batch(gamma_uniform=cfg.gamma if inp.gamma is None else 0, gamma=inp.gamma, row_off=inp.row_off)
    for label, call in (("three calls", r.step), ("one call", r.step_one_call), ("static workspace", r.step_static)):
        call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, 31, 2)
        check(label)
        assert_parity(r.results(inp.draft.shape[0]), ref, what=label)
    r.step_one_call(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp, 31, 2, greedy=True)
    check("greedy one call")
    r.step_greedy(batch, inp.draft, inp.target, inp.draft_tokens, inp.comp)
    check("greedy three calls")
    rows = inp.draft.shape[0]
    bt, tok = _guarded(torch.zeros(rows, dtype=torch.int32, device=DEV), -77)
    bp, prob = _guarded(torch.zeros(rows, dtype=torch.float32, device=DEV), -7.5)
    bf, flg = _guarded(torch.zeros(rows, dtype=torch.int32, device=DEV), -77)
    sk.sample_draft(batch, inp.draft, pkg.binding.TORCH_TO_DTYPE[inp.draft.dtype], 31, 2, 0, tok, prob, flg)
    torch.cuda.synchronize()
    for big in (bt, bp, bf):
        assert (big[:_GUARD] == big[0]).all() and (big[_GUARD + rows:] == big[0]).all()
    assert ((tok >= 0) & (tok < cfg.V)).all()


# --------------------------------------------------------------------------- randomised sweep
def _random_case(rng):
    """One random small configuration with random edits of the logits (masked blocks, ties,
    constant rows, spikes, NaN / inf, unusable tokens, p == q on a sequence)."""
    dtype = str(rng.choice(["f32", "f16", "bf16"]))
    V = int(rng.choice([1, 2, 3, 5, 17, 63, 64, 65, 255, 1000, 4031, 4032, 4033, 8064, 8191, 12345, 33333, 70001]))
    B = int(rng.choice([1, 2, 3, 7, 8, 9, 31, 33, 64]))
    gmax = int(rng.choice([1, 2, 4, 8, 16]))
    ragged = bool(rng.integers(0, 2))
    name = str(rng.choice(["C1", "C2", "C3", "C4", "C5"]))
    mode = str(rng.choice(["pos0", "agg4"]))
    form, nh = int(rng.integers(0, 2)), int(rng.choice([0, 1, 16, 33, 64]))
    cfg = config(name, B=B, V=V, dtype=dtype, gamma=int(rng.integers(1, gmax + 1)), gamma_max=gmax)
    gamma = torch.as_tensor(rng.integers(1, gmax + 1, size=B), dtype=torch.int32) if ragged else None
    inp = make_step(cfg, device=DEV, gamma=gamma, step=int(rng.integers(0, 5)))

    def fn(d, t, tok):
        for _ in range(int(rng.integers(0, 6))):
            kind = int(rng.integers(0, 8))
            side = d if rng.integers(0, 2) else t
            r = int(rng.integers(0, side.shape[0])); a = int(rng.integers(0, V)); b2 = int(rng.integers(a, V)) + 1
            if kind == 0: side[r, a:b2] = -float("inf")
            elif kind == 1: side[r, :] = float(rng.normal())
            elif kind == 2: side[r, a] = side[r, b2 - 1] = float(side[r].max()) + 1.0
            elif kind == 3: side[r, a] = 80.0 * float(rng.random())
            elif kind == 4: side[r, a] = float("nan")
            elif kind == 5: side[r, a] = float("inf")
            elif kind == 6: side[r, :] = -float("inf")
            elif kind == 7: tok[int(rng.integers(0, tok.numel()))] = int(rng.choice([-1, V, V + 5]))
        if rng.integers(0, 3) == 0:
            g0 = inp.gamma_host(); off = np.concatenate([[0], np.cumsum(g0)]); bb = int(rng.integers(0, B))
            t[off[bb] + bb: off[bb] + bb + g0[bb]] = d[off[bb]: off[bb] + g0[bb]]
    inp = _edit(inp, fn)
    inp.mlp = workloads.make_mlp(int(rng.integers(0, 1 << 30)), n_in=5 if mode == "pos0" else 7, n_hidden=nh, form=form)
    what = f"{name} {dtype} V={V} B={B} gamma_max={gmax} ragged={ragged} {mode} form={form} n_hidden={nh}"
    return inp, mode, what


def _sweep_seeds():
    """Two seeds by default; SPECKV_SWEEP_SEEDS=first:last adds that range for a longer run."""
    import os
    seeds = [20260527, 7]
    extra = os.environ.get("SPECKV_SWEEP_SEEDS")
    if extra:
        first, last = (int(x) for x in extra.split(":"))
        seeds += list(range(first, last))
    return seeds


@pytest.mark.parametrize("sweep_seed", _sweep_seeds())
def test_randomised_sweep_of_small_configurations(sk, sweep_seed):
    # Every case goes through both ways of issuing a step (which must agree bit for bit and match the
    # oracle) and through the proposal kernel.  Sweeps of this kind found a NaN inside a masked
    # region that went unflagged, a rejection at V = 1, and a score that cancels to 1e-3.
    rng = np.random.default_rng(sweep_seed)
    oracle.set_threads(16)
    total = dict(rows=0, excused_accept=0, excused_cdf=0, excused_gamma=0, excused_mass=0, accept_outside_relative_band=0)
    for it in range(120):
        inp, mode, what = _random_case(rng)
        seed, step, sb = int(rng.integers(0, 1 << 62)), int(rng.integers(0, 1 << 31)), int(rng.integers(0, 1 << 20))
        print("case", it, what, flush=True)
        ref = oracle_step(inp, seed, step, mode, seq_base=sb)
        a, _ = run_gpu(sk, inp, seed, step, mode, seq_base=sb, one_call=True)
        b, _ = run_gpu(sk, inp, seed, step, mode, seq_base=sb, one_call=False)
        problems, counts = compare(a, ref)
        assert not problems, (what, problems[:5])
        for k in total:
            total[k] += counts[k]
        for k in a:
            assert a[k].tobytes() == b[k].tobytes(), (what, k)
        smp = _run_sample(sk, inp, seed=seed, step=step, pos0=3, seq_base=sb)
        rs = oracle.sample_draft(workloads.stored_bits(inp.draft), inp.cfg.dtype, inp.cfg.B, inp.cfg.V, seed, step=step,
                                 gamma=inp.gamma_host(), seq_base=sb, pos0=3)
        _compare_sample(smp, rs)
        assert ((smp["tokens"] >= 0) & (smp["tokens"] < inp.cfg.V)).all()
    # excused rows over the whole sweep (about 2000 sequences, many of them built to sit on an edge:
    # tied maxima, p == q, masked rows): printed, and bounded per class
    print("sweep", sweep_seed, total, flush=True)
    assert total["excused_accept"] <= total["rows"] // 100 + 2
    assert total["excused_cdf"] <= total["rows"] // 100 + 2
    assert total["excused_gamma"] <= total["rows"] // 100 + 2
    assert total["excused_mass"] == 0 and total["accept_outside_relative_band"] == 0
