"""ctypes/numpy front end of the float64 C oracle (test infrastructure only).

Logits are handed over as the stored bits: ``float32`` arrays for fp32,
``uint16`` arrays holding binary16 or bfloat16 patterns otherwise, always with an
explicit dtype name so both sides of a parity test read identical bytes.
"""
import ctypes
import os

import numpy as np

from . import build as _build

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2}
FLAG_NONFINITE, FLAG_BAD_TOKEN, FLAG_FALLBACK = 1, 2, 4
RESID_FLOOR = 1e-6   # residual mass below which the correction is drawn from p_n (SKO_RESID_FLOOR)
GAMMAS = (2, 4, 6, 8)

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        lib.sko_load_logit.restype = ctypes.c_double
        lib.sko_residual.restype = ctypes.c_double
        lib.sko_inverse_cdf.restype = ctypes.c_int32
        lib.sko_inverse_cdf.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_double,
                                        ctypes.c_void_p]
        _lib = lib
    return _lib


def set_threads(n: int) -> None:
    """Number of host threads the oracle spreads sequences over (results do not depend on it)."""
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _as_logits(a, dtype):
    code = DTYPE_CODES[dtype]
    want = np.float32 if code == 0 else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"{dtype} logits must be passed as {want.__name__} bits, got {a.dtype}")
    return a, code


def _shape(B, gamma, gamma_uniform):
    if gamma is None:
        gamma = np.full(B, gamma_uniform, dtype=np.int32)
    gamma = np.ascontiguousarray(gamma, dtype=np.int32)
    if gamma.shape != (B,) or (gamma < 1).any():
        raise ValueError("gamma must be [B] with entries >= 1")
    row_off = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(gamma, out=row_off[1:])
    return gamma, row_off


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _load().sko_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def load_logits(bits, dtype):
    """Decode stored logits to float64, one by one, the way every oracle routine reads them."""
    a, code = _as_logits(bits, dtype)
    lib = _load()
    flat = a.reshape(-1)
    return np.array([lib.sko_load_logit(_ptr(flat), code, ctypes.c_int64(i))
                     for i in range(flat.size)], dtype=np.float64).reshape(a.shape)


def row_softmax(logits, dtype, row, V):
    """Softmax of one V-row -> (prob[V], H_bits, conf, argmax, has_nonfinite)."""
    a, code = _as_logits(logits, dtype)
    prob = np.zeros(V, dtype=np.float64)
    H = ctypes.c_double()
    c = ctypes.c_double()
    am = ctypes.c_int32()
    bad = _load().sko_row_softmax(_ptr(a), code, ctypes.c_int64(row), int(V), _ptr(prob),
                                  ctypes.byref(H), ctypes.byref(c), ctypes.byref(am))
    return prob, H.value, c.value, am.value, bool(bad)


def signals(draft, dtype, B, V, gamma=None, gamma_uniform=None):
    """Per-row entropy (bits), confidence, argmax and per-sequence aggregates."""
    a, code = _as_logits(draft, dtype)
    gamma, row_off = _shape(B, gamma, gamma_uniform)
    rows = int(row_off[-1])
    if a.size != rows * V:
        raise ValueError("draft logits size does not match sum(gamma)*V")
    H = np.zeros(rows)
    conf = np.zeros(rows)
    argmax = np.zeros(rows, dtype=np.int32)
    agg = np.zeros((B, 4))
    st = _load().sko_signals(_ptr(a), code, int(B), int(V), _ptr(gamma), _ptr(row_off),
                             _ptr(H), _ptr(conf), _ptr(argmax), _ptr(agg))
    if st:
        raise MemoryError("oracle signals failed")
    return dict(H=H, conf=conf, argmax=argmax, agg=agg, row_off=row_off, gamma=gamma)


def verify(draft, target, dtype, B, V, draft_tokens, seed, step=0, gamma=None,
           gamma_uniform=None, gamma_max=None, seq_base=0, debug=False):
    """Accept/reject and the one extra token of every sequence."""
    d, code = _as_logits(draft, dtype)
    t, _ = _as_logits(target, dtype)
    gamma, row_off = _shape(B, gamma, gamma_uniform)
    rows = int(row_off[-1])
    if gamma_max is None:
        gamma_max = int(gamma.max())
    if (gamma > gamma_max).any():
        raise ValueError("gamma exceeds gamma_max")
    if d.size != rows * V or t.size != (rows + B) * V:
        raise ValueError("logits sizes do not match the batch shape")
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    if tok.shape != (rows,):
        raise ValueError("draft_tokens must be [sum(gamma)]")
    n_acc = np.zeros(B, dtype=np.int32)
    tokens = np.zeros((B, gamma_max + 1), dtype=np.int32)
    num = np.zeros(B, dtype=np.int32)
    rate = np.zeros(B)
    flags = np.zeros(B, dtype=np.uint32)
    macc = np.zeros(B)
    mcdf = np.zeros(B)
    rmass = np.zeros(B)
    dbg = np.full((B, gamma_max, 3), np.nan) if debug else None
    st = _load().sko_verify(_ptr(d), _ptr(t), code, int(B), int(V), _ptr(gamma), _ptr(row_off),
                            _ptr(tok), ctypes.c_uint64(seed), ctypes.c_uint32(step),
                            ctypes.c_uint32(seq_base), int(gamma_max), _ptr(n_acc), _ptr(tokens),
                            _ptr(num), _ptr(rate), _ptr(flags), _ptr(macc), _ptr(mcdf), _ptr(rmass), _ptr(dbg))
    if st:
        raise MemoryError("oracle verify failed")
    out = dict(n_accepted=n_acc, tokens=tokens, num_tokens=num, accept_rate=rate,
               row_flags=flags, marg_acc=macc, marg_cdf=mcdf, resid_mass=rmass, row_off=row_off, gamma=gamma)
    if debug:
        out["dbg"] = dbg
    return out


def sample_draft(draft, dtype, B, V, seed, step=0, gamma=None, gamma_uniform=None, seq_base=0, pos0=0):
    """Draft-side proposal: one token per draft row by inverse CDF in vocabulary order."""
    a, code = _as_logits(draft, dtype)
    gamma, row_off = _shape(B, gamma, gamma_uniform)
    rows = int(row_off[-1])
    if a.size != rows * V:
        raise ValueError("draft logits size does not match sum(gamma)*V")
    tokens = np.zeros(rows, dtype=np.int32)
    prob = np.zeros(rows)
    flags = np.zeros(rows, dtype=np.uint32)
    margin = np.zeros(rows)
    st = _load().sko_sample_draft(_ptr(a), code, int(B), int(V), _ptr(gamma), _ptr(row_off),
                                  ctypes.c_uint64(seed), ctypes.c_uint32(step), ctypes.c_uint32(seq_base),
                                  ctypes.c_uint32(pos0), _ptr(tokens), _ptr(prob), _ptr(flags), _ptr(margin))
    if st:
        raise MemoryError("oracle sample_draft failed")
    return dict(tokens=tokens, prob=prob, flags=flags, margin=margin, row_off=row_off, gamma=gamma)


def verify_greedy(target, dtype, B, V, draft_tokens, gamma=None, gamma_uniform=None, gamma_max=None):
    """Greedy verification (target top-1 must equal the drafted token)."""
    t, code = _as_logits(target, dtype)
    gamma, row_off = _shape(B, gamma, gamma_uniform)
    rows = int(row_off[-1])
    if gamma_max is None:
        gamma_max = int(gamma.max())
    if (gamma > gamma_max).any() or gamma_max > 63:
        raise ValueError("gamma exceeds gamma_max")
    if t.size != (rows + B) * V:
        raise ValueError("target logits size does not match the batch shape")
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    if tok.shape != (rows,):
        raise ValueError("draft_tokens must be [sum(gamma)]")
    n_acc = np.zeros(B, dtype=np.int32)
    tokens = np.zeros((B, gamma_max + 1), dtype=np.int32)
    num = np.zeros(B, dtype=np.int32)
    rate = np.zeros(B)
    flags = np.zeros(B, dtype=np.uint32)
    _load().sko_verify_greedy(_ptr(t), code, int(B), int(V), _ptr(gamma), _ptr(row_off), _ptr(tok),
                              int(gamma_max), _ptr(n_acc), _ptr(tokens), _ptr(num), _ptr(rate), _ptr(flags))
    return dict(n_accepted=n_acc, tokens=tokens, num_tokens=num, accept_rate=rate, row_flags=flags,
                row_off=row_off, gamma=gamma)


def mlp_shapes(n_in, n_hidden, form):
    """Expected array shapes (W1, b1, W2, b2) of a controller; W1 / b1 are None without a hidden layer."""
    if form == 0:
        if n_hidden:
            return (n_hidden, n_in), (n_hidden,), (4, n_hidden), (4,)
        return None, None, (4, n_in), (4,)
    if n_hidden:
        return (n_hidden, n_in + 1), (n_hidden,), (1, n_hidden), (1,)
    return None, None, (1, n_in + 1), (1,)


def select_gamma(mlp, mode, H, conf, agg, row_off, comp):
    """mlp: dict with float32 W1, b1, W2, b2 and optionally 'form' (0: four outputs, 1: f([x, gamma])
    evaluated per candidate) -- shapes as mlp_shapes(); W1 = b1 = None for a linear predictor.
    mode: 'pos0' | 'agg4'."""
    m = {"pos0": 0, "agg4": 1}[mode]
    form = int(mlp.get("form", 0))
    n_in = 5 if m == 0 else 7
    W2 = np.ascontiguousarray(mlp["W2"], dtype=np.float32)
    b2 = np.ascontiguousarray(mlp["b2"], dtype=np.float32)
    if mlp.get("W1") is None:
        n_hidden, W1, b1 = 0, None, None
    else:
        W1 = np.ascontiguousarray(mlp["W1"], dtype=np.float32)
        b1 = np.ascontiguousarray(mlp["b1"], dtype=np.float32)
        n_hidden = W1.shape[0]
    want = mlp_shapes(n_in, n_hidden, form)
    have = (None if W1 is None else W1.shape, None if b1 is None else b1.shape, W2.shape, b2.shape)
    if have != want:
        raise ValueError(f"MLP shapes {have} do not match the feature mode and form (want {want})")
    H = np.ascontiguousarray(H, dtype=np.float64)
    conf = np.ascontiguousarray(conf, dtype=np.float64)
    agg = np.ascontiguousarray(agg, dtype=np.float64)
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    comp = np.ascontiguousarray(comp, dtype=np.uint8)
    B = comp.shape[0]
    gamma_next = np.zeros(B, dtype=np.int32)
    scores = np.zeros((B, 4))
    gap = np.zeros(B)
    st = _load().sko_select_gamma_form(form, m, int(n_hidden), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2),
                                       _ptr(H), _ptr(conf), _ptr(agg), _ptr(row_off), _ptr(comp),
                                       int(B), _ptr(gamma_next), _ptr(scores), _ptr(gap))
    if st:
        raise ValueError("oracle select_gamma rejected the MLP shape")
    return dict(gamma_next=gamma_next, scores=scores, gap=gap)


def residual(p, q):
    """r = max(0, p - q) (q None: bonus case r = p) and its mass R."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    qq = None if q is None else np.ascontiguousarray(q, dtype=np.float64)
    r = np.zeros_like(p)
    R = _load().sko_residual(_ptr(p), _ptr(qq), int(p.size), _ptr(r))
    return r, R


def inverse_cdf(r, tau):
    r = np.ascontiguousarray(r, dtype=np.float64)
    margin = ctypes.c_double()
    y = _load().sko_inverse_cdf(_ptr(r), int(r.size), float(tau), ctypes.byref(margin))
    return int(y), margin.value
