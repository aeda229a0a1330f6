"""ctypes binding of the C ABI declared in include/speckv.h.

Argument marshalling only: every step of the path runs in the library's HIP kernels.  Tensors
are torch tensors on the GPU (torch is used for device memory and streams, nothing else); the
binding passes their ``data_ptr()`` and the current stream's handle across the ABI.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspeckv.so")

STATUS_NAMES = {0: "OK", 1: "ERR_NULL", 2: "ERR_SHAPE", 3: "ERR_DTYPE", 4: "ERR_ALIGN",
                5: "ERR_WORKSPACE", 6: "ERR_GAMMA", 7: "ERR_STATE", 8: "ERR_DEVICE"}
DTYPES = {"f32": 0, "f16": 1, "bf16": 2}
TORCH_TO_DTYPE = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
FEATURES = {"pos0": 0, "agg4": 1}
FLAG_NONFINITE, FLAG_BAD_TOKEN, FLAG_FALLBACK, FLAG_BAD_GAMMA = 1, 2, 4, 8
GAMMA_LIMIT = 16
STATIC_WS_BYTES = 16 << 20


class SpecKVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"speckv: {STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class _CBatch(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("V", ctypes.c_int32), ("gamma_max", ctypes.c_int32),
                ("gamma_uniform", ctypes.c_int32), ("gamma", ctypes.c_void_p),
                ("row_off", ctypes.c_void_p), ("seq_base", ctypes.c_uint32)]


class _CMlp(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_int32), ("n_hidden", ctypes.c_int32), ("W1", ctypes.c_void_p),
                ("b1", ctypes.c_void_p), ("W2", ctypes.c_void_p), ("b2", ctypes.c_void_p), ("form", ctypes.c_int32)]


class _CStepArgs(ctypes.Structure):
    _fields_ = [("draft_logits", ctypes.c_void_p), ("target_logits", ctypes.c_void_p), ("dtype", ctypes.c_int),
                ("draft_tokens", ctypes.c_void_p), ("comp", ctypes.c_void_p), ("seed", ctypes.c_uint64),
                ("step", ctypes.c_uint32), ("mode", ctypes.c_int), ("H", ctypes.c_void_p), ("conf", ctypes.c_void_p),
                ("argmax", ctypes.c_void_p), ("agg", ctypes.c_void_p), ("n_accepted", ctypes.c_void_p),
                ("tokens", ctypes.c_void_p), ("num_tokens", ctypes.c_void_p), ("accept_rate", ctypes.c_void_p),
                ("row_flags", ctypes.c_void_p), ("gamma_next", ctypes.c_void_p), ("scores", ctypes.c_void_p),
                ("greedy", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libspeckv.so from the package directory; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_02888_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, u32, u64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t
    lib.speckv_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.speckv_destroy.argtypes = [vp]
    lib.speckv_last_error.argtypes = [vp]
    lib.speckv_last_error.restype = ctypes.c_char_p
    lib.speckv_workspace_bytes.argtypes = [i32, i32]
    lib.speckv_workspace_bytes.restype = sz
    lib.speckv_row_offsets.argtypes = [vp, vp, i32, vp, vp]
    lib.speckv_signals.argtypes = [vp, ctypes.POINTER(_CBatch), vp, ctypes.c_int, vp, sz, vp, vp, vp, vp, vp]
    lib.speckv_verify.argtypes = [vp, ctypes.POINTER(_CBatch), vp, vp, ctypes.c_int, vp, u64, u32, vp, sz,
                                  vp, vp, vp, vp, vp, vp]
    lib.speckv_verify_greedy.argtypes = [vp, ctypes.POINTER(_CBatch), vp, ctypes.c_int, vp, vp, sz, vp, vp, vp, vp,
                                         vp, vp]
    lib.speckv_select_gamma.argtypes = [vp, ctypes.POINTER(_CBatch), ctypes.POINTER(_CMlp), ctypes.c_int,
                                        vp, vp, vp, vp, vp, vp, vp]
    lib.speckv_step.argtypes = [vp, ctypes.POINTER(_CBatch), ctypes.POINTER(_CMlp), ctypes.POINTER(_CStepArgs), vp, sz, vp]
    lib.speckv_step_static.argtypes = [vp, ctypes.POINTER(_CBatch), ctypes.POINTER(_CMlp), ctypes.POINTER(_CStepArgs), vp]
    lib.speckv_sample_draft.argtypes = [vp, ctypes.POINTER(_CBatch), vp, ctypes.c_int, u64, u32, u32, vp, vp, vp, vp]
    lib.speckv_set_option.argtypes = [vp, ctypes.c_char_p, i32]
    lib.speckv_get_option.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(i32)]
    lib.speckv_profile.argtypes = [vp, i32]
    lib.speckv_profile_read.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(i32),
                                        ctypes.POINTER(ctypes.c_double)]
    lib.speckv_trace.argtypes = [vp, vp, sz]
    lib.speckv_probe_read.argtypes = [vp, vp, sz, vp, vp]
    lib.speckv_probe_copy.argtypes = [vp, vp, vp, sz, vp]
    for name in ("speckv_create", "speckv_destroy", "speckv_row_offsets", "speckv_signals",
                 "speckv_verify", "speckv_verify_greedy", "speckv_select_gamma", "speckv_step", "speckv_step_static", "speckv_sample_draft", "speckv_set_option", "speckv_get_option",
                 "speckv_profile", "speckv_profile_read", "speckv_trace", "speckv_probe_read", "speckv_probe_copy"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def workspace_bytes(B: int, gamma_max: int) -> int:
    return int(load_library().speckv_workspace_bytes(B, gamma_max))


@dataclass
class Batch:
    """Shape of one step's batch; gamma/row_off are device tensors for ragged batches."""
    B: int
    V: int
    gamma_max: int
    gamma_uniform: int = 0
    gamma: Optional[torch.Tensor] = None     # int32 [B]
    row_off: Optional[torch.Tensor] = None   # int64 [B+1]
    seq_base: int = 0

    def c_struct(self) -> _CBatch:
        return _CBatch(self.B, self.V, self.gamma_max, self.gamma_uniform, _ptr(self.gamma),
                       _ptr(self.row_off), self.seq_base)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _c_mlp(mlp: dict) -> _CMlp:
    """mlp: n_in, n_hidden, device tensors (or addresses) W1, b1, W2, b2, optional form (0 vector, 1 scalar)."""
    return _CMlp(mlp["n_in"], mlp["n_hidden"], _ptr(mlp.get("W1")), _ptr(mlp.get("b1")), _ptr(mlp["W2"]),
                 _ptr(mlp["b2"]), int(mlp.get("form", 0)))


def _stream():
    return torch.cuda.current_stream().cuda_stream


class SpecKV:
    """One library handle bound to a GPU.  device=-1 gives a handle that only validates arguments."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        h = ctypes.c_void_p()
        st = self.lib.speckv_create(ctypes.byref(h), device)
        if st:
            raise SpecKVError(st, self.lib.speckv_last_error(None).decode())
        self.h = h
        self.device = device

    def close(self):
        if getattr(self, "h", None):
            self.lib.speckv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st:
            raise SpecKVError(st, self.lib.speckv_last_error(self.h).decode())

    # ---- the three calls of a step ---------------------------------------------------------
    def signals(self, batch: Batch, draft, dtype: int, ws, H, conf, argmax, agg, ws_bytes=None, stream=None):
        self._check(self.lib.speckv_signals(
            self.h, ctypes.byref(batch.c_struct()), _ptr(draft), dtype, _ptr(ws),
            ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes,
            _stream() if stream is None else stream, _ptr(H), _ptr(conf), _ptr(argmax), _ptr(agg)))

    def verify(self, batch: Batch, target, draft, dtype: int, draft_tokens, seed: int, step: int, ws,
               n_accepted, tokens, num_tokens, accept_rate=None, row_flags=None, ws_bytes=None, stream=None):
        self._check(self.lib.speckv_verify(
            self.h, ctypes.byref(batch.c_struct()), _ptr(target), _ptr(draft), dtype, _ptr(draft_tokens),
            seed, step, _ptr(ws), ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes,
            _stream() if stream is None else stream, _ptr(n_accepted), _ptr(tokens), _ptr(num_tokens),
            _ptr(accept_rate), _ptr(row_flags)))

    def verify_greedy(self, batch: Batch, target, dtype: int, draft_tokens, ws, n_accepted, tokens, num_tokens,
                      accept_rate=None, row_flags=None, ws_bytes=None, stream=None):
        self._check(self.lib.speckv_verify_greedy(
            self.h, ctypes.byref(batch.c_struct()), _ptr(target), dtype, _ptr(draft_tokens), _ptr(ws),
            ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes,
            _stream() if stream is None else stream, _ptr(n_accepted), _ptr(tokens), _ptr(num_tokens),
            _ptr(accept_rate), _ptr(row_flags)))

    def select_gamma(self, batch: Batch, mlp: dict, mode: int, H, conf, agg, comp, gamma_next, scores=None,
                     stream=None):
        m = _c_mlp(mlp)
        self._check(self.lib.speckv_select_gamma(
            self.h, ctypes.byref(batch.c_struct()), ctypes.byref(m), mode, _ptr(H), _ptr(conf), _ptr(agg),
            _ptr(comp), _stream() if stream is None else stream, _ptr(gamma_next), _ptr(scores)))

    def step(self, batch: Batch, mlp: dict, mode: int, draft, target, dtype: int, draft_tokens, comp, seed: int,
             step: int, ws, H, conf, argmax, agg, n_accepted, tokens, num_tokens, accept_rate, row_flags,
             gamma_next, scores=None, ws_bytes=None, stream=None, greedy=False):
        """The whole step in one call (same results as signals + verify + select_gamma; with greedy=True
        as signals + verify_greedy + select_gamma)."""
        m = _c_mlp(mlp)
        a = _CStepArgs(_ptr(draft), _ptr(target), dtype, _ptr(draft_tokens), _ptr(comp), seed, step, mode, _ptr(H),
                       _ptr(conf), _ptr(argmax), _ptr(agg), _ptr(n_accepted), _ptr(tokens), _ptr(num_tokens),
                       _ptr(accept_rate), _ptr(row_flags), _ptr(gamma_next), _ptr(scores), int(greedy))
        self._check(self.lib.speckv_step(
            self.h, ctypes.byref(batch.c_struct()), ctypes.byref(m), ctypes.byref(a), _ptr(ws),
            ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes,
            _stream() if stream is None else stream))

    def step_static(self, batch: Batch, mlp: dict, mode: int, draft, target, dtype: int, draft_tokens, comp,
                    seed: int, step: int, H, conf, argmax, agg, n_accepted, tokens, num_tokens, accept_rate,
                    row_flags, gamma_next, scores=None, stream=None, greedy=False):
        """speckv_step with the library's own workspace (the call allocates nothing)."""
        m = _c_mlp(mlp)
        a = _CStepArgs(_ptr(draft), _ptr(target), dtype, _ptr(draft_tokens), _ptr(comp), seed, step, mode, _ptr(H),
                       _ptr(conf), _ptr(argmax), _ptr(agg), _ptr(n_accepted), _ptr(tokens), _ptr(num_tokens),
                       _ptr(accept_rate), _ptr(row_flags), _ptr(gamma_next), _ptr(scores), int(greedy))
        self._check(self.lib.speckv_step_static(
            self.h, ctypes.byref(batch.c_struct()), ctypes.byref(m), ctypes.byref(a),
            _stream() if stream is None else stream))

    def sample_draft(self, batch: Batch, draft, dtype: int, seed: int, step: int, pos0: int, tokens, prob=None,
                     row_flags=None, stream=None):
        """One token per draft row from softmax(row) (the draft model's proposal step)."""
        self._check(self.lib.speckv_sample_draft(
            self.h, ctypes.byref(batch.c_struct()), _ptr(draft), dtype, seed, step, pos0,
            _stream() if stream is None else stream, _ptr(tokens), _ptr(prob), _ptr(row_flags)))

    def row_offsets(self, gamma, B: int, row_off, stream=None):
        self._check(self.lib.speckv_row_offsets(self.h, _ptr(gamma), B, _ptr(row_off),
                                                _stream() if stream is None else stream))

    # ---- options, profiling, probes ----------------------------------------------------------
    def set_option(self, name: str, value: int):
        self._check(self.lib.speckv_set_option(self.h, name.encode(), value))

    def get_option(self, name: str) -> int:
        v = ctypes.c_int32()
        self._check(self.lib.speckv_get_option(self.h, name.encode(), ctypes.byref(v)))
        return v.value

    def profile(self, level: int):
        self._check(self.lib.speckv_profile(self.h, level))

    def profile_read(self, kernel: str):
        n = ctypes.c_int32()
        ms = ctypes.c_double()
        self._check(self.lib.speckv_profile_read(self.h, kernel.encode(), ctypes.byref(n), ctypes.byref(ms)))
        return n.value, ms.value

    def trace(self, buf):
        """Record per-workgroup clock readings of speckv_step into buf (uint64 device tensor), or stop (None)."""
        self._check(self.lib.speckv_trace(self.h, _ptr(buf), 0 if buf is None else buf.numel() * buf.element_size()))

    def probe_read(self, src, nbytes: int, sink, stream=None):
        self._check(self.lib.speckv_probe_read(self.h, _ptr(src), nbytes, _ptr(sink),
                                               _stream() if stream is None else stream))

    def probe_copy(self, dst, src, nbytes: int, stream=None):
        self._check(self.lib.speckv_probe_copy(self.h, _ptr(dst), _ptr(src), nbytes,
                                               _stream() if stream is None else stream))
