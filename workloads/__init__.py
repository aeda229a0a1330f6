"""Seeded synthetic inputs for the SpecKV verify-and-select stage.

This module only *draws inputs*: logits with the shapes, dtypes and draft/target
agreement regimes of the five benchmark configurations, drafted token ids, the
compression-level labels and random controller weights.  It contains none of the
method's arithmetic (no softmax, entropy, accept test, residual or MLP) and is
the one module both the CPU oracle's tests and the HIP path's tests import, so
that both sides read identical bytes.

The paper measured on 20 private prompts run through Llama-3.2 1B/3B
(vocabulary 128,256; Section 4.1).  Neither prompts nor models are available
here; these draws stand in for them.

Drafted tokens are drawn from softmax(draft row) with the Gumbel-max identity
(argmax of logits plus Gumbel noise), which needs no softmax.
"""
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20260527
TORCH_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
GAMMAS = (2, 4, 6, 8)


@dataclass
class Config:
    name: str
    B: int
    V: int
    dtype: str
    gamma: int                 # uniform speculation length (ragged batches override per row)
    law: str                   # "normal" | "zipf"
    draft_sigma: float = 3.0
    noise_sigma: tuple = (1.0,)  # target-noise sigma, cycled over rows (emulates FP16/INT8/NF4 targets)
    temperature: float = 1.0   # logits are divided by this before storage
    comp_cycle: bool = True    # compression label = b mod 3, else all FP16
    seed: int = BASE_SEED
    gamma_max: int = 8


def config(name: str, **over) -> Config:
    """The five benchmark configurations, in the benchmark spec order; keyword overrides shrink them."""
    table = {
        "C1": Config("C1", B=1, V=32000, dtype="f32", gamma=4, law="normal", comp_cycle=False,
                     seed=BASE_SEED + 1),
        "C2": Config("C2", B=64, V=32000, dtype="bf16", gamma=4, law="normal",
                     noise_sigma=(0.5, 1.0, 2.0), seed=BASE_SEED + 2),
        "C3": Config("C3", B=256, V=128256, dtype="bf16", gamma=8, law="zipf", seed=BASE_SEED + 3),
        "C4": Config("C4", B=1024, V=151936, dtype="f16", gamma=4, law="normal", draft_sigma=2.5,
                     noise_sigma=(1.5,), seed=BASE_SEED + 4),
        "C5": Config("C5", B=4096, V=50257, dtype="f32", gamma=8, law="normal", draft_sigma=3.0,
                     noise_sigma=(0.3,), temperature=0.3, seed=BASE_SEED + 5),
    }
    cfg = table[name]
    for k, v in over.items():
        setattr(cfg, k, v)
    return cfg


@dataclass
class StepInputs:
    cfg: Config
    gamma: Optional[torch.Tensor]      # int32 [B] on device for ragged batches, else None
    row_off: Optional[torch.Tensor]    # int64 [B+1] draft-row offsets for ragged batches, else None
    draft: torch.Tensor                # [sum gamma_b, V] stored dtype
    target: torch.Tensor               # [sum (gamma_b+1), V] stored dtype
    draft_tokens: torch.Tensor         # int32 [sum gamma_b]
    comp: torch.Tensor                 # uint8 [B]
    mlp: Dict[str, np.ndarray] = field(default_factory=dict)

    def gamma_host(self) -> np.ndarray:
        if self.gamma is None:
            return np.full(self.cfg.B, self.cfg.gamma, dtype=np.int32)
        return self.gamma.cpu().numpy().astype(np.int32)


def stored_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a logits tensor as the bits the oracle reads (float32, or uint16 patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


def make_mlp(seed: int, n_in: int = 5, n_hidden: int = 16, form: int = 0) -> Dict[str, np.ndarray]:
    """Controller weights N(0, 0.5^2), drawn in the order W1, b1, W2, b2.
    form 0: four outputs from the context vector; form 1: one output from [context, gamma].
    n_hidden = 0: no hidden layer (W1 = b1 = None, W2 maps the input directly)."""
    rng = np.random.default_rng(seed)
    n_x = n_in + (1 if form == 1 else 0)
    n_out = 4 if form == 0 else 1
    out: Dict[str, np.ndarray] = {"form": form}
    if n_hidden:
        out["W1"] = (0.5 * rng.standard_normal((n_hidden, n_x))).astype(np.float32)
        out["b1"] = (0.5 * rng.standard_normal(n_hidden)).astype(np.float32)
        out["W2"] = (0.5 * rng.standard_normal((n_out, n_hidden))).astype(np.float32)
    else:
        out["W1"] = out["b1"] = None
        out["W2"] = (0.5 * rng.standard_normal((n_out, n_x))).astype(np.float32)
    out["b2"] = (0.5 * rng.standard_normal(n_out)).astype(np.float32)
    return out


def _gumbel_argmax(x32: torch.Tensor, gen: torch.Generator) -> torch.Tensor:
    e = torch.empty_like(x32).exponential_(generator=gen)
    return torch.argmax(x32 - torch.log(e), dim=-1).to(torch.int32)


def _draw_full(cfg: Config, device, step: int, b0: int, b1: int):
    """Logits for sequences [b0, b1) at gamma_max positions: draft [n, G, V], target [n, G+1, V]
    in the stored dtype, plus drafted tokens [n, G] sampled from the stored draft rows."""
    G, V, n = cfg.gamma_max, cfg.V, b1 - b0
    dt = TORCH_DTYPES[cfg.dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed * 1000003 + step * 7919 + b0)
    T = cfg.temperature
    sig = torch.tensor([cfg.noise_sigma[b % len(cfg.noise_sigma)] for b in range(b0, b1)],
                       dtype=torch.float32, device=device).view(n, 1, 1)
    if cfg.law == "normal":
        d32 = cfg.draft_sigma * torch.randn(n, G, V, generator=gen, device=device)
        t32 = torch.empty(n, G + 1, V, dtype=torch.float32, device=device)
        t32[:, :G] = d32 + sig * torch.randn(n, G, V, generator=gen, device=device)
        t32[:, G] = cfg.draft_sigma * torch.randn(n, V, generator=gen, device=device)
        d32 = d32 / T
        t32 = t32 / T
    elif cfg.law == "zipf":
        # rank r = 1..V gets -1.1 ln r + N(0, 0.5^2), scattered by a fresh permutation per V-row;
        # the target shares permutation and ranks and adds elementwise N(0, 1); bonus row is fresh.
        base = -1.1 * torch.log(torch.arange(1, V + 1, dtype=torch.float32, device=device))
        d32 = torch.empty(n, G, V, dtype=torch.float32, device=device)
        t32 = torch.empty(n, G + 1, V, dtype=torch.float32, device=device)
        for s in range(n):
            for i in range(G + 1):
                perm = torch.randperm(V, generator=gen, device=device)
                row = base + 0.5 * torch.randn(V, generator=gen, device=device)
                if i < G:
                    d32[s, i, perm] = row
                    t32[s, i, perm] = row
                else:
                    t32[s, i, perm] = row
        t32[:, :G] += sig * torch.randn(n, G, V, generator=gen, device=device)
    else:
        raise ValueError(cfg.law)
    draft = d32.to(dt)
    target = t32.to(dt)
    tokens = _gumbel_argmax(draft.float(), gen)
    return draft, target, tokens


def make_step(cfg: Config, device="cpu", step: int = 0, gamma: Optional[torch.Tensor] = None,
              chunk: int = 16) -> StepInputs:
    """One step's inputs.  gamma: optional int [B] of per-row speculation lengths (ragged, packed)."""
    B, V, G = cfg.B, cfg.V, cfg.gamma_max
    dt = TORCH_DTYPES[cfg.dtype]
    if gamma is None:
        g_host = np.full(B, cfg.gamma, dtype=np.int64)
    else:
        g_host = gamma.detach().cpu().numpy().astype(np.int64)
        if g_host.shape != (B,) or g_host.min() < 1 or g_host.max() > G:
            raise ValueError("gamma must be [B] within [1, gamma_max]")
    off = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(g_host, out=off[1:])
    rows = int(off[-1])
    draft = torch.empty(rows, V, dtype=dt, device=device)
    target = torch.empty(rows + B, V, dtype=dt, device=device)
    tokens = torch.empty(rows, dtype=torch.int32, device=device)
    for b0 in range(0, B, chunk):
        b1 = min(B, b0 + chunk)
        d, t, tok = _draw_full(cfg, device, step, b0, b1)
        for b in range(b0, b1):
            g = int(g_host[b])
            draft[off[b]:off[b] + g] = d[b - b0, :g]
            tokens[off[b]:off[b] + g] = tok[b - b0, :g]
            # target rows 0..g-1 pair with the drafts; the bonus row is the independent one
            target[off[b] + b:off[b] + b + g] = t[b - b0, :g]
            target[off[b] + b + g] = t[b - b0, G]
    comp = (torch.arange(B) % 3).to(torch.uint8) if cfg.comp_cycle else torch.zeros(B, dtype=torch.uint8)
    ragged = gamma is not None
    return StepInputs(
        cfg=cfg,
        gamma=torch.as_tensor(g_host, dtype=torch.int32).to(device) if ragged else None,
        row_off=torch.as_tensor(off, dtype=torch.int64).to(device) if ragged else None,
        draft=draft, target=target, draft_tokens=tokens, comp=comp.to(device),
        mlp=make_mlp(cfg.seed),
    )
