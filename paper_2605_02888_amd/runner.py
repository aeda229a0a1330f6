"""Convenience around the binding: owns the output tensors and workspace of one batch shape and
issues the calls of a step on the current stream.  Allocation and marshalling only."""
from typing import Dict, Optional

import numpy as np
import torch

from .binding import Batch, SpecKV, TORCH_TO_DTYPE, FEATURES, workspace_bytes


class StepRunner:
    def __init__(self, sk: SpecKV, B: int, V: int, gamma_max: int, torch_dtype, mlp: Dict[str, np.ndarray],
                 mode: str = "pos0", device="cuda:0", max_draft_rows: Optional[int] = None, seq_base: int = 0,
                 with_argmax: bool = True):
        self.sk, self.B, self.V, self.gamma_max = sk, B, V, gamma_max
        self.dtype = TORCH_TO_DTYPE[torch_dtype]
        self.mode = FEATURES[mode]
        self.seq_base = seq_base
        self.with_argmax = with_argmax  # argmax of the draft rows is an optional output of speckv_signals
        dev = torch.device(device)
        rows = B * gamma_max if max_draft_rows is None else max_draft_rows
        self.ws = torch.empty(workspace_bytes(B, gamma_max), dtype=torch.uint8, device=dev)
        self.H = torch.zeros(rows, dtype=torch.float32, device=dev)
        self.conf = torch.zeros(rows, dtype=torch.float32, device=dev)
        self.argmax = torch.zeros(rows, dtype=torch.int32, device=dev)
        self.agg = torch.zeros(B, 4, dtype=torch.float32, device=dev)
        self.n_accepted = torch.zeros(B, dtype=torch.int32, device=dev)
        self.tokens = torch.zeros(B, gamma_max + 1, dtype=torch.int32, device=dev)
        self.num_tokens = torch.zeros(B, dtype=torch.int32, device=dev)
        self.accept_rate = torch.zeros(B, dtype=torch.float32, device=dev)
        self.row_flags = torch.zeros(B, dtype=torch.int32, device=dev)
        self.gamma_next = torch.zeros(B, dtype=torch.int32, device=dev)
        self.scores = torch.zeros(B, 4, dtype=torch.float32, device=dev)
        self.mlp = {k: torch.as_tensor(np.ascontiguousarray(v, dtype=np.float32)).to(dev)
                    for k, v in mlp.items() if k in ("W1", "b1", "W2", "b2") and v is not None}
        self.mlp["form"] = int(mlp.get("form", 0))
        self.mlp["n_in"] = 5 if mode == "pos0" else 7
        self.mlp["n_hidden"] = int(self.mlp["b1"].shape[0]) if "b1" in self.mlp else 0

    def batch(self, gamma_uniform: int = 0, gamma=None, row_off=None) -> Batch:
        return Batch(B=self.B, V=self.V, gamma_max=self.gamma_max, gamma_uniform=gamma_uniform, gamma=gamma,
                     row_off=row_off, seq_base=self.seq_base)

    def step(self, batch: Batch, draft, target, draft_tokens, comp, seed: int, step: int = 0):
        """signals -> verify -> select_gamma on the current stream; results stay on the device."""
        sk = self.sk
        sk.signals(batch, draft, self.dtype, self.ws, self.H, self.conf, self.argmax if self.with_argmax else None,
                   self.agg)
        sk.verify(batch, target, draft, self.dtype, draft_tokens, seed, step, self.ws, self.n_accepted,
                  self.tokens, self.num_tokens, self.accept_rate, self.row_flags)
        sk.select_gamma(batch, self.mlp, self.mode, self.H, self.conf, self.agg, comp, self.gamma_next,
                        self.scores)

    def step_one_call(self, batch: Batch, draft, target, draft_tokens, comp, seed: int, step: int = 0,
                      greedy: bool = False):
        """The same step through speckv_step: one ABI call, two launches."""
        self.sk.step(batch, self.mlp, self.mode, draft, target, self.dtype, draft_tokens, comp, seed, step, self.ws,
                     self.H, self.conf, self.argmax if self.with_argmax else None, self.agg, self.n_accepted,
                     self.tokens, self.num_tokens, self.accept_rate, self.row_flags, self.gamma_next, self.scores,
                     greedy=greedy)

    def step_static(self, batch: Batch, draft, target, draft_tokens, comp, seed: int, step: int = 0,
                    greedy: bool = False):
        """The same step through speckv_step_static: the library's own workspace, no allocation in the call."""
        self.sk.step_static(batch, self.mlp, self.mode, draft, target, self.dtype, draft_tokens, comp, seed, step,
                            self.H, self.conf, self.argmax if self.with_argmax else None, self.agg, self.n_accepted,
                            self.tokens, self.num_tokens, self.accept_rate, self.row_flags, self.gamma_next,
                            self.scores, greedy=greedy)

    def step_greedy(self, batch: Batch, draft, target, draft_tokens, comp):
        """signals -> verify_greedy -> select_gamma (the accept rule as the paper words it), three calls."""
        sk = self.sk
        sk.signals(batch, draft, self.dtype, self.ws, self.H, self.conf, self.argmax if self.with_argmax else None,
                   self.agg)
        sk.verify_greedy(batch, target, self.dtype, draft_tokens, self.ws, self.n_accepted, self.tokens,
                         self.num_tokens, self.accept_rate, self.row_flags)
        sk.select_gamma(batch, self.mlp, self.mode, self.H, self.conf, self.agg, comp, self.gamma_next,
                        self.scores)

    def results(self, n_draft_rows: int) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize()
        out = {k: getattr(self, k).cpu().numpy() for k in
               ("agg", "n_accepted", "tokens", "num_tokens", "accept_rate", "row_flags", "gamma_next", "scores")}
        for k in ("H", "conf", "argmax"):
            out[k] = getattr(self, k)[:n_draft_rows].cpu().numpy()
        return out
