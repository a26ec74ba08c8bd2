"""Helpers for the GPU parity tests: upload a stack, run switches through the C ABI, fetch rows,
and compare them with the CPU oracle under the rule of oracle/compare.py."""
from __future__ import annotations

import numpy as np
import torch

from oracle import compare as C
from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L


def bits_to_device(W_bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(W_bits.view(np.int16).copy()).cuda().view(torch.bfloat16)


def device_to_bits(W: torch.Tensor) -> np.ndarray:
    return W.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceStack:
    """A stack of adapted linears resident on the GPU plus the library context for it."""

    def __init__(self, stack, shapes, E, r, scale=1.0, kernel=L.KERNEL_AUTO):
        self.stack, self.shapes, self.E, self.r, self.scale = stack, shapes, E, r, scale
        self.ctx = L.create_from_tensors(stack, shapes, E, r, scale)
        if kernel != L.KERNEL_AUTO:
            L.lsw_set_option(self.ctx, L.LSW_OPT_KERNEL, kernel)

    @classmethod
    def from_host(cls, host_stack, shapes, E, r, scale=1.0, kernel=L.KERNEL_AUTO, bf16_factors=False):
        """bf16_factors: upload A and B as bf16 tensors (the host arrays must already hold bf16-representable values,
        see bf16_factor_stack), so that the library is created with LSW_FACTOR_BF16."""
        conv = (lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)) if bf16_factors else (lambda x: torch.from_numpy(x).cuda())
        dev = [(bits_to_device(W), conv(A), conv(B)) for W, A, B in host_stack]
        if bf16_factors:
            for (_, A, B), (_, Ad, Bd) in zip(host_stack, dev):
                assert torch.equal(Ad.float().cpu(), torch.from_numpy(A)) and torch.equal(Bd.float().cpu(), torch.from_numpy(B))
        return cls(dev, shapes, E, r, scale, kernel)

    def switch(self, old, new, layers=None):
        L.lsw_switch(self.ctx, old[0], old[1], new[0], new[1], layers=layers,
                     stream=torch.cuda.current_stream().cuda_stream)

    def rows(self, p, rows=None) -> np.ndarray:
        W = self.stack[p][0]
        if rows is not None:
            W = W.index_select(0, torch.as_tensor(rows, device=W.device))
        return device_to_bits(W)

    def close(self):
        if self.ctx:
            torch.cuda.synchronize()
            L.lsw_destroy(self.ctx)
            self.ctx = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def bf16_factor_stack(host_stack):
    """The same stack with every factor rounded to the nearest bf16 value (kept in fp32 arrays for the oracle)."""
    def rnd(x):
        return torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    return [(W, rnd(A), rnd(B)) for W, A, B in host_stack]


def check_step(prev_bits, got_bits, A, B, old, new, scale=1.0, rows=None):
    """Teacher-forced check of one switch of one linear: oracle applied to the GPU's own previous state."""
    want = O.switch_step(prev_bits, A, B, old[0], old[1], new[0], new[1], scale, rows)
    S = O.switch_magnitude(A, B, old[0], old[1], new[0], new[1], scale, rows)
    return C.switch_parity(got_bits, want, prev_bits, S), want


def merge_reports(reports):
    tot = {k: 0 for k in ("n", "exact", "within_1ulp", "needed_clause2", "fail")}
    mx = 0
    for r in reports:
        for k in tot:
            tot[k] += r[k]
        mx = max(mx, r["max_dist"])
    tot["max_dist"] = mx
    tot["exact_frac"] = tot["exact"] / max(tot["n"], 1)
    return tot
