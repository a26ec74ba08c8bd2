"""Seeded synthetic inputs for the adapter-switch workloads.

This module only draws random tensors of the right shapes and value
distributions.  It holds none of the method's arithmetic (no routing, no
merge), so the CPU oracle's tests and the GPU harness can both take their
inputs from here without sharing any computation.

Workloads (std = standard deviation of a zero-mean normal):

  tiny   1 layer, one linear 256x256; 8 experts, rank 8; W std 0.02 (bf16),
         A std 1/16, B std 0.01 (fp32); 16 switch steps, top-2.
  7b     32 layers x {q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008};
         8 experts rank 8; A std 1/64; 64 switch steps.
  7b_r64 as 7b with rank 64.
  13b    40 layers, hidden 5120, FFN 13824; 16 experts rank 16; A std
         1/sqrt(5120); about half of the steps are forced to keep one of the
         previous step's experts.
  70b    80 layers, hidden 8192, FFN 28672, k/v 1024x8192; 8 experts rank 16;
         A std 1/sqrt(8192).

Weights are [out, in] row-major, A is [E, r, in], B is [E, out, r].
"""

from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

KINDS = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    hidden: int
    ffn: int
    kv: int
    experts: int
    rank: int
    top_k: int
    steps: int
    w_std: float
    a_std: float
    b_std: float
    seed: int
    reuse_prob: float = 0.0
    kinds: tuple = KINDS

    def linear_shapes(self):
        """[(layer, kind_index, out, in)] in launch order."""
        dims = {
            "q": (self.hidden, self.hidden), "k": (self.kv, self.hidden),
            "v": (self.kv, self.hidden), "o": (self.hidden, self.hidden),
            "gate": (self.ffn, self.hidden), "up": (self.ffn, self.hidden),
            "down": (self.hidden, self.ffn),
        }
        out = []
        for layer in range(self.layers):
            for kind in self.kinds:
                o, i = dims[kind]
                out.append((layer, KINDS.index(kind), o, i))
        return out

    def w_elements(self):
        return sum(o * i for _, _, o, i in self.linear_shapes())

    def factor_dims(self):
        return sum(o + i for _, _, o, i in self.linear_shapes())


WORKLOADS = {
    "tiny": Workload("tiny", 1, 256, 256, 256, 8, 8, 2, 16, 0.02, 1 / 16, 0.01, 1001, kinds=("q",)),
    "7b": Workload("7b", 32, 4096, 11008, 4096, 8, 8, 2, 64, 0.02, 1 / 64, 0.01, 1002),
    "7b_r64": Workload("7b_r64", 32, 4096, 11008, 4096, 8, 64, 2, 64, 0.02, 1 / 64, 0.01, 1003),
    "13b": Workload("13b", 40, 5120, 13824, 5120, 16, 16, 2, 64, 0.02, 1 / math.sqrt(5120), 0.01, 1004,
                    reuse_prob=0.5),
    "70b": Workload("70b", 80, 8192, 28672, 1024, 8, 16, 2, 16, 0.02, 1 / math.sqrt(8192), 0.01, 1005),
}


def scaled(wl: Workload, layers: int) -> Workload:
    """Same shapes with fewer layers (for tests that must finish in seconds)."""
    return Workload(**{**wl.__dict__, "layers": layers, "name": f"{wl.name}[{layers}L]"})


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Quantise drawn fp32 samples to bf16 storage; returns the uint16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def host_linear(rng: np.random.Generator, out: int, inn: int, experts: int, rank: int,
                w_std=0.02, a_std=None, b_std=0.01):
    """One adapted linear drawn on the host: (W bf16 bits [out,in], A fp32, B fp32)."""
    a_std = 1.0 / math.sqrt(inn) if a_std is None else a_std
    W = f32_to_bf16_bits(rng.normal(0.0, w_std, size=(out, inn)).astype(np.float32))
    A = rng.normal(0.0, a_std, size=(experts, rank, inn)).astype(np.float32)
    B = rng.normal(0.0, b_std, size=(experts, out, rank)).astype(np.float32)
    return W, A, B


def host_stack(wl: Workload):
    """Every linear of a (small) workload drawn on the host with wl.seed."""
    rng = np.random.default_rng(wl.seed)
    return [host_linear(rng, o, i, wl.experts, wl.rank, wl.w_std, wl.a_std, wl.b_std)
            for _, _, o, i in wl.linear_shapes()]


PAD_GUARD = -7.5          # what the padding columns of a W stored at a leading dimension > in are filled with


def device_stack(wl: Workload, device="cuda", factor_dtype=torch.float32, ld_of=None):
    """Every linear of a workload drawn on the device with wl.seed.

    Returns a list of (W bf16 [out,in], A [E,r,in], B [E,out,r]) torch tensors; the factors are drawn in
    fp32 and stored as `factor_dtype` (fp32, or bf16: each value rounded once to the nearest bf16).
    ld_of: optional function in -> leading dimension (elements).  Where it exceeds `in`, W is the first `in`
    columns of an [out, ld] buffer whose other columns hold PAD_GUARD; the drawn values are the same.
    """
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed)
    stack = []
    for _, _, o, i in wl.linear_shapes():
        W = (torch.randn(o, i, generator=g, device=device, dtype=torch.float32) * wl.w_std).to(torch.bfloat16)
        if ld_of is not None and ld_of(i) > i:
            full = torch.full((o, int(ld_of(i))), PAD_GUARD, device=device, dtype=torch.bfloat16)
            full[:, :i] = W
            W = full[:, :i]
        A = torch.randn(wl.experts, wl.rank, i, generator=g, device=device, dtype=torch.float32) * wl.a_std
        B = torch.randn(wl.experts, o, wl.rank, generator=g, device=device, dtype=torch.float32) * wl.b_std
        stack.append((W, A.to(factor_dtype), B.to(factor_dtype)))
    return stack


def router_logits(wl: Workload, steps=None) -> np.ndarray:
    """fp32 [steps, E] router logits ~ N(0,1), one row per token.

    With wl.reuse_prob > 0 the rows are built by rank instead of drawn in place: the step's E values are
    sorted, and a random order of the experts says which expert receives the largest value, the second
    largest, and so on (i.i.d. values in a uniformly random order are again i.i.d., so the distribution is
    the same).  A Bernoulli(reuse_prob) draw per step decides whether the step must keep one of the previous
    step's k highest-valued experts: if none of them is among this step's first k, the expert at place k-1 of
    the order exchanges places with a uniformly chosen one of them.  Nothing here selects experts from logits:
    the generator knows the places because it assigned them.
    """
    steps = wl.steps if steps is None else steps
    rng = np.random.default_rng(wl.seed + 7919)
    logits = rng.normal(0.0, 1.0, size=(steps, wl.experts)).astype(np.float32)
    if wl.reuse_prob > 0.0:
        k = wl.top_k
        force = rng.random(steps) < wl.reuse_prob
        pick = rng.integers(0, k, size=steps)
        values = -np.sort(-logits, axis=1)                        # descending per step
        order = np.stack([rng.permutation(wl.experts) for _ in range(steps)])
        for t in range(steps):
            if t > 0 and force[t] and not set(order[t, :k].tolist()) & set(order[t - 1, :k].tolist()):
                keep = int(order[t - 1, pick[t]])
                at = int(np.nonzero(order[t] == keep)[0][0])
                order[t, k - 1], order[t, at] = order[t, at], order[t, k - 1]
            logits[t, order[t]] = values[t]
    return logits


def sample_rows(rng: np.random.Generator, out: int, n_random=61) -> np.ndarray:
    """Rows 0, 1, out-1 plus n_random distinct random rows (sorted, unique)."""
    fixed = {0, min(1, out - 1), out - 1}
    extra = rng.choice(out, size=min(n_random, out), replace=False).tolist()
    return np.asarray(sorted(fixed | set(extra)), dtype=np.int64)
