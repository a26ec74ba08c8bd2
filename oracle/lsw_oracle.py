"""Plain CPU oracle for the per-token LoRA expert switch (LoRA-Switch, arXiv 2405.17741).

THIS IS TEST INFRASTRUCTURE. It is slow on purpose, shares no code with the
HIP library, and must never be imported by the product package: only tests,
the smoke check and the benchmark's cpu_baseline leg call it.

What it computes
----------------
The paper's fused switch (Sec. 3.3, Eq. 8 and Eq. 10) is an algebraic
rewriting of "take the merged weight of the previous token, subtract the
previous token's gated low-rank sum (Eq. 7), add the current token's gated
low-rank sum (Eq. 4)".  It is exact, not an approximation, so the oracle is
that definition written out element by element:

    W_t[i,j] = RNE_bf16( W_{t-1}[i,j]
                         + sum_{c in new} (scale*g_c) * sum_rho B[e_c][i,rho]*A[e_c][rho,j]
                         - sum_{c in old} (scale*g_c) * sum_rho B[e_c][i,rho]*A[e_c][rho,j] )

All arithmetic is float64 on exactly widened inputs and there is one
round-to-nearest-even to bfloat16 per element per switch (the paper states no
precision; storage types follow the workload definition: W bf16, factors and
gates fp32).  Layout reading: weights are [out, in] row-major, the update of
one expert is B @ A with B = LoRA_UP [out, r] and A = LoRA_DOWN [r, in].  The
sign of the "previous" half follows Eq. 8 (minus); Eq. 9 as printed carries
the minus on both factors, which would cancel, so only one factor is negated.

The router (definition of G under Eq. 1, reused by Eq. 2 for the single
token-wise router) is Softmax(TopK(logits)): pick the k largest logits, then
softmax over those k only, so the gates sum to one.

Parity pins for every function here live in tests/test_oracle_*.py (exact
rational brute force, hand-derived rounding cases, closed forms, invariants).
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "f64_to_bf16_bits",
    "route",
    "gated_lowrank_sum",
    "switch_step",
    "switch_magnitude",
    "gemv",
    "adapter_term",
    "adapter_forward",
    "adapter_magnitude",
]


# --------------------------------------------------------------------------
# bfloat16 <-> float64 (bf16 is carried as its 16-bit pattern in a uint16)
# --------------------------------------------------------------------------

def bf16_bits_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns to float64 exactly (bf16 = top half of an fp32)."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(v) -> np.ndarray:
    """Round float64 to the nearest bf16 (ties to even) in ONE step.

    No stop-over in fp32, so there is no double rounding.  bf16 has 8
    significant bits and the fp32 exponent range: a value whose leading bit
    is 2^E is rounded to a multiple of 2^(max(E,-126)-7) (the max() makes the
    subnormal range use the fixed quantum 2^-133).  Dividing by a power of
    two is exact, rint() rounds half to even, multiplying back is exact.
    Results at or beyond 2^128 become infinity; NaN stays NaN.
    """
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    with np.errstate(invalid="ignore", over="ignore"):
        _, e = np.frexp(a)                       # a = m * 2^e, m in [0.5, 1)  ->  leading bit 2^(e-1)
        qexp = np.maximum(e.astype(np.int64) - 1, -126) - 7
        q = np.ldexp(1.0, qexp)
        r = np.rint(a / q) * q                   # exactly a bf16 value, or 2^128
        r = np.where(np.isfinite(a), r, a)       # inf/nan pass through
        r32 = r.astype(np.float32)               # exact; 2^128 overflows to +inf as bf16 does
    bits = (r32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    bits = np.where(np.isnan(a), np.uint16(0x7FC0), bits).astype(np.uint16)
    sign = np.signbit(v).astype(np.uint16) << np.uint16(15)
    return (bits | sign).astype(np.uint16)


# --------------------------------------------------------------------------
# Router: G = Softmax(TopK(logits))           (definition of G under Eq. 1)
# --------------------------------------------------------------------------

def route(logits, k: int):
    """Top-k selection followed by a softmax over the selected logits only.

    Returns (ids int32[k], gates float32[k]) listed by descending logit.
    Equal logits: the lower index wins (+0 and -0 are equal).  The softmax is
    evaluated in float64 with the maximum subtracted and rounded once to fp32.
    NaN logits are rejected.
    """
    l = np.asarray(logits, dtype=np.float32).reshape(-1)
    n = l.shape[0]
    if not (0 <= k <= n):
        raise ValueError("k out of range")
    if np.isnan(l).any():
        raise ValueError("NaN logit")
    order = sorted(range(n), key=lambda i: (-float(l[i]), i))
    ids = np.asarray(order[:k], dtype=np.int32)
    if k == 0:
        return ids, np.zeros(0, dtype=np.float32)
    z = l[ids].astype(np.float64)
    z = z - z.max()
    w = np.exp(z)
    gates = (w / w.sum()).astype(np.float32)
    return ids, gates


# --------------------------------------------------------------------------
# Merge / unmerge / fused switch              (Eq. 4, Eq. 7, Eq. 8 == Eq. 10)
# --------------------------------------------------------------------------

def _rows(M, rows):
    return M if rows is None else M[rows]


def gated_lowrank_sum(A, B, ids, gates, scale=1.0, rows=None) -> np.ndarray:
    """sum_c (scale*g_c) * B[e_c] @ A[e_c] in float64      (Eq. 4, the sum only).

    A: fp32 [E, r, in] (LoRA_DOWN), B: fp32 [E, out, r] (LoRA_UP).  Only the
    listed experts contribute (the other gates are zero).  `rows` restricts
    the result to some output rows; every element is independent of the
    others so this is the same definition evaluated on fewer elements.
    """
    A = np.asarray(A)
    B = np.asarray(B)
    n_out = B.shape[1] if rows is None else len(rows)
    d = np.zeros((n_out, A.shape[2]), dtype=np.float64)
    for e, g in zip(np.asarray(ids).tolist(), np.asarray(gates).tolist()):
        coeff = np.float64(scale) * np.float64(np.float32(g))
        d += coeff * (_rows(B[e], rows).astype(np.float64) @ A[e].astype(np.float64))
    return d


def switch_step(W_bits, A, B, old_ids, old_gates, new_ids, new_gates,
                scale=1.0, rows=None) -> np.ndarray:
    """One in-place switch of one adapted linear          (Eq. 8, equal to Eq. 10).

    W_bits: uint16 [out, in] (or the selected `rows` of it) holding the bf16
    weight with the OLD set merged.  Returns the bf16 bits with the old set
    removed (Eq. 7) and the new set merged (Eq. 4), rounded once.
    Empty `old` is a pure merge, empty `new` restores the base weight.
    """
    w = bf16_bits_to_f64(W_bits)
    d = gated_lowrank_sum(A, B, new_ids, new_gates, scale, rows) \
        - gated_lowrank_sum(A, B, old_ids, old_gates, scale, rows)
    return f64_to_bf16_bits(w + d)


def switch_magnitude(A, B, old_ids, old_gates, new_ids, new_gates,
                     scale=1.0, rows=None) -> np.ndarray:
    """S[i,j] = sum over old and new of |scale*g_c| * sum_rho |B||A|  (float64).

    The size of the largest partial sums entering an element; used by the
    comparison rule for elements whose result cancels towards zero.
    """
    ids = list(np.asarray(old_ids).tolist()) + list(np.asarray(new_ids).tolist())
    gs = [abs(float(g)) for g in np.asarray(old_gates).tolist()] + \
         [abs(float(g)) for g in np.asarray(new_gates).tolist()]
    return gated_lowrank_sum(np.abs(np.asarray(A)), np.abs(np.asarray(B)), ids, gs,
                             abs(float(scale)), rows)


# --------------------------------------------------------------------------
# Decode through a merged weight              (Eq. 3: y = f*(x))
# --------------------------------------------------------------------------

def gemv(W_bits, x_bits) -> np.ndarray:
    """y[i] = sum_j W[i,j] * x[j] in float64, W and x given as bf16 bit patterns."""
    return bf16_bits_to_f64(W_bits) @ bf16_bits_to_f64(x_bits)


# --------------------------------------------------------------------------
# Un-merged adapter path for many tokens      (Eq. 2: y = f(x) + sum_i G(x1)_i E_i(x))
# --------------------------------------------------------------------------

def adapter_term(X_bits, A, B, ids, gates, scale=1.0) -> np.ndarray:
    """The dynamic-adapter sum of Eq. 2 for T tokens, float64 [T, out].

    term[t, i] = sum_c (scale*g[t,c]) * sum_rho B[e][i,rho] * (sum_j A[e][rho,j] * x[t,j]),  e = ids[t,c].
    X_bits: bf16 bit patterns [T, in]; ids int [T, k]; gates fp32 [T, k] (each token carries the gates its
    own router output gave it; with the token-wise pre-gated structure they are the same in every layer).
    E_i(x) = W_up (W_down x) as under Eq. 1: the down projection first, then the up projection.
    """
    X = bf16_bits_to_f64(X_bits)
    A = np.asarray(A)
    B = np.asarray(B)
    ids = np.asarray(ids).reshape(X.shape[0], -1)
    gates = np.asarray(gates, dtype=np.float32).reshape(X.shape[0], -1)
    out = np.zeros((X.shape[0], B.shape[1]), dtype=np.float64)
    for t in range(X.shape[0]):
        for c in range(ids.shape[1]):
            e = int(ids[t, c])
            coeff = np.float64(scale) * np.float64(gates[t, c])
            down = A[e].astype(np.float64) @ X[t]                 # [r]
            out[t] += coeff * (B[e].astype(np.float64) @ down)    # [out]
    return out


def adapter_forward(Y_bits, X_bits, A, B, ids, gates, scale=1.0) -> np.ndarray:
    """Y <- RNE_bf16(Y + adapter_term): the term added to the backbone's bf16 output f(x), one rounding."""
    return f64_to_bf16_bits(bf16_bits_to_f64(Y_bits) + adapter_term(X_bits, A, B, ids, gates, scale))


def adapter_magnitude(X_bits, A, B, ids, gates, scale=1.0) -> np.ndarray:
    """S[t,i] = sum_c |scale*g| sum_rho |B| sum_j |A||x|: the size of the partial sums entering an output."""
    Xa = f64_to_bf16_bits(np.abs(bf16_bits_to_f64(X_bits)))       # |x| is again a bf16 value
    return adapter_term(Xa, np.abs(np.asarray(A)), np.abs(np.asarray(B)), ids,
                        np.abs(np.asarray(gates, dtype=np.float32)), abs(float(scale)))
