"""Comparison rules used by the parity tests (test infrastructure only).

bf16 values are compared on the integer line: a bit pattern b maps to
key = -(b & 0x7FFF) if the sign bit is set, else (b & 0x7FFF).  The map is
monotone in the value and sends +0 and -0 to the same key, so |key_a - key_b|
counts representable values between a and b.

An element of a switched weight passes when
  (1) its key distance to the oracle is at most 1, or
  (2) |gpu - oracle| <= one bf16 ulp taken at the largest magnitude that
      entered that element's sum: max(|W_prev|, |W_oracle|, S), where
      S = sum_c |g_c| sum_rho |B||A| (oracle.lsw_oracle.switch_magnitude).
Rule (2) is the backward-error reading of "within one ulp": when W_prev + delta
cancels to a result much smaller than delta, an ulp of the RESULT is smaller
than the rounding error any finite-precision accumulation of delta carries.
"""

from __future__ import annotations

import numpy as np

from .lsw_oracle import bf16_bits_to_f64


def ulp_key(bits) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16).astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag).astype(np.int32)


def ulp_distance(a_bits, b_bits) -> np.ndarray:
    return np.abs(ulp_key(a_bits) - ulp_key(b_bits))


def bf16_ulp_at(mag) -> np.ndarray:
    """Spacing of bf16 values around magnitude `mag` (>= 0), float64.

    2^(E-7) for 2^E <= mag < 2^(E+1), with E clamped to -126 (subnormals).
    """
    mag = np.asarray(mag, dtype=np.float64)
    _, e = np.frexp(mag)
    e = np.where(mag == 0, -1000, e.astype(np.int64))        # frexp(0) reports exponent 0
    return np.ldexp(1.0, np.maximum(e - 1, -126) - 7)


def switch_parity(gpu_bits, oracle_bits, w_prev_bits, S):
    """Apply the two-clause rule.  Returns a dict of counts and the fail mask."""
    gpu_bits = np.asarray(gpu_bits, dtype=np.uint16)
    oracle_bits = np.asarray(oracle_bits, dtype=np.uint16)
    dist = ulp_distance(gpu_bits, oracle_bits)
    strict = dist <= 1
    g = bf16_bits_to_f64(gpu_bits)
    o = bf16_bits_to_f64(oracle_bits)
    scale_mag = np.maximum(np.maximum(np.abs(bf16_bits_to_f64(w_prev_bits)), np.abs(o)),
                           np.asarray(S, dtype=np.float64))
    with np.errstate(invalid="ignore"):
        relaxed = np.abs(g - o) <= bf16_ulp_at(scale_mag)
    ok = strict | relaxed
    return {
        "n": int(gpu_bits.size),
        "exact": int((dist == 0).sum()),
        "within_1ulp": int(strict.sum()),
        "needed_clause2": int((~strict & relaxed).sum()),
        "fail": int((~ok).sum()),
        "max_dist": int(dist.max()) if dist.size else 0,
        "fail_mask": ~ok,
    }
