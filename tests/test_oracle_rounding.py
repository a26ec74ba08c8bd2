"""Pins for the oracle's bf16 conversion routines.

Sources of truth used here, none of which is the oracle itself:
  * the bf16 format (8 significant bits, fp32 exponent range) written as literals,
  * an exact-rational rounding routine (tests/exact_rational.py),
  * torch's fp32 -> bf16 cast (a library RNE) on inputs that are exactly fp32.
"""
from fractions import Fraction

import numpy as np
import torch

from oracle import lsw_oracle as O
from tests.exact_rational import bf16_bits_to_fraction, fraction_to_bf16_bits


def test_widening_literals():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3FFF, 0x0000, 0x8000, 0x0001, 0x0080, 0x7F7F, 0x3DCD], dtype=np.uint16)
    got = O.bf16_bits_to_f64(bits)
    want = [1.0, -1.0, 2.0, 2 - 2.0 ** -7, 0.0, -0.0, 2.0 ** -133, 2.0 ** -126,
            (2 - 2.0 ** -7) * 2.0 ** 127, (1 + 77 / 128) * 2.0 ** -4]
    assert got.tolist() == want
    assert np.signbit(got[5]) and not np.signbit(got[4])


def test_widening_all_finite_patterns_against_rational():
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    b = bits[finite].astype(np.uint16)
    got = O.bf16_bits_to_f64(b)
    for bi, gi in zip(b[::97].tolist(), got[::97].tolist()):
        assert Fraction(gi) == bf16_bits_to_fraction(bi)


def test_round_trip_every_bf16_value():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    b = bits[finite]
    assert (O.f64_to_bf16_bits(O.bf16_bits_to_f64(b)) == b).all()


def test_rounding_literals():
    cases = [
        (1.0 + 2.0 ** -8, 0x3F80),                    # tie -> even
        (1.0 + 2.0 ** -7 + 2.0 ** -8, 0x3F82),        # tie -> even
        (1.0 + 2.0 ** -8 + 2.0 ** -40, 0x3F81),       # above the tie by less than an fp32 ulp: no double rounding
        (1.0 + 2.0 ** -7 + 2.0 ** -8 - 2.0 ** -40, 0x3F81),
        (2.0 - 2.0 ** -8, 0x4000),                    # tie at the binade edge -> 2.0
        (-(1.0 + 2.0 ** -8), 0xBF80),
        (-(1.0 + 3 * 2.0 ** -8), 0xBF82),
        (2.0 ** -133, 0x0001), (2.0 ** -134, 0x0000), (3 * 2.0 ** -134, 0x0002),
        (2.0 ** -134 * (1 + 2.0 ** -30), 0x0001),
        (-2.0 ** -140, 0x8000),
        ((2 - 2.0 ** -7) * 2.0 ** 127, 0x7F7F),
        ((2 - 2.0 ** -8) * 2.0 ** 127, 0x7F80),        # tie at the top rounds to 2^128 = inf
        ((2 - 2.0 ** -8) * 2.0 ** 127 * (1 - 2.0 ** -40), 0x7F7F),
        (1e300, 0x7F80), (-1e300, 0xFF80), (float("inf"), 0x7F80), (0.0, 0x0000), (-0.0, 0x8000),
    ]
    v = np.array([c[0] for c in cases])
    got = O.f64_to_bf16_bits(v).tolist()
    assert got == [c[1] for c in cases]
    assert int(O.f64_to_bf16_bits(np.array([float("nan")]))[0]) & 0x7FFF > 0x7F80


def test_rounding_against_rational_on_random_doubles():
    rng = np.random.default_rng(5)
    v = np.concatenate([
        rng.normal(0, 0.02, 300), rng.normal(0, 1e-38, 200), rng.normal(0, 1e-40, 200),
        rng.normal(0, 1e30, 100), rng.normal(0, 3e38, 100),
        # exact ties and their neighbours
        (1 + (2 * rng.integers(0, 128, 100) + 1) * 2.0 ** -8) * 2.0 ** rng.integers(-20, 20, 100),
    ])
    v = np.concatenate([v, np.nextafter(v, np.inf), np.nextafter(v, -np.inf)])
    got = O.f64_to_bf16_bits(v)
    for x, g in zip(v.tolist(), got.tolist()):
        assert g == fraction_to_bf16_bits(Fraction(x)), x


def test_rounding_against_torch_cast_on_fp32_inputs():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.normal(0, 0.02, 200000), rng.normal(0, 1e-39, 1000),
                        rng.normal(0, 1e37, 1000)]).astype(np.float32)
    # include every tie pattern: odd 16-bit tails of exactly 0x8000
    u = rng.integers(0, 0x7F00, 50000, dtype=np.uint32) << np.uint32(16) | np.uint32(0x8000)
    x = np.concatenate([x, u.view(np.float32), -u.view(np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.f64_to_bf16_bits(x.astype(np.float64))
    assert (got == want).all()
