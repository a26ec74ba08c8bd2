"""Exact rational arithmetic used to pin the oracle (tiny inputs only).

Everything here works on Python integers and fractions.Fraction, so there is no
floating-point rounding anywhere except the one, explicitly coded, rounding to
bf16.  It deliberately shares nothing with oracle/: different number system,
different rounding routine, plain triple loops.
"""

from fractions import Fraction


def bf16_bits_to_fraction(bits: int) -> Fraction:
    sign = -1 if bits & 0x8000 else 1
    exp = (bits >> 7) & 0xFF
    man = bits & 0x7F
    assert exp != 0xFF, "finite values only"
    if exp == 0:
        return sign * Fraction(man, 1 << 7) * Fraction(1, 1 << 126)
    val = Fraction((1 << 7) | man, 1 << 7)
    e = exp - 127
    return sign * (val * (1 << e) if e >= 0 else val / (1 << -e))


def fraction_to_bf16_bits(v: Fraction) -> int:
    """Nearest bf16, ties to the even significand; overflow gives infinity."""
    sign = 0x8000 if v < 0 else 0
    a = -v if v < 0 else v
    if a == 0:
        return sign
    # E = floor(log2(a)) by integer comparison
    E = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** E > a:
        E -= 1
    assert Fraction(2) ** E <= a < Fraction(2) ** (E + 1)
    qe = max(E, -126) - 7
    n = a / (Fraction(2) ** qe)                 # exact
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    # fl in [0, 256]; value = fl * 2^qe
    if fl == 0:
        return sign
    if E < -126:                                # subnormal range: exponent field 0 (or 1 if fl == 128)
        return sign | fl                        # fl == 128 encodes the smallest normal: 0x0080
    if fl == 256:
        fl, E = 128, E + 1
    if E > 127:
        return sign | 0x7F80
    return sign | ((E + 127) << 7) | (fl - 128)


def f32_to_fraction(x) -> Fraction:
    return Fraction(float(x))                   # float -> Fraction is exact


def exact_switch(W_bits, A, B, old, new, scale=1.0):
    """Definition of the switch, element by element, in exact arithmetic.

    W_bits: list of lists of ints; A[e][rho][j], B[e][i][rho] floats (fp32 values);
    old/new: lists of (expert, gate) pairs.
    """
    n_out, n_in = len(W_bits), len(W_bits[0])
    res = [[0] * n_in for _ in range(n_out)]
    sc = f32_to_fraction(scale)
    for i in range(n_out):
        for j in range(n_in):
            acc = bf16_bits_to_fraction(int(W_bits[i][j]))
            for sgn, pairs in ((1, new), (-1, old)):
                for e, g in pairs:
                    dot = Fraction(0)
                    for rho in range(len(A[e])):
                        dot += f32_to_fraction(B[e][i][rho]) * f32_to_fraction(A[e][rho][j])
                    acc += sgn * sc * f32_to_fraction(g) * dot
            res[i][j] = fraction_to_bf16_bits(acc)
    return res


def exact_adapter_forward(Y_bits, X_bits, A, B, ids, gates, scale=1.0):
    """Eq. 2's adapter sum added to Y, element by element, in exact arithmetic; one rounding to bf16.

    Y_bits [T][out], X_bits [T][in] ints; A[e][rho][j], B[e][i][rho] floats; ids[t][c], gates[t][c].
    """
    T, n_out, n_in = len(Y_bits), len(Y_bits[0]), len(X_bits[0])
    sc = f32_to_fraction(scale)
    res = [[0] * n_out for _ in range(T)]
    for t in range(T):
        x = [bf16_bits_to_fraction(int(X_bits[t][j])) for j in range(n_in)]
        for i in range(n_out):
            acc = bf16_bits_to_fraction(int(Y_bits[t][i]))
            for c in range(len(ids[t])):
                e = int(ids[t][c])
                up = Fraction(0)
                for rho in range(len(A[e])):
                    down = Fraction(0)
                    for j in range(n_in):
                        down += f32_to_fraction(A[e][rho][j]) * x[j]
                    up += f32_to_fraction(B[e][i][rho]) * down
                acc += sc * f32_to_fraction(gates[t][c]) * up
            res[t][i] = fraction_to_bf16_bits(acc)
    return res
