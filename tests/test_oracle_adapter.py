"""Pins for oracle.adapter_term / adapter_forward / adapter_magnitude (the un-merged adapter path of Eq. 2).

The paper prints no numbers for it, so the oracle is pinned to exact rational brute force on tiny inputs, to the
textbook LoRA forward x -> B (A x) as the k = 1, g = 1 special case, to the identity Eq. 2 == Eq. 3 (adapter path ==
decode through exactly merged weights, using the separately pinned gated_lowrank_sum), and to the invariants the
definition implies.  Planted mistakes fail at least one of them.
"""
import numpy as np
import pytest

from oracle import lsw_oracle as O
from paper_2405_17741_amd import inputs as I
from tests.exact_rational import exact_adapter_forward


def _case(seed, T=3, inn=5, out=4, E=3, r=2, k=2):
    rng = np.random.default_rng(seed)
    _, A, B = I.host_linear(rng, out, inn, E, r, 0.02, 0.3, 0.05)
    X = I.f32_to_bf16_bits(rng.normal(0, 1, (T, inn)).astype(np.float32))
    Y = I.f32_to_bf16_bits(rng.normal(0, 0.05, (T, out)).astype(np.float32))
    ids = np.stack([rng.choice(E, k, replace=False) for _ in range(T)]).astype(np.int32)
    g = rng.random((T, k)).astype(np.float32)
    gates = (g / g.sum(1, keepdims=True)).astype(np.float32)
    return Y, X, A, B, ids, gates


@pytest.mark.parametrize("seed", range(5))
def test_exact_rational_bruteforce(seed):
    Y, X, A, B, ids, gates = _case(seed)
    want = exact_adapter_forward(Y.tolist(), X.tolist(), A.tolist(), B.tolist(), ids.tolist(), gates.tolist(), 0.75)
    got = O.adapter_forward(Y, X, A, B, ids, gates, 0.75)
    assert got.tolist() == want


def test_single_expert_unit_gate_is_the_textbook_lora_forward():
    Y, X, A, B, _, _ = _case(11, T=6, inn=16, out=8, E=4, r=4)
    ids = np.full((6, 1), 2, np.int32)
    gates = np.ones((6, 1), np.float32)
    Xf = O.bf16_bits_to_f64(X)
    want = (Xf @ A[2].astype(np.float64).T) @ B[2].astype(np.float64).T
    assert np.allclose(O.adapter_term(X, A, B, ids, gates), want, rtol=1e-13, atol=1e-18)


def test_adapter_path_equals_decode_through_exactly_merged_weights():
    # Eq. 2 == Eq. 3 in exact arithmetic: f(x) + sum_c g_c B_c (A_c x) = (W0 + sum_c g_c B_c A_c) x
    rng = np.random.default_rng(12)
    W0, A, B = I.host_linear(rng, 24, 40, 6, 4, 0.02, 0.2, 0.05)
    X = I.f32_to_bf16_bits(rng.normal(0, 1, (5, 40)).astype(np.float32))
    routes = [O.route(rng.normal(0, 1, 6).astype(np.float32), 2) for _ in range(5)]
    ids = np.stack([r[0] for r in routes])
    gates = np.stack([r[1] for r in routes])
    term = O.adapter_term(X, A, B, ids, gates, 2.0)
    Xf, W0f = O.bf16_bits_to_f64(X), O.bf16_bits_to_f64(W0)
    for t in range(5):
        merged = W0f + O.gated_lowrank_sum(A, B, ids[t], gates[t], 2.0)
        assert np.allclose(W0f @ Xf[t] + term[t], merged @ Xf[t], rtol=1e-12, atol=1e-15)


def test_invariants():
    Y, X, A, B, ids, gates = _case(13, T=7, inn=24, out=16, E=5, r=3)
    base = O.adapter_term(X, A, B, ids, gates, 1.5)
    # tokens are independent: any sub-batch gives the same rows
    sel = [4, 0, 6]
    assert (O.adapter_term(X[sel], A, B, ids[sel], gates[sel], 1.5) == base[sel]).all()
    # order of the (id, gate) pairs of a token does not matter (up to fp64 summation order)
    assert np.allclose(O.adapter_term(X, A, B, ids[:, ::-1], gates[:, ::-1], 1.5), base, rtol=1e-13, atol=1e-18)
    # linear in the gates and in scale; zero gates give zero; k = 0 gives zero
    assert np.allclose(O.adapter_term(X, A, B, ids, 2 * gates, 1.5), 2 * base, rtol=1e-13)
    assert np.allclose(O.adapter_term(X, A, B, ids, gates, 3.0), 2 * base, rtol=1e-13)
    assert (O.adapter_term(X, A, B, ids, 0 * gates) == 0).all()
    assert (O.adapter_term(X, A, B, np.zeros((7, 0), np.int32), np.zeros((7, 0), np.float32)) == 0).all()
    assert (O.adapter_forward(Y, X, A, B, ids, 0 * gates) == Y).all()
    # the magnitude bounds the term
    S = O.adapter_magnitude(X, A, B, ids, gates, 1.5)
    assert (np.abs(base) <= S * (1 + 1e-12)).all() and (S > 0).all()


def test_planted_mistakes_are_caught():
    Y, X, A, B, ids, gates = _case(14, T=4, inn=6, out=5, E=4, r=2)
    want = exact_adapter_forward(Y.tolist(), X.tolist(), A.tolist(), B.tolist(), ids.tolist(), gates.tolist(), 0.5)
    mistakes = {
        "gates of another token": lambda: O.adapter_forward(Y, X, A, B, ids, np.roll(gates, 1, axis=0), 0.5),
        "experts of another token": lambda: O.adapter_forward(Y, X, A, B, np.roll(ids, 1, axis=0), gates, 0.5),
        "scale dropped": lambda: O.adapter_forward(Y, X, A, B, ids, gates, 1.0),
        "one slot dropped": lambda: O.adapter_forward(Y, X, A, B, ids[:, :1], gates[:, :1], 0.5),
        "sign": lambda: O.adapter_forward(Y, X, A, B, ids, -gates, 0.5),
        "up and down of different experts": lambda: O.adapter_forward(Y, X, A, np.roll(B, 1, axis=0), ids, gates, 0.5),
        "truncation": lambda: (O.f64_to_bf16_bits(O.bf16_bits_to_f64(Y) + O.adapter_term(X, A, B, ids, gates, 0.5)) & 0xFFFE),
    }
    assert O.adapter_forward(Y, X, A, B, ids, gates, 0.5).tolist() == want
    for name, f in mistakes.items():
        assert np.asarray(f()).tolist() != want, name


def test_adapter_magnitude_bruteforce_and_closed_form():
    # S pinned from BOTH sides: a quadruple loop over the definition sum_c |s g| sum_rho |B| sum_j |A||x| on a tiny case
    # (mixed signs everywhere, negative scale), and a closed form where every factor has magnitude one.
    Y, X, A, B, ids, gates = _case(15, T=3, inn=5, out=4, E=3, r=2)
    gates = gates * np.array([[1.0, -1.0]], np.float32)          # a negative gate: only its magnitude may enter
    S = O.adapter_magnitude(X, A, B, ids, gates, -1.5)
    Xf = O.bf16_bits_to_f64(X)
    for t in range(3):
        for i in range(4):
            s = 0.0
            for c in range(2):
                e = int(ids[t, c])
                up = 0.0
                for rho in range(2):
                    down = sum(abs(float(A[e, rho, j])) * abs(float(Xf[t, j])) for j in range(5))
                    up += abs(float(B[e, i, rho])) * down
                s += 1.5 * abs(float(gates[t, c])) * up
            assert S[t, i] == pytest.approx(s, rel=1e-14)
    # all |values| one: S = |scale| * (sum_c |g_c|) * r * in, whatever the signs
    T, inn, out, E, r, k = 2, 6, 3, 4, 3, 2
    rng = np.random.default_rng(16)
    sgn = lambda shape: rng.choice([-1.0, 1.0], size=shape).astype(np.float32)
    X1 = I.f32_to_bf16_bits(sgn((T, inn)))
    ids1 = np.array([[0, 3], [2, 1]], np.int32)
    g1 = np.array([[0.25, -0.5], [1.0, 0.125]], np.float32)
    S1 = O.adapter_magnitude(X1, sgn((E, r, inn)), sgn((E, out, r)), ids1, g1, -2.0)
    assert (S1 == 2.0 * np.abs(g1).sum(1, keepdims=True) * r * inn).all()


def test_a_wrong_magnitude_fails_its_pins():
    # planted mistakes in a copy of the definition: each one leaves the brute-force value
    Y, X, A, B, ids, gates = _case(17, T=3, inn=5, out=4, E=3, r=2)
    S = O.adapter_magnitude(X, A, B, ids, gates, 1.5)
    Xa = np.abs(O.bf16_bits_to_f64(X))
    def variant(factor=1.0, abs_x=True, abs_a=True, slots=2):
        out = np.zeros_like(S)
        for t in range(3):
            for c in range(slots):
                e = int(ids[t, c])
                Ae = np.abs(A[e]).astype(np.float64) if abs_a else A[e].astype(np.float64)
                x = Xa[t] if abs_x else O.bf16_bits_to_f64(X)[t]
                out[t] += factor * 1.5 * abs(float(gates[t, c])) * (np.abs(B[e]).astype(np.float64) @ (Ae @ x))
        return out
    assert np.allclose(variant(), S, rtol=1e-14, atol=0)
    for kw in ({"factor": 2.0}, {"factor": 0.5}, {"abs_x": False}, {"abs_a": False}, {"slots": 1}):
        assert not np.allclose(variant(**kw), S, rtol=1e-9, atol=0), kw
