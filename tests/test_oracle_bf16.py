"""The bfloat16-storage oracle (an extension: the paper's Section 3.2 only names low precision as future
work) against what fixes it: hand-rounded values, an independent narrowing routine, exact cases that
must coincide with the fp32-storage oracle, the rounding error bound, and planted mistakes."""
import numpy as np
import pytest
import torch

import oracle
from oracle import elastic_bf16 as ob
from conftest import read_golden

F = np.float32


def as16(x):
    """fp32 values that are exactly representable -> their bfloat16 patterns (no rounding happens)."""
    x = np.asarray(x, dtype=F)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "test input is not representable in bfloat16"
    return (u >> 16).astype(np.uint16)


# ---- narrowing ------------------------------------------------------------------------------------

def test_narrowing_matches_hand_rounded_values():
    g = read_golden("bf16_rounding_hand_values.txt")
    x = np.array(g["x"], dtype=np.float64).astype(F)
    want = np.array(g["rounded"], dtype=np.float64).astype(F)
    got = ob.bf16_widen(ob.bf16_round(x))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_narrowing_matches_an_independent_routine():
    """torch's CPU conversion to bfloat16 is written by other people: same bits on random values of
    every magnitude, on every tie of a binade, on subnormals and on infinities."""
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2**32, size=400_000, dtype=np.uint64).astype(np.uint32)
    bits = bits[(bits & 0x7FFFFFFF) <= 0x7F800000]                      # NaNs apart
    ties = (np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16) | 0x8000  # every tie in [1, 2)
    sub = rng.integers(0, 0x00800000, size=5000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0x7F800000, 0xFF800000, 0x7F7FFFFF, 0x7F7F8000, 0x7F7F7FFF, 0, 0x80000000], dtype=np.uint32)
    x = np.concatenate([bits, ties, ties | 0x80000000, sub, special]).view(F)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ob.bf16_round(x), want)


def test_narrowing_of_nan_is_a_quiet_nan_with_the_sign_kept():
    x = np.array([0x7FC00001, 0xFF800001, 0x7F800001], dtype=np.uint32).view(F)
    assert list(ob.bf16_round(x)) == [0x7FC0, 0xFFC0, 0x7FC0]


def test_widening_is_exact_and_narrowing_undoes_it():
    every = np.arange(0, 2**16, dtype=np.uint32).astype(np.uint16)
    every = every[(every & 0x7FFF) <= 0x7F80]                           # all finite patterns and infinities
    assert np.array_equal(ob.bf16_round(ob.bf16_widen(every)), every)


def test_rounding_error_is_at_most_half_a_spacing():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(100_000) * 10.0 ** rng.uniform(-6, 6, 100_000)).astype(F)
    r = ob.bf16_widen(ob.bf16_round(x)).astype(np.float64)
    assert np.all(np.abs(r - x) <= 2.0 ** -8 * np.abs(x.astype(np.float64)))


# ---- the round ------------------------------------------------------------------------------------

class Bf16Oracle:
    @staticmethod
    def measgd(W, V16, G16, Wc, eta, rho, mu):
        ob.measgd_round_bf16(W, V16, G16, Wc, eta, rho, mu)


def pin_hand_example(impl):
    g = read_golden("measgd_bf16_hand_example.txt")
    W = np.array(g["W"], dtype=F).reshape(1, 2); Wc = np.array(g["Wc"], dtype=F)
    V16 = as16(g["V"]).reshape(1, 2); G16 = as16(g["G"]).reshape(1, 2)
    impl.measgd(W, V16, G16, Wc, g["eta"], g["rho"], g["mu"])
    assert np.array_equal(ob.bf16_widen(V16).ravel(), np.array(g["V_next"], dtype=F))
    assert np.array_equal(W.ravel(), np.array(g["W_next"], dtype=F))
    assert np.array_equal(Wc, np.array(g["Wc_next"], dtype=F))


def pin_exact_case_equals_fp32_storage(impl):
    """Small dyadic inputs for which no operation rounds, in fp32 or in bfloat16: the round must give
    exactly what the fp32-storage oracle gives."""
    rng = np.random.default_rng(11)
    P, N = 5, 257
    W = (rng.integers(-16, 17, (P, N)) / 8.0).astype(F)
    Wc = (rng.integers(-16, 17, N) / 8.0).astype(F)
    V = (rng.integers(-8, 9, (P, N)) / 4.0).astype(F)
    G = (rng.integers(-8, 9, (P, N)) / 4.0).astype(F)
    eta, rho, mu = 0.5, 0.25, 0.5
    W2, V2, Wc2 = W.copy(), V.copy(), Wc.copy()
    oracle.measgd_round(W2, V2, G, Wc2, eta, rho, mu)
    assert np.all((V2.view(np.uint32) & 0xFFFF) == 0)                    # the result needs no rounding either
    V16, G16 = as16(V), as16(G)
    impl.measgd(W, V16, G16, Wc, eta, rho, mu)
    assert np.array_equal(ob.bf16_widen(V16), V2)
    assert np.array_equal(W, W2)
    assert np.array_equal(Wc, Wc2)


def pin_error_bound_against_fp32_storage(impl):
    """Random inputs: V differs from the fp32-storage oracle's by at most half a bfloat16 spacing, and W by
    the same amount as V, element by element, because Eq. (6) adds the stored V."""
    rng = np.random.default_rng(5)
    P, N = 6, 4099
    W = rng.standard_normal((P, N)).astype(F)
    Wc = rng.standard_normal(N).astype(F)
    V16 = ob.bf16_round((0.05 * rng.standard_normal((P, N))).astype(F))
    G16 = ob.bf16_round(rng.standard_normal((P, N)).astype(F))
    eta, rho, mu = 0.05, 0.3, 0.9
    W2, Wc2, V16_in = W.copy(), Wc.copy(), V16.copy()
    V2, G2 = ob.bf16_widen(V16).copy(), ob.bf16_widen(G16).copy()
    oracle.measgd_round(W2, V2, G2, Wc2, eta, rho, mu)
    impl.measgd(W, V16, G16, Wc, eta, rho, mu)
    v = ob.bf16_widen(V16).astype(np.float64)
    dv = v - V2
    # half a bfloat16 spacing, plus the fp32 roundings of the two products of Eq. (5) (they matter where the
    # products cancel)
    slop = 2.0 ** -22 * (np.abs(mu * ob.bf16_widen(V16_in)) + np.abs(eta * ob.bf16_widen(G16)))
    assert np.all(np.abs(dv) <= 2.0 ** -8 * np.abs(V2) * (1 + 1e-6) + slop)
    assert np.abs(dv).max() > 2.0 ** -12 * np.abs(V2).max()              # and rounding did happen
    np.testing.assert_allclose(W.astype(np.float64) - W2, dv, atol=3e-7)  # W carries exactly V's rounding
    np.testing.assert_allclose(Wc, Wc2, rtol=0, atol=0)                  # the center never sees V or G


def pin_mu_zero(impl):
    """mu = 0, eta a power of two: V' = -eta*g exactly, whatever V was."""
    rng = np.random.default_rng(2)
    P, N = 3, 130
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    V16 = ob.bf16_round(rng.standard_normal((P, N)).astype(F))
    G16 = ob.bf16_round(rng.standard_normal((P, N)).astype(F))
    g = ob.bf16_widen(G16)
    W0, c0 = W.astype(np.float64), Wc.astype(np.float64)
    impl.measgd(W, V16, G16, Wc, 0.25, 0.5, 0.0)
    assert np.array_equal(ob.bf16_widen(V16), F(-0.25) * g)
    want = W0 - 0.25 * g - 0.125 * (W0 - c0[None])
    np.testing.assert_allclose(W, want, rtol=2e-7, atol=1e-7)


PINS = [pin_hand_example, pin_exact_case_equals_fp32_storage, pin_error_bound_against_fp32_storage, pin_mu_zero]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(Bf16Oracle)


def test_plain_rule_with_bf16_gradients_is_the_fp32_rule_on_the_widened_gradients():
    rng = np.random.default_rng(4)
    P, N, ld = 4, 1001, 1004
    W = rng.standard_normal((P, ld)).astype(F); Wc = rng.standard_normal(N).astype(F)
    G16 = ob.bf16_round(rng.standard_normal((P, ld)).astype(F))
    W0, c0 = W[:, :N].astype(np.float64), Wc.astype(np.float64)
    pad = W[:, N:].copy()
    ob.easgd_round_bf16(W, G16, Wc, 0.05, 0.3)
    g = ob.bf16_widen(G16)[:, :N].astype(np.float64)
    d = W0 - c0[None]
    np.testing.assert_allclose(W[:, :N], W0 - 0.05 * (g + 0.3 * d), rtol=3e-7, atol=1e-7)
    np.testing.assert_allclose(Wc, c0 + 0.05 * 0.3 * d.sum(0), rtol=3e-7, atol=1e-7)
    assert np.array_equal(W[:, N:], pad)


# ---- planted mistakes: each variant must fail at least one pin ---------------------------------------

class Variant:
    def __init__(self, name):
        self.name = name

    def measgd(self, W, V16, G16, Wc, eta, rho, mu):
        m = self.name
        w, c = W.astype(np.float64), Wc.astype(np.float64)
        v, g = ob.bf16_widen(V16), ob.bf16_widen(G16)
        d = w - c[None]
        cand = F(mu) * v - F(eta) * g
        u = cand.view(np.uint32)
        if m == "truncate":                         # drops the low half instead of rounding
            v16 = (u >> 16).astype(np.uint16)
        elif m == "ties_away":                      # adds half a spacing and truncates
            v16 = ((u + np.uint32(0x8000)) >> 16).astype(np.uint16)
        else:
            v16 = ob.bf16_round(cand)
        v_new = ob.bf16_widen(v16).astype(np.float64)
        if m == "unrounded_v_in_w":                 # Eq. (6) with V' before it was narrowed
            v_for_w = cand.astype(np.float64)
        elif m == "old_v_in_w":
            v_for_w = v.astype(np.float64)
        else:
            v_for_w = v_new
        if m == "gradient_sign":
            v16 = ob.bf16_round(F(mu) * v + F(eta) * g)
            v_for_w = ob.bf16_widen(v16).astype(np.float64)
        V16[...] = v16
        W[...] = (w + v_for_w - eta * rho * d).astype(F)
        Wc[...] = (c + eta * rho * d.sum(0)).astype(F)


def test_correct_restatement_passes_every_pin():
    for pin in PINS:
        pin(Variant("correct"))


@pytest.mark.parametrize("name", ["truncate", "ties_away", "unrounded_v_in_w", "old_v_in_w", "gradient_sign"])
def test_planted_mistake_is_caught(name):
    failed = []
    for pin in PINS:
        try:
            pin(Variant(name))
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"no pin notices the mistake '{name}'"


def test_fp32_gradients_with_bf16_momentum():
    """Only V stored in 16 bits: representable fp32 gradients give what their 16-bit patterns give; for other
    gradients V stays within half a spacing of the fp32-storage oracle's and W carries exactly that rounding."""
    rng = np.random.default_rng(9)
    P, N = 4, 1031
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    V16 = ob.bf16_round((0.05 * rng.standard_normal((P, N))).astype(F))
    G16 = ob.bf16_round(rng.standard_normal((P, N)).astype(F))
    eta, rho, mu = 0.05, 0.3, 0.9
    a = (W.copy(), V16.copy(), Wc.copy()); b = (W.copy(), V16.copy(), Wc.copy())
    ob.measgd_round_bf16(a[0], a[1], G16, a[2], eta, rho, mu)
    ob.measgd_round_bf16(b[0], b[1], ob.bf16_widen(G16).copy(), b[2], eta, rho, mu)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    G = rng.standard_normal((P, N)).astype(F)                      # not representable in 16 bits
    W2, Wc2, V2 = W.copy(), Wc.copy(), ob.bf16_widen(V16).copy()
    oracle.measgd_round(W2, V2, G, Wc2, eta, rho, mu)
    W1, V1, Wc1 = W.copy(), V16.copy(), Wc.copy()
    ob.measgd_round_bf16(W1, V1, G, Wc1, eta, rho, mu)
    dv = ob.bf16_widen(V1).astype(np.float64) - V2
    slop = 2.0 ** -22 * (np.abs(mu * ob.bf16_widen(V16)) + np.abs(eta * G))
    assert np.all(np.abs(dv) <= 2.0 ** -8 * np.abs(V2) * (1 + 1e-6) + slop)
    np.testing.assert_allclose(W1.astype(np.float64) - W2, dv, atol=3e-7)
    assert np.array_equal(Wc1, Wc2)
