"""Pins of the oracle's synchronous data-parallel SGD round (Section 2.3 "Data Parallelism"; the replicated
form of Section 6.2; momentum Eq. (3),(4)): a hand-worked example, closed forms, invariants and special cases
that reduce to other routines -- and a check that each pin set rejects plausible wrong rules."""
import numpy as np
import pytest

import oracle

F = np.float32


def _oracle_impl(W, V, G, eta, mu):
    oracle.sync_sgd_round(W, G, eta, V=V, mu=mu)


# ---- pins: each takes an implementation impl(W, V or None, G, eta, mu) that works in place ----

def pin_hand_example(impl, golden):
    g = golden("sync_sgd_hand_example.txt")
    W = np.array([g["W0"], g["W1"]], F); G = np.array([g["G0"], g["G1"]], F)
    impl(W, None, G, g["eta"], 0.0)
    np.testing.assert_array_equal(W, np.array([g["W0_new"], g["W1_new"]], F))
    W = np.array([g["W0"], g["W1"]], F); V = np.array([g["V0"], g["V1"]], F)
    impl(W, V, G, g["eta"], g["mu"])
    np.testing.assert_array_equal(V, np.array([g["V0_new"], g["V1_new"]], F))
    np.testing.assert_array_equal(W, np.array([g["W0_mom"], g["W1_mom"]], F))


def pin_constant_gradient_closed_form(impl, golden):
    """T rounds with the same gradients: W_T = W_0 - eta*T*sum_i g_i; with momentum the geometric series
    V_T = -eta*S*(1-mu^T)/(1-mu), W_T = W_0 - eta*S*(T - mu*(1-mu^T)/(1-mu))/(1-mu)."""
    rng = np.random.default_rng(5)
    P, N, T, eta, mu = 5, 257, 12, 0.03, 0.8
    W0 = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    S = G.astype(np.float64).sum(axis=0)
    W = W0.copy()
    for _ in range(T):
        impl(W, None, G, eta, 0.0)
    np.testing.assert_allclose(W, W0.astype(np.float64) - eta * T * S, rtol=0, atol=2e-6 * T)
    W = W0.copy(); V = np.zeros_like(W)
    for _ in range(T):
        impl(W, V, G, eta, mu)
    geo = (1 - mu ** T) / (1 - mu)
    np.testing.assert_allclose(V, np.broadcast_to(-eta * S * geo, (P, N)), rtol=0, atol=2e-6 * T)
    np.testing.assert_allclose(W, W0.astype(np.float64) - eta * S * (T - mu * geo) / (1 - mu), rtol=0, atol=4e-6 * T)


def pin_replicas_stay_identical_and_padding_untouched(impl, golden):
    rng = np.random.default_rng(6)
    P, N, ld = 4, 100, 104
    w = rng.standard_normal(N).astype(F)
    W = np.full((P, ld), np.nan, F); W[:, :N] = w
    G = np.full((P, ld), np.nan, F); G[:, :N] = rng.standard_normal((P, N)).astype(F)
    V = np.full((P, ld), np.nan, F); V[:, :N] = 0
    # the oracle wrapper takes N; other implementations see the valid part only
    if impl is _oracle_impl:
        oracle.sync_sgd_round(W, G, 0.1, V=V, mu=0.9, N=N)
    else:
        Wv, Vv, Gv = W[:, :N].copy(), V[:, :N].copy(), G[:, :N].copy()
        impl(Wv, Vv, Gv, 0.1, 0.9); W[:, :N] = Wv; V[:, :N] = Vv
    assert np.isnan(W[:, N:]).all() and np.isnan(V[:, N:]).all()
    for i in range(1, P):
        np.testing.assert_array_equal(W[i, :N], W[0, :N])      # the "broadcast of W" holds by construction
        np.testing.assert_array_equal(V[i, :N], V[0, :N])
    assert not np.array_equal(W[0, :N], w)


def pin_special_cases(impl, golden):
    rng = np.random.default_rng(7)
    N = 300
    # one worker: plain SGD, which is also the elastic worker rule with rho = 0 (a different routine)
    W = rng.standard_normal((1, N)).astype(F); G = rng.standard_normal((1, N)).astype(F)
    W_e, Wc = W.copy(), np.zeros(N, F)
    oracle.easgd_round(W_e, G, Wc, 0.0625, 0.0)
    impl(W, None, G, 0.0625, 0.0)
    np.testing.assert_array_equal(W, W_e)
    # mu = 0 with momentum buffers is the plain rule; V ends as the step itself
    P = 3
    W1 = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    W2 = W1.copy(); V = rng.standard_normal((P, N)).astype(F)
    impl(W1, None, G, 0.05, 0.0)
    impl(W2, V, G, 0.05, 0.0)
    np.testing.assert_allclose(W2, W1, rtol=0, atol=1e-6)
    np.testing.assert_allclose(V, np.broadcast_to(-0.05 * G.astype(np.float64).sum(0), (P, N)), rtol=0, atol=1e-6)
    # zero gradients: nothing moves, momentum decays
    W3 = W1.copy(); V3 = np.ones((P, N), F)
    impl(W3, V3, np.zeros((P, N), F), 0.05, 0.5)
    np.testing.assert_array_equal(V3, np.full((P, N), 0.5, F))
    np.testing.assert_allclose(W3, W1.astype(np.float64) + 0.5, rtol=0, atol=1e-6)
    # the order of the workers only changes the rounding of the sum
    W4, W5 = W1.copy(), W1.copy()[::-1].copy()
    impl(W4, None, G, 0.05, 0.0)
    impl(W5, None, G[::-1].copy(), 0.05, 0.0)
    np.testing.assert_allclose(W5[::-1], W4, rtol=0, atol=1e-6)


PINS = [pin_hand_example, pin_constant_gradient_closed_form, pin_replicas_stay_identical_and_padding_untouched,
        pin_special_cases]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_passes_every_pin(pin, golden):
    pin(_oracle_impl, golden)


# ---- plausible wrong rules: every one must be caught by at least one pin ----

def _mutant(kind):
    def impl(W, V, G, eta, mu):
        W64, G64 = W.astype(np.float64), G.astype(np.float64)
        S = G64.sum(axis=0)
        if kind == "mean_instead_of_sum":
            S = S / W.shape[0]
        if kind == "own_gradient_only":
            S = G64
        if kind == "plus_sign":
            S = -S
        if V is None:
            W[...] = (W64 - eta * S).astype(F)
            return
        V64 = V.astype(np.float64)
        if kind == "momentum_on_gradient_term":      # V <- mu*(V - eta*S)
            Vn = mu * (V64 - eta * S)
        elif kind == "old_velocity_in_weight_step":  # W <- W + V_t instead of V_{t+1}
            W[...] = (W64 + V64).astype(F)
            V[...] = (mu * V64 - eta * S).astype(F)
            return
        else:
            Vn = mu * V64 - eta * S
        V[...] = np.broadcast_to(Vn, V.shape).astype(F)
        W[...] = (W64 + V.astype(np.float64)).astype(F)
    return impl


@pytest.mark.parametrize("kind", ["mean_instead_of_sum", "own_gradient_only", "plus_sign",
                                  "momentum_on_gradient_term", "old_velocity_in_weight_step"])
def test_planted_mistakes_are_caught(kind, golden):
    caught = []
    for pin in PINS:
        try:
            pin(_mutant(kind), golden)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the mistake '{kind}'"


def test_correct_restatement_passes():
    """The mutant harness itself: the unmodified restatement must pass all pins (so a failure above is the
    planted mistake's, not the harness's)."""
    from conftest import read_golden
    for pin in PINS:
        pin(_mutant("none"), read_golden)
