"""Pins of the oracle's one-worker-at-a-time exchange (Algorithm 1 "Original EASGD" in rank order; Section 5.1
"Async EASGD" / "Async MEASGD" in arrival order): a hand-worked example, special cases that reduce to the
separately pinned synchronous round, invariants, a closed form, a scalar brute force -- and a check that each
plausible wrong rule is rejected by at least one pin."""
import numpy as np
import pytest

import oracle

F = np.float32


def _oracle_impl(W, V, G, Wc, order, eta, rho, mu):
    oracle.async_easgd(W, G, Wc, order, eta, rho, V=V, mu=mu)


# ---- pins: each takes impl(W, V or None, G, Wc, order, eta, rho, mu), in place on W, V, Wc (all without padding) ----

def pin_hand_example(impl, golden):
    g = golden("async_easgd_hand_example.txt")
    col = lambda v: np.array(v, F).reshape(2, 1)
    for key, order in (("order01", [0, 1]), ("order10", [1, 0])):
        W, Wc = col(g["W"]), np.array([g["Wc"]], F)
        impl(W, None, col(g["G"]), Wc, order, g["eta"], g["rho"], 0.0)
        np.testing.assert_array_equal(W, col(g["W_" + key]))
        np.testing.assert_array_equal(Wc, np.array([g["Wc_" + key]], F))
    W, V, Wc = col(g["W"]), col(g["V"]), np.array([g["Wc"]], F)
    impl(W, V, col(g["G"]), Wc, [0, 1], g["eta"], g["rho"], g["mu"])
    np.testing.assert_array_equal(V, col(g["V_mom01"]))
    np.testing.assert_array_equal(W, col(g["W_mom01"]))
    np.testing.assert_array_equal(Wc, np.array([g["Wc_mom01"]], F))


def pin_turns_are_one_worker_synchronous_rounds(impl, golden):
    """A turn of worker j is the synchronous round Eq. (1),(2) of a system whose only worker is j; a schedule is
    that, turn after turn.  The synchronous oracle has pins of its own, so this ties every turn to them."""
    rng = np.random.default_rng(11)
    P, N = 5, 203
    W0 = rng.standard_normal((P, N)).astype(F); G = (rng.standard_normal((P, N)) * 0.1).astype(F)
    V0 = (rng.standard_normal((P, N)) * 0.01).astype(F); Wc0 = rng.standard_normal(N).astype(F)
    order = [3, 0, 4, 1, 2, 0, 3]
    for mom in (False, True):
        W, V, Wc = W0.copy(), V0.copy(), Wc0.copy()
        impl(W, V if mom else None, G, Wc, order, 0.05, 0.3, 0.9)
        Wr, Vr, Wcr = W0.copy(), V0.copy(), Wc0.copy()
        for j in order:
            wj, vj = Wr[j:j + 1].copy(), Vr[j:j + 1].copy()
            if mom:
                oracle.measgd_round(wj, vj, G[j:j + 1].copy(), Wcr, 0.05, 0.3, 0.9)
            else:
                oracle.easgd_round(wj, G[j:j + 1].copy(), Wcr, 0.05, 0.3)
            Wr[j], Vr[j] = wj[0], vj[0]
        np.testing.assert_array_equal(W, Wr)
        np.testing.assert_array_equal(Wc, Wcr)
        if mom:
            np.testing.assert_array_equal(V, Vr)


def pin_workers_not_served_are_untouched(impl, golden):
    rng = np.random.default_rng(12)
    P, N = 4, 64
    W0 = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    V0 = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    W, V = W0.copy(), V0.copy()
    impl(W, V, G, Wc, [2], 0.1, 0.2, 0.5)
    for i in (0, 1, 3):
        np.testing.assert_array_equal(W[i], W0[i])
        np.testing.assert_array_equal(V[i], V0[i])
    assert not np.array_equal(W[2], W0[2]) and not np.array_equal(V[2], V0[2])
    W, Wc2 = W0.copy(), Wc.copy()
    impl(W, None, G, Wc2, [], 0.1, 0.2, 0.0)                     # an empty schedule does nothing
    np.testing.assert_array_equal(W, W0)
    np.testing.assert_array_equal(Wc2, Wc)


def pin_zero_gradient_invariants_and_closed_form(impl, golden):
    """Zero gradients: every turn moves worker and center toward each other by the same amount, so the sum of all
    replicas and the center is conserved, and k turns of the same worker shrink its distance to the center by
    (1 - 2*eta*rho)^k."""
    rng = np.random.default_rng(13)
    P, N, eta, rho = 3, 101, 0.25, 0.5                            # alpha = 0.125
    W0 = rng.standard_normal((P, N)).astype(F); Wc0 = rng.standard_normal(N).astype(F)
    Z = np.zeros((P, N), F)
    W, Wc = W0.copy(), Wc0.copy()
    total = W0.astype(np.float64).sum(0) + Wc0
    for j in (1, 2, 0, 2):
        impl(W, None, Z, Wc, [j], eta, rho, 0.0)
        np.testing.assert_allclose(W.astype(np.float64).sum(0) + Wc, total, rtol=0, atol=2e-6)
    k = 6
    W, Wc = W0.copy(), Wc0.copy()
    impl(W, None, Z, Wc, [1] * k, eta, rho, 0.0)
    d0 = W0[1].astype(np.float64) - Wc0
    np.testing.assert_allclose(W[1].astype(np.float64) - Wc, (1 - 2 * eta * rho) ** k * d0, rtol=0, atol=2e-6)
    # the pair's mean stays where it was
    np.testing.assert_allclose(W[1].astype(np.float64) + Wc, W0[1].astype(np.float64) + Wc0, rtol=0, atol=2e-6)


def pin_brute_force_scalar_loop(impl, golden):
    """Tiny sizes against a loop written from the statements of Algorithm 1, with explicit temporaries for the
    values at the start of the turn."""
    rng = np.random.default_rng(14)
    P, N, eta, rho, mu = 3, 5, 0.1, 0.4, 0.7
    W0 = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    V0 = rng.standard_normal((P, N)).astype(F); Wc0 = rng.standard_normal(N).astype(F)
    order = [2, 0, 1, 2, 2, 0]
    for mom in (False, True):
        W, V, Wc = W0.copy(), V0.copy(), Wc0.copy()
        impl(W, V if mom else None, G, Wc, order, eta, rho, mu)
        Wb, Vb, Wcb = W0.copy(), V0.copy(), Wc0.copy()
        for j in order:
            for p in range(N):
                w_fetched = float(Wb[j, p])                       # the master gets W^j before the worker updates it
                c_sent = float(Wcb[p])                            # the worker got the center before the master updates it
                grad = float(G[j, p])
                if mom:
                    v_new = F(mu * float(Vb[j, p]) - eta * grad)
                    Vb[j, p] = v_new
                    Wb[j, p] = F(w_fetched + float(v_new) - eta * rho * (w_fetched - c_sent))
                else:
                    Wb[j, p] = F(w_fetched - eta * (grad + rho * (w_fetched - c_sent)))
                Wcb[p] = F(c_sent + eta * rho * (w_fetched - c_sent))
        np.testing.assert_array_equal(W, Wb)
        np.testing.assert_array_equal(Wc, Wcb)
        if mom:
            np.testing.assert_array_equal(V, Vb)


def pin_momentum_special_cases(impl, golden):
    rng = np.random.default_rng(15)
    P, N = 3, 77
    W0 = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    Wc0 = rng.standard_normal(N).astype(F)
    order = [0, 2, 1]
    # mu = 0 from V = 0: the plain rule (to rounding: Eq. (6) adds the rounded step instead of fusing it)
    W1, Wc1 = W0.copy(), Wc0.copy(); impl(W1, None, G, Wc1, order, 0.05, 0.2, 0.0)
    W2, Wc2, V = W0.copy(), Wc0.copy(), np.zeros((P, N), F); impl(W2, V, G, Wc2, order, 0.05, 0.2, 0.0)
    np.testing.assert_allclose(W2, W1, rtol=0, atol=1e-6)
    np.testing.assert_array_equal(Wc2, Wc1)
    np.testing.assert_allclose(V, -0.05 * G.astype(np.float64), rtol=0, atol=1e-7)
    # rho = 0: every served worker takes a momentum SGD step Eq. (3),(4), the center stays
    W3, Wc3, V3 = W0.copy(), Wc0.copy(), np.ones((P, N), F); impl(W3, V3, G, Wc3, order, 0.05, 0.0, 0.5)
    np.testing.assert_array_equal(Wc3, Wc0)
    np.testing.assert_allclose(V3, 0.5 - 0.05 * G.astype(np.float64), rtol=0, atol=1e-6)
    np.testing.assert_allclose(W3, W0.astype(np.float64) + V3, rtol=0, atol=1e-6)


PINS = [pin_hand_example, pin_turns_are_one_worker_synchronous_rounds, pin_workers_not_served_are_untouched,
        pin_zero_gradient_invariants_and_closed_form, pin_brute_force_scalar_loop, pin_momentum_special_cases]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_passes_every_pin(pin, golden):
    pin(_oracle_impl, golden)


def test_padding_is_never_touched():
    rng = np.random.default_rng(16)
    P, N, ld = 3, 50, 56
    W = np.full((P, ld), np.nan, F); W[:, :N] = rng.standard_normal((P, N))
    G = np.full((P, ld), np.nan, F); G[:, :N] = rng.standard_normal((P, N))
    V = np.full((P, ld), np.nan, F); V[:, :N] = 0
    Wc = rng.standard_normal(N).astype(F)
    oracle.async_easgd(W, G, Wc, [0, 1, 2, 1], 0.1, 0.3, V=V, mu=0.9, N=N)
    assert np.isnan(W[:, N:]).all() and np.isnan(V[:, N:]).all()
    assert np.isfinite(W[:, :N]).all() and np.isfinite(V[:, :N]).all() and np.isfinite(Wc).all()
    with pytest.raises(ValueError):
        oracle.async_easgd(W, G, Wc, [0, 3], 0.1, 0.3, N=N)


def test_rank_order_differs_from_the_synchronous_round_at_second_order():
    """Serving the workers one at a time is not the synchronous round: the center a later worker sees has already
    moved, which changes results at O((eta*rho)^2) (the hand example shows the same with exact numbers)."""
    rng = np.random.default_rng(17)
    P, N, eta, rho = 4, 300, 0.1, 0.5
    W0 = rng.standard_normal((P, N)).astype(F); Wc0 = rng.standard_normal(N).astype(F)
    G = np.zeros((P, N), F)
    Wa, Wca = W0.copy(), Wc0.copy(); oracle.async_easgd(Wa, G, Wca, list(range(P)), eta, rho)
    Ws, Wcs = W0.copy(), Wc0.copy(); oracle.easgd_round(Ws, G, Wcs, eta, rho)
    alpha = eta * rho
    spread = np.abs(W0.astype(np.float64) - Wc0).sum(0).max()
    diff = np.abs(Wca.astype(np.float64) - Wcs).max()
    assert 1e-4 < diff <= alpha * alpha * P * spread
    np.testing.assert_array_equal(Wa[0], Ws[0])                   # the first worker served saw the time-t center


# ---- plausible wrong rules: every one must be caught by at least one pin ----

def _mutant(kind):
    def impl(W, V, G, Wc, order, eta, rho, mu):
        seq = list(order)
        if kind == "rank_order_whatever_the_schedule":
            seq = sorted(seq)
        c_frozen = Wc.astype(np.float64).copy()
        for j in seq:
            w = W[j].astype(np.float64); c = Wc.astype(np.float64)
            g = G[(j + 1) % W.shape[0] if kind == "neighbours_gradient" else j].astype(np.float64)
            c_for_worker = c
            if kind == "all_workers_see_the_first_center":       # the synchronous reading
                c_for_worker = c_frozen
            if kind == "worker_sees_center_after_master":
                c_for_worker = c + eta * rho * (w - c)
            d = w - c_for_worker
            if V is None:
                w_new = (w - eta * (g + rho * d)).astype(F)
            else:
                v_new = (mu * V[j].astype(np.float64) - eta * g).astype(F)
                V[j] = v_new
                w_new = (w + v_new.astype(np.float64) - eta * rho * d).astype(F)
            w_for_master = w_new.astype(np.float64) if kind == "master_uses_updated_weights" else w
            sign = -1.0 if kind == "center_moves_away" else 1.0
            c_base = c_frozen if kind == "all_workers_see_the_first_center" else c
            Wc[...] = (c + sign * eta * rho * (w_for_master - c_base)).astype(F)
            W[j] = w_new
    return impl


MISTAKES = ["rank_order_whatever_the_schedule", "neighbours_gradient", "all_workers_see_the_first_center",
            "worker_sees_center_after_master", "master_uses_updated_weights", "center_moves_away"]


@pytest.mark.parametrize("kind", MISTAKES)
def test_planted_mistakes_are_caught(kind, golden):
    caught = []
    for pin in PINS:
        try:
            pin(_mutant(kind), golden)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the mistake '{kind}'"


def test_correct_restatement_passes():
    """The mutant harness itself: the unmodified restatement must pass all pins."""
    from conftest import read_golden
    for pin in PINS:
        pin(_mutant("none"), read_golden)
