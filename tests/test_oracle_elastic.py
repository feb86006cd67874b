"""The elastic-update oracle against what the paper and the mathematics fix."""
import numpy as np
import pytest

import oracle
from elastic_pins import ALL_PINS, INDEPENDENT_PINS

F = np.float32


class OracleImpl:
    @staticmethod
    def easgd(W, G, Wc, eta, rho):
        oracle.easgd_round(W, G, Wc, eta, rho)

    @staticmethod
    def measgd(W, V, G, Wc, eta, rho, mu):
        oracle.measgd_round(W, V, G, Wc, eta, rho, mu)


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(OracleImpl)


# ---------------------------------------------------------------------------
# Wrong variants: each plants one plausible mistake into a numpy re-statement
# of the round.  Every one of them must be caught by an independent pin.
# ---------------------------------------------------------------------------

class Variant:
    def __init__(self, name):
        self.name = name

    def easgd(self, W, G, Wc, eta, rho):
        m = self.name
        w, g, c = W.astype(np.float64), G.astype(np.float64), Wc.astype(np.float64)
        P = w.shape[0]
        d = w - c[None]
        a = eta * rho
        if m == "correct" or m.startswith("m_"):
            w_n, c_n = w - eta * (g + rho * d), c + a * d.sum(0)
        elif m == "sequential":            # gradient step first, spring on the stepped weights
            w1 = w - eta * g
            w_n, c_n = w1 - a * (w1 - c[None]), c + a * (w1 - c[None]).sum(0)
        elif m == "center_sees_new_workers":
            w_n = w - eta * (g + rho * d)
            c_n = c + a * (w_n - c[None]).sum(0)
        elif m == "workers_see_new_center":
            c_n = c + a * d.sum(0)
            w_n = w - eta * (g + rho * (w - c_n[None]))
        elif m == "spring_sign":
            w_n, c_n = w - eta * (g - rho * d), c + a * d.sum(0)
        elif m == "center_sign":
            w_n, c_n = w - eta * (g + rho * d), c - a * d.sum(0)
        elif m == "grad_sign":
            w_n, c_n = w + eta * (g - rho * d), c + a * d.sum(0)
        elif m == "center_mean":           # averages instead of summing over the workers
            w_n, c_n = w - eta * (g + rho * d), c + a * d.mean(0)
        elif m == "center_no_eta":
            w_n, c_n = w - eta * (g + rho * d), c + rho * d.sum(0)
        elif m == "rho_outside":           # eta*g + rho*d instead of eta*(g + rho*d)
            w_n, c_n = w - eta * g - rho * d, c + a * d.sum(0)
        elif m == "wrong_worker_grad":     # gradient of the neighbouring worker
            w_n, c_n = w - eta * (np.roll(g, 1, axis=0) + rho * d), c + a * d.sum(0)
        elif m == "center_sum_of_weights": # forgets to subtract P*Wc after reducing sum_i W_i
            w_n, c_n = w - eta * (g + rho * d), c + a * w.sum(0)
        else:
            raise KeyError(m)
        W[...] = w_n.astype(F)
        Wc[...] = c_n.astype(F)

    def measgd(self, W, V, G, Wc, eta, rho, mu):
        m = self.name
        w, v, g, c = (x.astype(np.float64) for x in (W, V, G, Wc))
        d = w - c[None]
        a = eta * rho
        c_n = c + a * d.sum(0)
        if m == "m_old_velocity":          # Eq. (6) with V_t instead of V_{t+1}
            v_n = mu * v - eta * g
            w_n = w + v - a * d
        elif m == "m_grad_sign":
            v_n = mu * v + eta * g
            w_n = w + v_n - a * d
        elif m == "m_momentum_on_grad":    # mu multiplies the wrong term
            v_n = v - mu * eta * g
            w_n = w + v_n - a * d
        elif m == "m_spring_in_velocity":  # elastic force folded into V
            v_n = mu * v - eta * (g + rho * d)
            w_n = w + v_n
        elif m == "m_spring_no_eta":
            v_n = mu * v - eta * g
            w_n = w + v_n - rho * d
        elif m == "m_center_sees_new_workers":
            v_n = mu * v - eta * g
            w_n = w + v_n - a * d
            c_n = c + a * (w_n - c[None]).sum(0)
        else:                              # easgd-only mistakes: momentum part is right
            v_n = mu * v - eta * g
            w_n = w + v_n - a * d
        V[...] = v_n.astype(F)
        W[...] = w_n.astype(F)
        Wc[...] = c_n.astype(F)


def _failed_pins(impl):
    failed = []
    for pin in INDEPENDENT_PINS:
        try:
            pin(impl)
        except AssertionError:
            failed.append(pin.__name__)
    return failed


def test_correct_restatement_passes_all_pins():
    assert _failed_pins(Variant("correct")) == []


@pytest.mark.parametrize("name", [
    "sequential", "center_sees_new_workers", "workers_see_new_center", "spring_sign", "center_sign",
    "grad_sign", "center_mean", "center_no_eta", "rho_outside", "wrong_worker_grad",
    "center_sum_of_weights",
    "m_old_velocity", "m_grad_sign", "m_momentum_on_grad", "m_spring_in_velocity", "m_spring_no_eta",
    "m_center_sees_new_workers",
])
def test_planted_mistake_is_caught(name):
    assert _failed_pins(Variant(name)), f"no independent pin catches the mistake '{name}'"


# ---------------------------------------------------------------------------
# Properties specific to the oracle's interface
# ---------------------------------------------------------------------------

def test_conservation_needs_matching_coefficients():
    rng = np.random.default_rng(0)
    W = rng.standard_normal((3, 10)).astype(F); Wc = rng.standard_normal(10).astype(F)
    G = np.zeros((3, 10), F)
    total0 = W.astype(np.float64).sum(0) + Wc
    oracle.easgd_round(W, G, Wc, 0.1, 0.5, center_coef=0.02)      # worker coefficient is 0.05
    assert np.abs(W.astype(np.float64).sum(0) + Wc - total0).max() > 1e-3


def test_padding_columns_untouched():
    rng = np.random.default_rng(1)
    P, N, ld = 3, 10, 16
    W = rng.standard_normal((P, ld)).astype(F); G = rng.standard_normal((P, ld)).astype(F)
    V = rng.standard_normal((P, ld)).astype(F)
    W[:, N:] = np.nan; G[:, N:] = np.nan; V[:, N:] = 7.0
    Wc = rng.standard_normal(N).astype(F)
    Wd, Gd, Wcd = W[:, :N].copy(), G[:, :N].copy(), Wc.copy()
    oracle.easgd_round(W, G, Wc, 0.1, 0.5)
    oracle.easgd_round(Wd, Gd, Wcd, 0.1, 0.5)
    assert np.isnan(W[:, N:]).all()
    np.testing.assert_array_equal(W[:, :N], Wd)
    np.testing.assert_array_equal(Wc, Wcd)
    oracle.measgd_round(W, V, G, Wc, 0.1, 0.5, 0.9)
    assert np.isnan(W[:, N:]).all() and (V[:, N:] == 7.0).all()
    assert np.isfinite(W[:, :N]).all() and np.isfinite(Wc).all()


def test_order_of_workers_does_not_matter():
    """The sum over i in Eq. (2) is order-free in exact arithmetic; in double it is order-free to fp32 rounding."""
    rng = np.random.default_rng(2)
    P, N = 16, 200
    W = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
    Wc = rng.standard_normal(N).astype(F)
    perm = rng.permutation(P)
    W2, G2, Wc2 = W[perm].copy(), G[perm].copy(), Wc.copy()
    oracle.easgd_round(W, G, Wc, 0.01, 0.1)
    oracle.easgd_round(W2, G2, Wc2, 0.01, 0.1)
    np.testing.assert_array_equal(W[perm], W2)
    np.testing.assert_allclose(Wc, Wc2, rtol=2e-7)
