"""Pins for an implementation of one elastic exchange-and-update round.

Each pin takes `impl`, an object with
    easgd(W, G, Wc, eta, rho)            -> None (in place, fp32 numpy arrays)
    measgd(W, V, G, Wc, eta, rho, mu)    -> None (in place)
and raises AssertionError if `impl` disagrees with something the paper or the
mathematics fixes.  The same pins are run on the real oracle (must all pass)
and on deliberately wrong variants (each must fail at least one), so that the
pins are known to be sensitive to plausible mistakes.
"""
import numpy as np

from conftest import read_golden

F = np.float32


def _a(x, shape=None):
    a = np.array(x, dtype=F)
    return a.reshape(shape) if shape is not None else a


# ---- values printed in tests/golden (hand-evaluated Eq. (1),(2),(5),(6)) ----

def pin_hand_example_easgd(impl):
    g = read_golden("easgd_hand_example.txt")
    W = _a(g["W"], (2, 1)); G = _a(g["G"], (2, 1)); Wc = _a([g["Wc"]])
    impl.easgd(W, G, Wc, g["eta"], g["rho"])
    np.testing.assert_allclose(W.ravel(), g["W_next"], rtol=2e-7)
    np.testing.assert_allclose(Wc, [g["Wc_next"]], rtol=2e-7)


def pin_hand_example_measgd(impl):
    g = read_golden("measgd_hand_example.txt")
    W = _a(g["W"], (2, 1)); V = _a(g["V"], (2, 1)); G = _a(g["G"], (2, 1)); Wc = _a([g["Wc"]])
    impl.measgd(W, V, G, Wc, g["eta"], g["rho"], g["mu"])
    np.testing.assert_allclose(V.ravel(), g["V_next"], rtol=1e-6)
    np.testing.assert_allclose(W.ravel(), g["W_next"], rtol=2e-7)
    np.testing.assert_allclose(Wc, [g["Wc_next"]], rtol=2e-7)


def pin_zero_grad_trajectory(impl):
    g = read_golden("easgd_zero_grad_closed_form.txt")
    W = _a([1.0, 3.0], (2, 1)); G = np.zeros((2, 1), F); Wc = _a([0.0])
    for k, wc_k, gap_k in zip(g["rounds"], g["Wc"], g["W2_minus_W1"]):
        impl.easgd(W, G, Wc, 0.1, 0.5)
        np.testing.assert_allclose(Wc[0], wc_k, rtol=1e-6)
        np.testing.assert_allclose(W[1, 0] - W[0, 0], gap_k, rtol=1e-6)


# ---- special cases that reduce to textbook rules ----

def pin_plain_sgd(impl):
    """P = 1 and rho = 0: Eq. (1) is the SGD step W - eta*dW (Section 2.2); the center does not move."""
    rng = np.random.default_rng(1)
    W = rng.standard_normal((1, 37)).astype(F); G = rng.standard_normal((1, 37)).astype(F)
    Wc = rng.standard_normal(37).astype(F)
    W0, Wc0 = W.copy(), Wc.copy()
    impl.easgd(W, G, Wc, 0.03, 0.0)
    np.testing.assert_allclose(W, (W0.astype(np.float64) - 0.03 * G.astype(np.float64)).astype(F), rtol=0, atol=0)
    np.testing.assert_array_equal(Wc, Wc0)


def pin_rho_zero_any_P(impl):
    rng = np.random.default_rng(2)
    W = rng.standard_normal((5, 11)).astype(F); G = rng.standard_normal((5, 11)).astype(F)
    Wc = rng.standard_normal(11).astype(F)
    W0, Wc0 = W.copy(), Wc.copy()
    impl.easgd(W, G, Wc, 0.2, 0.0)
    np.testing.assert_array_equal(W, (W0.astype(np.float64) - 0.2 * G.astype(np.float64)).astype(F))
    np.testing.assert_array_equal(Wc, Wc0)


def pin_identical_start(impl):
    """All replicas and the center start as copies of one W (Algorithms 1-3):
    every difference is zero, so round 1 is a pure SGD step and Wc is unchanged bit for bit."""
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal(29).astype(F)
    W = np.tile(w0, (6, 1)); Wc = w0.copy()
    G = rng.standard_normal((6, 29)).astype(F)
    impl.easgd(W, G, Wc, 0.05, 0.3)
    np.testing.assert_array_equal(Wc, w0)
    np.testing.assert_array_equal(W, (w0.astype(np.float64)[None] - 0.05 * G.astype(np.float64)).astype(F))


def pin_measgd_identical_start(impl):
    rng = np.random.default_rng(4)
    w0 = rng.standard_normal(17).astype(F)
    W = np.tile(w0, (3, 1)); Wc = w0.copy()
    G = rng.standard_normal((3, 17)).astype(F); V = rng.standard_normal((3, 17)).astype(F)
    V0 = V.copy()
    impl.measgd(W, V, G, Wc, 0.05, 0.3, 0.9)
    np.testing.assert_array_equal(Wc, w0)
    v1 = (0.9 * V0.astype(np.float64) - 0.05 * G.astype(np.float64)).astype(F)         # Eq. (3)
    np.testing.assert_array_equal(V, v1)
    np.testing.assert_allclose(W, w0.astype(np.float64)[None] + v1, rtol=3e-7, atol=1e-7)   # Eq. (4)


def pin_measgd_mu_zero_is_easgd(impl):
    """mu = 0 and any V: Eq. (5),(6) collapse to Eq. (1)."""
    rng = np.random.default_rng(5)
    W = rng.standard_normal((4, 23)).astype(F); G = rng.standard_normal((4, 23)).astype(F)
    Wc = rng.standard_normal(23).astype(F); V = rng.standard_normal((4, 23)).astype(F)
    W2, Wc2 = W.copy(), Wc.copy()
    impl.measgd(W, V, G, Wc, 0.07, 0.4, 0.0)
    impl.easgd(W2, G, Wc2, 0.07, 0.4)
    np.testing.assert_allclose(W, W2, rtol=3e-7, atol=1e-7)
    np.testing.assert_array_equal(Wc, Wc2)
    np.testing.assert_array_equal(V, (-0.07 * G.astype(np.float64)).astype(F))


def pin_measgd_rho_zero_is_msgd(impl):
    """rho = 0: Eq. (5),(6) are momentum SGD, Eq. (3),(4), per replica, for several rounds."""
    rng = np.random.default_rng(6)
    W = rng.standard_normal((3, 13)).astype(F); V = np.zeros((3, 13), F)
    Wc = rng.standard_normal(13).astype(F); Wc0 = Wc.copy()
    w_ref, v_ref = W.astype(np.float64), np.zeros((3, 13))
    for t in range(4):
        G = rng.standard_normal((3, 13)).astype(F)
        impl.measgd(W, V, G, Wc, 0.1, 0.0, 0.9)
        v_ref = 0.9 * v_ref - 0.1 * G.astype(np.float64)
        w_ref = w_ref + v_ref
    np.testing.assert_allclose(V, v_ref, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(W, w_ref, rtol=1e-5, atol=1e-6)
    np.testing.assert_array_equal(Wc, Wc0)


# ---- invariants ----

def pin_conservation(impl):
    """Zero gradients: sum_i W_i + Wc is conserved (the -alpha*S of the workers cancels the +alpha*S of the center)."""
    rng = np.random.default_rng(7)
    P, N = 7, 41
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    G = np.zeros((P, N), F)
    total0 = W.astype(np.float64).sum(0) + Wc
    for _ in range(20):
        impl.easgd(W, G, Wc, 0.1, 0.3)
    total = W.astype(np.float64).sum(0) + Wc
    np.testing.assert_allclose(total, total0, rtol=0, atol=2e-5)
    # and with momentum, zero V and zero gradients
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    V = np.zeros((P, N), F)
    total0 = W.astype(np.float64).sum(0) + Wc
    for _ in range(20):
        impl.measgd(W, V, G, Wc, 0.1, 0.3, 0.9)
    np.testing.assert_allclose(W.astype(np.float64).sum(0) + Wc, total0, rtol=0, atol=2e-5)
    np.testing.assert_array_equal(V, np.zeros_like(V))


def pin_closed_form(impl):
    """Zero gradients, k rounds, alpha = eta*rho, lambda = 1 - alpha*(P+1):
       S_k = lambda^k S_0;  Wc_k = Wc_0 + S_0 (1 - lambda^k)/(P+1);
       W_i,k = Wc_k + (1-alpha)^k (d_i,0 - S_0/P) + S_k/P,   d_i = W_i - Wc, S = sum_i d_i."""
    rng = np.random.default_rng(8)
    P, N, k = 5, 19, 12
    eta, rho = 0.25, 0.2
    alpha = eta * rho
    lam = 1.0 - alpha * (P + 1)
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    G = np.zeros((P, N), F)
    d0 = W.astype(np.float64) - Wc.astype(np.float64)
    S0 = d0.sum(0)
    wc_k = Wc + S0 * (1 - lam ** k) / (P + 1)
    w_k = wc_k[None] + (1 - alpha) ** k * (d0 - S0 / P) + lam ** k * S0 / P
    for _ in range(k):
        impl.easgd(W, G, Wc, eta, rho)
    np.testing.assert_allclose(Wc, wc_k, rtol=0, atol=3e-6)
    np.testing.assert_allclose(W, w_k, rtol=0, atol=3e-6)


def pin_contraction(impl):
    """Zero gradients, 0 < alpha < 2/(P+1): all replicas and the center contract to (sum_i W_i + Wc)/(P+1)."""
    rng = np.random.default_rng(9)
    P, N = 4, 9
    W = rng.standard_normal((P, N)).astype(F); Wc = rng.standard_normal(N).astype(F)
    G = np.zeros((P, N), F)
    fixed = (W.astype(np.float64).sum(0) + Wc) / (P + 1)
    spread_prev = np.inf
    for r in range(400):
        impl.easgd(W, G, Wc, 0.5, 0.2)
        if r % 50 == 49:
            spread = np.abs(W - Wc[None]).max()
            assert spread < spread_prev or spread < 1e-6
            spread_prev = spread
    np.testing.assert_allclose(Wc, fixed, atol=2e-5)
    np.testing.assert_allclose(W, np.tile(fixed, (P, 1)), atol=2e-5)


# ---- brute force ----

def _brute_easgd(W, G, Wc, eta, rho):
    """Scalar loops straight from Eq. (1),(2); all time-t values are copied first."""
    P, N = len(W), len(Wc)
    W_t = [[float(W[i][j]) for j in range(N)] for i in range(P)]
    Wc_t = [float(Wc[j]) for j in range(N)]
    W_n = [[0.0] * N for _ in range(P)]
    Wc_n = [0.0] * N
    for i in range(P):
        for j in range(N):
            W_n[i][j] = W_t[i][j] - eta * (float(G[i][j]) + rho * (W_t[i][j] - Wc_t[j]))
    for j in range(N):
        s = 0.0
        for i in range(P):
            s += rho * (W_t[i][j] - Wc_t[j])
        Wc_n[j] = Wc_t[j] + eta * s
    return W_n, Wc_n


def _brute_measgd(W, V, G, Wc, eta, rho, mu):
    P, N = len(W), len(Wc)
    W_t = [[float(W[i][j]) for j in range(N)] for i in range(P)]
    V_t = [[float(V[i][j]) for j in range(N)] for i in range(P)]
    Wc_t = [float(Wc[j]) for j in range(N)]
    V_n = [[mu * V_t[i][j] - eta * float(G[i][j]) for j in range(N)] for i in range(P)]
    W_n = [[W_t[i][j] + V_n[i][j] - eta * rho * (W_t[i][j] - Wc_t[j]) for j in range(N)] for i in range(P)]
    Wc_n = [Wc_t[j] + eta * sum(rho * (W_t[i][j] - Wc_t[j]) for i in range(P)) for j in range(N)]
    return W_n, V_n, Wc_n


def pin_brute_force(impl):
    rng = np.random.default_rng(10)
    for P, N in [(1, 1), (2, 3), (3, 8), (4, 5)]:
        for _ in range(3):
            W = rng.standard_normal((P, N)).astype(F); G = rng.standard_normal((P, N)).astype(F)
            Wc = rng.standard_normal(N).astype(F); V = rng.standard_normal((P, N)).astype(F)
            eta, rho, mu = 0.13, 0.37, 0.8
            W_n, Wc_n = _brute_easgd(W, G, Wc, eta, rho)
            W1, Wc1 = W.copy(), Wc.copy()
            impl.easgd(W1, G, Wc1, eta, rho)
            np.testing.assert_allclose(W1, np.array(W_n), rtol=2e-7, atol=1e-7)
            np.testing.assert_allclose(Wc1, np.array(Wc_n), rtol=2e-7, atol=1e-7)
            W_n, V_n, Wc_n = _brute_measgd(W, V, G, Wc, eta, rho, mu)
            W2, V2, Wc2 = W.copy(), V.copy(), Wc.copy()
            impl.measgd(W2, V2, G, Wc2, eta, rho, mu)
            np.testing.assert_allclose(V2, np.array(V_n), rtol=2e-7, atol=1e-7)
            np.testing.assert_allclose(W2, np.array(W_n), rtol=3e-7, atol=2e-7)
            np.testing.assert_allclose(Wc2, np.array(Wc_n), rtol=2e-7, atol=1e-7)


# pins that do not re-type the update rule (brute force is listed separately)
INDEPENDENT_PINS = [
    pin_hand_example_easgd, pin_hand_example_measgd, pin_zero_grad_trajectory,
    pin_plain_sgd, pin_rho_zero_any_P, pin_identical_start, pin_measgd_identical_start,
    pin_measgd_mu_zero_is_easgd, pin_measgd_rho_zero_is_msgd,
    pin_conservation, pin_closed_form, pin_contraction,
]
ALL_PINS = INDEPENDENT_PINS + [pin_brute_force]
