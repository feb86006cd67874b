"""HIP async_easgd_round (the master serving one worker at a time: Algorithm 1 in rank order, Async EASGD / Async
MEASGD of Section 5.1 in arrival order) against the CPU oracle, and hogwild_easgd_round (Section 5.1, "Hogwild
EASGD": lock-free, not reproducible) against what every interleaving must satisfy.  Through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32
ETA, RHO, MU = F(0.01), F(0.1), F(0.9)


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


# (P, N, ld): one element, ragged tails (N % 4 = 1, 2, 3), ld > N, several tiles, many workers, a size that takes the
# die-interleaved tiles
SHAPES = [(1, 1, 4), (2, 3, 4), (9, 261, 264), (4, 7850, 7852), (3, 4099, 4100), (8, 100_003, 100_004),
          (16, 33_333, 33_336), (5, 1 << 20, 1 << 20), (64, 65_537, 65_540), (7, 1026, 2048), (3, 4_500_003, 4_500_004)]


def _schedule(P, seed, turns=None):
    """Arrival order: a shuffle of the workers plus a few that come up a second time."""
    rng = np.random.default_rng(seed)
    order = list(rng.permutation(P)) + list(rng.integers(0, P, size=min(P, 3)))
    return [int(j) for j in (order if turns is None else order[:turns])]


@pytest.mark.parametrize("P,N,ld", SHAPES)
@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_schedule_matches_oracle(hip, P, N, ld, momentum):
    W, Wc = workloads.update_state(P, N, ld, seed=51)
    G = workloads.update_gradients(P, N, 0, ld, seed=51)
    V = workloads.update_gradients(P, N, 99, ld, seed=51, std=0.005)
    order = _schedule(P, 51)
    dW, dG, dV, dWc = to_dev(W), to_dev(G), to_dev(V), to_dev(Wc)
    hip.async_easgd_round(dW, dG, dWc, order, float(ETA), float(RHO), V=dV if momentum else None, delta=float(MU), N=N)
    oracle.async_easgd(W, G, Wc, order, ETA, RHO, V=V if momentum else None, mu=MU, N=N)
    assert normwise(to_host(dW), W) <= PER_ROUND_TOL           # also checks that NaN padding stayed NaN
    assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
    if momentum:
        assert normwise(to_host(dV), V) <= PER_ROUND_TOL
    else:
        np.testing.assert_array_equal(to_host(dV), V)         # untouched without momentum
    np.testing.assert_array_equal(to_host(dG), G)              # gradients are read-only


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_one_launch_equals_the_turns_one_by_one(hip, momentum):
    """The schedule in one launch gives the bits of one launch per turn, and a turn of worker j gives the bits of the
    synchronous round of a system whose only worker is j (the fused kernel with P = 1 on that row)."""
    P, N, ld = 6, 300_001, 300_004
    W, Wc = workloads.update_state(P, N, ld, seed=52)
    G = workloads.update_gradients(P, N, 0, ld, seed=52)
    V = workloads.update_gradients(P, N, 9, ld, seed=52, std=0.005)
    order = _schedule(P, 52)
    aW, aV, aWc, dG = to_dev(W), to_dev(V), to_dev(Wc), to_dev(G)
    hip.async_easgd_round(aW, dG, aWc, order, float(ETA), float(RHO), V=aV if momentum else None, delta=float(MU), N=N)
    bW, bV, bWc = to_dev(W), to_dev(V), to_dev(Wc)
    cW, cV, cWc = to_dev(W), to_dev(V), to_dev(Wc)
    for j in order:
        hip.async_easgd_round(bW, dG, bWc, [j], float(ETA), float(RHO), V=bV if momentum else None, delta=float(MU), N=N)
        if momentum:
            hip.measgd_round(cW[j:j + 1], cV[j:j + 1], dG[j:j + 1], cWc, float(ETA), float(RHO), float(MU), N=N)
        else:
            hip.easgd_sync_round(cW[j:j + 1], dG[j:j + 1], cWc, float(ETA), float(RHO), N=N)
    for x, y_, z in ((aW, bW, cW), (aWc, bWc, cWc), (aV, bV, cV)):
        np.testing.assert_array_equal(to_host(x), to_host(y_))
        np.testing.assert_array_equal(to_host(x), to_host(z))


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_unaligned_operands_take_the_scalar_path(hip, momentum):
    P, N = 3, 1001
    for ld, shift in [(1003, 0), (1004, 1), (1001, 3)]:
        W, Wc = workloads.update_state(P, N, ld, seed=53)
        G = workloads.update_gradients(P, N, 0, ld, seed=53)
        V = workloads.update_gradients(P, N, 5, ld, seed=53)

        def carve(a):   # operands at an element offset inside larger buffers: base not 16-byte aligned
            buf = torch.full((a.size + 8,), float("nan"), dtype=torch.float32, device="cuda")
            view = buf[shift:shift + a.size].view(a.shape)
            view.copy_(torch.from_numpy(a))
            return buf, view
        bW, dW = carve(W); bG, dG = carve(G); bV, dV = carve(V); bWc, dWc = carve(Wc)
        order = [2, 0, 1, 2]
        hip.async_easgd_round(dW, dG, dWc, order, float(ETA), float(RHO), V=dV if momentum else None, delta=float(MU), N=N)
        oracle.async_easgd(W, G, Wc, order, ETA, RHO, V=V if momentum else None, mu=MU, N=N)
        assert normwise(to_host(dW), W) <= PER_ROUND_TOL and normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
        if momentum:
            assert normwise(to_host(dV), V) <= PER_ROUND_TOL
        for buf, a in ((bW, W), (bWc, Wc)):                    # nothing outside the operands was written
            h = to_host(buf)
            assert np.isnan(h[:shift]).all() and np.isnan(h[shift + a.size:]).all()


def test_hundred_rounds_in_rank_order(hip):
    """Original EASGD's schedule (worker t mod P in round t), 100 turns with fresh gradients, free-running."""
    P, N, ld = 4, 50_001, 50_004
    W, Wc = workloads.update_state(P, N, ld, seed=54)
    dW, dWc = to_dev(W), to_dev(Wc)
    for t in range(100):
        G = workloads.update_gradients(P, N, t, ld, seed=54)
        hip.async_easgd_round(dW, to_dev(G), dWc, [t % P], float(ETA), float(RHO), N=N)
        oracle.async_easgd(W, G, Wc, [t % P], ETA, RHO, N=N)
    assert normwise(to_host(dW), W) <= HUNDRED_ROUND_TOL and normwise(to_host(dWc), Wc) <= HUNDRED_ROUND_TOL


def test_bad_schedules_are_rejected(hip):
    W = torch.zeros(2, 8, device="cuda"); G = torch.zeros_like(W); Wc = torch.zeros(8, device="cuda")
    for order in ([0, 2], [-1], list(range(2)) * 129):
        with pytest.raises(hip.EasgdError):
            hip.async_easgd_round(W, G, Wc, order, 0.1, 0.1)
    hip.async_easgd_round(W, G, Wc, [], 0.1, 0.1)             # nobody served: a no-op, not an error
    assert float(W.abs().sum()) == 0.0


def test_full_size_on_sampled_columns(hip):
    """AlexNet-sized replicas (P = 8 x 61 M), the rank-order schedule, on sampled columns."""
    wl = workloads.WORKLOADS["cfg4"]
    P, N = wl.P, wl.N
    ld = workloads.round_up(N, 256)
    dW = workloads.device_normal((P, ld), workloads.WEIGHT_STD, 77, 1)
    dWc = workloads.device_normal((N,), workloads.WEIGHT_STD, 77, 2)
    dG = workloads.device_normal((P, ld), workloads.GRADIENT_STD, 77, 3)
    rng = np.random.default_rng(77)
    cols = np.unique(np.concatenate([np.arange(0, 4096), np.arange(N - 4096, N), rng.integers(0, N, 200_000)]))
    tc = torch.from_numpy(cols).cuda()
    W = np.ascontiguousarray(to_host(dW[:, tc])); G = np.ascontiguousarray(to_host(dG[:, tc])); Wc = to_host(dWc[tc]).copy()
    order = list(range(P))
    hip.async_easgd_round(dW, dG, dWc, order, wl.eta, wl.rho, N=N)
    oracle.async_easgd(W, G, Wc, order, F(wl.eta), F(wl.rho))
    assert normwise(to_host(dW[:, tc]), W) <= PER_ROUND_TOL and normwise(to_host(dWc[tc]), Wc) <= PER_ROUND_TOL
    assert bool(torch.isfinite(dWc).all())


# ---- Hogwild EASGD: what is the same under every interleaving is compared exactly (to the fp32 bar); the rest
# ---- must lie inside the interval that the interleavings span

def _hogwild_bounds(W, Wc, G, eta, rho):
    """Per element, a radius r such that every center value any worker can see lies within r of the time-t center:
    the center only moves by additions of alpha*(W_i - c_i), and |W_i - c_i| <= |W_i - Wc| + r."""
    alpha = float(eta) * float(rho)
    P = W.shape[0]
    spread = np.abs(W.astype(np.float64) - Wc.astype(np.float64)).sum(0)
    return alpha * spread / (1.0 - alpha * P)


@pytest.mark.parametrize("P,N,ld", [(1, 1, 4), (2, 3, 4), (9, 261, 264), (4, 7850, 7852), (16, 33_333, 33_336),
                                    (5, 1 << 20, 1 << 20), (7, 1026, 2048)])
@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_hogwild_round_stays_inside_what_interleavings_allow(hip, P, N, ld, momentum):
    eta, rho, mu = F(0.05), F(0.2), F(0.9)                      # a large alpha, so that the interval is not trivial
    W, Wc = workloads.update_state(P, N, ld, seed=61)
    G = workloads.update_gradients(P, N, 0, ld, seed=61)
    V = workloads.update_gradients(P, N, 99, ld, seed=61, std=0.005)
    dW, dG, dV, dWc = to_dev(W), to_dev(G), to_dev(V), to_dev(Wc)
    hip.hogwild_easgd_round(dW, dG, dWc, float(eta), float(rho), V=dV if momentum else None, delta=float(mu), N=N)
    hW, hV, hWc = to_host(dW), to_host(dV), to_host(dWc)
    # the synchronous round from the same state: every worker sees the time-t center
    sW, sV, sWc = W.copy(), V.copy(), Wc.copy()
    if momentum:
        oracle.measgd_round(sW, sV, G, sWc, eta, rho, mu, N=N)
        assert normwise(hV, sV) <= PER_ROUND_TOL                # Eq. (5) does not involve the center
    else:
        oracle.easgd_round(sW, G, sWc, eta, rho, N=N)
        np.testing.assert_array_equal(hV, V)
    assert np.isnan(hW[:, N:]).all()
    alpha = float(eta) * float(rho)
    r = _hogwild_bounds(W[:, :N], Wc, G[:, :N], eta, rho)       # radius of the center values a worker can see
    scale_w, scale_c = np.abs(sW[:, :N]).max(), np.abs(sWc).max()
    # a worker's result is affine in the center value it saw, with slope alpha
    assert (np.abs(hW[:, :N].astype(np.float64) - sW[:, :N]) <= alpha * r + PER_ROUND_TOL * scale_w).all()
    # the center receives alpha*(W_i - c_i) from every worker: each c_i within r of the time-t center
    assert (np.abs(hWc.astype(np.float64) - sWc) <= alpha * P * r + PER_ROUND_TOL * scale_c).all()
    # what a worker loses the center gains: sum_i W_i + Wc is the same under every interleaving
    total_h = hW[:, :N].astype(np.float64).sum(0) + hWc
    total_s = sW[:, :N].astype(np.float64).sum(0) + sWc
    assert np.abs(total_h - total_s).max() <= PER_ROUND_TOL * (P + 1) * max(scale_w, scale_c)
    if P == 1:                                                  # one worker: nothing to interleave
        assert normwise(hW, sW) <= PER_ROUND_TOL and normwise(hWc, sWc) <= PER_ROUND_TOL


def test_hogwild_unaligned_operands_and_zero_gradient_contraction(hip):
    """The scalar kernel (operands not 16-byte aligned), and the fixed point: with zero gradients repeated lock-free
    rounds still pull every replica and the center to the conserved mean (sum_i W_i + Wc) / (P + 1)."""
    P, N, ld, shift = 3, 1001, 1003, 1
    W, Wc = workloads.update_state(P, N, ld, seed=62)
    buf = torch.full((W.size + 8,), float("nan"), dtype=torch.float32, device="cuda")
    dW = buf[shift:shift + W.size].view(W.shape); dW.copy_(torch.from_numpy(W))
    dWc = to_dev(Wc); dG = torch.zeros_like(dW)
    mean = (W[:, :N].astype(np.float64).sum(0) + Wc) / (P + 1)
    eta, rho = 0.5, 0.25
    for _ in range(400):
        hip.hogwild_easgd_round(dW, dG, dWc, eta, rho, N=N)
    hW, hWc = to_host(dW), to_host(dWc)
    assert np.abs(hWc - mean).max() <= 1e-5 and np.abs(hW[:, :N] - mean).max() <= 1e-5
    h = to_host(buf)
    assert np.isnan(h[:shift]).all() and np.isnan(h[shift + W.size:]).all() and np.isnan(hW[:, N:]).all()
