"""HIP elastic update (easgd_sync_round / measgd_round) against the CPU oracle, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu

F = np.float32
ETA, RHO, DELTA = F(0.01), F(0.1), F(0.9)


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


# (P, N, ld): small N with P >= 4 takes the kernel that splits the workers over wavefronts, the others the
# one-thread-per-group kernel; one element, ragged tails (N % 4 = 1, 2, 3), ld > N, several 1024-element tiles
SHAPES = [(1, 1, 4), (2, 3, 4), (6, 3, 4), (9, 261, 264), (4, 7850, 7852), (3, 4099, 4100), (8, 100_003, 100_004),
          (16, 33_333, 33_336), (5, 1 << 20, 1 << 20), (32, 65_537, 65_540), (7, 1026, 2048)]


@pytest.mark.parametrize("P,N,ld", SHAPES)
@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_one_round_matches_oracle(hip, P, N, ld, momentum):
    W, Wc = workloads.update_state(P, N, ld, seed=11)
    G = workloads.update_gradients(P, N, 0, ld, seed=11)
    V = workloads.update_gradients(P, N, 99, ld, seed=11, std=0.005)
    dW, dG, dWc, dV = to_dev(W), to_dev(G), to_dev(Wc), to_dev(V)
    if momentum:
        hip.measgd_round(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
        oracle.measgd_round(W, V, G, Wc, ETA, RHO, DELTA, N=N)
        assert normwise(to_host(dV), V) <= PER_ROUND_TOL
    else:
        hip.easgd_sync_round(dW, dG, dWc, float(ETA), float(RHO), N=N)
        oracle.easgd_round(W, G, Wc, ETA, RHO, N=N)
    assert normwise(to_host(dW), W) <= PER_ROUND_TOL      # also checks that NaN padding stayed NaN
    assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
    np.testing.assert_array_equal(to_host(dG), G)           # gradients are read-only


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_unaligned_operands_take_the_scalar_path(hip, momentum):
    P, N = 3, 1001
    for ld, shift in [(1003, 0), (1004, 1), (1001, 3)]:
        W, Wc = workloads.update_state(P, N, ld, seed=12)
        G = workloads.update_gradients(P, N, 0, ld, seed=12)
        V = workloads.update_gradients(P, N, 5, ld, seed=12)
        # carve the operands out of larger buffers at an element offset -> base not 16-byte aligned
        def carve(a):
            buf = torch.full((a.size + 8,), float("nan"), dtype=torch.float32, device="cuda")
            view = buf[shift:shift + a.size].view(a.shape)
            view.copy_(torch.from_numpy(a))
            return buf, view
        bW, dW = carve(W); bG, dG = carve(G); bV, dV = carve(V); bWc, dWc = carve(Wc)
        if momentum:
            hip.measgd_round(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
            oracle.measgd_round(W, V, G, Wc, ETA, RHO, DELTA, N=N)
            assert normwise(to_host(dV), V) <= PER_ROUND_TOL
        else:
            hip.easgd_sync_round(dW, dG, dWc, float(ETA), float(RHO), N=N)
            oracle.easgd_round(W, G, Wc, ETA, RHO, N=N)
        assert normwise(to_host(dW), W) <= PER_ROUND_TOL
        assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
        # nothing outside the operands was written
        for buf, a in ((bW, W), (bWc, Wc)):
            h = to_host(buf)
            assert np.isnan(h[:shift]).all() and np.isnan(h[shift + a.size:]).all()


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_hundred_rounds_free_running_and_teacher_forced(hip, momentum):
    P, N = 8, (1 << 18) + 3
    ld = workloads.round_up(N, 4)
    W, Wc = workloads.update_state(P, N, ld, seed=13)
    V = np.zeros_like(W); V[:, N:] = np.nan
    dW, dWc, dV = to_dev(W), to_dev(Wc), to_dev(V)
    worst_forced = 0.0
    for t in range(100):
        G = workloads.update_gradients(P, N, t, ld, seed=13)
        dG = to_dev(G)
        if t % 10 == 0:
            # teacher-forced: one GPU round from the oracle's state of this round
            fW, fWc, fV = to_dev(W), to_dev(Wc), to_dev(V)
        if momentum:
            if t % 10 == 0:
                hip.measgd_round(fW, fV, dG, fWc, float(ETA), float(RHO), float(DELTA), N=N)
            hip.measgd_round(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
            oracle.measgd_round(W, V, G, Wc, ETA, RHO, DELTA, N=N)
        else:
            if t % 10 == 0:
                hip.easgd_sync_round(fW, dG, fWc, float(ETA), float(RHO), N=N)
            hip.easgd_sync_round(dW, dG, dWc, float(ETA), float(RHO), N=N)
            oracle.easgd_round(W, G, Wc, ETA, RHO, N=N)
        if t % 10 == 0:
            worst_forced = max(worst_forced, normwise(to_host(fW), W), normwise(to_host(fWc), Wc))
            if momentum:
                worst_forced = max(worst_forced, normwise(to_host(fV), V))
    assert worst_forced <= PER_ROUND_TOL
    assert normwise(to_host(dW), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= HUNDRED_ROUND_TOL
    if momentum:
        assert normwise(to_host(dV), V) <= HUNDRED_ROUND_TOL


def test_bitwise_reproducible_and_independent_of_launch_shape(hip):
    P, N = 16, 1_200_007        # large enough for the one-thread-per-group kernel, which the options shape
    ld = workloads.round_up(N, 4)
    W, Wc = workloads.update_state(P, N, ld, seed=14)
    G = workloads.update_gradients(P, N, 0, ld, seed=14)
    V = workloads.update_gradients(P, N, 1, ld, seed=14)
    results = []
    saved = [hip.get_option(o) for o in (1, 2, 3, 9)]
    try:
        for blocks_per_cu, nt, groups, layout in [(0, 1, 0, 2), (0, 1, 0, 2), (4, 0, 2, 0), (1, 1, 1, 0), (8, 0, 4, 0),
                                                  (0, 1, 4, 1), (0, 0, 8, 1), (2, 1, 8, 1), (3, 0, 1, 1), (0, 1, 2, 1),
                                                  (0, 1, 8, 0)]:
            hip.set_option(hip.OPT_UPDATE_BLOCKS_PER_CU, blocks_per_cu)
            hip.set_option(hip.OPT_UPDATE_NONTEMPORAL, nt)
            hip.set_option(hip.OPT_UPDATE_GROUPS, groups)
            hip.set_option(hip.OPT_UPDATE_LAYOUT, layout)
            dW, dG, dWc, dV = to_dev(W), to_dev(G), to_dev(Wc), to_dev(V)
            hip.easgd_sync_round(dW, dG, dWc, 0.01, 0.1, N=N)
            hip.measgd_round(dW, dV, dG, dWc, 0.01, 0.1, 0.9, N=N)
            results.append((to_host(dW), to_host(dV), to_host(dWc)))
    finally:
        for o, v in zip((1, 2, 3, 9), saved):
            hip.set_option(o, v)
    for r in results[1:]:
        for a, b in zip(results[0], r):
            assert np.array_equal(a, b, equal_nan=True)


def test_invariants_on_the_gpu(hip):
    """Identical start: the center must not move; zero gradients: sum_i W_i + Wc is conserved."""
    P, N = 6, 5000
    w0 = (np.random.default_rng(0).standard_normal(N) * 0.1).astype(F)
    dW = to_dev(np.tile(w0, (P, 1))); dWc = to_dev(w0)
    G = workloads.update_gradients(P, N, 0, seed=15)
    hip.easgd_sync_round(dW, to_dev(G), dWc, 0.05, 0.3)
    np.testing.assert_array_equal(to_host(dWc), w0)
    W, Wc = workloads.update_state(P, N, seed=15, std=1.0)
    dW, dWc = to_dev(W), to_dev(Wc)
    zero = torch.zeros_like(dW)
    total0 = W.astype(np.float64).sum(0) + Wc
    for _ in range(50):
        hip.easgd_sync_round(dW, zero, dWc, 0.1, 0.3)
    total = to_host(dW).astype(np.float64).sum(0) + to_host(dWc)
    assert np.abs(total - total0).max() < 5e-5


def _full_size_sampled(hip, name, rounds):
    """Full-size update-only workload: the GPU runs every column, the oracle the sampled ones."""
    wl = workloads.WORKLOADS[name]
    P, N = wl.P, wl.N
    eta, rho = F(wl.eta), F(wl.rho)
    idx = workloads.sample_columns(N)
    tidx = torch.from_numpy(idx).cuda()
    dW = workloads.device_normal((P, N), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 1)
    dWc = workloads.device_normal((N,), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 2)
    dV = torch.zeros_like(dW) if wl.momentum else None
    W = to_host(dW[:, tidx]).copy(); Wc = to_host(dWc[tidx]).copy()
    V = np.zeros_like(W)
    for t in range(rounds):
        dG = workloads.device_normal((P, N), workloads.GRADIENT_STD, workloads.DEFAULT_SEED, 100 + t)
        G = to_host(dG[:, tidx]).copy()
        if wl.momentum:
            hip.measgd_round(dW, dV, dG, dWc, float(eta), float(rho), float(wl.delta))
            oracle.measgd_round(W, V, G, Wc, eta, rho, F(wl.delta))
        else:
            hip.easgd_sync_round(dW, dG, dWc, float(eta), float(rho))
            oracle.easgd_round(W, G, Wc, eta, rho)
        if t == 0:
            assert normwise(to_host(dW[:, tidx]), W) <= PER_ROUND_TOL
            assert normwise(to_host(dWc[tidx]), Wc) <= PER_ROUND_TOL
        del dG
    assert normwise(to_host(dW[:, tidx]), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc[tidx]), Wc) <= HUNDRED_ROUND_TOL
    if wl.momentum:
        assert normwise(to_host(dV[:, tidx]), V) <= HUNDRED_ROUND_TOL
    assert bool(torch.isfinite(dW).all()) and bool(torch.isfinite(dWc).all())


def test_cfg4_full_size_100_rounds_sampled(hip):
    _full_size_sampled(hip, "cfg4", 100)


def test_cfg5_full_size_100_rounds_sampled(hip):
    _full_size_sampled(hip, "cfg5", 100)


def _nearest_f32(x):
    """The float32 nearest to the exact rational x, ties to the even mantissa."""
    from fractions import Fraction
    guess = np.float32(float(x))
    cands = (np.nextafter(guess, np.float32(-np.inf)), guess, np.nextafter(guess, np.float32(np.inf)))
    return min(cands, key=lambda c: (abs(Fraction(float(c)) - x), int(np.float32(c).view(np.uint32)) & 1))


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_bits_are_those_of_the_arithmetic_the_header_states(hip, momentum):
    """include/easgd.h fixes which products of the rules are fused.  Exact rational arithmetic, rounded where the
    header says a rounding happens, must give the kernels' bits: the 128-bit path (two tiles and their ragged end),
    the scalar tail and, through an unaligned ld, the scalar kernel."""
    from fractions import Fraction as Q
    P, N = 3, 2307
    rnd, q = _nearest_f32, lambda a: Q(float(a))
    fma = lambda a, b, c: rnd(q(a) * q(b) + q(c))
    alpha = F(ETA * RHO)
    for ld in (2308, 2309):
        W, Wc = workloads.update_state(P, N, ld, seed=19)
        G = workloads.update_gradients(P, N, 0, ld, seed=19)
        V = workloads.update_gradients(P, N, 7, ld, seed=19, std=0.005)
        dW, dG, dWc, dV = to_dev(W), to_dev(G), to_dev(Wc), to_dev(V)
        if momentum:
            hip.measgd_round(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
        else:
            hip.easgd_sync_round(dW, dG, dWc, float(ETA), float(RHO), N=N)
        gW, gV, gWc = to_host(dW), to_host(dV), to_host(dWc)
        for j in range(N):
            c, acc = Wc[j], F(0)
            for i in range(P):
                d = rnd(q(W[i, j]) - q(c))
                acc = d if i == 0 else rnd(q(acc) + q(d))
                if momentum:
                    v = fma(DELTA, V[i, j], -rnd(q(ETA) * q(G[i, j])))                # Eq. (5)
                    w = fma(-alpha, d, rnd(q(W[i, j]) + q(v)))                          # Eq. (6)
                    assert gV[i, j].view(np.uint32) == F(v).view(np.uint32), (ld, i, j)
                else:
                    w = fma(-ETA, fma(RHO, d, G[i, j]), W[i, j])                        # Eq. (1)
                assert gW[i, j].view(np.uint32) == F(w).view(np.uint32), (ld, i, j)
            assert gWc[j].view(np.uint32) == F(fma(alpha, acc, c)).view(np.uint32), (ld, j)   # Eq. (2)
