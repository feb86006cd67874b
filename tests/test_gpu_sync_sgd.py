"""HIP sync_sgd_round (synchronous data-parallel SGD on the replicas: every replica moves by the sum of all
workers' gradients, Section 2.3 / Section 6.2; momentum Eq. (3),(4)) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32
ETA, MU = F(0.01), F(0.9)


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


# (P, N, ld): one element, ragged tails (N % 4 = 1, 2, 3), ld > N, several tiles, many workers
SHAPES = [(1, 1, 4), (2, 3, 4), (9, 261, 264), (4, 7850, 7852), (3, 4099, 4100), (8, 100_003, 100_004),
          (16, 33_333, 33_336), (5, 1 << 20, 1 << 20), (64, 65_537, 65_540), (7, 1026, 2048)]


@pytest.mark.parametrize("P,N,ld", SHAPES)
@pytest.mark.parametrize("momentum", [False, True], ids=["sgd", "msgd"])
def test_one_round_matches_oracle(hip, P, N, ld, momentum):
    W, _ = workloads.update_state(P, N, ld, seed=41)
    G = workloads.update_gradients(P, N, 0, ld, seed=41)
    V = workloads.update_gradients(P, N, 99, ld, seed=41, std=0.005)
    dW, dG, dV = to_dev(W), to_dev(G), to_dev(V)
    if momentum:
        hip.sync_sgd_round(dW, dG, float(ETA), V=dV, delta=float(MU), N=N)
        oracle.sync_sgd_round(W, G, ETA, V=V, mu=MU, N=N)
        assert normwise(to_host(dV), V) <= PER_ROUND_TOL
    else:
        hip.sync_sgd_round(dW, dG, float(ETA), N=N)
        oracle.sync_sgd_round(W, G, ETA, N=N)
        np.testing.assert_array_equal(to_host(dV), V)        # untouched without momentum
    assert normwise(to_host(dW), W) <= PER_ROUND_TOL          # also checks that NaN padding stayed NaN
    np.testing.assert_array_equal(to_host(dG), G)              # gradients are read-only


@pytest.mark.parametrize("momentum", [False, True], ids=["sgd", "msgd"])
def test_unaligned_operands_take_the_scalar_path(hip, momentum):
    P, N = 3, 1001
    for ld, shift in [(1003, 0), (1004, 1), (1001, 3)]:
        W, _ = workloads.update_state(P, N, ld, seed=42)
        G = workloads.update_gradients(P, N, 0, ld, seed=42)
        V = workloads.update_gradients(P, N, 5, ld, seed=42)

        def carve(a):   # operands at an element offset inside larger buffers: base not 16-byte aligned
            buf = torch.full((a.size + 8,), float("nan"), dtype=torch.float32, device="cuda")
            view = buf[shift:shift + a.size].view(a.shape)
            view.copy_(torch.from_numpy(a))
            return buf, view
        bW, dW = carve(W); bG, dG = carve(G); bV, dV = carve(V)
        hip.sync_sgd_round(dW, dG, float(ETA), V=dV if momentum else None, delta=float(MU), N=N)
        oracle.sync_sgd_round(W, G, ETA, V=V if momentum else None, mu=MU, N=N)
        assert normwise(to_host(dW), W) <= PER_ROUND_TOL
        if momentum:
            assert normwise(to_host(dV), V) <= PER_ROUND_TOL
        for buf, a in ((bW, W), (bG, G), (bV, V)):             # nothing outside the operands was written
            h = buf.cpu().numpy()
            assert np.isnan(h[:shift]).all() and np.isnan(h[shift + a.size:]).all()


def test_identical_replicas_stay_identical_over_100_rounds(hip):
    """The broadcast of W holds by construction: replicas that start equal stay equal bit for bit; and 100
    free-running rounds stay within the 100-round tolerance of the oracle."""
    P, N = 8, 300_007
    ld = workloads.round_up(N, 4)
    w0 = (np.random.default_rng(43).standard_normal(N) * 0.01).astype(F)
    W = workloads.replicate(w0, P, ld)
    V = np.zeros_like(W); V[:, N:] = np.nan
    dW, dV = to_dev(W), to_dev(V)
    for t in range(100):
        G = workloads.update_gradients(P, N, t, ld, seed=43)
        hip.sync_sgd_round(dW, to_dev(G), float(ETA), V=dV, delta=float(MU), N=N)
        oracle.sync_sgd_round(W, G, ETA, V=V, mu=MU, N=N)
    hW, hV = to_host(dW), to_host(dV)
    for i in range(1, P):
        np.testing.assert_array_equal(hW[i, :N], hW[0, :N])
        np.testing.assert_array_equal(hV[i, :N], hV[0, :N])
    assert normwise(hW, W) <= HUNDRED_ROUND_TOL and normwise(hV, V) <= HUNDRED_ROUND_TOL


def test_results_do_not_depend_on_launch_shape_options(hip):
    P, N = 6, 1_200_007
    ld = workloads.round_up(N, 4)
    W, _ = workloads.update_state(P, N, ld, seed=44)
    G = workloads.update_gradients(P, N, 0, ld, seed=44)
    ref = None
    old = (hip.get_option(hip.OPT_UPDATE_GROUPS), hip.get_option(hip.OPT_UPDATE_NONTEMPORAL), hip.get_option(hip.OPT_UPDATE_LAYOUT))
    try:
        for groups, layout in ((0, 2), (1, 0), (2, 0), (4, 0), (8, 0), (1, 1), (2, 1), (4, 1), (8, 1)):
            for nt in (0, 1):
                hip.set_option(hip.OPT_UPDATE_GROUPS, groups); hip.set_option(hip.OPT_UPDATE_NONTEMPORAL, nt)
                hip.set_option(hip.OPT_UPDATE_LAYOUT, layout)
                dW = to_dev(W)
                hip.sync_sgd_round(dW, to_dev(G), float(ETA), N=N)
                out = to_host(dW)
                if ref is None:
                    ref = out
                else:
                    np.testing.assert_array_equal(out, ref)
    finally:
        hip.set_option(hip.OPT_UPDATE_GROUPS, old[0]); hip.set_option(hip.OPT_UPDATE_NONTEMPORAL, old[1])
        hip.set_option(hip.OPT_UPDATE_LAYOUT, old[2])


def test_full_size_on_sampled_columns(hip):
    """AlexNet-size replicas (P = 8 x 61 M, the launch configuration the benchmark times): 20 rounds, compared
    with the oracle on sampled parameter columns (the update is independent per parameter)."""
    P, N = 8, 61_000_000
    cols = torch.from_numpy(workloads.sample_columns(N, seed=45)).cuda()
    dW = workloads.device_normal((P, N), workloads.WEIGHT_STD, 45, 1)
    dV = torch.zeros_like(dW)
    W = dW[:, cols].cpu().numpy().copy(); V = np.zeros_like(W)
    for t in range(20):
        dG = workloads.device_normal((P, N), workloads.GRADIENT_STD, 45, 100 + t)
        G = dG[:, cols].cpu().numpy().copy()
        hip.sync_sgd_round(dW, dG, float(ETA), V=dV, delta=float(MU))
        oracle.sync_sgd_round(W, G, ETA, V=V, mu=MU)
        del dG
    assert normwise(dW[:, cols].cpu().numpy(), W) <= HUNDRED_ROUND_TOL
    assert normwise(dV[:, cols].cpu().numpy(), V) <= HUNDRED_ROUND_TOL
