"""HIP easgd_grad (batched MFMA forward/backward) against the CPU gradient oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import PER_ROUND_TOL, match_gradient, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


def _problem(dims, P, b, ld_pad=0, seed=21, x_dist="normal", distinct=True):
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=0.1, rho=0.1, rounds=1, dims=tuple(dims), batch=b, N=N, x_dist=x_dist)
    w0 = workloads.init_packed_weights(wl, seed=seed)
    ld = workloads.round_up(N, 4) + ld_pad
    W = workloads.replicate(w0, P, ld)
    if distinct:   # replicas drift apart during training: give every worker its own weights and non-zero biases
        rng = np.random.default_rng(seed)
        W[:, :N] += (rng.standard_normal((P, N)) * 0.02).astype(F)
    X, y = workloads.minibatch(wl, 0, seed=seed)
    return N, ld, W, X, y


def _run(hip, dims, W, X, y, loss=True):
    P, ld = W.shape
    dW, dX, dy = to_dev(W), to_dev(X), to_dev(y)
    dG = torch.full((P, ld), float("nan"), dtype=torch.float32, device="cuda")
    dloss = torch.full((P,), float("nan"), dtype=torch.float32, device="cuda") if loss else None
    hip.easgd_grad(dims, dW, dX, dy, dG, dloss)
    np.testing.assert_array_equal(to_host(dW), W)     # weights are read-only
    return to_host(dG), (to_host(dloss) if loss else None)


# dims, P, b: tiny; softmax regression (cfg1 shape); widths not multiples of 4 (scalar loads);
# batch 100 (ragged against the 32-row MFMA tile); 3 hidden layers; 64x64 and 128x128 tile routes
CASES = [
    ((5, 4, 3), 2, 3),
    ((784, 10), 4, 64),
    ((33, 17, 10), 3, 25),
    ((50, 70, 30, 7), 2, 100),
    ((784, 256, 128, 10), 3, 100),
    ((96, 200, 136, 64, 12), 5, 37),
    ((512, 384, 10), 40, 128),
    ((130, 1000), 2, 9),
]


@pytest.mark.parametrize("dims,P,b", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_gradient_matches_oracle(hip, dims, P, b):
    N, ld, W, X, y = _problem(dims, P, b, ld_pad=4)
    G, loss = _run(hip, dims, W, X, y)
    G_ref, loss_ref = oracle.mlp_grad_all_workers(dims, W, X, y)
    assert np.isnan(G[:, N:]).all()                   # padding untouched
    assert np.isfinite(G[:, :N]).all()                # every valid entry written
    sl = oracle.layer_slices(dims)
    for i in range(P):
        assert normwise(G[i], G_ref[i]) <= PER_ROUND_TOL
        for w_sl, b_sl in sl:                         # and per layer block, so that small blocks count
            assert normwise(G[i, w_sl], G_ref[i, w_sl]) <= 2 * PER_ROUND_TOL
            assert normwise(G[i, b_sl], G_ref[i, b_sl]) <= 2 * PER_ROUND_TOL
    np.testing.assert_allclose(loss, loss_ref, rtol=1e-5)


def test_loss_pointer_may_be_null_and_runs_are_bitwise_reproducible(hip):
    dims = (784, 256, 128, 10)
    N, ld, W, X, y = _problem(dims, 3, 100)
    G1, _ = _run(hip, dims, W, X, y, loss=False)
    G2, loss = _run(hip, dims, W, X, y, loss=True)
    assert np.array_equal(G1, G2, equal_nan=True)


def test_zero_weights_closed_form(hip):
    dims = (64, 32, 10)
    N = workloads.mlp_num_params(dims)
    P, b = 2, 16
    W = np.zeros((P, N), F)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((P, b, 64)).astype(F)
    y = rng.integers(0, 10, size=(P, b)).astype(np.int32)
    G, loss = _run(hip, dims, W, X, y)
    np.testing.assert_allclose(loss, np.log(10.0), rtol=1e-6)
    sl = oracle.layer_slices(dims)
    for i in range(P):
        freq = np.bincount(y[i], minlength=10) / b
        np.testing.assert_allclose(G[i, sl[1][1]], 0.1 - freq, atol=1e-7)
        assert not G[i, sl[0][0]].any() and not G[i, sl[1][0]].any()


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_full_shape_one_round(hip, name):
    """The benchmark shapes, in the launch configuration the benchmark times."""
    wl = workloads.WORKLOADS[name]
    N, ld, W, X, y = _problem(wl.dims, wl.P, wl.batch, seed=22, x_dist=wl.x_dist)
    G, loss = _run(hip, wl.dims, W, X, y)
    # the oracle handles a sample of the workers (every worker is an independent problem)
    for i in sorted({0, 1, wl.P // 2, wl.P - 1}):
        _, loss_ref, flipped = match_gradient(G[i], wl.dims, W[i], X[i], y[i], PER_ROUND_TOL)
        print(f"{name} worker {i}: {flipped} near-zero ReLU gate(s) decided differently in fp32")
        assert abs(loss[i] - loss_ref) <= 1e-5 * abs(loss_ref)
    assert np.isfinite(G[:, :N]).all()


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
def test_every_tile_shape_gives_the_same_gradient(hip, tile):
    """The block-tile option only changes the launch shape: each forced shape must match the oracle."""
    dims, P, b = (200, 264, 136, 10), 3, 100
    N, ld, W, X, y = _problem(dims, P, b)
    old = hip.get_option(hip.OPT_GEMM_TILE)
    try:
        hip.set_option(hip.OPT_GEMM_TILE, tile)
        G, loss = _run(hip, dims, W, X, y)
    finally:
        hip.set_option(hip.OPT_GEMM_TILE, old)
    for i in range(P):
        _, loss_ref, _ = match_gradient(G[i], dims, W[i], X[i], y[i], PER_ROUND_TOL)
        assert abs(loss[i] - loss_ref) <= 1e-5 * abs(loss_ref)


# Last layers that take the single-launch head (at most 16 classes) and ones that do not; a single-layer network;
# one class; 16 and 17 classes; widths that are no multiple of 4 or of the 256 columns the threads of a block
# cover; hidden layers wider than one pass of 1024 columns (one, two and several passes); a single row and a
# ragged last row group per worker.
HEAD_CASES = [
    ((784, 10), 4, 64),
    ((300, 3), 2, 7),
    ((12, 9, 1), 2, 5),
    ((40, 64, 16), 3, 8),
    ((40, 64, 17), 3, 8),
    ((31, 1027, 10), 2, 9),
    ((64, 2050, 7), 2, 1),
    ((16, 3000, 10), 2, 19),
    ((16, 3300, 10), 1, 4),
    ((20, 1024, 12), 8, 16),
    ((20, 1025, 5), 9, 17),
]


@pytest.mark.parametrize("dims,P,b", HEAD_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_head_of_the_network_in_one_launch_or_three(hip, dims, P, b):
    """EASGD_OPT_MLP_HEAD only changes how the last layer is launched: both ways match the oracle."""
    N, ld, W, X, y = _problem(dims, P, b, ld_pad=4)
    G_ref, loss_ref = oracle.mlp_grad_all_workers(dims, W, X, y)
    sl = oracle.layer_slices(dims)
    old = hip.get_option(hip.OPT_MLP_HEAD)
    got = {}
    try:
        for head in (1, 0):
            hip.set_option(hip.OPT_MLP_HEAD, head)
            G, loss = _run(hip, dims, W, X, y)
            got[head] = G
            assert np.isnan(G[:, N:]).all() and np.isfinite(G[:, :N]).all()
            for i in range(P):
                assert normwise(G[i], G_ref[i]) <= PER_ROUND_TOL
                for w_sl, b_sl in sl:
                    assert normwise(G[i, w_sl], G_ref[i, w_sl]) <= 2 * PER_ROUND_TOL
                    assert normwise(G[i, b_sl], G_ref[i, b_sl]) <= 2 * PER_ROUND_TOL
            np.testing.assert_allclose(loss, loss_ref, rtol=1e-5)
    finally:
        hip.set_option(hip.OPT_MLP_HEAD, old)
    for i in range(P):
        assert normwise(got[1][i], got[0][i]) <= PER_ROUND_TOL
