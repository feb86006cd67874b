"""The gradient oracle against closed forms, finite differences and torch autograd (CPU, fp64)."""
import numpy as np
import pytest
import torch

import oracle
import workloads

F = np.float32


def _random_problem(dims, b, seed, scale=0.5):
    rng = np.random.default_rng(seed)
    N = workloads.mlp_num_params(dims)
    w = (rng.standard_normal(N) * scale).astype(F)
    X = rng.standard_normal((b, dims[0])).astype(F)
    y = rng.integers(0, dims[-1], size=b).astype(np.int32)
    return w, X, y


def _loss_double(dims, w64, X, y):
    """Independent forward pass in double with explicit Python loops (tiny sizes only)."""
    off = 0
    a = [[float(v) for v in row] for row in X]
    L = len(dims) - 1
    for l in range(L):
        d_in, d_out = dims[l], dims[l + 1]
        Wl = w64[off:off + d_in * d_out]; off += d_in * d_out
        bl = w64[off:off + d_out]; off += d_out
        z = [[sum(a[n][k] * Wl[k * d_out + j] for k in range(d_in)) + bl[j] for j in range(d_out)]
             for n in range(len(a))]
        a = z if l == L - 1 else [[max(v, 0.0) for v in row] for row in z]
    total = 0.0
    for n, row in enumerate(a):
        m = max(row)
        lse = m + np.log(sum(np.exp(v - m) for v in row))
        total += lse - row[int(y[n])]
    return total / len(a)


def test_layer_slices_cover_the_packed_vector():
    dims = (7, 5, 3)
    sl = oracle.layer_slices(dims)
    assert sl[0] == (slice(0, 35), slice(35, 40))
    assert sl[1] == (slice(40, 55), slice(55, 58))
    for name, wl in workloads.WORKLOADS.items():
        if wl.dims:
            assert oracle.layer_slices(wl.dims)[-1][1].stop == wl.N
    assert workloads.WORKLOADS["cfg1"].N == 7850
    assert workloads.WORKLOADS["cfg2"].N == 1863690
    assert workloads.WORKLOADS["cfg3"].N == 10510346


def test_zero_weights_give_uniform_prediction():
    """All-zero parameters: p is uniform, loss = ln(C), dZ = (1/C - onehot)/b,
    so the last bias gradient is (count-independent) 1/C - freq(class) and hidden-layer gradients vanish."""
    dims = (6, 5, 4)
    b, C = 8, 4
    N = workloads.mlp_num_params(dims)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((b, 6)).astype(F)
    y = rng.integers(0, C, size=b).astype(np.int32)
    g, loss = oracle.mlp_grad(dims, np.zeros(N, F), X, y)
    assert abs(loss - np.log(C)) < 1e-12
    sl = oracle.layer_slices(dims)
    freq = np.bincount(y, minlength=C) / b
    np.testing.assert_allclose(g[sl[1][1]], 1.0 / C - freq, atol=1e-7)
    assert not g[sl[0][0]].any() and not g[sl[0][1]].any() and not g[sl[1][0]].any()


def test_softmax_regression_closed_form():
    """One layer: dW = X^T (p - onehot)/b, db = column sums; written with explicit loops."""
    dims = (4, 3)
    w, X, y = _random_problem(dims, b=5, seed=1)
    g, _ = oracle.mlp_grad(dims, w, X, y)
    Wm = w[:12].astype(np.float64).reshape(4, 3); bias = w[12:15].astype(np.float64)
    dW = np.zeros((4, 3)); db = np.zeros(3)
    for n in range(5):
        z = [sum(float(X[n, k]) * Wm[k, j] for k in range(4)) + bias[j] for j in range(3)]
        e = [np.exp(v - max(z)) for v in z]
        p = [v / sum(e) for v in e]
        for j in range(3):
            dz = (p[j] - (1.0 if y[n] == j else 0.0)) / 5
            db[j] += dz
            for k in range(4):
                dW[k, j] += float(X[n, k]) * dz
    np.testing.assert_allclose(g[:12].reshape(4, 3), dW, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(g[12:], db, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("dims,b", [((5, 4, 3), 3), ((6, 7, 5, 4), 4)])
def test_central_finite_differences(dims, b):
    w, X, y = _random_problem(dims, b, seed=2)
    g, loss = oracle.mlp_grad(dims, w, X, y)
    w64 = w.astype(np.float64)
    assert abs(loss - _loss_double(dims, w64, X, y)) < 1e-12
    h = 1e-6
    fd = np.zeros_like(w64)
    for k in range(len(w64)):
        wp, wm = w64.copy(), w64.copy()
        wp[k] += h; wm[k] -= h
        fd[k] = (_loss_double(dims, wp, X, y) - _loss_double(dims, wm, X, y)) / (2 * h)
    np.testing.assert_allclose(g, fd, rtol=0, atol=2e-7)


@pytest.mark.parametrize("dims,b", [((784, 10), 64), ((20, 33, 17, 10), 25), ((48, 64, 64, 10), 100)])
def test_against_torch_autograd(dims, b):
    """torch's cross_entropy (mean reduction) + autograd in fp64 is an independent library route
    to the same gradient; per-layer results concatenated must equal the packed gradient."""
    w, X, y = _random_problem(dims, b, seed=3, scale=0.2)
    g, loss = oracle.mlp_grad(dims, w, X, y)
    params = []
    off = 0
    for d_in, d_out in zip(dims[:-1], dims[1:]):
        Wl = torch.tensor(w[off:off + d_in * d_out].astype(np.float64).reshape(d_in, d_out), requires_grad=True)
        off += d_in * d_out
        bl = torch.tensor(w[off:off + d_out].astype(np.float64), requires_grad=True)
        off += d_out
        params += [Wl, bl]
    a = torch.tensor(X.astype(np.float64))
    for l in range(len(dims) - 1):
        a = a @ params[2 * l] + params[2 * l + 1]
        if l < len(dims) - 2:
            a = torch.relu(a)
    tl = torch.nn.functional.cross_entropy(a, torch.tensor(y.astype(np.int64)))
    tl.backward()
    ref = np.concatenate([p.grad.numpy().reshape(-1) for p in params])
    assert abs(loss - tl.item()) < 1e-12
    np.testing.assert_allclose(g, ref.astype(F), rtol=1e-6, atol=1e-9)


def test_last_bias_gradient_sums_to_zero_and_workers_are_independent():
    wl = workloads.Workload("t", P=3, eta=0.1, rho=0.1, rounds=1, dims=(12, 9, 4), batch=6,
                            N=workloads.mlp_num_params((12, 9, 4)))
    w0 = workloads.init_packed_weights(wl, seed=5)
    W = workloads.replicate(w0, wl.P, ld=wl.N + 3)
    W[1, :wl.N] += 0.1
    X, y = workloads.minibatch(wl, 0, seed=5)
    G, loss = oracle.mlp_grad_all_workers(wl.dims, W, X, y)
    assert np.isnan(G[:, wl.N:]).all()
    sl = oracle.layer_slices(wl.dims)
    np.testing.assert_allclose(G[:, sl[-1][1]].astype(np.float64).sum(1), 0, atol=1e-7)
    g1, l1 = oracle.mlp_grad(wl.dims, W[1], X[1], y[1])
    np.testing.assert_array_equal(G[1, :wl.N], g1)
    assert loss[1] == l1


def test_near_zero_gates_are_reported_and_flippable():
    """A hidden unit with pre-activation exactly 0 is a tie of the ReLU gate: the oracle reports it,
    and flipping its gate changes the gradient by that unit's back-propagated signal only."""
    dims = (3, 2, 2)
    w = np.array([1, 0, -1, 1, 0, 1, 0, 0,      # W0 (3x2), b0
                  1, -1, 2, 1, 0, 0], dtype=F)   # W1 (2x2), b1
    X = np.array([[2, 2, 1], [1, 1, 1]], dtype=F)   # sample 0: z = (0, 3); sample 1: z = (0, 2)
    y = np.array([0, 1], dtype=np.int32)
    near = []
    g0, _ = oracle.mlp_grad(dims, w, X, y, near_zero=near, near_zero_rel=1e-9)
    assert near == [(0, 0, 0), (0, 1, 0)]
    g1, _ = oracle.mlp_grad(dims, w, X, y, gate_flips=[(0, 0, 0)])
    changed = np.nonzero(g0 != g1)[0]
    # only column 0 of W0 (packed indices 0, 2, 4) and b0[0] (index 6) may change
    assert set(changed) <= {0, 2, 4, 6} and len(changed) > 0
    # gate closed (default, z == 0): no signal reaches column 0 from either sample
    assert g0[0] == 0 and g0[6] == 0
