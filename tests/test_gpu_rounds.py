"""Whole Sync EASGD rounds (gradient + elastic update) on the GPU against the oracle: the three
training workloads, free-running over all their rounds and teacher-forced per round."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


def _oracle_round(wl, W, V, Wc, X, y):
    G, loss = oracle.mlp_grad_all_workers(wl.dims, W, X, y)
    if wl.momentum:
        oracle.measgd_round(W, V, G, Wc, F(wl.eta), F(wl.rho), F(wl.delta), N=wl.N)
    else:
        oracle.easgd_round(W, G, Wc, F(wl.eta), F(wl.rho), N=wl.N)
    return loss


def _gpu_round(hip, wl, dW, dV, dWc, dG, dX, dy, ws):
    hip.easgd_grad(wl.dims, dW, dX, dy, dG, None, workspace=ws)
    if wl.momentum:
        hip.measgd_round(dW, dV, dG, dWc, wl.eta, wl.rho, wl.delta, N=wl.N)
    else:
        hip.easgd_sync_round(dW, dG, dWc, wl.eta, wl.rho, N=wl.N)


@pytest.mark.parametrize("name,rounds,forced_every", [("cfg1", 10, 1), ("cfg2", 50, 10), ("cfg3", 20, 10)])
def test_training_rounds(hip, name, rounds, forced_every):
    wl = workloads.WORKLOADS[name]
    assert rounds == wl.rounds
    ld = workloads.round_up(wl.N, 4)
    w0 = workloads.init_packed_weights(wl)
    W = workloads.replicate(w0, wl.P, ld); Wc = w0.copy()
    V = np.zeros_like(W); V[:, wl.N:] = np.nan
    dW, dWc, dV = to_dev(W), to_dev(Wc), to_dev(V)
    dG = torch.full_like(dW, float("nan"))
    ws = torch.empty(hip.easgd_grad_workspace_bytes(wl.dims, wl.P, wl.batch), dtype=torch.uint8, device="cuda")
    worst_forced = 0.0
    first_loss = last_loss = None
    for t in range(rounds):
        X, y = workloads.minibatch(wl, t)
        dX, dy = to_dev(X), to_dev(y)
        forced = (t % forced_every == 0) or t == rounds - 1
        if forced:      # one GPU round started from the oracle's state of this round
            fW, fWc, fV = to_dev(W), to_dev(Wc), to_dev(V)
            _gpu_round(hip, wl, fW, fV, fWc, dG, dX, dy, ws)
        _gpu_round(hip, wl, dW, dV, dWc, dG, dX, dy, ws)
        loss = _oracle_round(wl, W, V, Wc, X, y)
        first_loss = loss.mean() if first_loss is None else first_loss
        last_loss = loss.mean()
        if forced:
            worst_forced = max(worst_forced, normwise(to_host(fW), W), normwise(to_host(fWc), Wc))
            if wl.momentum:
                worst_forced = max(worst_forced, normwise(to_host(fV), V))
        if t == 0:      # identical start: the center does not move in the first round
            np.testing.assert_array_equal(to_host(dWc), w0)
    assert worst_forced <= PER_ROUND_TOL
    assert normwise(to_host(dW), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= HUNDRED_ROUND_TOL
    if wl.momentum:
        assert normwise(to_host(dV), V) <= HUNDRED_ROUND_TOL
    assert np.isfinite(last_loss) and np.isfinite(first_loss)
