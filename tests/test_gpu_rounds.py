"""Whole Sync EASGD rounds (gradient + elastic update) on the GPU against the oracle: the three
training workloads over all their rounds, free-running and teacher-forced.

A hidden unit whose pre-activation is within fp32 rounding of zero has a ReLU gate that fp32 and fp64
arithmetic may decide differently; both gradients are valid.  The oracle side therefore resolves such
ties per worker and per round towards the valid alternative that the GPU gradient matches
(gpu_util.match_gradient enumerates the oracle's own near-zero units); everything else is unique and is
compared at the stated tolerance."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import (HUNDRED_ROUND_TOL, PER_ROUND_TOL, match_gradients_all_workers, normwise,
                      oracle_gradient_base, to_dev, to_host)

pytestmark = pytest.mark.gpu
F = np.float32
# free-running: the two trajectories already differ by rounding when their gradients are matched, so both
# the match tolerance and the "near zero" band of the ReLU gates are wider than in the teacher-forced check
FREE_RUNNING_MATCH_TOL = 5e-5
FREE_RUNNING_NEAR_REL = 4e-5


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


def _oracle_update(wl, W, V, Wc, G):
    if wl.momentum:
        oracle.measgd_round(W, V, G, Wc, F(wl.eta), F(wl.rho), F(wl.delta), N=wl.N)
    else:
        oracle.easgd_round(W, G, Wc, F(wl.eta), F(wl.rho), N=wl.N)


def _gpu_round(hip, wl, dW, dV, dWc, dG, dX, dy, ws, path):
    if path == "one_call":      # the fused whole-round entry point; the gradients are kept for the tie matching
        hip.easgd_mlp_round(wl.dims, dW, dWc, dX, dy, wl.eta, wl.rho, V=dV if wl.momentum else None,
                            delta=wl.delta or 0.0, G=dG, workspace=ws)
        return
    hip.easgd_grad(wl.dims, dW, dX, dy, dG, None, workspace=ws)
    if wl.momentum:
        hip.measgd_round(dW, dV, dG, dWc, wl.eta, wl.rho, wl.delta, N=wl.N)
    else:
        hip.easgd_sync_round(dW, dG, dWc, wl.eta, wl.rho, N=wl.N)


@pytest.mark.parametrize("path", ["two_calls", "one_call"])
@pytest.mark.parametrize("name,rounds,forced_every", [("cfg1", 10, 1), ("cfg2", 50, 1), ("cfg3", 20, 1)])
def test_training_rounds(hip, name, rounds, forced_every, path, progress):
    wl = workloads.WORKLOADS[name]
    assert rounds == wl.rounds
    ld = workloads.round_up(wl.N, 4)
    w0 = workloads.init_packed_weights(wl)
    W = workloads.replicate(w0, wl.P, ld); Wc = w0.copy()
    V = np.zeros_like(W); V[:, wl.N:] = np.nan
    dW, dWc, dV = to_dev(W), to_dev(Wc), to_dev(V)
    dG = torch.full_like(dW, float("nan"))
    fG = torch.full_like(dW, float("nan"))
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(wl.dims, wl.P, wl.batch), dtype=torch.uint8, device="cuda")
    worst_forced, ties = 0.0, 0
    losses = []
    for t in range(rounds):
        X, y = workloads.minibatch(wl, t)
        dX, dy = to_dev(X), to_dev(y)
        # the oracle's gradient at its own state: both comparisons of this round start from it
        bases = [oracle_gradient_base(wl.dims, W[i], X[i], y[i], FREE_RUNNING_NEAR_REL) for i in range(wl.P)]
        if (t % forced_every == 0) or t == rounds - 1:
            # teacher-forced: one GPU round started from the oracle's state of this round
            fW, fWc, fV = to_dev(W), to_dev(Wc), to_dev(V)
            _gpu_round(hip, wl, fW, fV, fWc, fG, dX, dy, ws, path)
            Gf, _, k = match_gradients_all_workers(to_host(fG), wl.dims, W, X, y, PER_ROUND_TOL, bases=bases)
            ties += k
            W1, V1, Wc1 = W.copy(), V.copy(), Wc.copy()
            _oracle_update(wl, W1, V1, Wc1, Gf)
            worst_forced = max(worst_forced, normwise(to_host(fW), W1), normwise(to_host(fWc), Wc1))
            if wl.momentum:
                worst_forced = max(worst_forced, normwise(to_host(fV), V1))
        # free-running: both sides continue from their own state
        _gpu_round(hip, wl, dW, dV, dWc, dG, dX, dy, ws, path)
        G, loss, k = match_gradients_all_workers(to_host(dG), wl.dims, W, X, y, FREE_RUNNING_MATCH_TOL,
                                                 FREE_RUNNING_NEAR_REL, bases=bases)
        ties += k
        if wl.N > 5_000_000 or t % 10 == 9:
            progress(f"  {name} {path} round {t + 1}/{rounds}: {ties} gate tie(s) so far, teacher-forced worst {worst_forced:.2e}")
        _oracle_update(wl, W, V, Wc, G)
        losses.append(loss.mean())
        if t == 0:      # identical start: the center does not move in the first round
            np.testing.assert_array_equal(to_host(dWc), w0)
    print(f"{name} {path}: {ties} near-zero ReLU gate(s) resolved; teacher-forced worst {worst_forced:.2e}; "
          f"free-running W {normwise(to_host(dW), W):.2e} Wc {normwise(to_host(dWc), Wc):.2e}; "
          f"loss {losses[0]:.4f} -> {losses[-1]:.4f}")
    assert worst_forced <= PER_ROUND_TOL
    assert normwise(to_host(dW), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= HUNDRED_ROUND_TOL
    if wl.momentum:
        assert normwise(to_host(dV), V) <= HUNDRED_ROUND_TOL
    assert np.isfinite(losses).all()


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_the_call_the_benchmark_times(hip, name):
    """The configuration the benchmark times: one easgd_mlp_round at the workload's full shape that stores no
    gradient (G = NULL), under the library's default options (center rule placed per call, die-interleaved block
    order, shared launches, single-launch head).  From a state a few rounds into training (replicas apart, a
    center of its own, non-zero momentum) it must give the bits of the same call with the gradient kept, and
    match the oracle's round, whose gate ties are resolved against that kept gradient."""
    wl = workloads.WORKLOADS[name]
    for opt, default in ((hip.OPT_ROUND_OVERLAP, 1), (hip.OPT_GEMM_XCD, 1), (hip.OPT_GEMM_PAIR, 1),
                         (hip.OPT_MLP_HEAD, 1), (hip.OPT_GEMM_TILE, 0)):
        assert hip.get_option(opt) == default
    N, P = wl.N, wl.P
    ld = workloads.round_up(N, 4)
    w0 = workloads.init_packed_weights(wl)
    rng = np.random.default_rng(77)
    W = workloads.replicate(w0, P, ld)
    for i in range(P):
        W[i, :N] += rng.standard_normal(N, dtype=F) * F(0.004)
    Wc = w0 + rng.standard_normal(N, dtype=F) * F(0.002)
    V = np.full_like(W, np.nan)
    for i in range(P):
        V[i, :N] = rng.standard_normal(N, dtype=F) * F(1e-3)
    X, y = workloads.minibatch(wl, 3)
    dX, dy = to_dev(X), to_dev(y)
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(wl.dims, P, wl.batch), dtype=torch.uint8, device="cuda")
    out = []
    for keep in (False, True):
        dW, dWc, dV = to_dev(W), to_dev(Wc), to_dev(V)
        dG = torch.full_like(dW, float("nan")) if keep else None
        dloss = torch.empty(P, device="cuda")
        hip.easgd_mlp_round(wl.dims, dW, dWc, dX, dy, wl.eta, wl.rho, V=dV if wl.momentum else None,
                            delta=wl.delta or 0.0, G=dG, loss=dloss, workspace=ws)
        out.append((to_host(dW), to_host(dWc), to_host(dV), to_host(dloss)))
        if keep:
            G_gpu = to_host(dG)
    for a, c in zip(out[0], out[1]):
        np.testing.assert_array_equal(a, c)                    # storing the gradient changes nothing else
    G, loss, ties = match_gradients_all_workers(G_gpu, wl.dims, W, X, y, PER_ROUND_TOL)
    oW, oV, oWc = W.copy(), V.copy(), Wc.copy()
    _oracle_update(wl, oW, oV, oWc, G)
    gW, gWc, gV, gloss = out[0]
    errs = {"W": normwise(gW, oW), "Wc": normwise(gWc, oWc)}
    if wl.momentum:
        errs["V"] = normwise(gV, oV)
    else:
        np.testing.assert_array_equal(gV, V)
    print(f"{name} as timed (G=NULL, default options): {ties} gate tie(s), errors {errs}")
    assert max(errs.values()) <= PER_ROUND_TOL
    np.testing.assert_allclose(gloss, loss, rtol=1e-5)
    assert not np.array_equal(gWc, Wc)
