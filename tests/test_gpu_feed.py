"""Rounds fed from pinned host memory through the double-buffered feeder (the data copy of the next round
overlaps the current round, Algorithm 3; the overlap of Sync EASGD3, Section 6.1.3): every fed round against the
oracle's round, and the fed rounds against rounds whose data is already resident (the same bits)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, match_gradients_all_workers, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32


def test_host_fed_rounds_equal_resident_rounds():
    import paper_1708_02983_amd as hip
    dims, P, b, rounds = (784, 160, 10), 8, 64, 9
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=0.05, rho=0.1, rounds=rounds, delta=0.9, dims=dims, batch=b, N=N)
    ld = workloads.round_up(N, 4)
    w0 = workloads.init_packed_weights(wl)
    W0 = workloads.replicate(w0, P, ld)
    batches = [workloads.minibatch(wl, t) for t in range(rounds)]

    def run(feed, snapshots=None, packed=False):
        W, Wc = to_dev(W0), to_dev(w0.copy())
        V = torch.zeros_like(W)
        V[:, N:] = float("nan")
        G = torch.full_like(W, float("nan")) if snapshots is not None else None
        ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(dims, P, b), dtype=torch.uint8, device="cuda")
        if not feed:
            for X, y in batches:
                hip.easgd_mlp_round(dims, W, Wc, to_dev(X), to_dev(y), wl.eta, wl.rho, V=V, delta=wl.delta, workspace=ws)
        else:
            feeder = hip.BatchFeeder(P, b, dims[0])
            if packed:                  # samples and labels back to back in one pinned buffer: one copy per round
                host = [feeder.host_batch() for _ in batches]
                for (hX, hy), (X, y) in zip(host, batches):
                    hX.copy_(torch.from_numpy(X)); hy.copy_(torch.from_numpy(y))
            else:
                host = [(torch.from_numpy(X).pin_memory(), torch.from_numpy(y).pin_memory()) for X, y in batches]
            feeder.submit(0, *host[0])
            for t in range(rounds):
                if t + 1 < rounds:
                    feeder.submit((t + 1) % 2, *host[t + 1])      # copy of round t+1 runs beside round t
                X, y = feeder.acquire(t % 2)
                hip.easgd_mlp_round(dims, W, Wc, X, y, wl.eta, wl.rho, V=V, delta=wl.delta, G=G, workspace=ws)
                feeder.release(t % 2)
                if snapshots is not None:      # device-side copies queued behind the round, read after the loop
                    snapshots.append((W.clone(), V.clone(), Wc.clone(), G.clone()))
        torch.cuda.synchronize()
        return to_host(W), to_host(V), to_host(Wc)

    ref = run(False)
    for attempt in range(3):        # a missing wait would show as a race, so run it more than once
        got = run(True, packed=(attempt % 2 == 1))
        for a, c in zip(ref, got):
            np.testing.assert_array_equal(a, c, err_msg=f"attempt {attempt}")
    assert np.isfinite(ref[2][:N]).all() and not np.array_equal(ref[2], w0)

    # the fed rounds against the oracle (Algorithm 3 with the five steps of Section 5.1; Eq. (5),(6),(2)):
    # teacher-forced (the oracle's round from the state the fed path held before round t) and free-running
    snaps = []
    kept = run(True, snaps, packed=True)
    for a, c in zip(ref, kept):
        np.testing.assert_array_equal(a, c)             # keeping the gradient changes nothing else
    V0 = np.zeros_like(W0); V0[:, N:] = np.nan
    W, V, Wc = W0.copy(), V0.copy(), w0.copy()           # free-running oracle state
    pW, pV, pWc = W0.copy(), V0.copy(), w0.copy()        # the fed path's state before round t
    worst = 0.0
    for t, (X, y) in enumerate(batches):
        gW, gV, gWc, gG = (to_host(a) for a in snaps[t])
        Gf, _, _ = match_gradients_all_workers(gG, dims, pW, X, y, PER_ROUND_TOL)
        oracle.measgd_round(pW, pV, Gf, pWc, F(wl.eta), F(wl.rho), F(wl.delta), N=N)
        worst = max(worst, normwise(gW, pW), normwise(gV, pV), normwise(gWc, pWc))
        pW, pV, pWc = gW.copy(), gV.copy(), gWc.copy()
        G, _ = oracle.mlp_grad_all_workers(dims, W, X, y)
        oracle.measgd_round(W, V, G, Wc, F(wl.eta), F(wl.rho), F(wl.delta), N=N)
    print(f"host-fed rounds against the oracle: teacher-forced worst {worst:.2e}; after {rounds} free-running rounds "
          f"W {normwise(kept[0], W):.2e} V {normwise(kept[1], V):.2e} Wc {normwise(kept[2], Wc):.2e}")
    assert worst <= PER_ROUND_TOL
    assert max(normwise(kept[0], W), normwise(kept[1], V), normwise(kept[2], Wc)) <= HUNDRED_ROUND_TOL


def test_several_rounds_per_copy_give_the_same_bits():
    """One copy, one wait and one release per three rounds (rounds_per_copy = 3): the same bits as rounds on
    resident data, with separate and with back-to-back host tensors."""
    import paper_1708_02983_amd as hip
    dims, P, b, rounds, g = (100, 48, 10), 4, 20, 9, 3
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=0.05, rho=0.1, rounds=rounds, delta=None, dims=dims, batch=b, N=N)
    ld = workloads.round_up(N, 4)
    w0 = workloads.init_packed_weights(wl)
    batches = [workloads.minibatch(wl, t) for t in range(rounds)]
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(dims, P, b), dtype=torch.uint8, device="cuda")
    W, Wc = to_dev(workloads.replicate(w0, P, ld)), to_dev(w0.copy())
    for X, y in batches:
        hip.easgd_mlp_round(dims, W, Wc, to_dev(X), to_dev(y), wl.eta, wl.rho, workspace=ws)
    ref = to_host(W), to_host(Wc)
    for packed in (False, True):
        feeder = hip.BatchFeeder(P, b, dims[0], rounds_per_copy=g)
        host = []
        for k in range(rounds // g):
            Xs = np.stack([batches[g * k + i][0] for i in range(g)]); ys = np.stack([batches[g * k + i][1] for i in range(g)])
            if packed:
                hX, hy = feeder.host_batch(); hX.copy_(torch.from_numpy(Xs)); hy.copy_(torch.from_numpy(ys))
            else:
                hX, hy = torch.from_numpy(Xs).pin_memory(), torch.from_numpy(ys).pin_memory()
            host.append((hX, hy))
        W, Wc = to_dev(workloads.replicate(w0, P, ld)), to_dev(w0.copy())
        feeder.submit(0, *host[0])
        for k in range(rounds // g):
            if k + 1 < rounds // g:
                feeder.submit((k + 1) % 2, *host[k + 1])
            X, y = feeder.acquire(k % 2)
            for i in range(g):
                hip.easgd_mlp_round(dims, W, Wc, X[i], y[i], wl.eta, wl.rho, workspace=ws)
            feeder.release(k % 2)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(to_host(W), ref[0])
        np.testing.assert_array_equal(to_host(Wc), ref[1])
    with pytest.raises(ValueError):
        hip.BatchFeeder(P, b, dims[0], rounds_per_copy=0)


def test_feeder_rejects_pageable_memory_and_wrong_shapes():
    import paper_1708_02983_amd as hip
    feeder = hip.BatchFeeder(2, 4, 8)
    X = torch.zeros(2, 4, 8); y = torch.zeros(2, 4, dtype=torch.int32)
    with pytest.raises(ValueError):
        feeder.submit(0, X, y)                                   # not pinned
    with pytest.raises(ValueError):
        feeder.submit(0, torch.zeros(2, 4, 9).pin_memory(), y.pin_memory())
    with pytest.raises(ValueError):
        hip.BatchFeeder(2, 4, 8, slots=1)
