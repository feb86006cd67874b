"""The single-launch round of a single-layer network (softmax regression; Section 5.1 steps (1)-(5) in one grid with a
grid-wide barrier) through the C ABI: gradient, loss and updated state against the CPU oracle, against the path of
separate launches it replaces, and the barrier's bookkeeping."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import PER_ROUND_TOL, normwise, to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32
ETA, RHO, DELTA = 0.05, 0.1, 0.9


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    old = hip.get_option(hip.OPT_ROUND_SINGLE_LAUNCH)
    hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 1)               # the path under test is opt-in
    yield hip
    hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, old)


def _state(dims, P, b, seed, ld_pad=4):
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=ETA, rho=RHO, rounds=1, dims=tuple(dims), batch=b, N=N)
    w0 = workloads.init_packed_weights(wl, seed=seed)
    ld = workloads.round_up(N, 4) + ld_pad
    rng = np.random.default_rng(seed)
    W = workloads.replicate(w0, P, ld)
    W[:, :N] += (rng.standard_normal((P, N)) * 0.02).astype(F)
    Wc = (w0 + (rng.standard_normal(N) * 0.01).astype(F)).astype(F)
    V = workloads.replicate((rng.standard_normal(N) * 0.001).astype(F), P, ld)
    V[:, :N] += (rng.standard_normal((P, N)) * 0.001).astype(F)
    X, y = workloads.minibatch(wl, 0, seed=seed)
    return N, ld, W, V, Wc, X, y


# the cfg1 shape; one class; widths and batches that leave ragged slices, rows and tails; sixteen classes (the
# narrowest slices); a batch that lets only one worker into a pass; more workers than one pass holds; more (worker,
# rows) items and more slices than the grid has blocks
CASES = [
    ((784, 10), 4, 64),
    ((5, 1), 2, 3),
    ((33, 7), 3, 25),
    ((130, 16), 5, 37),
    ((61, 10), 5, 200),
    ((100, 4), 19, 50),
    ((3000, 12), 16, 128),
    ((8100, 16), 2, 8),
    ((20, 10), 11, 8),
]
IDS = [str(c).replace(" ", "") for c in CASES]


def _launches(hip, fn):
    n0 = hip.launch_count()
    fn()
    return hip.launch_count() - n0


@pytest.mark.parametrize("dims,P,b", CASES, ids=IDS)
def test_gradient_and_loss_match_oracle(hip, dims, P, b):
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=7)
    dW, dX, dy = to_dev(W), to_dev(X), to_dev(y)
    dG = torch.full_like(dW, float("nan")); dloss = torch.full((P,), float("nan"), device="cuda")
    assert _launches(hip, lambda: hip.easgd_grad(dims, dW, dX, dy, dG, dloss)) == 1
    G, loss = to_host(dG), to_host(dloss)
    np.testing.assert_array_equal(to_host(dW), W)                # the replicas are read-only here
    G_ref, loss_ref = oracle.mlp_grad_all_workers(dims, W, X, y)
    assert np.isnan(G[:, N:]).all() and np.isfinite(G[:, :N]).all()
    (w_sl, b_sl), = oracle.layer_slices(dims)
    for i in range(P):
        assert normwise(G[i], G_ref[i]) <= PER_ROUND_TOL
        assert normwise(G[i, w_sl], G_ref[i, w_sl]) <= 2 * PER_ROUND_TOL
        assert normwise(G[i, b_sl], G_ref[i, b_sl]) <= 2 * PER_ROUND_TOL
    np.testing.assert_allclose(loss, loss_ref, rtol=1e-5)
    assert hip.round_barrier_timeouts() == 0


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
@pytest.mark.parametrize("dims,P,b", CASES, ids=IDS)
def test_round_matches_oracle_and_separate_launches(hip, dims, P, b, momentum):
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=11)
    dX, dy = to_dev(X), to_dev(y)
    # the oracle's round: its own gradient, then its update rule
    G_ref, loss_ref = oracle.mlp_grad_all_workers(dims, W, X, y)
    oW, oV, oWc = W.copy(), V.copy(), Wc.copy()
    if momentum:
        oracle.measgd_round(oW, oV, G_ref, oWc, F(ETA), F(RHO), F(DELTA), N=N)
    else:
        oracle.easgd_round(oW, G_ref, oWc, F(ETA), F(RHO), N=N)

    def run(keep_g):
        fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
        fG = torch.full_like(fW, float("nan")) if keep_g else None
        floss = torch.full((P,), float("nan"), device="cuda")
        n = _launches(hip, lambda: hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV if momentum else None,
                                                       delta=DELTA, G=fG, loss=floss))
        return n, to_host(fW), to_host(fV), to_host(fWc), (to_host(fG) if keep_g else None), to_host(floss)

    one = [run(True), run(False)]
    try:
        hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 0)
        n_sep, sW, sV, sWc, sG, sloss = run(True)
    finally:
        hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 1)
    assert n_sep >= 2
    for n, fW, fV, fWc, fG, floss in one:
        assert n == 1
        assert normwise(fW[:, :N], oW[:, :N]) <= PER_ROUND_TOL
        assert normwise(fWc, oWc) <= PER_ROUND_TOL
        assert np.isnan(fW[:, N:]).all()                          # padding is never written
        np.testing.assert_allclose(floss, loss_ref, rtol=1e-5)
        if momentum:
            assert normwise(fV[:, :N], oV[:, :N]) <= PER_ROUND_TOL
            assert np.isnan(fV[:, N:]).all() == np.isnan(V[:, N:]).all()
        else:
            np.testing.assert_array_equal(fV, V)                  # untouched without momentum
        if fG is not None:
            for i in range(P):
                assert normwise(fG[i], G_ref[i]) <= PER_ROUND_TOL
            assert np.isnan(fG[:, N:]).all()
        # the two paths sum the minibatch in different fixed orders: equal to rounding
        assert normwise(fW[:, :N], sW[:, :N]) <= 2e-6 and normwise(fWc, sWc) <= 2e-6
    # storing the gradient or not changes nothing else
    np.testing.assert_array_equal(one[0][1], one[1][1])
    np.testing.assert_array_equal(one[0][3], one[1][3])
    assert hip.round_barrier_timeouts() == 0


def test_local_step_leaves_the_center_alone(hip):
    dims, P, b = (784, 10), 4, 64
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=3)
    dX, dy = to_dev(X), to_dev(y)
    G_ref, _ = oracle.mlp_grad_all_workers(dims, W, X, y)
    for momentum in (False, True):
        oW, oV, oWc = W.copy(), V.copy(), Wc.copy()
        if momentum:
            oracle.measgd_round(oW, oV, G_ref, oWc, F(ETA), F(0.0), F(DELTA), N=N)
        else:
            oracle.easgd_round(oW, G_ref, oWc, F(ETA), F(0.0), N=N)
        np.testing.assert_array_equal(oWc, Wc)                    # Eq. (2) with rho = 0
        fW, fV = to_dev(W), to_dev(V)
        fWc = to_dev(np.full_like(Wc, np.nan))                    # must be neither read into a result nor written
        assert _launches(hip, lambda: hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, 0.0, V=fV if momentum else None,
                                                          delta=DELTA)) == 1
        assert np.isnan(to_host(fWc)).all()
        assert normwise(to_host(fW)[:, :N], oW[:, :N]) <= PER_ROUND_TOL
        if momentum:
            assert normwise(to_host(fV)[:, :N], oV[:, :N]) <= PER_ROUND_TOL


def test_ten_training_rounds_follow_the_oracle(hip):
    """cfg1 as a whole: ten Sync EASGD rounds from identical replicas, every round started from the oracle's state."""
    wl = workloads.WORKLOADS["cfg1"]
    dims, P, N = wl.dims, wl.P, wl.N
    ld = workloads.round_up(N, 4)
    w0 = workloads.init_packed_weights(wl)
    W = workloads.replicate(w0, P, ld); Wc = w0.copy()
    fW, fWc = to_dev(W), to_dev(Wc)                               # free-running on the GPU
    for t in range(wl.rounds):
        X, y = workloads.minibatch(wl, t)
        dX, dy = to_dev(X), to_dev(y)
        G_ref, loss_ref = oracle.mlp_grad_all_workers(dims, W, X, y)
        tW, tWc = to_dev(W), to_dev(Wc)                           # teacher-forced: from the oracle's state
        tloss = torch.empty(P, device="cuda")
        hip.easgd_mlp_round(dims, tW, tWc, dX, dy, wl.eta, wl.rho, loss=tloss)
        hip.easgd_mlp_round(dims, fW, fWc, dX, dy, wl.eta, wl.rho)
        oracle.easgd_round(W, G_ref, Wc, F(wl.eta), F(wl.rho), N=N)
        assert normwise(to_host(tW)[:, :N], W[:, :N]) <= PER_ROUND_TOL, t
        assert normwise(to_host(tWc), Wc) <= PER_ROUND_TOL, t
        np.testing.assert_allclose(to_host(tloss), loss_ref, rtol=1e-5)
    assert normwise(to_host(fW)[:, :N], W[:, :N]) <= 1e-4 and normwise(to_host(fWc), Wc) <= 1e-4
    assert hip.round_barrier_timeouts() == 0


def test_rounds_on_two_streams_do_not_share_a_barrier(hip):
    """Each stream has barrier words of its own: rounds enqueued on two streams at the same time give the results of
    the same rounds run one after the other."""
    dims, P, b = (784, 10), 4, 64
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=5)
    dX, dy = to_dev(X), to_dev(y)
    ref = []
    for k in range(2):
        rW, rWc = to_dev(W), to_dev(Wc)
        for _ in range(20):
            hip.easgd_mlp_round(dims, rW, rWc, dX, dy, ETA, RHO)
        ref.append((to_host(rW), to_host(rWc)))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    state = [(to_dev(W), to_dev(Wc)) for _ in streams]
    torch.cuda.synchronize()
    for _ in range(20):
        for s, (sW, sWc) in zip(streams, state):
            with torch.cuda.stream(s):
                hip.easgd_mlp_round(dims, sW, sWc, dX, dy, ETA, RHO)
    torch.cuda.synchronize()
    for (sW, sWc), (rW, rWc), s in zip(state, ref, streams):
        np.testing.assert_array_equal(to_host(sW), rW)
        np.testing.assert_array_equal(to_host(sWc), rWc)
        assert hip.round_barrier_timeouts(s) == 0


def test_a_captured_round_takes_the_separate_launches(hip):
    """A launch whose blocks wait for each other is not recorded into a graph: under capture the call falls back to
    the separate launches, and the replayed graph gives their result."""
    dims, P, b = (784, 10), 4, 64
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=9)
    dX, dy = to_dev(X), to_dev(y)
    try:
        hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 0)
        rW, rWc = to_dev(W), to_dev(Wc)
        hip.easgd_mlp_round(dims, rW, rWc, dX, dy, ETA, RHO)
    finally:
        hip.set_option(hip.OPT_ROUND_SINGLE_LAUNCH, 1)
    gW, gWc = to_dev(W), to_dev(Wc)
    ws = torch.empty(hip.easgd_mlp_round_workspace_bytes(dims, P, b), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    n0 = hip.launch_count()
    with torch.cuda.graph(graph):
        hip.easgd_mlp_round(dims, gW, gWc, dX, dy, ETA, RHO, workspace=ws)
    assert hip.launch_count() - n0 >= 2
    torch.cuda.synchronize()
    gW.copy_(to_dev(W)); gWc.copy_(to_dev(Wc))                    # whatever the capture run did is not relied upon
    graph.replay()
    np.testing.assert_array_equal(to_host(gW), to_host(rW))
    np.testing.assert_array_equal(to_host(gWc), to_host(rWc))


def test_bfloat16_storage_forms_take_the_same_launch(hip):
    """The forms that store the gradient or the momentum buffers as bfloat16 (an extension) through the single
    launch: the narrowed gradient is the fp32 gradient of the same launch rounded to nearest even (the oracle's
    narrowing), and a round with bfloat16 momentum buffers equals the gradient call followed by the streaming
    update with bfloat16 momentum buffers, bit for bit in W and V."""
    dims, P, b = (784, 10), 4, 64
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=13)
    dX, dy = to_dev(X), to_dev(y)
    dW = to_dev(W)
    dG = torch.full_like(dW, float("nan"))
    hip.easgd_grad(dims, dW, dX, dy, dG)
    G = to_host(dG)
    dG16 = torch.zeros(dW.shape, dtype=torch.bfloat16, device="cuda")
    assert _launches(hip, lambda: hip.easgd_grad(dims, dW, dX, dy, dG16)) == 1
    got = to_host(dG16.view(torch.int16)).view(np.uint16)[:, :N]
    np.testing.assert_array_equal(got, oracle.bf16_round(np.ascontiguousarray(G[:, :N])))
    V16 = oracle.bf16_round(np.ascontiguousarray(V))
    V16[:, N:] = 0x7fc0

    def dev16(a):
        return torch.from_numpy(a.view(np.int16).copy()).cuda().view(torch.bfloat16)

    rW, rWc, rV = to_dev(W), to_dev(Wc), dev16(V16)
    hip.measgd_round_bf16v(rW, rV, dG, rWc, ETA, RHO, DELTA, N=N)
    fW, fWc, fV = to_dev(W), to_dev(Wc), dev16(V16)
    assert _launches(hip, lambda: hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV, delta=DELTA)) == 1
    np.testing.assert_array_equal(to_host(fW), to_host(rW))
    np.testing.assert_array_equal(to_host(fV.view(torch.int16)), to_host(rV.view(torch.int16)))
    assert normwise(to_host(fWc), to_host(rWc)) <= 1e-6
    # and the oracle's rule on the same gradient bits
    oW, oWc, oV = np.ascontiguousarray(W[:, :N]), Wc.copy(), np.ascontiguousarray(V16[:, :N])
    oracle.measgd_round_bf16(oW, oV, np.ascontiguousarray(G[:, :N]), oWc, F(ETA), F(RHO), F(DELTA))
    np.testing.assert_array_equal(to_host(fV.view(torch.int16)).view(np.uint16)[:, :N], oV)
    assert normwise(to_host(fW)[:, :N], oW) <= PER_ROUND_TOL and normwise(to_host(fWc), oWc) <= PER_ROUND_TOL
    assert hip.round_barrier_timeouts() == 0
