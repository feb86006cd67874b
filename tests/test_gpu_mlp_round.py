"""HIP easgd_mlp_round (the whole round in one call, the elastic update fused into backward propagation)
through the C ABI: against the two-call path it must reproduce, and against the CPU oracle's update rules."""
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
    return hip


def _state(dims, P, b, seed, ld_pad=4):
    """Replicas that have drifted apart, a center of its own and non-zero momentum buffers; NaN padding."""
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


# tiny; softmax regression; widths that force the scalar loaders; batch ragged against the MFMA tile;
# several hidden layers; enough workers for every tile route; a wide last layer
CASES = [
    ((5, 4, 3), 2, 3),
    ((784, 10), 4, 64),
    ((33, 17, 10), 3, 25),
    ((50, 70, 30, 7), 9, 100),
    ((784, 256, 128, 10), 3, 100),
    ((512, 384, 10), 40, 128),
    ((130, 1000), 2, 9),
]


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
@pytest.mark.parametrize("dims,P,b", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_fused_round_equals_gradient_then_update(hip, dims, P, b, momentum):
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=31)
    dX, dy = to_dev(X), to_dev(y)
    # reference: the two calls
    rW, rV, rWc = to_dev(W), to_dev(V), to_dev(Wc)
    rG = torch.full_like(rW, float("nan")); rloss = torch.empty(P, device="cuda")
    hip.easgd_grad(dims, rW, dX, dy, rG, rloss)
    if momentum:
        hip.measgd_round(rW, rV, rG, rWc, ETA, RHO, DELTA, N=N)
    else:
        hip.easgd_sync_round(rW, rG, rWc, ETA, RHO, N=N)
    G = to_host(rG)
    # the oracle's update rules applied to the same gradients
    oW, oV, oWc = W.copy(), V.copy(), Wc.copy()
    if momentum:
        oracle.measgd_round(oW, oV, G, oWc, F(ETA), F(RHO), F(DELTA), N=N)
    else:
        oracle.easgd_round(oW, G, oWc, F(ETA), F(RHO), N=N)
    old = hip.get_option(hip.OPT_ROUND_OVERLAP)
    try:
        for keep_g, overlap in ((True, 0), (False, 0), (True, 2), (False, 2), (True, 3), (False, 3), (False, 1)):
            hip.set_option(hip.OPT_ROUND_OVERLAP, overlap)
            fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
            fG = torch.full_like(fW, float("nan")) if keep_g else None
            floss = torch.empty(P, device="cuda")
            hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV if momentum else None, delta=DELTA,
                                G=fG, loss=floss)
            what = f"keep_g={keep_g} overlap={overlap}"
            if keep_g:      # same products, same accumulators: the stored gradient is the same bits
                np.testing.assert_array_equal(to_host(fG), G, err_msg=what)
            np.testing.assert_array_equal(to_host(floss), to_host(rloss), err_msg=what)
            # the worker rule is element-wise on the same inputs: the same bits as the streaming kernel
            np.testing.assert_array_equal(to_host(fW), to_host(rW), err_msg=what)
            # the center sums the workers in ascending order; the streaming kernel uses another fixed
            # order when N is small and P >= 4, so the two may differ by rounding
            assert normwise(to_host(fWc), to_host(rWc)) <= 1e-6, what
            assert normwise(to_host(fW)[:, :N], oW[:, :N]) <= PER_ROUND_TOL, what
            assert normwise(to_host(fWc), oWc) <= PER_ROUND_TOL, what
            assert np.isnan(to_host(fW)[:, N:]).all(), what          # padding is never written
            if momentum:
                np.testing.assert_array_equal(to_host(fV), to_host(rV), err_msg=what)
                assert normwise(to_host(fV)[:, :N], oV[:, :N]) <= PER_ROUND_TOL, what
            else:
                np.testing.assert_array_equal(to_host(fV), V, err_msg=what)   # untouched without momentum
    finally:
        hip.set_option(hip.OPT_ROUND_OVERLAP, old)


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
def test_every_tile_shape_gives_the_same_round(hip, tile):
    dims, P, b = (300, 260, 200, 10), 6, 70
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=32)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_GEMM_TILE)
    out = []
    try:
        for t in (0, tile):
            hip.set_option(hip.OPT_GEMM_TILE, t)
            fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
            hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV, delta=DELTA)
            out.append((to_host(fW), to_host(fV), to_host(fWc)))
    finally:
        hip.set_option(hip.OPT_GEMM_TILE, old)
    # a tile shape changes the slab depth (the order of the k sums) only: results agree to rounding
    for a, c in zip(out[0], out[1]):
        assert normwise(a[..., :N], c[..., :N]) <= 1e-6


@pytest.mark.parametrize("tile", [1, 3, 4])
def test_center_rule_rides_on_every_forward_tile(hip, tile):
    """The center rule on extra blocks of the first forward launch, whatever tile shape that launch uses (by default the
    extra blocks are only attached to 64x64 launches): same bits as the rule run as a kernel of its own."""
    dims, P, b = (300, 260, 200, 10), 6, 100
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=33)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_GEMM_TILE), hip.get_option(hip.OPT_ROUND_OVERLAP)
    out = []
    try:
        hip.set_option(hip.OPT_GEMM_TILE, tile)
        for overlap in (0, 3):
            hip.set_option(hip.OPT_ROUND_OVERLAP, overlap)
            fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
            hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV, delta=DELTA)
            out.append((to_host(fW), to_host(fV), to_host(fWc)))
    finally:
        hip.set_option(hip.OPT_GEMM_TILE, old[0])
        hip.set_option(hip.OPT_ROUND_OVERLAP, old[1])
    for a, c in zip(out[0], out[1]):
        np.testing.assert_array_equal(a, c)


@pytest.mark.parametrize("dims,P,b,ld_pad", [((1024, 1100, 10), 2, 8, 0), ((512, 600, 10), 3, 16, 1)],
                         ids=["vector", "scalar"])
def test_center_rule_beside_forward_walks_the_range(hip, dims, P, b, ld_pad):
    """On the second stream the center rule of a long parameter vector takes one block per compute unit that walks
    the range (128-bit form, and the scalar form for a row stride that is no multiple of 4): same bits as the rule
    as a kernel of its own, padding untouched."""
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=34, ld_pad=ld_pad)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_ROUND_OVERLAP)
    out = []
    try:
        for overlap in (0, 2):
            hip.set_option(hip.OPT_ROUND_OVERLAP, overlap)
            fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
            hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV, delta=DELTA)
            out.append((to_host(fW), to_host(fV), to_host(fWc)))
    finally:
        hip.set_option(hip.OPT_ROUND_OVERLAP, old)
    for a, c in zip(out[0], out[1]):
        np.testing.assert_array_equal(a, c)
    assert not np.array_equal(out[1][2], Wc)                    # the center did move
    assert np.isnan(out[1][0][:, N:]).all()


def test_consecutive_rounds_on_one_stream_and_reproducibility(hip):
    """Several fused rounds back to back, overlapped and not: the rounds are ordered correctly on the
    caller's stream (each starts from the previous one's results) and runs are bitwise reproducible."""
    dims, P, b = (784, 128, 10), 8, 64
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=33)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_ROUND_OVERLAP)
    results = []
    try:
        for overlap in (0, 2, 2, 3, 1):
            hip.set_option(hip.OPT_ROUND_OVERLAP, overlap)
            fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
            ws = None
            for _ in range(12):
                ws = hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV, delta=DELTA, workspace=ws)
            results.append((to_host(fW), to_host(fV), to_host(fWc)))
    finally:
        hip.set_option(hip.OPT_ROUND_OVERLAP, old)
    for other in results[1:]:
        for a, c in zip(results[0], other):
            np.testing.assert_array_equal(a, c)
    # and the same 12 rounds through the two-call path
    rW, rV, rWc = to_dev(W), to_dev(V), to_dev(Wc)
    rG = torch.empty_like(rW)
    for _ in range(12):
        hip.easgd_grad(dims, rW, dX, dy, rG)
        hip.measgd_round(rW, rV, rG, rWc, ETA, RHO, DELTA, N=N)
    assert normwise(results[0][0][:, :N], to_host(rW)[:, :N]) <= 1e-5
    assert normwise(results[0][2], to_host(rWc)) <= 1e-5


@pytest.mark.parametrize("overlap", [0, 2, 3], ids=["one_stream", "two_streams", "extra_blocks"])
def test_round_can_be_captured_in_a_hip_graph(hip, overlap):
    """The call allocates nothing, records no memset and never synchronises, so a caller may capture it.
    The graph is replayed several times with eager library work and synchronisations in between, and every
    replay is checked against the same rounds run eagerly (with the second stream in use, its fork and join
    events become edges of the graph)."""
    dims, P, b = (784, 96, 10), 6, 32
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=34)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_ROUND_OVERLAP)
    hip.set_option(hip.OPT_ROUND_OVERLAP, overlap)
    try:
        eW, eV, eWc = to_dev(W), to_dev(V), to_dev(Wc)
        gW, gV, gWc = to_dev(W), to_dev(V), to_dev(Wc)
        ws_e = torch.empty(hip.easgd_mlp_round_workspace_bytes(dims, P, b), dtype=torch.uint8, device="cuda")
        ws_g = torch.empty_like(ws_e)

        def two_rounds(Wt, Vt, Wct, ws):
            hip.easgd_mlp_round(dims, Wt, Wct, dX, dy, ETA, RHO, V=Vt, delta=DELTA, workspace=ws)
            hip.easgd_mlp_round(dims, Wt, Wct, dX, dy, ETA, RHO, workspace=ws)

        # eager warm-up on both states: creates the library's stream and events, caches the device properties
        two_rounds(eW, eV, eWc, ws_e)
        two_rounds(gW, gV, gWc, ws_g)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            two_rounds(gW, gV, gWc, ws_g)
        torch.cuda.synchronize()
        two_rounds(eW, eV, eWc, ws_e)       # what the capture run did, if it ran at all, is not relied upon:
        gW.copy_(eW); gV.copy_(eV); gWc.copy_(eWc)   # both states restart from the same point
        for replay in range(4):
            two_rounds(eW, eV, eWc, ws_e)
            graph.replay()
            torch.cuda.synchronize()
            for a, c in ((eW, gW), (eV, gV), (eWc, gWc)):
                np.testing.assert_array_equal(to_host(a), to_host(c), err_msg=f"replay {replay}")
            # eager library work between the replays
            scratch = torch.empty_like(eW)
            hip.easgd_grad(dims, eW, dX, dy, scratch)
            torch.cuda.synchronize()
    finally:
        hip.set_option(hip.OPT_ROUND_OVERLAP, old)


@pytest.mark.parametrize("dims,P,b", [((784, 256, 128, 10), 3, 100), ((300, 260, 10), 5, 64), ((128, 200, 136, 64, 12), 4, 37),
                                      ((130, 96, 1000), 2, 9), ((512, 384, 10), 40, 128)],
                         ids=lambda v: str(v).replace(" ", ""))
def test_shared_launches_change_nothing(hip, dims, P, b):
    """Independent products of backward propagation may share a launch (the narrow last layer's weight gradient
    with the input gradient below it, the weight gradients of two layers); every block still does exactly the work
    it does in a launch of its own, so gradients and rounds are the same bits with the sharing on and off."""
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=35)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_GEMM_PAIR)
    out = []
    try:
        for pair in (0, 1):
            hip.set_option(hip.OPT_GEMM_PAIR, pair)
            res = []
            for momentum in (False, True):
                fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
                fG = torch.full_like(fW, float("nan"))
                hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV if momentum else None, delta=DELTA, G=fG)
                res += [to_host(fW), to_host(fV), to_host(fWc), to_host(fG)]
            gW = to_dev(W); gG = torch.full_like(gW, float("nan"))
            hip.easgd_grad(dims, gW, dX, dy, gG)
            res.append(to_host(gG))
            out.append(res)
    finally:
        hip.set_option(hip.OPT_GEMM_PAIR, old)
    for a, c in zip(out[0], out[1]):
        np.testing.assert_array_equal(a, c)
    np.testing.assert_array_equal(out[0][3], out[0][-1])      # the round's stored gradient is easgd_grad's


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_local_steps_between_exchanges(hip, momentum):
    """rho = 0 makes the call a local step (no exchange): with a period of 3 the center changes only every third
    round and stays bit for bit what it was in between (negative zeros included); every round matches the
    oracle's rules applied to the stored gradients, with rho = 0 in the local rounds (Eq. (1) / (5),(6) at rho = 0
    are the plain rules Eq. (3),(4) of one worker)."""
    dims, P, b, tau = (40, 48, 10), 5, 20, 3
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=41)
    Wc[::7] = F(-0.0)
    wl = workloads.Workload("t", P=P, eta=ETA, rho=RHO, rounds=6, dims=tuple(dims), batch=b, N=N)
    dW, dV, dWc = to_dev(W), to_dev(V), to_dev(Wc)
    oW, oV, oWc = W.copy(), V.copy(), Wc.copy()
    for t in range(6):
        X, y = workloads.minibatch(wl, t, seed=41)
        rho = RHO if (t + 1) % tau == 0 else 0.0
        before = to_host(dWc).copy()
        dG = torch.full_like(dW, float("nan"))
        hip.easgd_mlp_round(dims, dW, dWc, to_dev(X), to_dev(y), ETA, rho, V=dV if momentum else None,
                            delta=DELTA, G=dG)
        G = to_host(dG)
        if momentum:
            oracle.measgd_round(oW, oV, G, oWc, F(ETA), F(rho), F(DELTA), N=N)
        else:
            oracle.easgd_round(oW, G, oWc, F(ETA), F(rho), N=N)
        after = to_host(dWc)
        if rho == 0.0:
            assert after.tobytes() == before.tobytes(), f"round {t}: a local step wrote the center"
            np.testing.assert_array_equal(oWc, before)          # and so says Eq. (2) at rho = 0
        else:
            assert not np.array_equal(after, before)
        assert normwise(to_host(dW)[:, :N], oW[:, :N]) <= PER_ROUND_TOL, t
        assert normwise(after, oWc) <= PER_ROUND_TOL, t
        if momentum:
            assert normwise(to_host(dV)[:, :N], oV[:, :N]) <= PER_ROUND_TOL, t
        # teacher forcing: the next round starts from the device's state on both sides
        oW[:, :N] = to_host(dW)[:, :N]; oWc[:] = after
        if momentum:
            oV[:, :N] = to_host(dV)[:, :N]


@pytest.mark.parametrize("dims,P,b", [((200, 264, 136, 10), 8, 100), ((512, 384, 10), 40, 128), ((300, 260, 10), 16, 64),
                                      ((200, 512, 256, 10), 8, 36)],
                         ids=lambda v: str(v).replace(" ", ""))
def test_block_order_changes_nothing(hip, dims, P, b):
    """EASGD_OPT_GEMM_XCD only renumbers the blocks of a product (plain order; whole workers per die; a die's workers
    interleaved tile by tile in the products that apply the worker rule, in bands of tile columns or in row-major
    tile order): every block computes the same tile the same way, so rounds and gradients are the same bits under
    all four orders (P a multiple of 8 makes the interleaved orders differ from the second; at 64-wide tiles the
    widths 512, 256 and 384 give bands of 8, 4 and 2 tile columns, the others none)."""
    N, ld, W, V, Wc, X, y = _state(dims, P, b, seed=37)
    dX, dy = to_dev(X), to_dev(y)
    old = hip.get_option(hip.OPT_GEMM_XCD)
    out = []
    try:
        for order in (0, 1, 2, 3):
            hip.set_option(hip.OPT_GEMM_XCD, order)
            res = []
            for momentum in (False, True):
                fW, fV, fWc = to_dev(W), to_dev(V), to_dev(Wc)
                fG = torch.full_like(fW, float("nan"))
                hip.easgd_mlp_round(dims, fW, fWc, dX, dy, ETA, RHO, V=fV if momentum else None, delta=DELTA, G=fG)
                res += [to_host(fW), to_host(fV), to_host(fWc), to_host(fG)]
            gW = to_dev(W); gG = torch.full_like(gW, float("nan"))
            hip.easgd_grad(dims, gW, dX, dy, gG)
            res.append(to_host(gG))
            out.append(res)
    finally:
        hip.set_option(hip.OPT_GEMM_XCD, old)
    for other in out[1:]:
        for a, c in zip(out[0], other):
            np.testing.assert_array_equal(a, c)
