"""HIP elastic update with bfloat16-stored gradients and momentum buffers (easgd_sync_round_bf16 /
measgd_round_bf16, an extension) against the CPU oracle, through the C ABI.

The stored momentum code is an integer decided by fp32 arithmetic whose order both sides fix, so V must
agree bit for bit (also after 100 free-running rounds: V_{t+1} depends on V_t and G only); W and Wc are
fp32 results with the usual bar."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import HUNDRED_ROUND_TOL, PER_ROUND_TOL, normwise, to_host

pytestmark = pytest.mark.gpu

F = np.float32
ETA, RHO, DELTA = F(0.01), F(0.1), F(0.9)
PAD16 = np.uint16(0x7FC0)          # what the padding of a bfloat16 row holds (a NaN pattern)


@pytest.fixture(scope="module")
def hip():
    import paper_1708_02983_amd as hip
    hip.lib()
    return hip


def narrow(a32: np.ndarray) -> np.ndarray:
    """Input preparation: fp32 draws (NaN padding) -> bfloat16 patterns with PAD16 padding."""
    out = oracle.bf16_round(np.nan_to_num(a32, nan=0.0))
    out[np.isnan(a32)] = PAD16
    return out


def dev16(a16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a16).view(np.int16)).cuda().view(torch.bfloat16)


def host16(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def dev32(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# one element, ragged tails (N % 4 = 1, 2, 3), ld > N, several tiles, every GROUPS choice of the launch
SHAPES = [(1, 1, 4), (2, 3, 4), (6, 3, 4), (9, 261, 264), (4, 7850, 7852), (3, 4099, 4100), (8, 100_003, 100_004),
          (16, 33_333, 33_336), (5, 1 << 20, 1 << 20), (32, 65_537, 65_540), (7, 1026, 2048), (4, 1 << 22, 1 << 22)]


@pytest.mark.parametrize("P,N,ld", SHAPES)
@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_one_round_matches_oracle(hip, P, N, ld, momentum):
    W, Wc = workloads.update_state(P, N, ld, seed=21)
    G16 = narrow(workloads.update_gradients(P, N, 0, ld, seed=21))
    V16 = narrow(workloads.update_gradients(P, N, 99, ld, seed=21, std=0.005))
    dW, dWc, dG, dV = dev32(W), dev32(Wc), dev16(G16), dev16(V16)
    G_before = G16.copy()
    if momentum:
        hip.measgd_round_bf16(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
        Wv, V16v, G16v = W[:, :N].copy(), V16[:, :N].copy(), G16[:, :N].copy()
        oracle.measgd_round_bf16(Wv, V16v, G16v, Wc, ETA, RHO, DELTA)
        W[:, :N] = Wv
        V16[:, :N] = V16v
        np.testing.assert_array_equal(host16(dV), V16)      # stored codes bit for bit, padding untouched
    else:
        hip.easgd_sync_round_bf16(dW, dG, dWc, float(ETA), float(RHO), N=N)
        Wv = W[:, :N].copy()
        oracle.easgd_round_bf16(Wv, np.ascontiguousarray(G16[:, :N]), Wc, ETA, RHO)
        W[:, :N] = Wv
    assert normwise(to_host(dW), W) <= PER_ROUND_TOL      # also checks that NaN padding stayed NaN
    assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
    np.testing.assert_array_equal(host16(dG), G_before)     # gradients are read-only


@pytest.mark.parametrize("momentum", [False, True], ids=["easgd", "measgd"])
def test_unaligned_operands_take_the_scalar_path(hip, momentum):
    P, N = 3, 1001
    # (ld, element offset of the fp32 buffers, element offset of the bfloat16 buffers)
    for ld, s32, s16 in [(1003, 0, 0), (1004, 1, 0), (1004, 0, 1), (1004, 0, 2), (1001, 3, 3)]:
        W, Wc = workloads.update_state(P, N, ld, seed=22)
        G16 = narrow(workloads.update_gradients(P, N, 0, ld, seed=22))
        V16 = narrow(workloads.update_gradients(P, N, 5, ld, seed=22))

        def carve32(a):
            buf = torch.full((a.size + 8,), float("nan"), dtype=torch.float32, device="cuda")
            view = buf[s32:s32 + a.size].view(a.shape)
            view.copy_(torch.from_numpy(a))
            return buf, view

        def carve16(a):
            buf = torch.full((a.size + 8,), float("nan"), dtype=torch.bfloat16, device="cuda")
            view = buf[s16:s16 + a.size].view(a.shape)
            view.copy_(dev16(a))
            return buf, view

        bW, dW = carve32(W); bWc, dWc = carve32(Wc); bG, dG = carve16(G16); bV, dV = carve16(V16)
        Wv, V16v, G16v = W[:, :N].copy(), V16[:, :N].copy(), G16[:, :N].copy()
        if momentum:
            hip.measgd_round_bf16(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
            oracle.measgd_round_bf16(Wv, V16v, G16v, Wc, ETA, RHO, DELTA)
            V16[:, :N] = V16v
            np.testing.assert_array_equal(host16(dV), V16)
        else:
            hip.easgd_sync_round_bf16(dW, dG, dWc, float(ETA), float(RHO), N=N)
            oracle.easgd_round_bf16(Wv, G16v, Wc, ETA, RHO)
        W[:, :N] = Wv
        assert normwise(to_host(dW), W) <= PER_ROUND_TOL
        assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
        # nothing outside the operands was written
        for buf, a, s in ((bW, W, s32), (bWc, Wc, s32)):
            h = to_host(buf)
            assert np.isnan(h[:s]).all() and np.isnan(h[s + a.size:]).all()
        h = host16(bV)
        assert (h[:s16] == PAD16).all() and (h[s16 + V16.size:] == PAD16).all()


@pytest.mark.parametrize("P,N,ld", [(2, 3, 4), (9, 261, 264), (3, 4099, 4100), (8, 100_003, 100_004), (4, 1 << 22, 1 << 22),
                                    (3, 1001, 1003)])
def test_fp32_gradients_with_bf16_momentum(hip, P, N, ld):
    """measgd_round_bf16v: only V is stored in 16 bits; the last shape takes the scalar path (ld % 4 != 0)."""
    W, Wc = workloads.update_state(P, N, ld, seed=25)
    G = workloads.update_gradients(P, N, 0, ld, seed=25)
    V16 = narrow(workloads.update_gradients(P, N, 99, ld, seed=25, std=0.005))
    dW, dWc, dG, dV = dev32(W), dev32(Wc), dev32(G), dev16(V16)
    hip.measgd_round_bf16v(dW, dV, dG, dWc, float(ETA), float(RHO), float(DELTA), N=N)
    Wv, V16v, Gv = W[:, :N].copy(), V16[:, :N].copy(), G[:, :N].copy()
    oracle.measgd_round_bf16(Wv, V16v, Gv, Wc, ETA, RHO, DELTA)
    W[:, :N] = Wv
    V16[:, :N] = V16v
    np.testing.assert_array_equal(host16(dV), V16)
    assert normwise(to_host(dW), W) <= PER_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
    np.testing.assert_array_equal(to_host(dG), G)


def test_training_rounds_with_bf16_momentum(hip):
    """easgd_grad + measgd_round_bf16v over 30 rounds of a small MLP: the update of every round is checked against
    the oracle on the gradient bits the GPU produced (the gradient itself has its own parity tests), and the
    loss follows the run with fp32 momentum buffers."""
    wl = workloads.WORKLOADS["cfg1"]
    dims, P, b = list(wl.dims), wl.P, wl.batch
    N = workloads.mlp_num_params(dims)
    ld = workloads.round_up(N, 4)
    w0 = workloads.init_packed_weights(wl)
    W = workloads.replicate(w0, P, ld); Wc = w0.copy()
    eta, rho, delta = 0.05, 0.1, 0.9
    dW, dWc = dev32(W), dev32(Wc)
    dW32, dWc32 = dev32(W), dev32(Wc)
    dV16 = torch.zeros((P, ld), dtype=torch.bfloat16, device="cuda")
    dV32 = torch.zeros((P, ld), dtype=torch.float32, device="cuda")
    dG = torch.zeros((P, ld), dtype=torch.float32, device="cuda")
    dloss = torch.zeros(P, dtype=torch.float32, device="cuda")
    ws = torch.empty(hip.easgd_grad_workspace_bytes(dims, P, b), dtype=torch.uint8, device="cuda")
    V16 = np.zeros((P, N), dtype=np.uint16)
    Wh = np.ascontiguousarray(W[:, :N]); Wch = Wc.copy()
    losses16, losses32 = [], []
    X, y = workloads.minibatch(wl, 0)          # the same minibatch every round, so that the loss has to fall
    dX, dy = dev32(X), torch.from_numpy(y).cuda()
    for t in range(30):
        hip.easgd_grad(dims, dW, dX, dy, dG, loss=dloss, workspace=ws)
        losses16.append(float(dloss.mean()))
        G = np.ascontiguousarray(to_host(dG)[:, :N])
        hip.measgd_round_bf16v(dW, dV16, dG, dWc, eta, rho, delta, N=N)
        # teacher-forced on the replicas the GPU had at the start of this round
        oracle.measgd_round_bf16(Wh, V16, G, Wch, F(eta), F(rho), F(delta))
        np.testing.assert_array_equal(host16(dV16)[:, :N], V16)
        assert normwise(to_host(dW)[:, :N], Wh) <= PER_ROUND_TOL
        assert normwise(to_host(dWc), Wch) <= PER_ROUND_TOL
        Wh = np.ascontiguousarray(to_host(dW)[:, :N]); Wch = to_host(dWc).copy()
        hip.easgd_grad(dims, dW32, dX, dy, dG, loss=dloss, workspace=ws)
        losses32.append(float(dloss.mean()))
        hip.measgd_round(dW32, dV32, dG, dWc32, eta, rho, delta, N=N)
    assert losses16[-1] < 0.8 * losses16[0]                        # it trains
    assert abs(losses16[-1] - losses32[-1]) < 0.02 * losses32[0]   # and tracks the fp32-momentum run


def test_hundred_rounds_free_running(hip):
    P, N = 8, (1 << 18) + 3
    ld = workloads.round_up(N, 4)
    W, Wc = workloads.update_state(P, N, ld, seed=23)
    W = np.ascontiguousarray(W[:, :N]); pad = ld - N
    V16 = np.zeros((P, N), dtype=np.uint16)

    def padded32(a):
        return np.concatenate([a, np.full((P, pad), np.nan, dtype=F)], axis=1)

    def padded16(a):
        return np.concatenate([a, np.full((P, pad), PAD16, dtype=np.uint16)], axis=1)

    dW, dWc, dV = dev32(padded32(W)), dev32(Wc), dev16(padded16(V16))
    for t in range(100):
        G16 = narrow(workloads.update_gradients(P, N, t, seed=23))
        hip.measgd_round_bf16(dW, dV, dev16(padded16(G16)), dWc, float(ETA), float(RHO), float(DELTA), N=N)
        oracle.measgd_round_bf16(W, V16, G16, Wc, ETA, RHO, DELTA)
        if t in (0, 9):
            np.testing.assert_array_equal(host16(dV), padded16(V16))
            assert normwise(to_host(dW), padded32(W)) <= PER_ROUND_TOL * (t + 1)
    np.testing.assert_array_equal(host16(dV), padded16(V16))       # still the same codes after 100 rounds
    assert normwise(to_host(dW), padded32(W)) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= HUNDRED_ROUND_TOL


def test_bitwise_reproducible_and_independent_of_launch_shape(hip):
    P, N = 16, 1_200_007
    ld = workloads.round_up(N, 4)
    W, Wc = workloads.update_state(P, N, ld, seed=24)
    G16 = narrow(workloads.update_gradients(P, N, 0, ld, seed=24))
    V16 = narrow(workloads.update_gradients(P, N, 1, ld, seed=24))
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
            dW, dWc, dG, dV = dev32(W), dev32(Wc), dev16(G16), dev16(V16)
            hip.easgd_sync_round_bf16(dW, dG, dWc, 0.01, 0.1, N=N)
            hip.measgd_round_bf16(dW, dV, dG, dWc, 0.01, 0.1, 0.9, N=N)
            results.append((to_host(dW), host16(dV), to_host(dWc)))
    finally:
        for o, v in zip((1, 2, 3, 9), saved):
            hip.set_option(o, v)
    for r in results[1:]:
        for a, b in zip(results[0], r):
            assert np.array_equal(a, b, equal_nan=True)


def test_bad_arguments_are_rejected(hip):
    W = torch.zeros(2, 8, device="cuda"); Wc = torch.zeros(8, device="cuda")
    G16 = torch.zeros(2, 8, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        hip.measgd_round_bf16(W, torch.zeros(2, 8, device="cuda"), G16, Wc, 0.1, 0.1, 0.9)   # fp32 momentum buffers
    with pytest.raises(ValueError):
        hip.easgd_sync_round_bf16(W, G16, Wc, 0.1, 0.1, N=9)                                  # rows too short
    lib = hip.lib()
    assert lib.easgd_sync_round_bf16(W.data_ptr(), G16.data_ptr(), Wc.data_ptr(), 2, 9, 8, 0.1, 0.1, None) == -1
    assert b"ld (8) < N (9)" in lib.easgd_last_error()
    assert lib.measgd_round_bf16(W.data_ptr(), None, G16.data_ptr(), Wc.data_ptr(), 2, 8, 8, 0.1, 0.1, 0.9, None) == -1


def test_cfg5_full_size_sampled(hip):
    """P = 16 x 61 M with bfloat16 G and V: the GPU runs every column, the oracle the sampled ones."""
    wl = workloads.WORKLOADS["cfg5"]
    P, N = wl.P, wl.N
    eta, rho, delta = F(wl.eta), F(wl.rho), F(wl.delta)
    idx = workloads.sample_columns(N)
    tidx = torch.from_numpy(idx).cuda()
    dW = workloads.device_normal((P, N), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 1)
    dWc = workloads.device_normal((N,), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 2)
    dV = torch.zeros((P, N), dtype=torch.bfloat16, device="cuda")
    W = to_host(dW[:, tidx]).copy(); Wc = to_host(dWc[tidx]).copy()
    V16 = np.zeros(W.shape, dtype=np.uint16)
    for t in range(10):
        dG = workloads.device_normal((P, N), workloads.GRADIENT_STD, workloads.DEFAULT_SEED, 100 + t).to(torch.bfloat16)
        G16 = host16(dG[:, tidx].contiguous()).copy()
        hip.measgd_round_bf16(dW, dV, dG, dWc, float(eta), float(rho), float(delta))
        oracle.measgd_round_bf16(W, V16, G16, Wc, eta, rho, delta)
        if t == 0:
            assert normwise(to_host(dW[:, tidx]), W) <= PER_ROUND_TOL
            assert normwise(to_host(dWc[tidx]), Wc) <= PER_ROUND_TOL
        del dG
    np.testing.assert_array_equal(host16(dV[:, tidx].contiguous()), V16)
    assert normwise(to_host(dW[:, tidx]), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc[tidx]), Wc) <= HUNDRED_ROUND_TOL
    assert bool(torch.isfinite(dW).all()) and bool(torch.isfinite(dWc).all())


def test_cfg4_full_size_sampled(hip):
    """P = 8 x 61 M with bfloat16 G (Eq. (1)): the GPU runs every column, the oracle the sampled ones."""
    wl = workloads.WORKLOADS["cfg4"]
    P, N = wl.P, wl.N
    eta, rho = F(wl.eta), F(wl.rho)
    idx = workloads.sample_columns(N)
    tidx = torch.from_numpy(idx).cuda()
    dW = workloads.device_normal((P, N), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 1)
    dWc = workloads.device_normal((N,), workloads.WEIGHT_STD, workloads.DEFAULT_SEED, 2)
    W = to_host(dW[:, tidx]).copy(); Wc = to_host(dWc[tidx]).copy()
    for t in range(10):
        dG = workloads.device_normal((P, N), workloads.GRADIENT_STD, workloads.DEFAULT_SEED, 100 + t).to(torch.bfloat16)
        G16 = host16(dG[:, tidx].contiguous()).copy()
        hip.easgd_sync_round_bf16(dW, dG, dWc, float(eta), float(rho))
        oracle.easgd_round_bf16(W, G16, Wc, eta, rho)
        if t == 0:
            assert normwise(to_host(dW[:, tidx]), W) <= PER_ROUND_TOL
            assert normwise(to_host(dWc[tidx]), Wc) <= PER_ROUND_TOL
        del dG
    assert normwise(to_host(dW[:, tidx]), W) <= HUNDRED_ROUND_TOL
    assert normwise(to_host(dWc[tidx]), Wc) <= HUNDRED_ROUND_TOL
    assert bool(torch.isfinite(dW).all()) and bool(torch.isfinite(dWc).all())


# ---- the whole round in one call with bfloat16 momentum buffers --------------------------------------

ROUND_CASES = [
    ((5, 4, 3), 2, 3),
    ((784, 10), 4, 64),
    ((33, 17, 10), 3, 25),
    ((50, 70, 30, 7), 9, 100),
    ((784, 256, 128, 10), 3, 100),
    ((512, 384, 10), 16, 128),
    ((130, 1000), 2, 9),
    ((784, 1024, 1024, 10), 16, 128),
]


@pytest.mark.parametrize("dims,P,b", ROUND_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_whole_round_with_bf16_momentum(hip, dims, P, b):
    """easgd_mlp_round with a bfloat16 V against easgd_grad + measgd_round_bf16v (same bits for W, V and the
    stored gradient) and against the oracle's rule on the gradient bits the GPU produced; two rounds, the second
    from the state the first one left, with and without storing the gradient, and a local step (rho = 0)."""
    eta, rho, delta = 0.05, 0.1, 0.9
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=eta, rho=rho, rounds=1, dims=tuple(dims), batch=b, N=N)
    w0 = workloads.init_packed_weights(wl, seed=41)
    ld = workloads.round_up(N, 4) + 4
    rng = np.random.default_rng(41)
    W = workloads.replicate(w0, P, ld)
    W[:, :N] += (rng.standard_normal((P, N)) * 0.02).astype(F)
    Wc = (w0 + (rng.standard_normal(N) * 0.01).astype(F)).astype(F)
    V16 = np.full((P, ld), PAD16, dtype=np.uint16)
    V16[:, :N] = oracle.bf16_round((rng.standard_normal((P, N)) * 0.002).astype(F))
    rW, rWc, rV = dev32(W), dev32(Wc), dev16(V16)           # two calls
    fW, fWc, fV = dev32(W), dev32(Wc), dev16(V16)           # one call
    oW, oWc, oV = np.ascontiguousarray(W[:, :N]), Wc.copy(), np.ascontiguousarray(V16[:, :N])
    rG = torch.full_like(rW, float("nan")); rloss = torch.empty(P, device="cuda")
    for t, (keep_g, rho_t) in enumerate(((True, rho), (False, rho), (True, 0.0))):
        X, y = workloads.minibatch(wl, t, seed=41)
        dX, dy = dev32(X), torch.from_numpy(y).cuda()
        hip.easgd_grad(dims, rW, dX, dy, rG, rloss)
        G = to_host(rG)
        if rho_t == 0.0:
            c_before = to_host(rWc).copy()
        hip.measgd_round_bf16v(rW, rV, rG, rWc, eta, rho_t, delta, N=N)
        fG = torch.full_like(fW, float("nan")) if keep_g else None
        floss = torch.empty(P, device="cuda")
        hip.easgd_mlp_round(dims, fW, fWc, dX, dy, eta, rho_t, V=fV, delta=delta, G=fG, loss=floss)
        what = f"round {t} keep_g={keep_g} rho={rho_t}"
        if keep_g:
            np.testing.assert_array_equal(to_host(fG), G, err_msg=what)
        np.testing.assert_array_equal(to_host(floss), to_host(rloss), err_msg=what)
        np.testing.assert_array_equal(host16(fV), host16(rV), err_msg=what)       # padding included
        np.testing.assert_array_equal(to_host(fW), to_host(rW), err_msg=what)
        assert normwise(to_host(fWc), to_host(rWc)) <= 1e-6, what
        if rho_t == 0.0:
            np.testing.assert_array_equal(to_host(fWc), c_before, err_msg=what)   # a local step leaves the center alone
        # the oracle on the same gradient bits, from the state this round started with
        oracle.measgd_round_bf16(oW, oV, np.ascontiguousarray(G[:, :N]), oWc, F(eta), F(rho_t), F(delta))
        np.testing.assert_array_equal(host16(fV)[:, :N], oV, err_msg=what)
        assert normwise(to_host(fW)[:, :N], oW) <= PER_ROUND_TOL, what
        assert normwise(to_host(fWc), oWc) <= PER_ROUND_TOL, what
        oW, oWc = np.ascontiguousarray(to_host(fW)[:, :N]), to_host(fWc).copy()
    assert np.isnan(to_host(fW)[:, N:]).all()


GRAD_CASES = [((5, 4, 3), 2, 3), ((784, 10), 4, 64), ((33, 17, 10), 3, 25), ((50, 70, 30, 7), 9, 100),
              ((784, 256, 128, 10), 3, 100), ((130, 1000), 2, 9), ((784, 1024, 1024, 10), 16, 128)]


@pytest.mark.parametrize("dims,P,b", GRAD_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_gradient_stored_as_bf16_is_the_narrowed_fp32_gradient(hip, dims, P, b):
    """easgd_grad with a bfloat16 G: the same accumulators as the fp32 form (which has its own parity tests against
    the oracle), narrowed once: bit for bit the oracle's narrowing of the fp32 result; then one update from it."""
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=0.05, rho=0.1, rounds=1, dims=tuple(dims), batch=b, N=N)
    w0 = workloads.init_packed_weights(wl, seed=43)
    ld = workloads.round_up(N, 4) + 4
    rng = np.random.default_rng(43)
    W = workloads.replicate(w0, P, ld)
    W[:, :N] += (rng.standard_normal((P, N)) * 0.02).astype(F)
    X, y = workloads.minibatch(wl, 0, seed=43)
    dW, dX, dy = dev32(W), dev32(X), torch.from_numpy(y).cuda()
    G32 = torch.full_like(dW, float("nan")); l32 = torch.empty(P, device="cuda")
    hip.easgd_grad(dims, dW, dX, dy, G32, l32)
    G16 = torch.full((P, ld), float("nan"), dtype=torch.bfloat16, device="cuda"); l16 = torch.empty(P, device="cuda")
    hip.easgd_grad(dims, dW, dX, dy, G16, l16)
    want = np.full((P, ld), PAD16, dtype=np.uint16)
    want[:, :N] = oracle.bf16_round(to_host(G32)[:, :N])
    np.testing.assert_array_equal(host16(G16), want)              # padding untouched
    np.testing.assert_array_equal(to_host(l16), to_host(l32))
    # and the update that consumes it
    Wc = w0.copy()
    V16 = np.zeros((P, ld), dtype=np.uint16)
    dWc, dV = dev32(Wc), dev16(V16)
    hip.measgd_round_bf16(dW, dV, G16, dWc, 0.05, 0.1, 0.9, N=N)
    oW, oV = np.ascontiguousarray(W[:, :N]), np.ascontiguousarray(V16[:, :N])
    oracle.measgd_round_bf16(oW, oV, np.ascontiguousarray(want[:, :N]), Wc, F(0.05), F(0.1), F(0.9))
    np.testing.assert_array_equal(host16(dV)[:, :N], oV)
    assert normwise(to_host(dW)[:, :N], oW) <= PER_ROUND_TOL
    assert normwise(to_host(dWc), Wc) <= PER_ROUND_TOL
