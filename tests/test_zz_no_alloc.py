"""easgd_grad_static, the entry point for callers that cannot allocate: called through the raw C ABI it must give
the bits of easgd_grad (same kernels, the workspace being the library's own static device array), on two calls
in a row of which the second is smaller (the array still holds the first call's contents), reject shapes beyond
the array before launching anything, and leave the amount of free device memory as it was."""
import ctypes

import numpy as np
import pytest
import torch

import workloads
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu
F = np.float32


def _inputs(dims, P, b, seed):
    N = workloads.mlp_num_params(dims)
    wl = workloads.Workload("t", P=P, eta=0.05, rho=0.1, rounds=1, dims=tuple(dims), batch=b, N=N)
    ld = workloads.round_up(N, 4) + 4
    W = workloads.replicate(workloads.init_packed_weights(wl, seed=seed), P, ld)
    W[:, :N] += (np.random.default_rng(seed).standard_normal((P, N)) * 0.02).astype(F)
    X, y = workloads.minibatch(wl, 0, seed=seed)
    return N, ld, to_dev(W), to_dev(X), to_dev(y)


def test_static_workspace_entry_point_matches_easgd_grad():
    import paper_1708_02983_amd as hip
    lib = hip.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    limit = hip.STATIC_SCRATCH_BYTES

    def both(dims, P, b, seed):
        N, ld, dW, dX, dy = _inputs(dims, P, b, seed)
        arr = (ctypes.c_int * len(dims))(*dims)
        L = len(dims) - 1
        need = lib.easgd_grad_workspace_bytes(arr, L, P, b)
        assert 0 < need <= limit
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        G0 = torch.full_like(dW, float("nan")); l0 = torch.empty(P, device="cuda")
        G1 = torch.full_like(dW, float("nan")); l1 = torch.empty(P, device="cuda")
        rc = lib.easgd_grad(arr, L, dW.data_ptr(), ld, dX.data_ptr(), dy.data_ptr(), P, b, G0.data_ptr(), l0.data_ptr(),
                            ws.data_ptr(), need, stream)
        assert rc == 0, lib.easgd_last_error()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rc = lib.easgd_grad_static(arr, L, dW.data_ptr(), ld, dX.data_ptr(), dy.data_ptr(), P, b, G1.data_ptr(),
                                   l1.data_ptr(), stream)
        assert rc == 0, lib.easgd_last_error()
        torch.cuda.synchronize()
        free_after = torch.cuda.mem_get_info()[0]
        g0, g1 = to_host(G0), to_host(G1)
        assert np.isfinite(g0[:, :N]).all() and np.isnan(g0[:, N:]).all()
        np.testing.assert_array_equal(g1, g0)                 # bit for bit, padding untouched
        np.testing.assert_array_equal(to_host(l1), to_host(l0))
        return free_before, free_after

    # first call: three layers, ragged batch, 12.6 MB of workspace; second call: a smaller network on fewer rows,
    # whose buffers overlay what the first call left in the array; third: the second again, memory watched
    print("static workspace: call 1", flush=True)
    both((784, 1024, 512, 10), 6, 100, seed=5)
    print("static workspace: call 2 (smaller)", flush=True)
    both((130, 70, 10), 3, 25, seed=6)
    print("static workspace: call 3 (repeat)", flush=True)
    before, after = both((130, 70, 10), 3, 25, seed=6)
    assert after == before, f"free device memory changed across the call: {before} -> {after}"

    # beyond the array: cfg3's shape needs about 131 MB
    dims = (3072, 2048, 2048, 10)
    arr = (ctypes.c_int * 4)(*dims)
    assert lib.easgd_grad_workspace_bytes(arr, 3, 32, 100) > limit
    fake = 0x1000   # never dereferenced: the call must fail before it touches anything
    rc = lib.easgd_grad_static(arr, 3, fake, 10510348, fake, fake, 32, 100, fake, None, stream)
    assert rc == -3 and b"static workspace holds" in lib.easgd_last_error()
    assert lib.easgd_grad_static(arr, 0, fake, 10510348, fake, fake, 32, 100, fake, None, stream) == -1
    assert lib.easgd_grad_static((ctypes.c_int * 2)(784, 10), 1, fake, 7852, fake, fake, 4, 64, None, None, stream) == -1
