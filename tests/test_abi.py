"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
before touching the GPU (no kernel is launched in this file)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1708_02983_amd", "libeasgd_hip.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libeasgd_hip.so not built (run __graft_entry__.build())")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "easgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:m?easgd|sync_sgd)_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"easgd_sync_round", "measgd_round", "easgd_grad", "easgd_grad_workspace_bytes",
            "easgd_mlp_num_params", "easgd_last_error", "easgd_version", "easgd_set_option",
            "easgd_get_option", "easgd_stream_copy", "easgd_stream_triad", "easgd_mlp_round", "easgd_mlp_round_bf16v",
            "easgd_mlp_round_workspace_bytes", "easgd_sync_round_bf16", "measgd_round_bf16", "measgd_round_bf16v",
            "easgd_grad_bf16", "easgd_grad_static", "sync_sgd_round", "easgd_stream_mix32",
            "easgd_launch_count", "easgd_layer_product", "easgd_mfma_probe"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/easgd.h but not exported"


def test_num_params_and_workspace(lib):
    lib.easgd_mlp_num_params.restype = ctypes.c_size_t
    lib.easgd_grad_workspace_bytes.restype = ctypes.c_size_t
    for dims, n in [((784, 10), 7850), ((784, 1024, 1024, 10), 1863690), ((3072, 2048, 2048, 10), 10510346)]:
        arr = (ctypes.c_int * len(dims))(*dims)
        assert lib.easgd_mlp_num_params(arr, len(dims) - 1) == n
        ws = lib.easgd_grad_workspace_bytes(arr, len(dims) - 1, 4, 64)
        assert ws > 0 and ws % 256 == 0
        # the whole-round call also keeps the new center (N floats) in the workspace
        lib.easgd_mlp_round_workspace_bytes.restype = ctypes.c_size_t
        wr = lib.easgd_mlp_round_workspace_bytes(arr, len(dims) - 1, 4, 64)
        assert wr % 256 == 0 and 4 * n <= wr - ws < 4 * n + 256
    bad = (ctypes.c_int * 2)(784, 0)
    assert lib.easgd_mlp_num_params(bad, 1) == 0
    assert lib.easgd_grad_workspace_bytes(bad, 1, 4, 64) == 0
    assert lib.easgd_mlp_round_workspace_bytes(bad, 1, 4, 64) == 0


def test_bad_arguments_are_rejected_without_a_launch(lib):
    lib.easgd_last_error.restype = ctypes.c_char_p
    f, sz, vp = ctypes.c_float, ctypes.c_size_t, ctypes.c_void_p
    lib.easgd_sync_round.argtypes = [vp, vp, vp, ctypes.c_int, sz, sz, f, f, vp]
    lib.measgd_round.argtypes = [vp, vp, vp, vp, ctypes.c_int, sz, sz, f, f, f, vp]
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    assert lib.easgd_sync_round(None, fake, fake, 1, 4, 4, 0.1, 0.1, None) == -1
    assert b"NULL" in lib.easgd_last_error()
    assert lib.easgd_sync_round(fake, fake, fake, 0, 4, 4, 0.1, 0.1, None) == -1
    assert lib.easgd_sync_round(fake, fake, fake, 1, 0, 4, 0.1, 0.1, None) == -1
    assert lib.easgd_sync_round(fake, fake, fake, 1, 8, 4, 0.1, 0.1, None) == -1
    assert b"ld" in lib.easgd_last_error()
    assert lib.measgd_round(fake, None, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
    # the bfloat16-storage forms validate the same way
    lib.easgd_sync_round_bf16.argtypes = [vp, vp, vp, ctypes.c_int, sz, sz, f, f, vp]
    for fn in (lib.measgd_round_bf16, lib.measgd_round_bf16v):
        fn.argtypes = [vp, vp, vp, vp, ctypes.c_int, sz, sz, f, f, f, vp]
        assert fn(fake, None, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
        assert b"NULL" in lib.easgd_last_error()
        assert fn(fake, fake, fake, fake, 0, 4, 4, 0.1, 0.1, 0.9, None) == -1
        assert fn(fake, fake, fake, fake, 1, 0, 4, 0.1, 0.1, 0.9, None) == -1
        assert fn(fake, fake, fake, fake, 1, 8, 4, 0.1, 0.1, 0.9, None) == -1
    assert b"measgd_round_bf16v: ld (4) < N (8)" in lib.easgd_last_error()
    assert lib.easgd_sync_round_bf16(fake, None, fake, 1, 4, 4, 0.1, 0.1, None) == -1
    assert lib.easgd_sync_round_bf16(fake, fake, fake, 1, 8, 4, 0.1, 0.1, None) == -1
    assert b"easgd_sync_round_bf16" in lib.easgd_last_error()
    # pointers that are not aligned to their element type are rejected (fp32: 4 bytes, bfloat16: 2 bytes)
    for bad in (0x1001, 0x1002):
        assert lib.easgd_sync_round(bad, fake, fake, 1, 4, 4, 0.1, 0.1, None) == -1
        assert b"4-byte aligned" in lib.easgd_last_error()
        assert lib.easgd_sync_round(fake, bad, fake, 1, 4, 4, 0.1, 0.1, None) == -1
        assert lib.easgd_sync_round(fake, fake, bad, 1, 4, 4, 0.1, 0.1, None) == -1
        assert lib.measgd_round(fake, bad, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
        assert lib.measgd_round_bf16v(fake, fake, bad, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
        assert lib.measgd_round_bf16(bad, fake, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
    assert lib.measgd_round_bf16(fake, 0x1001, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
    assert b"2-byte aligned" in lib.easgd_last_error()
    assert lib.measgd_round_bf16(fake, fake, 0x1001, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
    assert lib.measgd_round_bf16v(fake, 0x1003, fake, fake, 1, 4, 4, 0.1, 0.1, 0.9, None) == -1
    assert lib.easgd_sync_round_bf16(fake, 0x1001, fake, 1, 4, 4, 0.1, 0.1, None) == -1
    lib.sync_sgd_round.argtypes = [vp, vp, vp, ctypes.c_int, sz, sz, f, f, vp]
    assert lib.sync_sgd_round(0x1002, None, fake, 1, 4, 4, 0.1, 0.0, None) == -1
    assert lib.sync_sgd_round(fake, 0x1001, fake, 1, 4, 4, 0.1, 0.9, None) == -1
    assert lib.sync_sgd_round(None, None, fake, 1, 4, 4, 0.1, 0.0, None) == -1
    assert lib.sync_sgd_round(fake, None, None, 1, 4, 4, 0.1, 0.0, None) == -1
    assert lib.sync_sgd_round(fake, None, fake, 0, 4, 4, 0.1, 0.0, None) == -1
    assert lib.sync_sgd_round(fake, None, fake, 1, 0, 4, 0.1, 0.0, None) == -1
    assert lib.sync_sgd_round(fake, fake, fake, 1, 8, 4, 0.1, 0.9, None) == -1
    assert b"sync_sgd_round" in lib.easgd_last_error()
    ip = ctypes.POINTER(ctypes.c_int)
    lib.easgd_grad.argtypes = [ip, ctypes.c_int, vp, sz, vp, vp, ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, vp]
    dims = (ctypes.c_int * 2)(784, 10)
    assert lib.easgd_grad(dims, 1, None, 7850, fake, fake, 1, 1, fake, None, fake, 1 << 30, None) == -1
    assert lib.easgd_grad(dims, 1, fake, 7000, fake, fake, 1, 1, fake, None, fake, 1 << 30, None) == -1   # ld < N
    assert lib.easgd_grad(dims, 0, fake, 7850, fake, fake, 1, 1, fake, None, fake, 1 << 30, None) == -1
    assert lib.easgd_grad(dims, 1, fake, 7850, fake, fake, 1, 1, fake, None, None, 0, None) == -3          # workspace
    assert lib.easgd_grad(dims, 1, fake, 7850, fake, fake, 1, 1, fake, None, 0x1000, 16, None) == -3
    lib.easgd_grad_bf16.argtypes = lib.easgd_grad.argtypes
    assert lib.easgd_grad_bf16(dims, 1, fake, 7850, fake, fake, 1, 1, None, None, fake, 1 << 30, None) == -1
    assert b"easgd_grad_bf16: NULL" in lib.easgd_last_error()
    assert lib.easgd_grad_bf16(dims, 1, fake, 7850, fake, fake, 1, 1, 0x1001, None, fake, 1 << 30, None) == -1
    assert lib.easgd_grad_bf16(dims, 1, fake, 7000, fake, fake, 1, 1, fake, None, fake, 1 << 30, None) == -1
    assert lib.easgd_grad_bf16(dims, 1, fake, 7850, fake, fake, 1, 1, fake, None, None, 0, None) == -3
    lib.easgd_mlp_round.argtypes = [ip, ctypes.c_int, vp, vp, vp, sz, vp, vp, ctypes.c_int, ctypes.c_int, vp, vp, f, f, f, vp, sz, vp]
    big = 1 << 30
    assert lib.easgd_mlp_round(dims, 1, fake, None, None, 7850, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.0, fake, big, None) == -1
    assert b"NULL" in lib.easgd_last_error()
    assert lib.easgd_mlp_round(dims, 1, None, None, fake, 7850, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.0, fake, big, None) == -1
    assert lib.easgd_mlp_round(dims, 1, fake, None, fake, 7000, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.0, fake, big, None) == -1
    lib.easgd_mlp_round_bf16v.argtypes = lib.easgd_mlp_round.argtypes
    assert lib.easgd_mlp_round_bf16v(dims, 1, fake, None, fake, 7850, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.9, fake, big, None) == -1
    assert b"easgd_mlp_round_bf16v: NULL" in lib.easgd_last_error()
    assert lib.easgd_mlp_round_bf16v(dims, 1, fake, 0x1001, fake, 7850, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.9, fake, big, None) == -1
    assert b"2-byte aligned" in lib.easgd_last_error()
    assert lib.easgd_mlp_round_bf16v(dims, 1, fake, fake, fake, 7000, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.9, fake, big, None) == -1
    lib.easgd_grad_workspace_bytes.restype = ctypes.c_size_t
    short = lib.easgd_grad_workspace_bytes(dims, 1, 1, 1)     # enough for easgd_grad, not for the whole round
    assert lib.easgd_mlp_round(dims, 1, fake, None, fake, 7850, fake, fake, 1, 1, None, None, 0.1, 0.1, 0.0, fake, short, None) == -3
    many = (ctypes.c_int * 2)(784, 5000)
    assert lib.easgd_grad(many, 1, fake, 784 * 5000 + 5000, fake, fake, 1, 1, fake, None, 0x1000, 1 << 30, None) == -1


def test_options_roundtrip(lib):
    lib.easgd_set_option.argtypes = [ctypes.c_int, ctypes.c_long]
    lib.easgd_get_option.restype = ctypes.c_long
    old = lib.easgd_get_option(3)
    assert old == 0
    assert lib.easgd_set_option(3, 2) == 0 and lib.easgd_get_option(3) == 2
    assert lib.easgd_set_option(3, 8) == 0 and lib.easgd_set_option(3, 5) == -1 and lib.easgd_get_option(3) == 8
    assert lib.easgd_get_option(9) == 2 and lib.easgd_set_option(9, 3) == -1
    assert lib.easgd_set_option(9, 0) == 0 and lib.easgd_get_option(9) == 0 and lib.easgd_set_option(9, 2) == 0
    assert lib.easgd_set_option(99, 1) == -1
    assert lib.easgd_set_option(3, old) == 0
    assert lib.easgd_get_option(5) == 1 and lib.easgd_set_option(5, 4) == -1
    assert lib.easgd_set_option(5, 2) == 0 and lib.easgd_get_option(5) == 2 and lib.easgd_set_option(5, 1) == 0
    assert lib.easgd_get_option(6) == 1 and lib.easgd_set_option(6, 4) == -1 and lib.easgd_set_option(6, 3) == 0 and lib.easgd_set_option(6, 1) == 0
    assert lib.easgd_set_option(6, 0) == 0 and lib.easgd_get_option(6) == 0 and lib.easgd_set_option(6, 1) == 0
    assert lib.easgd_get_option(4) == 0 and lib.easgd_set_option(4, 5) == -1
    assert lib.easgd_set_option(4, 4) == 0 and lib.easgd_get_option(4) == 4 and lib.easgd_set_option(4, 0) == 0
    assert lib.easgd_get_option(7) == 1 and lib.easgd_set_option(7, 2) == -1 and lib.easgd_set_option(7, 1) == 0
    assert lib.easgd_get_option(8) == 1 and lib.easgd_set_option(8, 2) == -1
    assert lib.easgd_set_option(8, 0) == 0 and lib.easgd_get_option(8) == 0 and lib.easgd_set_option(8, 1) == 0
    # non-temporal accesses of the update kernels: 2 = chosen per call (default), 0 and 1 force
    assert lib.easgd_get_option(2) == 2 and lib.easgd_set_option(2, 3) == -1 and lib.easgd_set_option(2, -1) == -1
    assert lib.easgd_set_option(2, 0) == 0 and lib.easgd_get_option(2) == 0 and lib.easgd_set_option(2, 2) == 0
    assert lib.easgd_version() >= 100
