"""Thin ctypes binding of libeasgd_hip.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks their
dtype / device / contiguity / size on the host, and passes raw device pointers
and the current HIP stream through the C ABI declared in ``include/easgd.h``.
All arithmetic of the round runs inside the library's kernels; there is no
fallback: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import functools
import os
from typing import Optional, Sequence

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libeasgd_hip.so")

EASGD_OK = 0
OPT_UPDATE_BLOCKS_PER_CU = 1
OPT_UPDATE_NONTEMPORAL = 2
OPT_UPDATE_GROUPS = 3
OPT_GEMM_TILE = 4
OPT_ROUND_OVERLAP = 5
OPT_GEMM_XCD = 6
OPT_GEMM_PAIR = 7
OPT_MLP_HEAD = 8
OPT_UPDATE_LAYOUT = 9
OPT_ROUND_SINGLE_LAUNCH = 10
OPT_ROUND_SPIN_LIMIT = 11


class EasgdError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"easgd error {code}: {message}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build the HIP library first "
            "(python -m paper_1708_02983_amd.build); there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, f, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int
    lib.easgd_sync_round.argtypes = [vp, vp, vp, i, sz, sz, f, f, vp]
    lib.easgd_sync_round.restype = i
    lib.measgd_round.argtypes = [vp, vp, vp, vp, i, sz, sz, f, f, f, vp]
    lib.measgd_round.restype = i
    lib.easgd_sync_round_bf16.argtypes = [vp, vp, vp, i, sz, sz, f, f, vp]
    lib.easgd_sync_round_bf16.restype = i
    lib.measgd_round_bf16.argtypes = [vp, vp, vp, vp, i, sz, sz, f, f, f, vp]
    lib.measgd_round_bf16.restype = i
    lib.measgd_round_bf16v.argtypes = [vp, vp, vp, vp, i, sz, sz, f, f, f, vp]
    lib.measgd_round_bf16v.restype = i
    lib.sync_sgd_round.argtypes = [vp, vp, vp, i, sz, sz, f, f, vp]
    lib.sync_sgd_round.restype = i
    lib.async_easgd_round.argtypes = [vp, vp, vp, vp, i, sz, sz, ctypes.POINTER(ctypes.c_int), i, f, f, f, vp]
    lib.async_easgd_round.restype = i
    lib.hogwild_easgd_round.argtypes = [vp, vp, vp, vp, i, sz, sz, f, f, f, vp]
    lib.hogwild_easgd_round.restype = i
    ip = ctypes.POINTER(ctypes.c_int)
    lib.easgd_grad_workspace_bytes.argtypes = [ip, i, i, i]
    lib.easgd_grad_workspace_bytes.restype = sz
    lib.easgd_grad.argtypes = [ip, i, vp, sz, vp, vp, i, i, vp, vp, vp, sz, vp]
    lib.easgd_grad.restype = i
    lib.easgd_grad_static.argtypes = [ip, i, vp, sz, vp, vp, i, i, vp, vp, vp]
    lib.easgd_grad_static.restype = i
    lib.easgd_grad_bf16.argtypes = [ip, i, vp, sz, vp, vp, i, i, vp, vp, vp, sz, vp]
    lib.easgd_grad_bf16.restype = i
    lib.easgd_mlp_round_workspace_bytes.argtypes = [ip, i, i, i]
    lib.easgd_mlp_round_workspace_bytes.restype = sz
    lib.easgd_mlp_round.argtypes = [ip, i, vp, vp, vp, sz, vp, vp, i, i, vp, vp, f, f, f, vp, sz, vp]
    lib.easgd_mlp_round.restype = i
    lib.easgd_mlp_round_bf16v.argtypes = [ip, i, vp, vp, vp, sz, vp, vp, i, i, vp, vp, f, f, f, vp, sz, vp]
    lib.easgd_mlp_round_bf16v.restype = i
    lib.easgd_layer_product.argtypes = [i, i, i, i, i, vp, vp, sz, vp, vp, sz, i, vp]
    lib.easgd_layer_product.restype = i
    lib.easgd_mlp_num_params.argtypes = [ip, i]
    lib.easgd_mlp_num_params.restype = sz
    lib.easgd_stream_copy.argtypes = [vp, vp, sz, vp]
    lib.easgd_stream_copy.restype = i
    lib.easgd_stream_triad.argtypes = [vp, vp, vp, sz, f, vp]
    lib.easgd_stream_triad.restype = i
    lib.easgd_stream_mix32.argtypes = [vp, vp, vp, vp, vp, sz, f, vp]
    lib.easgd_stream_mix32.restype = i
    lib.easgd_mfma_probe.argtypes = [vp, sz, i, i, i, vp, sz, ctypes.POINTER(ctypes.c_uint), vp]
    lib.easgd_mfma_probe.restype = i
    lib.easgd_round_barrier_timeouts.argtypes = [vp]
    lib.easgd_round_barrier_timeouts.restype = ctypes.c_long
    lib.easgd_launch_count.argtypes = []
    lib.easgd_launch_count.restype = ctypes.c_ulonglong
    lib.easgd_set_option.argtypes = [i, ctypes.c_long]
    lib.easgd_set_option.restype = i
    lib.easgd_get_option.argtypes = [i]
    lib.easgd_get_option.restype = ctypes.c_long
    lib.easgd_last_error.restype = ctypes.c_char_p
    lib.easgd_version.restype = i
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (for callers that want the raw entry points)."""
    return _lib


def _check(code: int) -> None:
    if code != EASGD_OK:
        raise EasgdError(code, _lib.easgd_last_error().decode())


_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream) -> ctypes.c_void_p:
    # the current stream of the current device; torch.cuda.current_stream() builds a Stream object through several
    # layers of Python (8 us per call here, more than the library's own share of a small round), the raw query does not
    if stream is None:
        if _raw_current_stream is not None:
            return ctypes.c_void_p(_raw_current_stream(torch.cuda.current_device()))
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(name: str, t: torch.Tensor, dtype, min_numel: int) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if t.numel() < min_numel:
        raise ValueError(f"{name} holds {t.numel()} elements, needs {min_numel}")
    return t.data_ptr()


def _replica_shape(W: torch.Tensor, N: Optional[int]):
    if W.dim() != 2:
        raise ValueError("replica matrices must be [P][ld]")
    P, ld = W.shape
    return P, ld, (ld if N is None else int(N))


def easgd_sync_round(W, G, Wc, eta: float, rho: float, N: Optional[int] = None, stream=None) -> None:
    """Steps (2)-(5) of a Sync EASGD round, in place on W[P][ld] and Wc[N] (Eq. (1), Eq. (2))."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.easgd_sync_round(_dev("W", W, torch.float32, need), _dev("G", G, torch.float32, need),
                                 _dev("Wc", Wc, torch.float32, N), P, N, ld, eta, rho, _stream(stream)))


def measgd_round(W, V, G, Wc, eta: float, rho: float, delta: float, N: Optional[int] = None,
                 stream=None) -> None:
    """The same round with the momentum worker rule, in place on W, V and Wc (Eq. (5), (6), (2))."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.measgd_round(_dev("W", W, torch.float32, need), _dev("V", V, torch.float32, need),
                             _dev("G", G, torch.float32, need), _dev("Wc", Wc, torch.float32, N),
                             P, N, ld, eta, rho, delta, _stream(stream)))


def easgd_sync_round_bf16(W, G16, Wc, eta: float, rho: float, N: Optional[int] = None, stream=None) -> None:
    """easgd_sync_round with the gradients stored as bfloat16 (torch.bfloat16 tensor [P][ld]); an extension."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.easgd_sync_round_bf16(_dev("W", W, torch.float32, need), _dev("G16", G16, torch.bfloat16, need),
                                      _dev("Wc", Wc, torch.float32, N), P, N, ld, eta, rho, _stream(stream)))


def measgd_round_bf16(W, V16, G16, Wc, eta: float, rho: float, delta: float, N: Optional[int] = None,
                      stream=None) -> None:
    """measgd_round with gradients and momentum buffers stored as bfloat16 (torch.bfloat16 tensors [P][ld]);
    an extension."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.measgd_round_bf16(_dev("W", W, torch.float32, need), _dev("V16", V16, torch.bfloat16, need),
                                  _dev("G16", G16, torch.bfloat16, need), _dev("Wc", Wc, torch.float32, N),
                                  P, N, ld, eta, rho, delta, _stream(stream)))


def measgd_round_bf16v(W, V16, G, Wc, eta: float, rho: float, delta: float, N: Optional[int] = None,
                       stream=None) -> None:
    """measgd_round with only the momentum buffers stored as bfloat16; the gradients are fp32; an extension."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.measgd_round_bf16v(_dev("W", W, torch.float32, need), _dev("V16", V16, torch.bfloat16, need),
                                   _dev("G", G, torch.float32, need), _dev("Wc", Wc, torch.float32, N),
                                   P, N, ld, eta, rho, delta, _stream(stream)))


def sync_sgd_round(W, G, eta: float, V=None, delta: float = 0.0, N: Optional[int] = None, stream=None) -> None:
    """Synchronous data-parallel SGD on the replicas: every replica moves by the sum of all gradients
    (Section 2.3, Section 6.2); V selects the momentum rule Eq. (3),(4)."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.sync_sgd_round(_dev("W", W, torch.float32, need),
                               None if V is None else _dev("V", V, torch.float32, need),
                               _dev("G", G, torch.float32, need), P, N, ld, eta, delta, _stream(stream)))


def async_easgd_round(W, G, Wc, order: Sequence[int], eta: float, rho: float, V=None, delta: float = 0.0,
                      N: Optional[int] = None, stream=None) -> None:
    """The master serving one worker at a time in the sequence `order` (Algorithm 1 in rank order; Async EASGD /
    Async MEASGD in arrival order), one launch for the whole schedule; V selects Eq. (5),(6)."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    seq = (ctypes.c_int * len(order))(*[int(j) for j in order])
    _check(_lib.async_easgd_round(_dev("W", W, torch.float32, need),
                                  None if V is None else _dev("V", V, torch.float32, need),
                                  _dev("G", G, torch.float32, need), _dev("Wc", Wc, torch.float32, N),
                                  P, N, ld, seq, len(order), eta, rho, delta, _stream(stream)))


def hogwild_easgd_round(W, G, Wc, eta: float, rho: float, V=None, delta: float = 0.0, N: Optional[int] = None,
                        stream=None) -> None:
    """Hogwild EASGD: all workers exchange with the center at once, lock-free (atomic adds into the center);
    W and Wc are not reproducible from run to run."""
    P, ld, N = _replica_shape(W, N)
    need = (P - 1) * ld + N
    _check(_lib.hogwild_easgd_round(_dev("W", W, torch.float32, need),
                                    None if V is None else _dev("V", V, torch.float32, need),
                                    _dev("G", G, torch.float32, need), _dev("Wc", Wc, torch.float32, N),
                                    P, N, ld, eta, rho, delta, _stream(stream)))


# What the marshalling derives from the layer widths alone is kept per tuple of widths: a round of a small network
# takes some 15 us on the device, and rebuilding the C array and asking the library for N and the workspace size on
# every call cost more than that on the host.
@functools.lru_cache(maxsize=256)
def _dims_cached(dims: tuple):
    arr = (ctypes.c_int * len(dims))(*dims)
    return arr, len(dims) - 1


def _dims(dims: Sequence[int]):
    return _dims_cached(tuple(int(d) for d in dims))


@functools.lru_cache(maxsize=256)
def _num_params_cached(dims: tuple) -> int:
    arr, L = _dims_cached(dims)
    return int(_lib.easgd_mlp_num_params(arr, L))


def easgd_mlp_num_params(dims: Sequence[int]) -> int:
    return _num_params_cached(tuple(int(d) for d in dims))


@functools.lru_cache(maxsize=256)
def _workspace_cached(dims: tuple, P: int, b: int, whole_round: bool) -> int:
    arr, L = _dims_cached(dims)
    fn = _lib.easgd_mlp_round_workspace_bytes if whole_round else _lib.easgd_grad_workspace_bytes
    return int(fn(arr, L, P, b))


def easgd_grad_workspace_bytes(dims: Sequence[int], P: int, b: int) -> int:
    return _workspace_cached(tuple(int(d) for d in dims), int(P), int(b), False)


def easgd_grad(dims: Sequence[int], W, X, y, G, loss=None, workspace=None, stream=None):
    """Step (1): gradients of all P workers into G[P][ld]; returns the workspace used.
    A torch.bfloat16 G selects the form that stores the gradients in 16 bits (an extension)."""
    arr, L = _dims(dims)
    if W.dim() != 2 or X.dim() != 3 or y.dim() != 2:
        raise ValueError("expected W[P][ld], X[P][b][d_in], y[P][b]")
    P, ld = W.shape
    b = X.shape[1]
    N = easgd_mlp_num_params(dims)
    if N == 0:
        raise ValueError(f"invalid layer widths {list(dims)}")
    if X.shape[0] != P or X.shape[2] != dims[0] or tuple(y.shape) != (P, b):
        raise ValueError("X / y shapes do not match W and dims")
    need = (P - 1) * ld + N
    nbytes = easgd_grad_workspace_bytes(dims, P, b)
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    g16 = G.dtype == torch.bfloat16
    entry = _lib.easgd_grad_bf16 if g16 else _lib.easgd_grad
    _check(entry(arr, L, _dev("W", W, torch.float32, need), ld,
                           _dev("X", X, torch.float32, P * b * dims[0]),
                           _dev("y", y, torch.int32, P * b), P, b,
                           _dev("G", G, torch.bfloat16 if g16 else torch.float32, need),
                           None if loss is None else _dev("loss", loss, torch.float32, P),
                           _dev("workspace", workspace, torch.uint8, nbytes), workspace.numel(),
                           _stream(stream)))
    return workspace


def easgd_layer_product(kind: int, d_in: int, d_out: int, A, out, Wl=None, dZ=None, ld: int = 0, out_ws: int = 0,
                        relu: bool = False, stream=None) -> None:
    """One product of forward / backward propagation alone (a testing aid): kind 0 forward, 1 weight gradient,
    2 input gradient; A[P][b][d_in], Wl[P][ld], dZ[P][b][d_out], out[P][out_ws]."""
    P, b = A.shape[0], A.shape[1]
    _check(_lib.easgd_layer_product(kind, d_in, d_out, P, b, _dev("A", A, torch.float32, P * b * d_in),
                                    None if Wl is None else _dev("Wl", Wl, torch.float32, (P - 1) * ld + (d_in + 1) * d_out),
                                    ld, None if dZ is None else _dev("dZ", dZ, torch.float32, P * b * d_out),
                                    _dev("out", out, torch.float32, (P - 1) * out_ws + 1), out_ws, int(relu),
                                    _stream(stream)))


STATIC_SCRATCH_BYTES = 64 << 20    # EASGD_STATIC_SCRATCH_BYTES of include/easgd.h


def easgd_grad_static(dims: Sequence[int], W, X, y, G, loss=None, stream=None) -> None:
    """easgd_grad on the library's own static workspace: nothing is allocated, here or in the library
    (for callers that cannot allocate; shapes beyond STATIC_SCRATCH_BYTES of workspace are rejected)."""
    arr, L = _dims(dims)
    if W.dim() != 2 or X.dim() != 3 or y.dim() != 2:
        raise ValueError("expected W[P][ld], X[P][b][d_in], y[P][b]")
    P, ld = W.shape
    b = X.shape[1]
    N = easgd_mlp_num_params(dims)
    if N == 0:
        raise ValueError(f"invalid layer widths {list(dims)}")
    if X.shape[0] != P or X.shape[2] != dims[0] or tuple(y.shape) != (P, b):
        raise ValueError("X / y shapes do not match W and dims")
    need = (P - 1) * ld + N
    _check(_lib.easgd_grad_static(arr, L, _dev("W", W, torch.float32, need), ld,
                                  _dev("X", X, torch.float32, P * b * dims[0]),
                                  _dev("y", y, torch.int32, P * b), P, b,
                                  _dev("G", G, torch.float32, need),
                                  None if loss is None else _dev("loss", loss, torch.float32, P),
                                  _stream(stream)))


def easgd_mlp_round_workspace_bytes(dims: Sequence[int], P: int, b: int) -> int:
    return _workspace_cached(tuple(int(d) for d in dims), int(P), int(b), True)


def easgd_mlp_round(dims: Sequence[int], W, Wc, X, y, eta: float, rho: float, V=None, delta: float = 0.0,
                    G=None, loss=None, workspace=None, stream=None):
    """Steps (1)-(5) in one call, the update fused into backward propagation; V selects Eq. (5),(6)
    (a torch.bfloat16 V selects the form that stores the momentum buffers in 16 bits, an extension);
    the gradients are stored only when G is given.  Returns the workspace used."""
    arr, L = _dims(dims)
    if W.dim() != 2 or X.dim() != 3 or y.dim() != 2:
        raise ValueError("expected W[P][ld], X[P][b][d_in], y[P][b]")
    P, ld = W.shape
    b = X.shape[1]
    N = easgd_mlp_num_params(dims)
    if N == 0:
        raise ValueError(f"invalid layer widths {list(dims)}")
    if X.shape[0] != P or X.shape[2] != dims[0] or tuple(y.shape) != (P, b):
        raise ValueError("X / y shapes do not match W and dims")
    if V is not None and tuple(V.shape) != (P, ld):
        raise ValueError("V must have the shape of W")
    need = (P - 1) * ld + N
    nbytes = easgd_mlp_round_workspace_bytes(dims, P, b)
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    v16 = V is not None and V.dtype == torch.bfloat16
    entry = _lib.easgd_mlp_round_bf16v if v16 else _lib.easgd_mlp_round
    _check(entry(arr, L, _dev("W", W, torch.float32, need),
                                None if V is None else _dev("V", V, torch.bfloat16 if v16 else torch.float32, need),
                                _dev("Wc", Wc, torch.float32, N), ld,
                                _dev("X", X, torch.float32, P * b * dims[0]),
                                _dev("y", y, torch.int32, P * b), P, b,
                                None if G is None else _dev("G", G, torch.float32, need),
                                None if loss is None else _dev("loss", loss, torch.float32, P),
                                eta, rho, delta,
                                _dev("workspace", workspace, torch.uint8, nbytes), workspace.numel(),
                                _stream(stream)))
    return workspace


def stream_copy(dst, src, stream=None) -> None:
    """Measurement aid: dst[:] = src with the library's streaming copy kernel."""
    n = src.numel()
    _check(_lib.easgd_stream_copy(_dev("dst", dst, torch.float32, n), _dev("src", src, torch.float32, n), n, _stream(stream)))


def stream_triad(a, b, c, s: float, stream=None) -> None:
    """Measurement aid: a[:] = b + s*c (two reads, one write per element)."""
    n = a.numel()
    _check(_lib.easgd_stream_triad(_dev("a", a, torch.float32, n), _dev("b", b, torch.float32, n),
                                   _dev("c", c, torch.float32, n), n, s, _stream(stream)))


def stream_mix32(a, b, c, d, e, s: float, stream=None) -> None:
    """Measurement aid: a[:] = c + s*d, b[:] = d + s*e (three reads, two writes per element)."""
    n = a.numel()
    _check(_lib.easgd_stream_mix32(_dev("a", a, torch.float32, n), _dev("b", b, torch.float32, n),
                                   _dev("c", c, torch.float32, n), _dev("d", d, torch.float32, n),
                                   _dev("e", e, torch.float32, n), n, s, _stream(stream)))


def mfma_probe(out, iters: int, mode, blocks_per_cu: int = 2, src=None, stream=None) -> int:
    """Measurement aid: the bare fp32 matrix-instruction loop (see include/easgd.h; mode 0, 1 or 2, a bool counts as
    0 or 1; mode 2 reads `src`).  Returns the flops of the launch."""
    blocks = ctypes.c_uint(0)
    mode = int(mode)
    src_ptr, src_len = (None, 0) if src is None else (_dev("src", src, torch.float32, 4096), src.numel())
    _check(_lib.easgd_mfma_probe(_dev("out", out, torch.float32, out.numel()), out.numel(), int(iters), mode,
                                 int(blocks_per_cu), src_ptr, src_len, ctypes.byref(blocks), _stream(stream)))
    return blocks.value * 4 * int(iters) * 16 * 4096


def round_barrier_timeouts(stream=None) -> int:
    """Blocks that ever gave up waiting at the barrier of a single-launch round on `stream` (synchronises it)."""
    n = int(_lib.easgd_round_barrier_timeouts(_stream(stream)))
    if n < 0:
        _check(n)
    return n


def launch_count() -> int:
    """Measurement aid: kernel launches issued by the library in this process so far."""
    return int(_lib.easgd_launch_count())


def set_option(option: int, value: int) -> None:
    _check(_lib.easgd_set_option(option, value))


def get_option(option: int) -> int:
    return int(_lib.easgd_get_option(option))


def version() -> int:
    return int(_lib.easgd_version())
