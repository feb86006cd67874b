"""CPU ORACLE (test infrastructure): ctypes front end of ``elastic.c``.

``easgd_round`` evaluates Eq. (1)+(2), ``measgd_round`` Eq. (5)+(6)+(2), once,
in place, on fp32 numpy arrays, with double arithmetic inside.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "elastic.c")
_LIB = os.path.join(_HERE, "liboracle_elastic.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile elastic.c with gcc into liboracle_elastic.so (beside the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.oracle_easgd_round.argtypes = [f32p, f32p, f32p, ctypes.c_int, ctypes.c_size_t,
                                           ctypes.c_size_t, ctypes.c_double, ctypes.c_double,
                                           ctypes.c_double]
        lib.oracle_easgd_round.restype = None
        lib.oracle_measgd_round.argtypes = [f32p, f32p, f32p, f32p, ctypes.c_int, ctypes.c_size_t,
                                            ctypes.c_size_t, ctypes.c_double, ctypes.c_double,
                                            ctypes.c_double, ctypes.c_double]
        lib.oracle_measgd_round.restype = None
        lib.oracle_sync_sgd_round.argtypes = [f32p, f32p, f32p, ctypes.c_int, ctypes.c_size_t,
                                              ctypes.c_size_t, ctypes.c_double, ctypes.c_double]
        lib.oracle_sync_sgd_round.restype = None
        lib.oracle_async_easgd.argtypes = [f32p, f32p, f32p, f32p, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_double, ctypes.c_double]
        lib.oracle_async_easgd.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads used by the C loops from now on (n < 1: all cores); only the timing of the oracle uses this."""
    _load().oracle_set_num_threads(int(n))


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _check(name, a, shape=None):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]):
        raise TypeError(f"{name} must be a C-contiguous float32 numpy array")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {a.shape}, expected {shape}")


def easgd_round(W: np.ndarray, G: np.ndarray, Wc: np.ndarray, eta: float, rho: float,
                N: Optional[int] = None, center_coef: Optional[float] = None) -> None:
    """One Sync EASGD exchange-and-update, in place on W[P][ld] and Wc[N].

    ``center_coef`` defaults to eta*rho, which is Eq. (2)."""
    _check("W", W)
    P, ld = W.shape
    N = Wc.shape[0] if N is None else N
    _check("G", G, (P, ld))
    _check("Wc", Wc, (N,))
    if ld < N:
        raise ValueError("ld < N")
    cc = float(eta) * float(rho) if center_coef is None else float(center_coef)
    _load().oracle_easgd_round(_ptr(W), _ptr(G), _ptr(Wc), P, N, ld, float(eta), float(rho), cc)


def measgd_round(W: np.ndarray, V: np.ndarray, G: np.ndarray, Wc: np.ndarray, eta: float,
                 rho: float, mu: float, N: Optional[int] = None,
                 center_coef: Optional[float] = None) -> None:
    """One Sync MEASGD exchange-and-update, in place on W, V [P][ld] and Wc[N]."""
    _check("W", W)
    P, ld = W.shape
    N = Wc.shape[0] if N is None else N
    _check("V", V, (P, ld))
    _check("G", G, (P, ld))
    _check("Wc", Wc, (N,))
    if ld < N:
        raise ValueError("ld < N")
    cc = float(eta) * float(rho) if center_coef is None else float(center_coef)
    _load().oracle_measgd_round(_ptr(W), _ptr(V), _ptr(G), _ptr(Wc), P, N, ld,
                                float(eta), float(rho), float(mu), cc)


def sync_sgd_round(W: np.ndarray, G: np.ndarray, eta: float, V: Optional[np.ndarray] = None,
                   mu: float = 0.0, N: Optional[int] = None) -> None:
    """One round of synchronous data-parallel SGD on P replicas, in place on W[P][ld] (and V):
    every replica moves by the sum of all workers' gradients (Section 2.3; Section 6.2); with V the
    sum drives the momentum rule Eq. (3),(4)."""
    _check("W", W)
    P, ld = W.shape
    N = ld if N is None else N
    _check("G", G, (P, ld))
    if V is not None:
        _check("V", V, (P, ld))
    if ld < N:
        raise ValueError("ld < N")
    _load().oracle_sync_sgd_round(_ptr(W), None if V is None else _ptr(V), _ptr(G), P, N, ld,
                                  float(eta), float(mu))


def async_easgd(W: np.ndarray, G: np.ndarray, Wc: np.ndarray, order, eta: float, rho: float,
                V: Optional[np.ndarray] = None, mu: float = 0.0, N: Optional[int] = None,
                center_coef: Optional[float] = None) -> None:
    """The master serving one worker at a time, in the sequence ``order`` (Algorithm 1 in rank order; Async
    EASGD / Async MEASGD in arrival order): per turn Eq. (1) (Eq. (5),(6) with V) for that worker and the
    one-worker form of Eq. (2) for the center, both from the values at the start of the turn.  In place."""
    _check("W", W)
    P, ld = W.shape
    N = Wc.shape[0] if N is None else N
    _check("G", G, (P, ld))
    _check("Wc", Wc, (N,))
    if V is not None:
        _check("V", V, (P, ld))
    if ld < N:
        raise ValueError("ld < N")
    seq = np.ascontiguousarray(np.asarray(order, dtype=np.int32))
    if seq.ndim != 1 or (seq.size and (seq.min() < 0 or seq.max() >= P)):
        raise ValueError("order must be a sequence of worker indices in [0, P)")
    cc = float(eta) * float(rho) if center_coef is None else float(center_coef)
    _load().oracle_async_easgd(_ptr(W), None if V is None else _ptr(V), _ptr(G), _ptr(Wc), P, N, ld,
                               seq.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), int(seq.size),
                               float(eta), float(rho), float(mu), cc)
