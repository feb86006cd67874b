"""CPU ORACLE (test infrastructure): the elastic exchange-and-update with gradients and momentum
buffers STORED as bfloat16 -- an extension, not in the paper, whose Section 3.2 only names
low-precision arithmetic as future work.  The rules are the paper's (Eq. (1), (2), (5), (6));
this file fixes what "stored as bfloat16" means so that a kernel can be checked against it.

* bfloat16 = the upper 16 bits of an IEEE fp32 (1 sign, 8 exponent, 7 fraction bits).  Widening is
  exact.  Narrowing rounds to nearest, ties to the even 16-bit pattern; values beyond the largest
  finite bfloat16 become infinity; a NaN becomes the quiet NaN 0x7FC0 with the input's sign.
* Replicas W and the center Wc stay fp32.  G16 is only read.
* Eq. (5) decides a stored 16-bit code, so it is evaluated the way the kernel is specified to: in
  fp32, as fl(fl(mu*v) - fl(eta*g)) with v, g the widened stored values and mu, eta rounded to fp32,
  then narrowed.  Eq. (6) uses V_{t+1} as stored (like the fp32 oracle); it and Eq. (2) are
  evaluated in double and rounded once to fp32.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""
from __future__ import annotations

import numpy as np

from . import elastic


def bf16_widen(b16: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 patterns -> the fp32 values they stand for (exact)."""
    b = np.ascontiguousarray(b16, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values -> uint16 bfloat16 patterns, round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    keep = u >> np.uint32(16)                       # the 16 bits that stay
    rest = u & np.uint32(0xFFFF)                    # the 16 bits that go
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint32(1)) == 1))
    out = (keep + up.astype(np.uint32)).astype(np.uint32)
    is_nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    out = np.where(is_nan, ((u >> np.uint32(16)) & np.uint32(0x8000)) | np.uint32(0x7FC0), out)
    return out.astype(np.uint16)


def _check16(name, a, shape):
    if not (isinstance(a, np.ndarray) and a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]):
        raise TypeError(f"{name} must be a C-contiguous uint16 numpy array")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {a.shape}, expected {shape}")


def easgd_round_bf16(W: np.ndarray, G16: np.ndarray, Wc: np.ndarray, eta: float, rho: float) -> None:
    """Eq. (1)+(2) in place on W[P][ld], Wc[N]; the gradients are the widened G16[P][ld]."""
    _check16("G16", G16, W.shape)
    elastic.easgd_round(W, bf16_widen(G16), Wc, eta, rho)


def measgd_round_bf16(W: np.ndarray, V16: np.ndarray, G16: np.ndarray, Wc: np.ndarray,
                      eta: float, rho: float, mu: float) -> None:
    """Eq. (5)+(6)+(2) in place on W[P][ld] (fp32), V16[P][ld] (bfloat16 patterns) and Wc[N] (fp32).
    G16[P][ld]: the gradients, as bfloat16 patterns (uint16) or, when only V is stored in 16 bits, as fp32."""
    if not (W.dtype == np.float32 and Wc.dtype == np.float32 and W.ndim == 2 and Wc.ndim == 1):
        raise TypeError("W[P][ld] and Wc[N] must be float32")
    P, ld = W.shape
    N = Wc.shape[0]
    if ld < N:
        raise ValueError("ld < N")
    _check16("V16", V16, W.shape)
    if G16.dtype == np.float32:
        if G16.shape != W.shape:
            raise ValueError("G has the wrong shape")
        g = np.ascontiguousarray(G16[:, :N])
    else:
        _check16("G16", G16, W.shape)
        g = bf16_widen(G16[:, :N])
    c = Wc.astype(np.float64)                                   # Wc_t, seen by every worker
    w = W[:, :N].astype(np.float64)
    d = w - c[None, :]                                          # W^i_t - Wc_t
    v = bf16_widen(V16[:, :N])
    # Eq. (5) in fp32, one rounding per operation, then narrowed: this is the value that is stored
    cand = np.float32(mu) * v - np.float32(eta) * g
    v16_new = bf16_round(cand)
    v_new = bf16_widen(v16_new).astype(np.float64)
    w_new = w + v_new - float(eta) * float(rho) * d             # Eq. (6) with the stored V_{t+1}
    sum_d = np.zeros(N, dtype=np.float64)
    for i in range(P):                                          # ascending worker order
        sum_d += d[i]
    V16[:, :N] = v16_new
    W[:, :N] = w_new.astype(np.float32)
    Wc[:] = (c + float(eta) * float(rho) * sum_d).astype(np.float32)   # Eq. (2)
