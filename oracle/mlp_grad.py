"""CPU ORACLE (test infrastructure): minibatch gradient of a dense ReLU MLP.

Step (1) of Sync EASGD (Section 5.1): worker i computes its sub-gradient
dW^i_t from its own minibatch at its own weights W^i_t, by forward and
backward propagation (Section 2.2).  The paper does not name the loss; the
workloads here are "softmax regression" and "MLP with ReLU", so the loss is
softmax cross-entropy averaged over the b samples of the worker's minibatch.

Everything is evaluated in double; inputs are widened from fp32 and the
gradient is rounded to fp32 once at the end.  The matrix products are numpy's
``@`` (a library primitive used as one step); there is no blocking or fusion.

Packed layout: per layer, weight W_l[d_in][d_out] row-major, then bias
b_l[d_out]; layers back to back (the packed single buffer of Section 5.2).
"""
from __future__ import annotations

from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np


def layer_slices(dims: Sequence[int]) -> List[Tuple[slice, slice]]:
    """(weight slice, bias slice) into the packed vector for every layer."""
    out, off = [], 0
    for d_in, d_out in zip(dims[:-1], dims[1:]):
        w = slice(off, off + d_in * d_out)
        b = slice(w.stop, w.stop + d_out)
        out.append((w, b))
        off = b.stop
    return out


def mlp_grad(dims: Sequence[int], w_packed: np.ndarray, X: np.ndarray, y: np.ndarray,
             gate_flips: Iterable[Tuple[int, int, int]] = (), near_zero: Optional[list] = None,
             near_zero_rel: float = 0.0, near_zero_ratio: Optional[list] = None):
    """Gradient (packed, fp32) and mean loss (float) for ONE worker.

    w_packed: [>=N] fp32, X: [b][dims[0]] fp32, y: [b] integer labels in [0, dims[-1]).

    The ReLU derivative is a step: a hidden unit whose pre-activation z is within
    rounding of zero has a gate (z > 0) that fp32 and fp64 arithmetic may decide
    differently, and either decision is a valid gradient of the fp32 computation.
    By default the gate is decided here in double.  For such ties a caller can
    ask which units are near zero (``near_zero`` list is filled with
    (layer, sample, unit) where |z| <= near_zero_rel * max|Z_layer|; ``near_zero_ratio``,
    if given, receives |z| / max|Z_layer| of each of them) and evaluate
    the other decision by passing those triples in ``gate_flips``."""
    sl = layer_slices(dims)
    L = len(sl)
    b = X.shape[0]
    Ws = [w_packed[w].astype(np.float64).reshape(dims[l], dims[l + 1]) for l, (w, _) in enumerate(sl)]
    bs = [w_packed[bb].astype(np.float64) for _, bb in sl]

    # forward propagation
    acts = [X.astype(np.float64)]          # A_0 = X, A_l = relu(Z_l)
    zs = []
    for l in range(L):
        z = acts[-1] @ Ws[l] + bs[l][None, :]
        zs.append(z)
        if l < L - 1:
            acts.append(np.maximum(z, 0.0))
    logits = zs[-1]
    shifted = logits - logits.max(axis=1, keepdims=True)
    log_p = shifted - np.log(np.exp(shifted).sum(axis=1, keepdims=True))
    rows = np.arange(b)
    loss = float(-log_p[rows, y].mean())

    flips = list(gate_flips)
    if near_zero is not None:
        for l in range(L - 1):
            zmax = np.abs(zs[l]).max()
            n_idx, u_idx = np.nonzero(np.abs(zs[l]) <= near_zero_rel * zmax)
            near_zero.extend((l, int(n), int(u)) for n, u in zip(n_idx, u_idx))
            if near_zero_ratio is not None:
                near_zero_ratio.extend(float(abs(zs[l][n, u]) / zmax) if zmax > 0 else 0.0 for n, u in zip(n_idx, u_idx))

    # backward propagation
    dz = np.exp(log_p)
    dz[rows, y] -= 1.0
    dz /= b                                 # d(mean loss)/d(logits)
    grad = np.zeros(sl[-1][1].stop, dtype=np.float64)
    for l in range(L - 1, -1, -1):
        w_sl, b_sl = sl[l]
        grad[w_sl] = (acts[l].T @ dz).reshape(-1)
        grad[b_sl] = dz.sum(axis=0)
        if l > 0:
            da = dz @ Ws[l].T
            gate = zs[l - 1] > 0.0          # ReLU derivative, 0 at z == 0
            for (fl, n, u) in flips:
                if fl == l - 1:
                    gate[n, u] = ~gate[n, u]
            dz = da * gate
    return grad.astype(np.float32), loss


def mlp_grad_all_workers(dims: Sequence[int], W: np.ndarray, X: np.ndarray, y: np.ndarray):
    """Step (1) for all P workers: W[P][ld], X[P][b][d_in], y[P][b] ->
    G[P][ld] (padding columns NaN) and loss[P]."""
    P, ld = W.shape
    N = layer_slices(dims)[-1][1].stop
    G = np.full((P, ld), np.nan, dtype=np.float32)
    loss = np.zeros(P, dtype=np.float64)
    for i in range(P):
        G[i, :N], loss[i] = mlp_grad(dims, W[i], X[i], y[i])
    return G, loss
