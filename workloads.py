"""Seeded synthetic inputs for the Sync EASGD hot path.

This module only *draws numbers and lays them out*: it contains none of the
method's arithmetic (no update rule, no forward/backward pass).  Both the CPU
oracle and the HIP library are fed from here so that they always see the same
bits; neither of them imports this module, the tests and the benchmark do.

The five workloads mirror the shapes of the paper's experiments (Table 1:
MNIST images are 28x28 = 784 pixels, CIFAR images 3x32x32 = 3072 pixels, both
with 10 classes; Section 6.1.1 quotes AlexNet at 249 MB, i.e. about 61 M fp32
words).  The real datasets are not used: inputs are random with the stated
distribution, labels are uniform over the classes.

Packed parameter layout (the paper's single-layer / packed-buffer idea,
Section 5.2): for each layer l in order, the weight matrix W_l[d_in][d_out]
row-major, followed by the bias b_l[d_out]; all layers back to back in one
flat fp32 vector of length N.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence, Tuple

import numpy as np

DEFAULT_SEED = 1234

# "N(0, s)" in the workload descriptions is read as mean 0, standard deviation s.
WEIGHT_STD = 0.01      # update-only replicas and the softmax-regression init
GRADIENT_STD = 1e-3    # update-only synthetic gradients
ALEXNET_SIZED_N = 61_000_000


@dataclass(frozen=True)
class Workload:
    name: str
    P: int                       # number of worker replicas
    eta: float                   # learning rate
    rho: float                   # elastic coefficient (worker and center both use eta*rho)
    rounds: int
    delta: Optional[float] = None            # momentum rate (paper's mu); None = plain EASGD
    dims: Optional[Tuple[int, ...]] = None   # MLP layer widths; None = update-only workload
    batch: int = 0                           # samples per worker per round
    x_dist: str = "normal"                   # "normal" = N(0,1), "uniform" = U[0,1]
    init: str = "he"                         # "he" = He-normal, "std" = N(0, WEIGHT_STD)
    N: int = 0                               # parameters per replica (derived for MLPs)

    @property
    def momentum(self) -> bool:
        return self.delta is not None

    @property
    def has_grad(self) -> bool:
        return self.dims is not None


def mlp_num_params(dims: Sequence[int]) -> int:
    return sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))


def _mlp(name, dims, **kw) -> Workload:
    return Workload(name=name, dims=tuple(dims), N=mlp_num_params(dims), **kw)


WORKLOADS = {
    "cfg1": _mlp("cfg1", (784, 10), P=4, batch=64, x_dist="normal", init="std",
                 eta=0.01, rho=0.1, rounds=10),
    "cfg2": _mlp("cfg2", (784, 1024, 1024, 10), P=16, batch=128, x_dist="uniform", init="he",
                 eta=0.05, rho=0.05, rounds=50),
    "cfg3": _mlp("cfg3", (3072, 2048, 2048, 10), P=32, batch=100, x_dist="normal", init="he",
                 eta=0.01, rho=0.05, delta=0.9, rounds=20),
    "cfg4": Workload("cfg4", P=8, N=ALEXNET_SIZED_N, eta=0.01, rho=0.1, rounds=100),
    "cfg5": Workload("cfg5", P=16, N=ALEXNET_SIZED_N, eta=0.01, rho=0.05, delta=0.9, rounds=100),
}


def _rng(seed: int, *stream: int) -> np.random.Generator:
    """Independent Philox stream per (seed, stream...) tuple."""
    return np.random.Generator(np.random.Philox(key=np.random.SeedSequence([seed, *stream]).generate_state(2, np.uint64)))


def round_up(n: int, m: int) -> int:
    return (n + m - 1) // m * m


# --------------------------------------------------------------------------
# MLP workloads (cfg1-cfg3): initial weights and per-round minibatches
# --------------------------------------------------------------------------

def init_packed_weights(wl: Workload, seed: int = DEFAULT_SEED) -> np.ndarray:
    """One packed initial parameter vector W0 of length N (fp32); biases are zero.

    Every replica and the center start as copies of this one vector (the
    initialisation loop of Algorithms 1-3)."""
    assert wl.dims is not None
    rng = _rng(seed, 0)
    out = np.zeros(wl.N, dtype=np.float32)
    off = 0
    for l in range(len(wl.dims) - 1):
        d_in, d_out = wl.dims[l], wl.dims[l + 1]
        std = WEIGHT_STD if wl.init == "std" else float(np.sqrt(2.0 / d_in))
        out[off:off + d_in * d_out] = (rng.standard_normal(d_in * d_out) * std).astype(np.float32)
        off += d_in * d_out + d_out          # bias stays 0
    assert off == wl.N
    return out


def replicate(w0: np.ndarray, P: int, ld: Optional[int] = None) -> np.ndarray:
    """[P][ld] array whose rows all start with w0; padding columns hold NaN so
    that a kernel touching them is caught."""
    N = w0.shape[0]
    ld = N if ld is None else ld
    out = np.full((P, ld), np.nan, dtype=np.float32)
    out[:, :N] = w0[None, :]
    return out


def minibatch(wl: Workload, t: int, seed: int = DEFAULT_SEED):
    """Inputs X[P][b][d_in] (fp32) and labels y[P][b] (int32) of round t."""
    assert wl.dims is not None
    rng = _rng(seed, 1, t)
    shape = (wl.P, wl.batch, wl.dims[0])
    if wl.x_dist == "uniform":
        X = rng.random(shape, dtype=np.float32)
    else:
        X = rng.standard_normal(shape, dtype=np.float32)
    y = rng.integers(0, wl.dims[-1], size=(wl.P, wl.batch), dtype=np.int32)
    return X, y


# --------------------------------------------------------------------------
# Update-only workloads (cfg4, cfg5) and generic elastic-update inputs
# --------------------------------------------------------------------------

def update_state(P: int, N: int, ld: Optional[int] = None, seed: int = DEFAULT_SEED,
                 std: float = WEIGHT_STD):
    """Independent draws for the replicas W[P][ld] and the center Wc[N]
    (identical replicas would make every elastic difference zero)."""
    ld = N if ld is None else ld
    rng = _rng(seed, 2)
    W = np.full((P, ld), np.nan, dtype=np.float32)
    W[:, :N] = rng.standard_normal((P, N), dtype=np.float32) * np.float32(std)
    Wc = rng.standard_normal(N, dtype=np.float32) * np.float32(std)
    return W, Wc


def update_gradients(P: int, N: int, t: int, ld: Optional[int] = None, seed: int = DEFAULT_SEED,
                     std: float = GRADIENT_STD) -> np.ndarray:
    """Synthetic gradients G[P][ld] of round t, regenerated from (seed, t)."""
    ld = N if ld is None else ld
    rng = _rng(seed, 3, t)
    G = np.full((P, ld), np.nan, dtype=np.float32)
    G[:, :N] = rng.standard_normal((P, N), dtype=np.float32) * np.float32(std)
    return G


def host_normal_rows(P: int, N: int, std: float, stream: int, seed: int = DEFAULT_SEED, threads: int = 8) -> np.ndarray:
    """[P][N] fp32 draws of N(0, std) in host memory, filled by several threads (one Philox stream per chunk):
    full-size update-only inputs for a host-side run, where a single stream would take a minute."""
    from concurrent.futures import ThreadPoolExecutor
    out = np.empty((P, N), dtype=np.float32)
    step = max(N // 4 + 1, 1)

    def fill(job):
        i, lo = job
        hi = min(lo + step, N)
        _rng(seed, stream, i, lo).standard_normal(out=out[i, lo:hi], dtype=np.float32)
        out[i, lo:hi] *= np.float32(std)

    with ThreadPoolExecutor(max(1, threads)) as ex:
        list(ex.map(fill, [(i, lo) for i in range(P) for lo in range(0, N, step)]))
    return out


# --------------------------------------------------------------------------
# Full-size update-only inputs drawn directly in device memory.
# torch is used purely as a seeded random-number source here.
# --------------------------------------------------------------------------

def device_normal(shape, std: float, seed: int, stream: int, device="cuda"):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1_000_003 + stream)
    out = torch.empty(shape, dtype=torch.float32, device=device)
    out.normal_(0.0, std, generator=g)
    return out


def sample_columns(N: int, n_blocks: int = 64, block: int = 1024, seed: int = DEFAULT_SEED) -> np.ndarray:
    """Sorted parameter indices used for sampled parity at full size: the first
    and last `block` indices plus `n_blocks` random contiguous runs."""
    rng = _rng(seed, 4)
    block = min(block, N)
    starts = [0, N - block] + list(rng.integers(0, max(N - block, 1), size=n_blocks))
    idx = np.unique(np.concatenate([np.arange(s, s + block) for s in starts]))
    return idx[idx < N].astype(np.int64)
