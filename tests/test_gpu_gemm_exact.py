"""The three matrix products of forward / backward propagation (Section 2.2), each alone, on integer-valued
operands: every product and every partial sum is then an integer below 2^24, exact in fp32 whatever the order of
the k sum, so the MFMA kernels must reproduce a plain triple loop BIT FOR BIT.  A k slab that is dropped, read
twice or read past its end, a wrong ones row (bias), a transposed operand or a tile written to the wrong place
cannot hide under a rounding tolerance here.  Every operand-layout combination (forward: k-contiguous x
n-contiguous; weight gradient: m-contiguous x n-contiguous; input gradient: k-contiguous x k-contiguous), every
tile shape (the 16x16x4 tiles in all three heights, forced and chosen by default), K not a multiple of the slab depth, ragged M and N, the tile that holds the ones row, operands that
rule out 128-bit loads, and enough workers for the die-aware block order."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host

F = np.float32

# (d_in, d_out, P, b): K = d_in + 1 (forward), b (weight gradient), d_out (input gradient)
SHAPES = [
    (64, 64, 1, 32),        # one tile, one slab pair; the ones row starts a tile of its own in the weight gradient
    (70, 50, 3, 37),        # nothing a multiple of 4: guarded scalar loaders
    (128, 96, 2, 100),      # ragged batch against the 32-row MFMA tile
    (257, 130, 9, 64),      # K = 258: partial last slab for both slab depths; ragged N
    (100, 10, 5, 128),      # narrow output: the 128x32 tile
    (36, 32, 4, 44),        # N = 32 exactly
    (512, 256, 8, 128),     # >= 64 tiles: die-aware renumbering; several k slabs per block
    (300, 260, 16, 70),     # many workers, ragged everything, multiples of 4
    (64, 2048, 32, 40),     # enough blocks for the 16-row MFMA tiles to be chosen by default: 48 rows for b = 40,
    (60, 2048, 32, 72),     # 80 rows for b = 72,
    (64, 2048, 32, 100),    # 112 rows for b = 100
]


def _ints(rng, shape, lo=-3, hi=3):
    return rng.integers(lo, hi + 1, size=shape).astype(F)


def _reference(kind, A, Wl, dZ, d_in, d_out, relu):
    """Plain definition in double (exact on these integers)."""
    P, b = A.shape[0], A.shape[1]
    A64 = A.astype(np.float64)
    if kind == 0:
        out = np.empty((P, b, d_out))
        for w in range(P):
            blk = Wl[w, :(d_in + 1) * d_out].astype(np.float64).reshape(d_in + 1, d_out)
            out[w] = A64[w] @ blk[:d_in] + blk[d_in][None, :]
        return np.maximum(out, 0.0) if relu else out
    if kind == 1:
        out = np.empty((P, d_in + 1, d_out))
        for w in range(P):
            out[w, :d_in] = A64[w].T @ dZ[w].astype(np.float64)
            out[w, d_in] = dZ[w].astype(np.float64).sum(axis=0)
        return out
    out = np.empty((P, b, d_in))
    for w in range(P):
        blk = Wl[w, :(d_in + 1) * d_out].astype(np.float64).reshape(d_in + 1, d_out)
        out[w] = (dZ[w].astype(np.float64) @ blk[:d_in].T) * (A64[w] > 0)
    return out


def test_reference_is_the_triple_loop():
    """The numpy reference above against literal loops on a tiny case (CPU arithmetic only)."""
    rng = np.random.default_rng(0)
    d_in, d_out, P, b = 5, 4, 2, 3
    A, dZ = _ints(rng, (P, b, d_in)), _ints(rng, (P, b, d_out))
    Wl = _ints(rng, (P, (d_in + 1) * d_out + 3))
    for kind in (0, 1, 2):
        ref = _reference(kind, A, Wl, dZ, d_in, d_out, relu=False)
        for w in range(P):
            blk = Wl[w, :(d_in + 1) * d_out].reshape(d_in + 1, d_out)
            if kind == 0:
                for r in range(b):
                    for n in range(d_out):
                        acc = float(blk[d_in, n])
                        for k in range(d_in):
                            acc += float(A[w, r, k]) * float(blk[k, n])
                        assert ref[w, r, n] == acc
            elif kind == 1:
                for m in range(d_in + 1):
                    for n in range(d_out):
                        acc = 0.0
                        for r in range(b):
                            acc += (float(A[w, r, m]) if m < d_in else 1.0) * float(dZ[w, r, n])
                        assert ref[w, m, n] == acc
            else:
                for r in range(b):
                    for k in range(d_in):
                        acc = 0.0
                        for n in range(d_out):
                            acc += float(dZ[w, r, n]) * float(blk[k, n])
                        assert ref[w, r, k] == (acc if A[w, r, k] > 0 else 0.0)


@pytest.mark.gpu
@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("d_in,d_out,P,b", SHAPES, ids=lambda v: str(v))
def test_each_product_is_exact_on_integers(d_in, d_out, P, b, tile):
    import paper_1708_02983_amd as hip
    rng = np.random.default_rng(1000 * d_in + d_out + P + b)
    block = (d_in + 1) * d_out
    ld = block + (4 - block % 4) % 4 + (4 if d_in % 4 == 0 else 3)     # padded; not a multiple of 4 for the odd shapes
    A, dZ = _ints(rng, (P, b, d_in)), _ints(rng, (P, b, d_out))
    Wl = np.full((P, ld), np.nan, dtype=F)
    Wl[:, :block] = _ints(rng, (P, block))
    dA_, dW_, dZ_ = to_dev(A), to_dev(Wl), to_dev(dZ)
    old = hip.get_option(hip.OPT_GEMM_TILE)
    try:
        hip.set_option(hip.OPT_GEMM_TILE, tile)
        for kind, relu in ((0, False), (0, True), (1, False), (2, False)):
            ref = _reference(kind, A, Wl, dZ, d_in, d_out, relu)
            assert np.abs(ref).max() < 2 ** 24
            width = ref.shape[1] * ref.shape[2]
            out_ws = width + 8                                          # padded worker stride, NaN-filled
            out = torch.full((P, out_ws), float("nan"), device="cuda")
            hip.easgd_layer_product(kind, d_in, d_out, dA_, out, Wl=dW_, dZ=dZ_, ld=ld, out_ws=out_ws, relu=relu)
            got = to_host(out)
            what = f"kind {kind} relu {relu} tile {tile}"
            assert np.isnan(got[:, width:]).all(), what                 # padding never written
            np.testing.assert_array_equal(got[:, :width].astype(np.float64), ref.reshape(P, width), err_msg=what)
    finally:
        hip.set_option(hip.OPT_GEMM_TILE, old)
