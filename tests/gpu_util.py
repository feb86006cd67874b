"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

PER_ROUND_TOL = 1e-5      # fp32, one round, max |x-y| / max |y| per tensor
HUNDRED_ROUND_TOL = 1e-4  # after 100 free-running rounds


def normwise(x: np.ndarray, y: np.ndarray) -> float:
    """max_j |x_j - y_j| / max_j |y_j| over the finite entries of the reference y
    (NaN padding must be NaN in both)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    pad = np.isnan(y)
    assert np.array_equal(np.isnan(x), pad), "padding / validity pattern differs"
    if pad.all():
        return 0.0
    scale = np.abs(y[~pad]).max()
    diff = np.abs(x[~pad] - y[~pad]).max()
    return float(diff / scale) if scale > 0 else float(diff)


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


# |z| <= NEAR_REL * max|Z_layer| counts as "within fp32 rounding of zero" in the teacher-forced checks.
# A length-K fp32 dot product accumulated in sequence has an rms rounding error of about
# (eps/2) * sigma_z * sqrt(K/2): for K = 3073, sigma_z = 1.4 that is 2e-6, and max|Z| is about 7, so 1e-5 * max|Z|
# leaves a factor of about 30 for the tail over millions of units and for error carried in from the layer below.
NEAR_REL = 1e-5


def match_gradient(g_gpu, dims, w, X, y, tol, near_rel=NEAR_REL, max_ties=14):
    """GPU gradient of one worker against the oracle.  Hidden units whose pre-activation is within
    rounding of zero (|z| <= near_rel * max|Z_layer|, judged on the oracle's own z) have a ReLU gate
    that either side may decide either way; if the plain comparison fails, the oracle is re-evaluated
    with gates of such units flipped and the GPU result must match one of these valid gradients.
    The search is narrowed to near-zero units whose bias gradient differs (a flipped gate (n, u)
    changes db[u] by exactly the signal that reached the unit), then runs over all subsets, smallest
    first.  Returns (matching oracle gradient, oracle loss, number of flipped gates)."""
    import itertools
    import oracle
    sl = oracle.layer_slices(dims)
    N = sl[-1][1].stop
    near = []
    g_ref, loss_ref = oracle.mlp_grad(dims, w, X, y, near_zero=near, near_zero_rel=near_rel)
    errs = [normwise(g_gpu[:N], g_ref)]
    if errs[0] <= tol:
        return g_ref, loss_ref, 0
    scale = np.abs(g_ref).max()

    def bias_residual(g_oracle):
        out = {}
        for l, (_, b_sl) in enumerate(sl[:-1]):
            r = np.abs(g_gpu[b_sl].astype(np.float64) - g_oracle[b_sl])
            out.update({(l, int(u)): float(r[u] / scale) for u in np.nonzero(r > 0.1 * tol * scale)[0]})
        return out

    suspicious = bias_residual(g_ref)
    cand = [t for t in near if (t[0], t[2]) in suspicious]
    assert cand, (f"gradient differs from the oracle by {errs[0]:.3e} and none of the {len(near)} near-zero "
                  f"ReLU gates sits in a unit whose bias gradient differs")
    assert len(cand) <= max_ties, f"{len(cand)} candidate gates: too many to enumerate"
    best = (errs[0], g_ref, ())
    for k in range(1, len(cand) + 1):
        for subset in itertools.combinations(cand, k):
            g_alt, _ = oracle.mlp_grad(dims, w, X, y, gate_flips=subset)
            e = normwise(g_gpu[:N], g_alt)
            if e < best[0]:
                best = (e, g_alt, subset)
            if e <= tol:
                return g_alt, loss_ref, k
    left = sorted(bias_residual(best[1]).items(), key=lambda kv: -kv[1])[:6]
    raise AssertionError(f"gradient matches no valid gate assignment of the {len(cand)} candidate units {cand}; "
                         f"best normwise error {best[0]:.3e} > {tol:g} with flips {best[2]} (plain {errs[0]:.3e}); "
                         f"hidden units whose bias gradient still differs (layer, unit): rel. residual = {left}")


def match_gradients_all_workers(G_gpu, dims, W, X, y, tol, near_rel=NEAR_REL):
    """match_gradient for every worker: oracle G[P][ld] (NaN padding), losses, total flipped gates."""
    P, ld = W.shape
    G = np.full((P, ld), np.nan, dtype=np.float32)
    N = None
    loss = np.zeros(P)
    flips = 0
    for i in range(P):
        g, loss[i], k = match_gradient(G_gpu[i], dims, W[i], X[i], y[i], tol, near_rel)
        G[i, :g.shape[0]] = g
        flips += k
    return G, loss, flips
