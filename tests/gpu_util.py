"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

PER_ROUND_TOL = 1e-5      # fp32, one round, max |x-y| / max |y| per tensor
HUNDRED_ROUND_TOL = 1e-4  # after 100 free-running rounds


def normwise(x: np.ndarray, y: np.ndarray) -> float:
    """max_j |x_j - y_j| / max_j |y_j| over the finite entries of the reference y
    (NaN padding must be NaN in both).  Evaluated in double, chunk by chunk on a few threads: the
    full-size tensors hold hundreds of millions of entries."""
    from concurrent.futures import ThreadPoolExecutor
    x = np.ascontiguousarray(x).reshape(-1)
    y = np.ascontiguousarray(y).reshape(-1)
    assert x.shape == y.shape, "shapes differ"
    chunk = 1 << 22

    def part(s):
        xc = x[s:s + chunk].astype(np.float64)
        yc = y[s:s + chunk].astype(np.float64)
        pad = np.isnan(yc)
        same = np.array_equal(np.isnan(xc), pad)
        if pad.any():
            xc[pad] = 0.0
            yc[pad] = 0.0
        return same, bool(pad.all()), float(np.abs(yc).max()), float(np.abs(xc - yc).max())

    starts = range(0, x.size, chunk)
    if x.size > 4 * chunk:
        with ThreadPoolExecutor(8) as ex:
            parts = list(ex.map(part, starts))
    else:
        parts = [part(s) for s in starts]
    assert all(p[0] for p in parts), "padding / validity pattern differs"
    if all(p[1] for p in parts):
        return 0.0
    scale = max(p[2] for p in parts)
    diff = max(p[3] for p in parts)
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


def oracle_gradient_base(dims, w, X, y, near_rel):
    """The oracle's gradient of one worker with its near-zero ReLU gates (|z| <= near_rel * max|Z_layer|) and their
    ratios |z| / max|Z_layer|: what match_gradient starts from.  Computed once when the same state is matched
    against two GPU results (teacher-forced and free-running rounds start from the same oracle state)."""
    import oracle
    near, ratio = [], []
    g_ref, loss_ref = oracle.mlp_grad(dims, w, X, y, near_zero=near, near_zero_rel=near_rel, near_zero_ratio=ratio)
    return g_ref, loss_ref, near, ratio, near_rel


def match_gradient(g_gpu, dims, w, X, y, tol, near_rel=NEAR_REL, max_ties=14, base=None):
    """GPU gradient of one worker against the oracle.  Hidden units whose pre-activation is within
    rounding of zero (|z| <= near_rel * max|Z_layer|, judged on the oracle's own z) have a ReLU gate
    that either side may decide either way; if the plain comparison fails, the oracle is re-evaluated
    with gates of such units flipped and the GPU result must match one of these valid gradients.

    A flipped gate (n, u) of hidden layer l changes the gradient blocks of layer l and of the layers
    below it, never those above, and it changes db_l[u] by exactly the signal that reached the unit.
    The search therefore goes from the top hidden layer down; in each layer the candidates are the
    near-zero units whose bias gradient still differs, and all their subsets are tried, smallest first,
    until the blocks of that layer agree.  Returns (matching oracle gradient, oracle loss, flipped gates)."""
    import itertools
    import oracle
    sl = oracle.layer_slices(dims)
    N = sl[-1][1].stop
    if base is None:
        base = oracle_gradient_base(dims, w, X, y, near_rel)
    assert base[4] >= near_rel
    g_ref, loss_ref = base[0], base[1]
    near = [t for t, r in zip(base[2], base[3]) if r <= near_rel]
    plain = normwise(g_gpu[:N], g_ref)
    if plain <= tol:
        return g_ref, loss_ref, 0
    scale = np.abs(g_ref).max()
    gpu64 = g_gpu[:N].astype(np.float64)

    def block_err(g_oracle, l):
        w_sl, b_sl = sl[l]
        return max(np.abs(gpu64[w_sl] - g_oracle[w_sl]).max(), np.abs(gpu64[b_sl] - g_oracle[b_sl]).max()) / scale

    flips, g_best = (), g_ref
    for l in range(len(sl) - 2, -1, -1):            # hidden layers, top down
        if block_err(g_best, l) <= tol:
            continue
        r = np.abs(gpu64[sl[l][1]] - g_best[sl[l][1]]) / scale
        units = set(int(u) for u in np.nonzero(r > 0.1 * tol)[0])
        cand = [t for t in near if t[0] == l and t[2] in units]
        assert cand, (f"layer {l} gradient differs from the oracle by {block_err(g_best, l):.3e} and none of the "
                      f"near-zero ReLU gates of that layer sits in a unit whose bias gradient differs")
        assert len(cand) <= max_ties, f"layer {l}: {len(cand)} candidate gates, too many to enumerate"
        found = False
        for k in range(1, len(cand) + 1):
            for subset in itertools.combinations(cand, k):
                g_alt, _ = oracle.mlp_grad(dims, w, X, y, gate_flips=flips + subset)
                if block_err(g_alt, l) <= tol:
                    flips, g_best, found = flips + subset, g_alt, True
                    break
            if found:
                break
        assert found, (f"layer {l} gradient matches no gate assignment of its {len(cand)} candidate near-zero units "
                       f"{cand}; error {block_err(g_best, l):.3e} > {tol:g}")
    final = normwise(g_gpu[:N], g_best)
    assert final <= tol, f"gradient differs from the oracle by {final:.3e} > {tol:g} after resolving {len(flips)} gate ties (plain {plain:.3e})"
    return g_best, loss_ref, len(flips)


def match_gradients_all_workers(G_gpu, dims, W, X, y, tol, near_rel=NEAR_REL, bases=None):
    """match_gradient for every worker: oracle G[P][ld] (NaN padding), losses, total flipped gates.
    bases: per worker what oracle_gradient_base returned for this state (with a near_rel at least as wide)."""
    P, ld = W.shape
    G = np.full((P, ld), np.nan, dtype=np.float32)
    N = None
    loss = np.zeros(P)
    flips = 0
    for i in range(P):
        g, loss[i], k = match_gradient(G_gpu[i], dims, W[i], X[i], y[i], tol, near_rel,
                                       base=None if bases is None else bases[i])
        G[i, :g.shape[0]] = g
        flips += k
    return G, loss, flips
