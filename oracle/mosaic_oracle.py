"""CPU oracle for projection-level importance scoring and mask construction.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP path must compute.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does, and this file
imports nothing from the product package.

Everything is written out in float64 NumPy, step by step, in the order and
notation of the paper (Mosaic, arXiv 2504.06323):

  * activation column norms      -- the l2 norm term of Eq. 5 / Eq. 3, gathered
                                    over all calibration samples (Algorithm 1,
                                    the loop over S that fills A)
  * weight metric  omega         -- Eq. 5
  * projection outliers O, C, R  -- Eq. 6 and the three assignments of
                                    Algorithm 1 that follow the weight metric
  * layer outliers               -- Eq. 3 and Eq. 4 (the layer-level rule)
  * normalize(R_LLM) + planner   -- Algorithm 1's return value and the
                                    Projection Planner of Section 3.3
  * unstructured masking         -- Section 4.1.3, category 1
  * structured removal           -- Section 4.1.3, categories 2 and 3, Fig. 4

Readings taken where the paper is silent (each is listed in the design notes):
per-input-channel norms of the tensor a projection multiplies; plain l2 norm
with no division by the token count; one omega per parameter; strict ">" in
Eq. 6; per-output-row selection of the k smallest omega with the lower column
index pruned first among equals; structured group magnitude = squared l2 norm
of the already-masked gate row + up row + down column.

Parity status of each function:
  column_sumsq / column_norms      pinned (closed forms, library norm)
  weight_metric                    pinned (hand example, magnitude special case)
  outlier_stats / count_above      pinned (hand example, brute force, strictness)
  layer_outlier_stats              pinned (hand example, brute force, one-projection special case)
  plan_sparsity                    PARITY UNPINNED against the paper: the paper gives no
                                   formula for normalize() or for the planner's scaling;
                                   pinned only by the invariants it states (mean = p,
                                   more outliers => pruned less, equal ranks => uniform p)
  layer_ratios / plan_sparsity_layerwise
                                   the pooled ratio is pinned (hand example, brute force); the spread inherits
                                   plan_sparsity's status (PARITY UNPINNED against the paper, same invariants)
  select_smallest_per_row          pinned (brute-force sort, library top-k special case)
  group_magnitude / struct_rank    PARITY UNPINNED against the paper (no formula given for
                                   "lowest-magnitude" groups); pinned by brute force and
                                   by the dense-equivalence invariant
  struct_compact                   pinned (dense-equivalence of the MLP, exact gather)
  coupled_group_magnitude          PARITY UNPINNED against the paper (same gap as group_magnitude); pinned by
                                   brute force and by reducing to group_magnitude for one-row / one-column groups
  coupled_group_compact            pinned (dense-equivalence of grouped-query attention, exact gather)
"""
from __future__ import annotations

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- norms

def column_sumsq(x) -> np.ndarray:
    """sumsq[j] = sum over tokens t of X[t, j]^2  (the square of Eq. 5's norm term)."""
    x = _f64(x)
    return (x * x).sum(axis=0)


def column_norms(x) -> np.ndarray:
    """||X[:, j]||_2 per input channel j, over every calibration token (Eq. 5, Alg. 1)."""
    return np.sqrt(column_sumsq(x))


# --------------------------------------------------------------------------- Eq. 5

def weight_metric(w, norms) -> np.ndarray:
    """omega[i, j] = ||A_j||_2 * |theta[i, j]|  (Eq. 5); the norm is broadcast over output rows."""
    w = _f64(w)
    norms = _f64(norms)
    assert w.ndim == 2 and norms.shape == (w.shape[1],)
    return np.abs(w) * norms[None, :]


# --------------------------------------------------------------------------- Eq. 6

def outlier_stats(omega, alpha: float):
    """Algorithm 1, the four steps after the weight metric.

    Returns (C, O, R, mean): parameter count, number of outliers
    #{omega_i > alpha * mean(omega)} with a strict comparison (Eq. 6),
    the projection rank R = O / C * 100, and the mean itself.
    """
    flat = _f64(omega).reshape(-1)          # flatten
    c = flat.size                           # C = numel
    mean = flat.sum() / c
    o = int(np.count_nonzero(flat > alpha * mean))
    return c, o, 100.0 * o / c, mean


def layer_outlier_stats(omegas, alpha: float):
    """Layer Outlier Distribution (Eq. 3, Eq. 4): the layer-level rule the projection rule refines.

    omegas are the weight metrics of all projections of one layer.  The metric
    vector of the layer is their concatenation; a parameter is an outlier if its
    metric exceeds alpha times the mean over the whole layer (strict).  Returns
    (C, O, R, mean, per-projection outlier counts).
    """
    flat = np.concatenate([_f64(o).reshape(-1) for o in omegas])
    c = flat.size
    mean = flat.sum() / c
    per_proj = [int(np.count_nonzero(_f64(o) > alpha * mean)) for o in omegas]
    o = int(np.count_nonzero(flat > alpha * mean))
    return c, o, 100.0 * o / c, mean, per_proj


def count_above(scores, tau) -> int:
    """#{scores > tau} evaluated in the dtype the scores already have.

    Used for the bit-exact protocol: the kernel's own score bits and its own
    float32 threshold go in, so the integer decision is taken in the kernel's
    precision on both sides.
    """
    scores = np.asarray(scores)
    tau = scores.dtype.type(tau)
    return int(np.count_nonzero(scores > tau))


def threshold_f32(alpha: float, score_sum: float, numel: int) -> np.float32:
    """tau = alpha * mean, formed in float64 and rounded once to float32."""
    return np.float32(np.float64(alpha) * np.float64(score_sum) / np.float64(numel))


# --------------------------------------------------------------------------- planner

def plan_sparsity(ratios, p: float, lam: float, scope: str = "global", cols=None):
    """normalize(R_LLM) and the Projection Planner: ranks -> per-projection sparsity targets.

    ratios is the N x M table R_LLM.  Within a comparison scope (all N*M
    entries, or one projection category m across the N layers) the ranks are
    min-max normalised to [0, 1] and spread about the scope mean:

        r_hat = (R - R_min) / (R_max - R_min)
        s     = p + 2 * lam * (mean(r_hat) - r_hat)

    so that the unweighted mean of s equals p (Eq. 1 and Eq. 2), projections
    with more outliers get a smaller target, and equal ranks give s == p
    everywhere (global pruning).  If cols is given (N x M input widths) each
    target is clamped to [0, 1 - 1/cols].  Returns (s, clamped_flag).
    """
    r = _f64(ratios)
    assert r.ndim == 2
    s = np.empty_like(r)

    def spread(block):
        lo, hi = block.min(), block.max()
        if hi == lo:
            return np.full_like(block, p)
        r_hat = (block - lo) / (hi - lo)
        return p + 2.0 * lam * (r_hat.mean() - r_hat)

    if scope == "global":
        s[:, :] = spread(r)
    elif scope == "category":
        for m in range(r.shape[1]):
            s[:, m] = spread(r[:, m])
    else:
        raise ValueError(scope)

    clamped = False
    if cols is not None:
        upper = 1.0 - 1.0 / _f64(cols)
        t = np.minimum(np.maximum(s, 0.0), upper)
        clamped = bool(np.any(t != s))
        s = t
    return s, clamped


def layer_ratios(counts, numels) -> np.ndarray:
    """R_n = 100 * (outliers of layer n) / (parameters of layer n), from the N x M tables of per-projection
    outlier counts and sizes: Algorithm 1's ratio taken over a whole layer, which is what the layer outlier
    distribution compares between layers (Eq. 3, Eq. 4).  The counts are meant to be those against the
    layer's mean (layer_outlier_stats)."""
    c = np.asarray(counts, dtype=np.int64)
    e = np.asarray(numels, dtype=np.int64)
    assert c.ndim == 2 and c.shape == e.shape
    return 100.0 * _f64(c.sum(axis=1)) / _f64(e.sum(axis=1))


def plan_sparsity_layerwise(counts, numels, p: float, lam: float, cols=None):
    """Layer pruning (Section 4.1.3, Pruning Methods, item 2; Section 3.1, layer / block-wise pruning):
    one target p_n per layer, derived from the N layer ratios by the same normalise-and-spread rule as the
    projection targets, and every projection of layer n is pruned by p_n.  The unweighted mean of p_n over
    the layers is p (Eq. 1).  Returns (s [N, M], clamped_flag) like plan_sparsity."""
    c = np.asarray(counts, dtype=np.int64)
    s_layer, _ = plan_sparsity(layer_ratios(counts, numels)[:, None], p, lam, "global")
    s = np.repeat(s_layer, c.shape[1], axis=1)
    clamped = False
    if cols is not None:
        upper = 1.0 - 1.0 / _f64(cols)
        t = np.minimum(np.maximum(s, 0.0), upper)
        clamped = bool(np.any(t != s))
        s = t
    return s, clamped


def zeros_per_row(sparsity: float, cols: int) -> int:
    """k = floor(s * cols) in float64."""
    return int(np.floor(np.float64(sparsity) * np.float64(cols)))


# --------------------------------------------------------------------------- unstructured

def select_smallest_per_row(omega, k: int) -> np.ndarray:
    """Boolean [rows, cols], True = pruned: in every output row the k smallest omega.

    A full stable ascending sort of each row by omega; among equal omega the
    lower column comes first, which makes the result unique.  Works on any
    real dtype (float64 oracle scores, or the kernel's float32 score bits).
    """
    omega = np.asarray(omega)
    rows, cols = omega.shape
    assert 0 <= k <= cols
    pruned = np.zeros((rows, cols), dtype=bool)
    if k == 0:
        return pruned
    order = np.argsort(omega, axis=1, kind="stable")
    np.put_along_axis(pruned, order[:, :k], True, axis=1)
    return pruned


def apply_mask(w, pruned) -> np.ndarray:
    """Unstructured pruning: pruned parameters are set to zero, survivors untouched."""
    out = np.array(w, copy=True)
    out[np.asarray(pruned, dtype=bool)] = 0
    return out


def pack_keep_bits(pruned) -> np.ndarray:
    """uint32 [rows, ceil(cols/32)]; bit b of word q is 1 iff column 32*q + b is kept."""
    pruned = np.asarray(pruned, dtype=bool)
    rows, cols = pruned.shape
    words = (cols + 31) // 32
    keep = np.zeros((rows, words * 32), dtype=np.uint64)
    keep[:, :cols] = ~pruned
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (keep.reshape(rows, words, 32) * weights).sum(axis=2).astype(np.uint32)


# --------------------------------------------------------------------------- structured

def group_magnitude(gate, up, down) -> np.ndarray:
    """g[c] = ||gate[c, :]||^2 + ||up[c, :]||^2 + ||down[:, c]||^2 on the (masked) weights.

    Channel c of the MLP intermediate dimension couples one row of gate, one
    row of up and one column of down; they are scored and removed as a group.
    """
    gate, up, down = _f64(gate), _f64(up), _f64(down)
    inter = gate.shape[0]
    assert up.shape == gate.shape and down.shape == (gate.shape[1], inter)
    return (gate * gate).sum(axis=1) + (up * up).sum(axis=1) + (down * down).sum(axis=0)


def struct_rank(g, r: int) -> np.ndarray:
    """Indices (ascending) of the channels kept after removing the r lowest-magnitude groups.

    Stable ascending sort by g, lower channel index first among equals.
    """
    g = np.asarray(g)
    n = g.shape[0]
    assert 0 <= r < n
    order = np.argsort(g, kind="stable")
    return np.sort(order[r:]).astype(np.int32)


def struct_compact(gate, up, down, kept_idx):
    """Physically remove the dropped channels: gate[kept, :], up[kept, :], down[:, kept]."""
    kept_idx = np.asarray(kept_idx)
    return (np.asarray(gate)[kept_idx, :].copy(),
            np.asarray(up)[kept_idx, :].copy(),
            np.asarray(down)[:, kept_idx].copy())


def coupled_group_magnitude(row_mats, row_per, col_mats, col_per, n_groups: int) -> np.ndarray:
    """Magnitude of groups that span several matrices (attention heads, feed-forward channels).

    Group g owns rows [g * row_per[i], (g + 1) * row_per[i]) of row_mats[i] and columns
    [g * col_per[i], (g + 1) * col_per[i]) of col_mats[i]; its magnitude is the sum of squares of
    all of them.  With one row per group in gate and up and one column in down this is
    group_magnitude(); with grouped-query attention a group is one key/value head: its k and v
    rows, the q rows of the query heads that share it, and the matching columns of o.
    """
    g = np.zeros(n_groups, dtype=np.float64)
    for m, per in zip(row_mats, row_per):
        m = _f64(m)
        assert m.shape[0] == n_groups * per
        g += (m * m).sum(axis=1).reshape(n_groups, per).sum(axis=1)
    for m, per in zip(col_mats, col_per):
        m = _f64(m)
        assert m.shape[1] == n_groups * per
        g += (m * m).sum(axis=0).reshape(n_groups, per).sum(axis=1)
    return g


def coupled_group_compact(row_mats, row_per, col_mats, col_per, kept_idx):
    """Keep only what the kept groups own: their rows of every row matrix, their columns of every column matrix."""
    kept_idx = np.asarray(kept_idx, dtype=np.int64)
    rows_out, cols_out = [], []
    for m, per in zip(row_mats, row_per):
        idx = (kept_idx[:, None] * per + np.arange(per)[None, :]).reshape(-1)
        rows_out.append(np.asarray(m)[idx, :].copy())
    for m, per in zip(col_mats, col_per):
        idx = (kept_idx[:, None] * per + np.arange(per)[None, :]).reshape(-1)
        cols_out.append(np.asarray(m)[:, idx].copy())
    return rows_out, cols_out


# --------------------------------------------------------------------------- whole path

def rank_projection(x, w, alpha: float):
    """Ranking Controller work for one projection: norms, omega, (C, O, R, mean)."""
    norms = column_norms(x)
    omega = weight_metric(w, norms)
    return (norms, omega) + outlier_stats(omega, alpha)


def prune_projection(w, omega, k: int):
    """Pruning Controller, unstructured category, one projection."""
    pruned = select_smallest_per_row(omega, k)
    return apply_mask(w, pruned), pruned
