"""CPU oracle for the Hessian-based one-shot pruner with per-projection targets.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this file; the product path never does, and this
file imports nothing from the product package.

The paper's experiments prune with "the inverse Hessian matrix and a subsequent
weight update in a one-shot manner" (Section 4.1.3, "Pruning Methods": the
SparseGPT pruner, an Optimal Brain Surgeon scheme), driven by the sparsity
target p_{n,m} that the Projection Planner assigns to each projection
(Section 3.3), with the 128 calibration samples also providing the Hessian
(Section 4.1.4, "Calibration").  The paper itself gives no formula for that
pruner; what follows is the published algorithm it cites, written out in
float64 step by step.  Every choice the paper leaves open is a reading:

  * Hessian of the layer-wise reconstruction problem min ||W X^T - W' X^T||^2:
    H = X^T X over all calibration tokens (any positive scaling of H gives the
    same result, because the damping below is relative to H's own diagonal).
  * An input channel that never fires (H_jj == 0) gets H_jj = 1 and its weight
    column is set to zero.
  * Damping: H += 0.01 * mean(diag H) * I.
  * Columns are processed left to right in blocks of 128.  When a block starts,
    its saliencies are (w_ij / U_jj)^2 with U the upper Cholesky factor of
    H^-1 (H^-1 = U^T U), and the floor(s * rows * width) entries of the block
    with the smallest saliency are pruned -- all rows of the block compete
    together, ties go to the lower (row, column) position in row-major order.
  * Inside the block, column by column: the pruned entries of the column are set
    to zero, the error e_i = (w_ij - w'_ij) / U_jj is spread over the columns to
    the right with row j of U (w_i,j+1: -= e_i * U_j,j+1:); after the block the
    same is applied to all later blocks at once (W[:, later] -= E U[block, later]).

Parity status:
  gram_matrix          pinned (brute-force loops, diagonal = column sums of squares, rank-1 closed form)
  damped_hessian       PARITY UNPINNED against the paper (it states no damping); pinned by hand example
  inverse_factor       pinned (U^T U H = I, triangular with positive diagonal, hand-worked 2 x 2)
  reverse_factor       pinned (R R^T = H, triangular, equals the Cholesky factor of the reversed matrix)
  select_block         pinned (brute-force sort)
  obs_sweep            pinned: identity Hessian reduces it to magnitude pruning without update; a single
                       pruned weight gives the closed-form Optimal Brain Surgeon update; for any mask the
                       weights agree with an independent elimination that inverts the trailing Hessian
                       explicitly; a pruned prefix of columns gives the least-squares optimum
"""
from __future__ import annotations

import numpy as np

BLOCK = 128
DAMP = 0.01


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def gram_matrix(x) -> np.ndarray:
    """H[i, j] = sum over tokens t of X[t, i] * X[t, j]."""
    x = _f64(x)
    return x.T @ x


def damped_hessian(h, damp: float = DAMP):
    """Dead channels get a unit diagonal, then damp * mean(diag) is added to the diagonal.
    Returns (H', dead) with dead[j] true where H_jj was zero."""
    h = _f64(h).copy()
    dead = np.diag(h) == 0.0
    h[dead, dead] = 1.0
    h[np.diag_indices_from(h)] += damp * np.mean(np.diag(h))
    return h, dead


def inverse_factor(h) -> np.ndarray:
    """Upper triangular U with positive diagonal and U^T U = H^-1."""
    return np.linalg.cholesky(np.linalg.inv(_f64(h))).T


def reverse_factor(h) -> np.ndarray:
    """Upper triangular R with positive diagonal and R R^T = H: the inverse of inverse_factor(h)."""
    return np.linalg.inv(inverse_factor(h))


def block_saliency(w_block, u_diag) -> np.ndarray:
    """(w_ij / U_jj)^2 for the columns of one block."""
    return (_f64(w_block) / _f64(u_diag)[None, :]) ** 2


def select_block(saliency, k: int) -> np.ndarray:
    """Boolean mask of the k smallest entries of the block, ties to the lower row-major position."""
    s = _f64(saliency)
    order = np.argsort(s.reshape(-1), kind="stable")
    pruned = np.zeros(s.size, dtype=bool)
    pruned[order[:k]] = True
    return pruned.reshape(s.shape)


def block_quota(sparsity: float, rows: int, width: int) -> int:
    return int(np.floor(sparsity * rows * width))


def obs_sweep(w, u, sparsity: float, block: int = BLOCK, forced_mask=None, saliency_fn=None):
    """Left-to-right pruning with error compensation.  Returns (W', pruned mask).

    forced_mask (bool, shape of W) replaces the per-block selection; saliency_fn(w_block, u_diag)
    replaces block_saliency (tests use it to take the selection in another precision)."""
    w = _f64(w).copy()
    u = _f64(u)
    rows, cols = w.shape
    pruned = np.zeros((rows, cols), dtype=bool)
    for c0 in range(0, cols, block):
        c1 = min(c0 + block, cols)
        d = np.diag(u)[c0:c1]
        if forced_mask is not None:
            m = np.asarray(forced_mask[:, c0:c1], dtype=bool)
        else:
            sal = (saliency_fn or block_saliency)(w[:, c0:c1], d)
            m = select_block(sal, block_quota(sparsity, rows, c1 - c0))
        pruned[:, c0:c1] = m
        err = np.zeros((rows, c1 - c0))
        for j in range(c0, c1):
            col = w[:, j].copy()
            kept = np.where(m[:, j - c0], 0.0, col)
            e = (col - kept) / u[j, j]
            w[:, j] = kept
            w[:, j + 1:c1] -= np.outer(e, u[j, j + 1:c1])
            err[:, j - c0] = e
        w[:, c1:] -= err @ u[c0:c1, c1:]
    return w, pruned


def obs_prune(x, w, sparsity: float, block: int = BLOCK, damp: float = DAMP):
    """The whole pruner for one projection: Hessian, damping, inverse factor, sweep."""
    h, dead = damped_hessian(gram_matrix(x), damp)
    w = _f64(w).copy()
    w[:, dead] = 0.0
    return obs_sweep(w, inverse_factor(h), sparsity, block)


def reconstruction_error(w, w_hat, h) -> float:
    """||(W - W') X^T||_F^2 = trace((W - W') H (W - W')^T)."""
    d = _f64(w) - _f64(w_hat)
    return float(np.einsum("ij,jk,ik->", d, _f64(h), d))
