"""CPU oracle for the feed-forward block whose projections are being pruned.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this file; the product path never does, and this
file imports nothing from the product package.

The models of Table 2 (Section 4.1.1) are LLaMA-style: every layer's feed-forward
block is  y = down( silu(gate(x)) * up(x) )  with three bias-free projections
(the gate / up / down projections whose outliers Section 3 measures and whose
coupled channels Fig. 4 removes).  The input of the down projection -- the
activation its weight metric (Eq. 5) and its Hessian are computed from -- is
therefore  h = silu(x gate^T) * (x up^T),  produced by a forward pass.
Plain float64 NumPy, no blocking.

Parity status:
  silu          pinned (closed-form values, the identity silu(a) - silu(-a) = a, limits)
  linear        pinned (brute-force loops)
  mlp_hidden    pinned (hand example, zero gate => zero)
  mlp_forward   pinned (hand example; removing channels from gate/up rows and down columns leaves the
                output unchanged iff the removed channels' hidden activations are dropped: dense equivalence)
"""
from __future__ import annotations

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def silu(a) -> np.ndarray:
    """a * sigmoid(a)."""
    a = _f64(a)
    return a / (1.0 + np.exp(-a))


def linear(x, w) -> np.ndarray:
    """y[t, n] = sum_k x[t, k] * w[n, k]   (a bias-free projection, weights [out, in])."""
    return _f64(x) @ _f64(w).T


def mlp_hidden(x, gate, up) -> np.ndarray:
    """h = silu(x gate^T) * (x up^T): the input of the down projection."""
    return silu(linear(x, gate)) * linear(x, up)


def mlp_forward(x, gate, up, down) -> np.ndarray:
    return linear(mlp_hidden(x, gate, up), down)
