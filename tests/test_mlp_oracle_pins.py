"""Pins for the feed-forward oracle."""
import numpy as np
import pytest

from oracle import mlp_oracle as mlp
from oracle import mosaic_oracle as orc


def test_silu_closed_forms():
    assert mlp.silu(0.0) == 0.0
    assert mlp.silu(1.0) == pytest.approx(1.0 / (1.0 + np.exp(-1.0)), rel=1e-15)          # 0.7310585786...
    assert mlp.silu(1.0) == pytest.approx(0.7310585786300049, rel=1e-14)
    assert mlp.silu(-1.0) == pytest.approx(-0.2689414213699951, rel=1e-14)
    a = np.linspace(-8, 8, 33)
    assert np.allclose(mlp.silu(a) - mlp.silu(-a), a, rtol=1e-13, atol=1e-15)            # sigmoid(a) + sigmoid(-a) = 1
    assert mlp.silu(40.0) == pytest.approx(40.0, rel=1e-15) and abs(mlp.silu(-40.0)) < 1e-15
    assert np.all(mlp.silu(a) >= -0.2785)                                                # the minimum of silu is -0.27846...


def test_linear_brute_force():
    rng = np.random.default_rng(0)
    x, w = rng.standard_normal((3, 5)), rng.standard_normal((4, 5))
    y = mlp.linear(x, w)
    for t in range(3):
        for n in range(4):
            assert y[t, n] == pytest.approx(sum(x[t, k] * w[n, k] for k in range(5)), rel=1e-13)


def test_mlp_hand_example():
    # one token x = [1, 2]; gate rows [1, 0], [0, -1]; up rows [2, 1], [1, 1]; down row [3, 5]
    x = np.array([[1.0, 2.0]])
    gate = np.array([[1.0, 0.0], [0.0, -1.0]])
    up = np.array([[2.0, 1.0], [1.0, 1.0]])
    down = np.array([[3.0, 5.0]])
    h = mlp.mlp_hidden(x, gate, up)
    want_h = [(1.0 / (1.0 + np.exp(-1.0))) * 4.0, (-2.0 / (1.0 + np.exp(2.0))) * 3.0]      # silu(1) * 4, silu(-2) * 3
    assert np.allclose(h, [want_h], rtol=1e-14)
    assert mlp.mlp_forward(x, gate, up, down)[0, 0] == pytest.approx(3.0 * want_h[0] + 5.0 * want_h[1], rel=1e-14)
    assert not mlp.mlp_hidden(x, np.zeros((2, 2)), up).any()                            # silu(0) = 0 closes the gate


def test_removed_channels_are_dense_equivalent():
    """Dropping channels (gate / up rows, down columns) gives the output of the full block with those channels'
    hidden activations set to zero: what structured removal of coupled channels means (Fig. 4)."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 8))
    gate, up, down = rng.standard_normal((10, 8)), rng.standard_normal((10, 8)), rng.standard_normal((8, 10))
    kept = np.array([0, 2, 3, 7, 9])
    g2, u2, d2 = orc.struct_compact(gate, up, down, kept)
    h = mlp.mlp_hidden(x, gate, up)
    h_zeroed = np.zeros_like(h)
    h_zeroed[:, kept] = h[:, kept]
    assert np.allclose(mlp.mlp_forward(x, g2, u2, d2), mlp.linear(h_zeroed, down), rtol=1e-12, atol=1e-12)
    assert np.allclose(mlp.mlp_hidden(x, g2, u2), h[:, kept], rtol=1e-13)
