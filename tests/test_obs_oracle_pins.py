"""Pins for the Hessian-based pruner's oracle: each checks it against something other than itself
(brute force, a hand-worked case, a closed form, or an independent formulation of the same optimum)."""
import numpy as np
import pytest

from oracle import mosaic_oracle as orc
from oracle import obs_oracle as obs


def _spd(n, seed, tokens=None):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((tokens or 4 * n, n))
    x[:, ::5] *= 3.0
    return x, x.T @ x


# ------------------------------------------------------------------ Hessian

def test_gram_brute_force_and_diagonal():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 5))
    h = obs.gram_matrix(x)
    for i in range(5):
        for j in range(5):
            assert h[i, j] == pytest.approx(sum(x[t, i] * x[t, j] for t in range(7)), rel=1e-13)
    assert np.allclose(np.diag(h), orc.column_sumsq(x), rtol=1e-13)      # the statistic of the metric path
    assert np.array_equal(h, h.T)
    v = np.array([[1.0, -2.0, 0.5]])
    assert np.allclose(obs.gram_matrix(np.repeat(v, 4, axis=0)), 4 * v.T @ v)   # rank one, closed form
    assert obs.gram_matrix(np.zeros((0, 3))).shape == (3, 3) and not obs.gram_matrix(np.zeros((0, 3))).any()


def test_damping_hand_example():
    h = np.array([[4.0, 0.0, 2.0], [0.0, 0.0, 0.0], [2.0, 0.0, 3.0]])
    got, dead = obs.damped_hessian(h, damp=0.03)
    # channel 1 never fired: unit diagonal; mean of the diagonal (4 + 1 + 3) / 3; 0.03 * 8 / 3 = 0.08 added
    assert dead.tolist() == [False, True, False]
    assert np.allclose(got, [[4.08, 0.0, 2.0], [0.0, 1.08, 0.0], [2.0, 0.0, 3.08]], rtol=1e-15)
    assert h[1, 1] == 0.0                                                       # input untouched


def test_inverse_factor_hand_example_and_identities():
    # H = [[4, 2], [2, 3]]: H^-1 = [[3, -2], [-2, 4]] / 8.  Lower Cholesky factor L of H^-1:
    # L11 = sqrt(3/8), L21 = (-2/8) / L11, L22 = sqrt(4/8 - L21^2) = sqrt(1/3); U = L^T
    u = obs.inverse_factor(np.array([[4.0, 2.0], [2.0, 3.0]]))
    l11 = np.sqrt(3.0 / 8.0)
    want = np.array([[l11, -0.25 / l11], [0.0, np.sqrt(1.0 / 3.0)]])
    assert np.allclose(u, want, rtol=1e-14, atol=1e-16)
    _, h = _spd(9, 1)
    u = obs.inverse_factor(h)
    assert np.allclose(u.T @ u @ h, np.eye(9), atol=1e-10)
    assert np.allclose(u, np.triu(u)) and (np.diag(u) > 0).all()
    # the same factor by another route: H = R R^T with R upper triangular (Cholesky of the reversed matrix), U = R^-1
    rev = np.linalg.cholesky(h[::-1, ::-1])[::-1, ::-1]
    assert np.allclose(rev, np.triu(rev)) and np.allclose(rev @ rev.T, h, rtol=1e-12)
    assert np.allclose(u, np.linalg.inv(rev), rtol=1e-9, atol=1e-12)
    r = obs.reverse_factor(h)
    assert np.allclose(r, rev, rtol=1e-9, atol=1e-12) and np.allclose(r @ r.T, h, rtol=1e-10)
    assert np.allclose(obs.inverse_factor(4.0 * np.eye(3)), 0.5 * np.eye(3))


# ------------------------------------------------------------------ selection

def test_select_block_brute_force_and_ties():
    rng = np.random.default_rng(2)
    s = rng.integers(0, 4, size=(5, 6)).astype(float)                          # many equal saliencies
    for k in (0, 1, 7, 29, 30):
        got = obs.select_block(s, k)
        order = sorted(range(30), key=lambda f: (s.reshape(-1)[f], f))         # value, then row-major position
        want = np.zeros(30, dtype=bool)
        want[order[:k]] = True
        assert np.array_equal(got.reshape(-1), want) and got.sum() == k
    assert obs.block_quota(0.5, 3, 5) == 7 and obs.block_quota(0.0, 3, 5) == 0 and obs.block_quota(0.999, 2, 2) == 3


# ------------------------------------------------------------------ sweep

def test_identity_hessian_is_magnitude_pruning_without_update():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((6, 10))
    u = obs.inverse_factor(2.5 * np.eye(10))
    got, pruned = obs.obs_sweep(w, u, 0.4, block=5)
    for c0 in (0, 5):                                                           # per block: the 12 smallest |w| go
        blk = np.abs(w[:, c0:c0 + 5])
        thresh = np.sort(blk.reshape(-1))[11]
        assert np.array_equal(pruned[:, c0:c0 + 5], blk <= thresh)
    assert np.array_equal(got, np.where(pruned, 0.0, w))                        # kept weights are untouched


def test_saliency_weighs_a_weight_by_its_channel_energy():
    # Diagonal Hessian diag(100, 1): the saliency w^2 / [H^-1]_jj is w^2 * H_jj, so w = [0.5, 1.0] costs 25 and 1:
    # the larger weight on the quiet channel goes, not the smaller weight on the loud one; nothing to compensate.
    u = obs.inverse_factor(np.diag([100.0, 1.0]))
    assert np.allclose(obs.block_saliency(np.array([[0.5, 1.0]]), np.diag(u)), [[25.0, 1.0]], rtol=1e-12)
    got, pruned = obs.obs_sweep(np.array([[0.5, 1.0]]), u, 0.5, block=2)
    assert pruned.tolist() == [[False, True]] and got.tolist() == [[0.5, 0.0]]


def test_single_pruned_weight_is_the_closed_form_obs_update():
    _, h = _spd(7, 4)
    rng = np.random.default_rng(4)
    w = rng.standard_normal((1, 7))
    u = obs.inverse_factor(h)
    hinv = np.linalg.inv(h)
    # first column pruned: delta = -(w_q / [H^-1]_qq) * H^-1[:, q]
    mask = np.zeros((1, 7), dtype=bool)
    mask[0, 0] = True
    got, _ = obs.obs_sweep(w, u, 0.0, block=4, forced_mask=mask)
    want = w[0] - w[0, 0] / hinv[0, 0] * hinv[:, 0]
    assert got[0, 0] == 0.0 and np.allclose(got[0], want, rtol=1e-10, atol=1e-12)
    # column q > 0 pruned with everything to its left frozen: the same formula on the trailing Hessian
    for q in (2, 5):
        mask[:] = False
        mask[0, q] = True
        got, _ = obs.obs_sweep(w, u, 0.0, block=4, forced_mask=mask)
        tinv = np.linalg.inv(h[q:, q:])
        want = w[0].copy()
        want[q:] -= w[0, q] / tinv[0, 0] * tinv[:, 0]
        assert np.allclose(got[0], want, rtol=1e-10, atol=1e-12) and got[0, q] == 0.0
        assert np.array_equal(got[0, :q], w[0, :q])


def _eliminate_with_trailing_inverses(w_row, h, mask_row):
    """Independent formulation: walk the columns; when one is pruned, compensate on the columns to its
    right with the explicit inverse of the Hessian restricted to the columns not yet visited."""
    w = w_row.copy()
    for q in range(len(w)):
        if mask_row[q]:
            tinv = np.linalg.inv(h[q:, q:])
            w[q:] -= w[q] / tinv[0, 0] * tinv[:, 0]
            w[q] = 0.0
    return w


@pytest.mark.parametrize("block", [3, 4, 16])
def test_sweep_equals_explicit_trailing_inverse_elimination(block):
    _, h = _spd(11, 5)
    rng = np.random.default_rng(5)
    w = rng.standard_normal((6, 11))
    u = obs.inverse_factor(h)
    got, pruned = obs.obs_sweep(w, u, 0.45, block=block)
    assert pruned.sum() == sum(obs.block_quota(0.45, 6, min(block, 11 - c)) for c in range(0, 11, block))
    assert (got[pruned] == 0).all()
    for i in range(6):
        want = _eliminate_with_trailing_inverses(w[i], h, pruned[i])
        assert np.allclose(got[i], want, rtol=1e-8, atol=1e-10), i


def test_later_blocks_select_on_compensated_weights():
    """Selection of a block re-derived without the factor: current weights from the explicit elimination above,
    saliency w^2 / [inverse of the trailing Hessian]_00.  With correlated channels the compensation of earlier
    blocks changes which entries of later blocks go."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((60, 12)) @ (np.eye(12) + 0.6 * rng.standard_normal((12, 12)))
    h = x.T @ x
    w = rng.standard_normal((5, 12))
    block, sparsity = 4, 0.5
    got, pruned = obs.obs_sweep(w, obs.inverse_factor(h), sparsity, block=block)
    mask = np.zeros_like(pruned)
    differs_from_static = False
    for c0 in range(0, 12, block):
        cur = np.stack([_eliminate_with_trailing_inverses(w[i], h, mask[i]) for i in range(5)])
        denom = np.array([np.linalg.inv(h[j:, j:])[0, 0] for j in range(c0, c0 + block)])
        sal = cur[:, c0:c0 + block] ** 2 / denom[None, :]
        mask[:, c0:c0 + block] = obs.select_block(sal, obs.block_quota(sparsity, 5, block))
        static = obs.select_block(w[:, c0:c0 + block] ** 2 / denom[None, :], obs.block_quota(sparsity, 5, block))
        differs_from_static |= not np.array_equal(static, mask[:, c0:c0 + block])
    assert np.array_equal(pruned, mask)
    assert differs_from_static                              # the example does exercise the difference


def test_pruned_prefix_gives_the_least_squares_optimum():
    x, h = _spd(8, 6, tokens=40)
    rng = np.random.default_rng(6)
    w = rng.standard_normal((3, 8))
    mask = np.zeros((3, 8), dtype=bool)
    mask[:, :3] = True                                                          # columns 0..2 pruned in every row
    got, _ = obs.obs_sweep(w, obs.inverse_factor(h), 0.0, block=2, forced_mask=mask)
    # argmin over w' (with w'[:3] = 0) of || (w - w') X^T ||: ordinary least squares on the kept channels
    target = w @ x.T
    sol, *_ = np.linalg.lstsq(x[:, 3:], target.T, rcond=None)
    assert np.allclose(got[:, 3:], sol.T, rtol=1e-8, atol=1e-10) and (got[:, :3] == 0).all()
    # and compensation never does worse than plain masking
    plain = np.where(mask, 0.0, w)
    assert obs.reconstruction_error(w, got, h) <= obs.reconstruction_error(w, plain, h)
    assert obs.reconstruction_error(w, got, h) == pytest.approx(np.sum((target - got @ x.T) ** 2), rel=1e-9)


def test_whole_pruner_dead_channel_and_sparsity():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((64, 12))
    x[:, 4] = 0.0                                                               # a channel that never fires
    w = rng.standard_normal((5, 12))
    got, pruned = obs.obs_prune(x, w, 0.5, block=4)
    assert (got[:, 4] == 0).all()                                               # its weights are dropped
    assert pruned.sum() == 3 * obs.block_quota(0.5, 5, 4)
    assert (got[pruned] == 0).all()
    h, _ = obs.damped_hessian(obs.gram_matrix(x))
    w0 = w.copy()
    w0[:, 4] = 0.0
    plain = np.where(pruned, 0.0, w0)
    assert obs.reconstruction_error(w0, got, h) < obs.reconstruction_error(w0, plain, h)
