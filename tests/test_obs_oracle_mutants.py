"""The pins of the Hessian-based pruner's oracle must notice plausible mistakes: each mutant below plants one
in oracle/obs_oracle.py (on the CPU) and at least one pin of test_obs_oracle_pins.py has to fail for it."""
import numpy as np
import pytest

import test_obs_oracle_pins as pins
from oracle import obs_oracle as obs

_PINS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]
_ORIG = {n: getattr(obs, n) for n in dir(obs) if callable(getattr(obs, n)) and not n.startswith("_")}


def _failed_pins():
    failed = []
    for fn in _PINS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:
            cases = [{**c, m.args[0]: v} for c in cases for v in m.args[1]]
        for kw in cases:
            try:
                fn(**kw)
            except Exception:                  # an assertion, or a crash caused by the mutant: both count as noticed
                failed.append(fn.__name__)
                break
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert _failed_pins() == []


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _sweep(w, u, sparsity, block=obs.BLOCK, forced_mask=None, saliency_fn=None, *, sign=-1.0, divide=True, lazy=True,
           start=1, frozen_mask=False):
    """The oracle's sweep with one switchable mistake."""
    w, u = _f64(w).copy(), _f64(u)
    rows, cols = w.shape
    pruned = np.zeros((rows, cols), dtype=bool)
    first = None
    for c0 in range(0, cols, block):
        c1 = min(c0 + block, cols)
        d = np.diag(u)[c0:c1]
        if forced_mask is not None:
            m = np.asarray(forced_mask[:, c0:c1], dtype=bool)
        else:
            src = first if (frozen_mask and first is not None) else w
            sal = (saliency_fn or obs.block_saliency)(src[:, c0:c1], d)
            m = obs.select_block(sal, obs.block_quota(sparsity, rows, c1 - c0))
        if first is None:
            first = w.copy()
        pruned[:, c0:c1] = m
        err = np.zeros((rows, c1 - c0))
        for j in range(c0, c1):
            col = w[:, j].copy()
            kept = np.where(m[:, j - c0], 0.0, col)
            e = (col - kept) / (u[j, j] if divide else 1.0)
            w[:, j] = kept
            w[:, j + start:c1] += sign * np.outer(e, u[j, j + start:c1])
            if start == 0:
                w[:, j] = kept
            err[:, j - c0] = e
        if lazy:
            w[:, c1:] += sign * (err @ u[c0:c1, c1:])
    return w, pruned


def _ties_high_first(saliency, k):
    s = _f64(saliency)
    flat = s.reshape(-1)
    order = sorted(range(flat.size), key=lambda f: (flat[f], -f))
    pruned = np.zeros(flat.size, dtype=bool)
    pruned[order[:k]] = True
    return pruned.reshape(s.shape)


MUTANTS = {
    "gram_of_rows": ("gram_matrix", lambda x: _f64(x) @ _f64(x).T),
    "gram_mean_not_sum": ("gram_matrix", lambda x: _f64(x).T @ _f64(x) / max(len(_f64(x)), 1)),
    "damping_by_largest_diagonal": ("damped_hessian", lambda h, damp=obs.DAMP: (
        lambda hh, dead: (hh + damp * np.max(np.diag(hh)) * np.eye(len(hh)), dead))(
        *(lambda hh: (np.where(np.eye(len(hh), dtype=bool) & (np.diag(hh) == 0)[:, None], 1.0, hh), np.diag(hh) == 0))(
            _f64(h).copy()))),
    "dead_channel_left_singular": ("damped_hessian", lambda h, damp=obs.DAMP: (
        _f64(h) + damp * np.mean(np.diag(_f64(h))) * np.eye(len(_f64(h))), np.diag(_f64(h)) == 0)),
    "factor_lower_triangular": ("inverse_factor", lambda h: np.linalg.cholesky(np.linalg.inv(_f64(h)))),
    "factor_of_h_not_inverse": ("inverse_factor", lambda h: np.linalg.cholesky(_f64(h)).T),
    "reverse_factor_is_plain_cholesky": ("reverse_factor", lambda h: np.linalg.cholesky(_f64(h)).T),
    "saliency_ignores_the_factor": ("block_saliency", lambda wb, ud: _f64(wb) ** 2),
    "saliency_multiplies_by_the_factor": ("block_saliency", lambda wb, ud: (_f64(wb) * _f64(ud)[None, :]) ** 2),
    "select_largest": ("select_block", lambda s, k: _ORIG["select_block"](-_f64(s), k)),
    "select_ties_high_position_first": ("select_block", _ties_high_first),
    "quota_rounds_up": ("block_quota", lambda s, rows, width: int(np.ceil(s * rows * width))),
    "sweep_update_wrong_sign": ("obs_sweep", lambda *a, **k: _sweep(*a, **k, sign=+1.0)),
    "sweep_error_not_divided": ("obs_sweep", lambda *a, **k: _sweep(*a, **k, divide=False)),
    "sweep_forgets_later_blocks": ("obs_sweep", lambda *a, **k: _sweep(*a, **k, lazy=False)),
    "sweep_selects_on_original_weights": ("obs_sweep", lambda *a, **k: _sweep(*a, **k, frozen_mask=True)),
}


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, monkeypatch):
    target, replacement = MUTANTS[name]
    monkeypatch.setattr(obs, target, replacement)
    failed = _failed_pins()
    assert failed, f"no pin notices the planted mistake '{name}' in {target}"
