"""The pins must notice plausible mistakes: each mutant below plants one in the oracle (on the CPU)
and at least one pin of test_oracle_pins.py has to fail for it."""
import json
import os

import numpy as np
import pytest

import test_oracle_pins as pins
from oracle import mosaic_oracle as orc

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")))

# pins that take no pytest fixture besides the golden file
_PLAIN = [getattr(pins, n) for n in dir(pins) if n.startswith("test_") and n not in
          ("test_model_shapes_match_table2",)]


def _run_all_pins():
    """Run every pin; return the names of those that fail."""
    failed = []
    for fn in _PLAIN:
        params = [()]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names, values = mark.args
                vals = [v if isinstance(v, tuple) else (v,) for v in values]
                params = [p + v for p in params for v in vals]
        argnames = fn.__code__.co_varnames[:fn.__code__.co_argcount]
        for p in params:
            kwargs = {}
            extra = list(p)
            # parametrize marks are stacked bottom-up; map by name instead of by position
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            flat_names = [m.args[0] for m in marks]
            kwargs = dict(zip(flat_names, extra))
            if "golden" in argnames:
                kwargs["golden"] = GOLDEN
            try:
                fn(**kwargs)
            except AssertionError:
                failed.append(fn.__name__)
                break
            except Exception:                      # a mutant may also crash a pin: that counts as noticed
                failed.append(fn.__name__)
                break
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert _run_all_pins() == []


def _f64(a):
    return np.asarray(a, dtype=np.float64)


MUTANTS = {
    # norms
    "norm_divided_by_tokens": ("column_sumsq", lambda x: (_f64(x) ** 2).mean(axis=0)),
    "norm_l1": ("column_sumsq", lambda x: np.abs(_f64(x)).sum(axis=0)),
    "norm_over_channels_not_tokens": ("column_sumsq", lambda x: np.resize((_f64(x) ** 2).sum(axis=1), _f64(x).shape[1])),
    "norm_squares_in_input_dtype": ("column_sumsq", lambda x: (np.asarray(x) * np.asarray(x)).sum(axis=0).astype(np.float64)),
    # Eq. 5
    "metric_without_abs": ("weight_metric", lambda w, n: _f64(w) * _f64(n)[None, :]),
    "metric_norm_per_row": ("weight_metric", lambda w, n: np.abs(_f64(w)) * np.resize(_f64(n), _f64(w).shape[0])[:, None]),
    "metric_squared_weight": ("weight_metric", lambda w, n: _f64(w) ** 2 * _f64(n)[None, :]),
    # Eq. 6
    "outlier_non_strict": ("outlier_stats", lambda om, a: (lambda f: (f.size, int((f >= a * f.mean()).sum()),
                                                                       100.0 * (f >= a * f.mean()).sum() / f.size, f.mean()))(_f64(om).reshape(-1))),
    "outlier_vs_median": ("outlier_stats", lambda om, a: (lambda f: (f.size, int((f > a * np.median(f)).sum()),
                                                                     100.0 * (f > a * np.median(f)).sum() / f.size, f.mean()))(_f64(om).reshape(-1))),
    "outlier_ratio_not_percent": ("outlier_stats", lambda om, a: (lambda f: (f.size, int((f > a * f.mean()).sum()),
                                                                            (f > a * f.mean()).sum() / f.size, f.mean()))(_f64(om).reshape(-1))),
    "outlier_alpha_added": ("outlier_stats", lambda om, a: (lambda f: (f.size, int((f > a + f.mean()).sum()),
                                                                       100.0 * (f > a + f.mean()).sum() / f.size, f.mean()))(_f64(om).reshape(-1))),
    # selection
    "select_largest": ("select_smallest_per_row", lambda om, k: _select(om, k, largest=True)),
    "select_unstable_ties_high_index_first": ("select_smallest_per_row", lambda om, k: _select(om, k, reverse_ties=True)),
    "select_per_column": ("select_smallest_per_row", lambda om, k: _select(np.asarray(om).T, min(k, np.asarray(om).shape[0])).T
                          if np.asarray(om).shape[0] != np.asarray(om).shape[1] else _select(np.asarray(om).T, k).T),
    "select_k_minus_one": ("select_smallest_per_row", lambda om, k: _select(om, max(k - 1, 0))),
    # planner
    "planner_more_outliers_pruned_more": ("plan_sparsity", lambda r, p, lam, scope="global", cols=None:
                                          (lambda s: (2 * p - s[0], s[1]))(_ORIG["plan_sparsity"](r, p, lam, scope, cols))),
    "layer_ratio_is_mean_of_projection_ratios": ("layer_ratios", lambda c, e: (100.0 * _f64(c) / _f64(e)).mean(axis=1)),
    "layer_ratio_not_in_percent_of_layer": ("layer_ratios", lambda c, e: 100.0 * _f64(c).sum(axis=1) / _f64(e)[:, 0]),
    "layer_plan_not_shared_within_layer": ("plan_sparsity_layerwise", lambda c, e, p, lam, cols=None:
                                           _ORIG["plan_sparsity"](100.0 * _f64(c) / _f64(e), p, lam, "global", cols)),
    "planner_no_recentering": ("plan_sparsity", lambda r, p, lam, scope="global", cols=None:
                               (p - 2 * lam * (_f64(r) - _f64(r).min()) / max(np.ptp(_f64(r)), 1e-300), False)),
    # structured
    "group_without_down": ("group_magnitude", lambda g, u, d: (_f64(g) ** 2).sum(1) + (_f64(u) ** 2).sum(1)),
    "group_down_rows_not_cols": ("group_magnitude", lambda g, u, d: (_f64(g) ** 2).sum(1) + (_f64(u) ** 2).sum(1) +
                                 np.resize((_f64(d) ** 2).sum(1), _f64(g).shape[0])),
    "rank_keeps_lowest": ("struct_rank", lambda g, r: np.sort(np.argsort(np.asarray(g), kind="stable")[:len(g) - r]).astype(np.int32)),
    "rank_ties_high_index_first": ("struct_rank", lambda g, r: np.sort(
        (len(g) - 1 - np.argsort(np.asarray(g)[::-1], kind="stable"))[r:]).astype(np.int32)),
    "compact_down_rows": ("struct_compact", lambda g, u, d, k: (np.asarray(g)[k], np.asarray(u)[k],
                                                                 np.asarray(d)[:, :len(k)])),
    "layer_rule_uses_projection_means": ("layer_outlier_stats", lambda oms, a: (lambda per: (
        sum(_f64(o).size for o in oms), sum(per), 100.0 * sum(per) / sum(_f64(o).size for o in oms),
        np.concatenate([_f64(o).reshape(-1) for o in oms]).mean(), per))(
        [int((_f64(o) > a * _f64(o).mean()).sum()) for o in oms])),
    "coupled_groups_ignore_column_matrices": ("coupled_group_magnitude", lambda rm, rp, cm, cp, n:
                                              _ORIG["coupled_group_magnitude"](rm, rp, [], [], n)),
}

_ORIG = {name: getattr(orc, name) for name in dir(orc) if callable(getattr(orc, name)) and not name.startswith("_")}


def _select(om, k, largest=False, reverse_ties=False):
    om = np.asarray(om, dtype=np.float64)
    rows, cols = om.shape
    pruned = np.zeros((rows, cols), dtype=bool)
    for i in range(rows):
        key = (lambda j: (-om[i, j], j)) if largest else ((lambda j: (om[i, j], -j)) if reverse_ties else
                                                          (lambda j: (om[i, j], j)))
        for j in sorted(range(cols), key=key)[:k]:
            pruned[i, j] = True
    return pruned


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, monkeypatch):
    target, replacement = MUTANTS[name]
    monkeypatch.setattr(orc, target, replacement)
    failed = _run_all_pins()
    assert failed, f"no pin notices the planted mistake '{name}' in {target}"
