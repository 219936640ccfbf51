"""Pins for the CPU oracle: hand-worked examples, closed forms, brute force, library special cases.

None of these re-type the oracle's formula: each expected value comes from a
hand derivation (tests/golden), a closed form, an independent pure-Python
brute force written with loops and sorted(), or a library routine reached
through a special case (np.linalg.norm, np.partition).
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import mosaic_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")


@pytest.fixture(scope="module")
def golden():
    with open(GOLDEN) as f:
        return json.load(f)


# ----------------------------------------------------------------- hand examples

def test_hand_metric_and_outliers(golden):
    ex = golden["metric_and_outliers"]
    x, w = np.array(ex["X"], float), np.array(ex["W"], float)
    np.testing.assert_allclose(orc.column_sumsq(x), ex["sumsq"], rtol=0, atol=0)
    np.testing.assert_allclose(orc.column_norms(x), ex["norms"], rtol=1e-15)
    omega = orc.weight_metric(w, orc.column_norms(x))
    np.testing.assert_allclose(omega, ex["omega"], rtol=1e-15)
    for case in ex["cases"]:
        c, o, r, mean = orc.outlier_stats(omega, case["alpha"])
        assert c == ex["C"]
        assert o == case["O"]
        assert r == pytest.approx(case["R"], rel=1e-14)
        assert mean == pytest.approx(ex["mean"], rel=1e-14)


def test_hand_strictness(golden):
    ex = golden["strictness"]
    omega = orc.weight_metric(np.array(ex["W"], float), orc.column_norms(np.array(ex["X"], float)))
    assert orc.outlier_stats(omega, ex["alpha"])[1] == ex["O"]
    # just below the mean every element is an outlier: the comparison really is at the mean
    assert orc.outlier_stats(omega, ex["alpha"] * (1 - 1e-12))[1] == omega.size


def test_hand_layer_outliers(golden):
    ex = golden["layer_outliers"]
    omegas = [np.array(o, float) for o in ex["omegas"]]
    for case in ex["cases"]:
        c, o, r, mean, per_proj = orc.layer_outlier_stats(omegas, case["alpha"])
        assert (c, o, per_proj) == (ex["C"], case["O"], case["per_projection"])
        assert mean == pytest.approx(ex["mean"], rel=1e-14) and r == pytest.approx(100.0 * case["O"] / ex["C"])


def test_layer_outliers_bruteforce_and_special_case():
    rng = np.random.default_rng(31)
    omegas = [np.abs(rng.standard_cauchy((5, 7))), np.abs(rng.standard_cauchy((3, 4))) * 10, np.abs(rng.standard_normal((6, 2)))]
    vals = [float(v) for o in omegas for v in o.reshape(-1)]
    mean = math.fsum(vals) / len(vals)
    for alpha in (0.5, 1.0, 5.0):
        c, o, r, m, per_proj = orc.layer_outlier_stats(omegas, alpha)
        assert c == len(vals) and m == pytest.approx(mean, rel=1e-13)
        assert o == sum(1 for v in vals if v > alpha * mean) == sum(per_proj)
        assert per_proj == [sum(1 for v in om.reshape(-1) if v > alpha * mean) for om in omegas]
        # a layer made of one projection is the projection rule
        assert orc.layer_outlier_stats(omegas[:1], alpha)[:4] == orc.outlier_stats(omegas[0], alpha)
    # the two rules differ when projections have different scales: the small-scale one has no layer outliers
    assert orc.layer_outlier_stats(omegas, 5.0)[4][2] == 0 < orc.outlier_stats(omegas[2], 2.0)[1]


def test_hand_row_selection(golden):
    ex = golden["row_selection"]
    omega, w = np.array(ex["omega"], float), np.array(ex["W"], float)
    for case in ex["cases"]:
        pruned = orc.select_smallest_per_row(omega, case["k"])
        for i, cols in enumerate(case["pruned_cols"]):
            assert sorted(np.nonzero(pruned[i])[0].tolist()) == cols
        np.testing.assert_array_equal(orc.apply_mask(w, pruned), np.array(case["W_out"], float))


def test_hand_structured(golden):
    ex = golden["structured"]
    gate, up, down = (np.array(ex[n], float) for n in ("gate", "up", "down"))
    g = orc.group_magnitude(gate, up, down)
    np.testing.assert_array_equal(g, ex["g"])
    for case in ex["cases"]:
        assert orc.struct_rank(g, case["r"]).tolist() == case["kept"]


def test_hand_planner(golden):
    ex = golden["planner"]
    s, clamped = orc.plan_sparsity(ex["R"], ex["p"], ex["lam"])
    np.testing.assert_allclose(s, ex["s"], rtol=1e-14)
    assert not clamped


def test_model_shapes_match_table2(golden):
    """The synthetic layer shapes reproduce the paper's parameter counts and target counts."""
    from paper_2504_06323_amd import synth
    for row in golden["model_shapes"]["rows"]:
        cfg = synth.CONFIGS[row["config"]]
        per_layer = synth.layer_numel(cfg)
        emb = row["vocab"] * cfg.hidden * (1 if row["tied_embeddings"] else 2)
        total = row["layers"] * per_layer + emb
        assert round(total / 1e9, 2) == pytest.approx(row["params_billion"], abs=0.011)
        assert row["layers"] * len(synth.projection_shapes(cfg)) == row["targets"]


# ----------------------------------------------------------------- norms

def test_norm_closed_forms():
    t, c = 37, 5
    x = np.full((t, c), -1.5)
    np.testing.assert_allclose(orc.column_norms(x), 1.5 * math.sqrt(t), rtol=1e-15)
    # one-hot rows: sumsq counts how often each channel fires
    rng = np.random.default_rng(1)
    hot = rng.integers(0, c, size=200)
    x = np.zeros((200, c))
    x[np.arange(200), hot] = 1.0
    np.testing.assert_array_equal(orc.column_sumsq(x), np.bincount(hot, minlength=c))


def test_norm_matches_library_and_axis():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((64, 7)) * np.arange(1, 8)      # distinct per-channel scales
    np.testing.assert_allclose(orc.column_norms(x), np.linalg.norm(x, axis=0), rtol=1e-14)
    assert orc.column_norms(x).shape == (7,)                 # per input channel, not per token
    # chunked accumulation over tokens adds up
    np.testing.assert_allclose(orc.column_sumsq(x[:20]) + orc.column_sumsq(x[20:]), orc.column_sumsq(x), rtol=1e-14)


def test_norm_widens_before_squaring():
    x = np.full((4, 1), 3e20, dtype=np.float32)   # squares overflow float32, not float64
    assert np.isfinite(orc.column_norms(x)).all()
    np.testing.assert_allclose(orc.column_norms(x), 2 * 3e20, rtol=1e-6)


# ----------------------------------------------------------------- Eq. 5

def test_metric_is_magnitude_when_norms_are_one():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((5, 9))
    np.testing.assert_array_equal(orc.weight_metric(w, np.ones(9)), np.abs(w))


def test_metric_elementwise_bruteforce():
    rng = np.random.default_rng(4)
    w = rng.standard_normal((3, 4))
    n = np.array([1.0, 2.0, 0.0, 10.0])
    omega = orc.weight_metric(w, n)
    for i in range(3):
        for j in range(4):
            assert omega[i, j] == abs(w[i, j]) * n[j]
    assert (omega >= 0).all()
    with pytest.raises(AssertionError):
        orc.weight_metric(w, np.ones(3))     # norms follow the input dimension (columns)


# ----------------------------------------------------------------- Eq. 6

def _brute_outliers(omega, alpha):
    vals = [float(v) for row in omega for v in row]
    mean = math.fsum(vals) / len(vals)
    return sum(1 for v in vals if v > alpha * mean), mean


@pytest.mark.parametrize("seed", range(5))
def test_outliers_bruteforce(seed):
    rng = np.random.default_rng(seed)
    omega = np.abs(rng.standard_cauchy((13, 17)))
    for alpha in (0.0, 0.5, 1.0, 3.0, 5.0):
        c, o, r, mean = orc.outlier_stats(omega, alpha)
        bo, bmean = _brute_outliers(omega, alpha)
        assert (c, o) == (13 * 17, bo)
        assert mean == pytest.approx(bmean, rel=1e-13)
        assert r == pytest.approx(100.0 * bo / (13 * 17), rel=1e-14)
        assert 0.0 <= r <= 100.0


def test_outliers_special_cases():
    rng = np.random.default_rng(7)
    w = rng.standard_normal((8, 6))
    w[2, 3] = 0.0
    omega = orc.weight_metric(w, np.ones(6))
    assert orc.outlier_stats(omega, 0.0)[1] == np.count_nonzero(omega > 0) == 47
    big = omega.max() / omega.mean()
    assert orc.outlier_stats(omega, big)[1] == 0            # alpha >= max/mean: nothing is above
    # planted: unit-magnitude weights, one input channel with a huge norm
    # => omega is 1e6 in that column and 1 elsewhere, 5 * mean ~ 7.3e5, so exactly
    # the column's nonzero entries (7 of its 8 rows) are outliers
    ws = np.sign(w)
    norms = np.ones(6)
    norms[3] = 1e6
    assert orc.outlier_stats(orc.weight_metric(ws, norms), 5.0)[1] == 7


def test_outliers_scale_invariance():
    """A power-of-two rescale of the activations changes neither the count nor the masks."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((50, 12)).astype(np.float32)
    w = rng.standard_normal((9, 12)).astype(np.float32)
    a = orc.weight_metric(w, orc.column_norms(x))
    b = orc.weight_metric(w, orc.column_norms(2.0 * x))
    assert orc.outlier_stats(a, 2.0)[1] == orc.outlier_stats(b, 2.0)[1]
    np.testing.assert_array_equal(orc.select_smallest_per_row(a, 5), orc.select_smallest_per_row(b, 5))


def test_count_above_uses_score_dtype():
    s = np.array([1.0, np.nextafter(np.float32(1.0), np.float32(2.0)), 2.0], dtype=np.float32)
    assert orc.count_above(s, np.float32(1.0)) == 2
    assert orc.count_above(s, 1.0 + 1e-12) == 2      # threshold is rounded to float32 first
    assert orc.threshold_f32(5.0, 12.0, 6) == np.float32(10.0)


# ----------------------------------------------------------------- planner (invariants only)

@pytest.mark.parametrize("scope", ["global", "category"])
@pytest.mark.parametrize("p", [0.3, 0.5, 0.7, 0.8])
def test_planner_invariants(scope, p):
    rng = np.random.default_rng(11)
    r = rng.uniform(0, 8, size=(32, 7))
    lam = 0.08
    s, clamped = orc.plan_sparsity(r, p, lam, scope)
    assert not clamped
    assert s.mean() == pytest.approx(p, abs=1e-12)                      # Eq. 1 / Eq. 2
    blocks = [(r, s)] if scope == "global" else [(r[:, m], s[:, m]) for m in range(7)]
    for rb, sb in blocks:
        assert sb.mean() == pytest.approx(p, abs=1e-12)
        order = np.argsort(rb, axis=None)
        assert (np.diff(sb.reshape(-1)[order]) <= 1e-15).all()          # more outliers => pruned less
        assert sb.max() - sb.min() == pytest.approx(2 * lam, rel=1e-12)


def test_planner_equal_ranks_is_global_pruning():
    s, _ = orc.plan_sparsity(np.full((4, 7), 3.25), 0.6, 0.08)
    np.testing.assert_array_equal(s, np.full((4, 7), 0.6))


def test_planner_clamp_reports():
    r = np.array([[0.0, 1.0]])
    s, clamped = orc.plan_sparsity(r, 0.95, 0.2, cols=np.array([[8, 8]]))
    assert clamped and s.max() <= 1 - 1 / 8 and s.min() >= 0
    assert orc.zeros_per_row(0.5, 688) == 344 and orc.zeros_per_row(0.4999, 256) == 127


def test_hand_layer_planner(golden):
    ex = golden["layer_planner"]
    np.testing.assert_allclose(orc.layer_ratios(ex["counts"], ex["numels"]), ex["R_layer"], rtol=1e-14)
    s, clamped = orc.plan_sparsity_layerwise(ex["counts"], ex["numels"], ex["p"], ex["lam"])
    np.testing.assert_allclose(s, np.repeat(np.array(ex["s_layer"])[:, None], 2, axis=1), rtol=1e-14)
    assert not clamped


@pytest.mark.parametrize("p", [0.3, 0.7])
def test_layer_planner_invariants(p):
    rng = np.random.default_rng(12)
    numels = rng.integers(1000, 100000, size=(32, 7))
    counts = (numels * rng.uniform(0, 0.05, size=numels.shape)).astype(np.int64)
    lam = 0.08
    s, clamped = orc.plan_sparsity_layerwise(counts, numels, p, lam)
    assert not clamped and s.shape == (32, 7)
    assert (s == s[:, :1]).all()                                        # one target per layer
    assert s[:, 0].mean() == pytest.approx(p, abs=1e-12)                # Eq. 1
    assert s[:, 0].max() - s[:, 0].min() == pytest.approx(2 * lam, rel=1e-12)
    # the layer ratio pools the layer's parameters: brute force over explicit outlier flags
    pooled = [100.0 * sum(int(c) for c in counts[n]) / sum(int(e) for e in numels[n]) for n in range(32)]
    np.testing.assert_allclose(orc.layer_ratios(counts, numels), pooled, rtol=1e-14)
    order = np.argsort(pooled)
    assert (np.diff(s[order, 0]) <= 1e-15).all()                        # more outliers => pruned less
    # one projection per layer: layer pruning and projection pruning are the same plan
    one, _ = orc.plan_sparsity_layerwise(counts[:, :1], numels[:, :1], p, lam)
    want, _ = orc.plan_sparsity(100.0 * counts[:, :1] / numels[:, :1], p, lam)
    np.testing.assert_allclose(one, want, rtol=0, atol=1e-15)
    # equal layer ratios: global (uniform) pruning
    flat, _ = orc.plan_sparsity_layerwise(np.full((4, 7), 5), np.full((4, 7), 100), p, lam)
    np.testing.assert_array_equal(flat, np.full((4, 7), p))
    # clamp by each projection's own width
    cl, flag = orc.plan_sparsity_layerwise([[0, 0], [9, 9]], [[10, 10], [10, 10]], 0.9, 0.2, cols=[[4, 100], [4, 100]])
    assert flag and cl[0, 0] == 0.75 and cl[0, 1] == pytest.approx(0.99) and cl[1, 0] == pytest.approx(0.7)


# ----------------------------------------------------------------- row selection

def _brute_select(row, k):
    order = sorted(range(len(row)), key=lambda j: (row[j], j))
    return set(order[:k])


@pytest.mark.parametrize("seed", range(6))
def test_selection_bruteforce_with_ties(seed):
    rng = np.random.default_rng(100 + seed)
    rows, cols = 7, 29
    omega = rng.integers(0, 6, size=(rows, cols)).astype(np.float64)   # few distinct values => many ties
    omega[0, :] = 0.0                                                 # a fully tied row
    for k in (0, 1, 5, 14, 28, 29):
        pruned = orc.select_smallest_per_row(omega, k)
        assert (pruned.sum(axis=1) == k).all()
        for i in range(rows):
            assert set(np.nonzero(pruned[i])[0].tolist()) == _brute_select(omega[i].tolist(), k)


def test_selection_properties_and_library_special_case():
    rng = np.random.default_rng(9)
    w = rng.standard_normal((16, 64))
    omega = orc.weight_metric(w, np.ones(64))            # = |W|: per-row magnitude pruning
    k = 32
    pruned = orc.select_smallest_per_row(omega, k)
    kth = np.partition(np.abs(w), k - 1, axis=1)[:, k - 1]
    assert (np.abs(w)[pruned].reshape(16, k).max(axis=1) == kth).all()
    assert (np.where(pruned, np.inf, omega).min(axis=1) >= np.where(pruned, omega, -np.inf).max(axis=1)).all()
    out = orc.apply_mask(w, pruned)
    np.testing.assert_array_equal(out[~pruned], w[~pruned])           # survivors bit-identical
    assert (out[pruned] == 0).all()
    assert pruned.mean() == k / 64                                    # sparsity equals the requested ratio


def test_keep_bits_layout():
    pruned = np.zeros((2, 40), dtype=bool)
    pruned[0, [0, 31, 33]] = True
    bits = orc.pack_keep_bits(pruned)
    assert bits.shape == (2, 2) and bits.dtype == np.uint32
    assert bits[0, 0] == 0xFFFFFFFF & ~(1 | (1 << 31))
    assert bits[0, 1] == 0xFF & ~(1 << 1)          # only 8 live columns in the tail word
    assert bits[1, 0] == 0xFFFFFFFF and bits[1, 1] == 0xFF


# ----------------------------------------------------------------- structured

def _silu(z):
    return z / (1.0 + np.exp(-z))


def _mlp(gate, up, down, x):
    return down @ (_silu(gate @ x) * (up @ x))


@pytest.mark.parametrize("seed", range(3))
def test_struct_bruteforce_and_dense_equivalence(seed):
    rng = np.random.default_rng(200 + seed)
    inter, hidden, r = 23, 11, 6
    gate, up = rng.standard_normal((inter, hidden)), rng.standard_normal((inter, hidden))
    down = rng.standard_normal((hidden, inter))
    g = orc.group_magnitude(gate, up, down)
    for c in range(inter):
        brute = sum(v * v for v in gate[c]) + sum(v * v for v in up[c]) + sum(down[i, c] ** 2 for i in range(hidden))
        assert g[c] == pytest.approx(brute, rel=1e-13)
    kept = orc.struct_rank(g, r)
    removed = sorted(sorted(range(inter), key=lambda c: (g[c], c))[:r])
    assert kept.tolist() == [c for c in range(inter) if c not in removed]
    assert (np.diff(kept) > 0).all() and kept.dtype == np.int32
    g2, u2, d2 = orc.struct_compact(gate, up, down, kept)
    assert g2.shape == (inter - r, hidden) and d2.shape == (hidden, inter - r)
    # removing the channels equals zeroing them in the full-size matrices (silu(0) * 0 == 0)
    gz, uz, dz = gate.copy(), up.copy(), down.copy()
    gz[removed], uz[removed], dz[:, removed] = 0, 0, 0
    x = rng.standard_normal(hidden)
    np.testing.assert_allclose(_mlp(g2, u2, d2, x), _mlp(gz, uz, dz, x), rtol=1e-12, atol=1e-12)


def test_struct_rank_ties_lower_index_first():
    g = np.array([1.0, 0.0, 0.0, 2.0, 0.0])
    assert orc.struct_rank(g, 2).tolist() == [0, 3, 4]
    assert orc.struct_rank(g, 0).tolist() == [0, 1, 2, 3, 4]


def test_composite_order_on_masked_weights():
    """Composite = unstructured first, then structured on what is left (Section 3.3 (c))."""
    rng = np.random.default_rng(5)
    inter, hidden = 12, 8
    gate, up = rng.standard_normal((inter, hidden)), rng.standard_normal((inter, hidden))
    down = rng.standard_normal((hidden, inter))
    down[:, 4] *= 1e-3                         # unstructured selection will empty most of this column
    ones_h, ones_i = np.ones(hidden), np.ones(inter)
    gm, _ = orc.prune_projection(gate, orc.weight_metric(gate, ones_h), 4)
    um, _ = orc.prune_projection(up, orc.weight_metric(up, ones_h), 4)
    dm, _ = orc.prune_projection(down, orc.weight_metric(down, ones_i), 6)
    g_after = orc.group_magnitude(gm, um, dm)
    g_before = orc.group_magnitude(gate, up, down)
    assert (g_after <= g_before + 1e-15).all() and (g_after < g_before).any()
    assert (dm[:, 4] == 0).all()


# ----------------------------------------------------------------- coupled groups (attention heads)

def _gqa_attention(q, k, v, o, x, n_groups, heads_per_group, d):
    """Grouped-query attention on a token sequence x [T, hidden] (float64, no masking)."""
    t = x.shape[0]
    out = np.zeros((t, o.shape[0]))
    for g in range(n_groups):
        kg, vg = x @ k[g * d:(g + 1) * d].T, x @ v[g * d:(g + 1) * d].T
        for j in range(heads_per_group):
            h = g * heads_per_group + j
            qh = x @ q[h * d:(h + 1) * d].T
            a = qh @ kg.T / math.sqrt(d)
            a = np.exp(a - a.max(axis=1, keepdims=True))
            a /= a.sum(axis=1, keepdims=True)
            out += (a @ vg) @ o[:, h * d:(h + 1) * d].T
    return out


@pytest.mark.parametrize("seed", range(3))
def test_coupled_groups_bruteforce_and_dense_equivalence(seed):
    rng = np.random.default_rng(300 + seed)
    n_groups, m, d, hidden = 4, 2, 3, 10                     # 4 key/value heads, 8 query heads of width 3
    q = rng.standard_normal((n_groups * m * d, hidden))
    k, v = rng.standard_normal((n_groups * d, hidden)), rng.standard_normal((n_groups * d, hidden))
    o = rng.standard_normal((hidden, n_groups * m * d))
    row_per, col_per = [m * d, d, d], [m * d]
    g = orc.coupled_group_magnitude([q, k, v], row_per, [o], col_per, n_groups)
    for grp in range(n_groups):
        brute = 0.0
        for mat, per in zip([q, k, v], row_per):
            for i in range(grp * per, (grp + 1) * per):
                brute += sum(float(val) ** 2 for val in mat[i])
        for j in range(grp * m * d, (grp + 1) * m * d):
            brute += sum(float(o[i, j]) ** 2 for i in range(hidden))
        assert g[grp] == pytest.approx(brute, rel=1e-13)
    r = 1
    kept = orc.struct_rank(g, r)
    removed = [grp for grp in range(n_groups) if grp not in kept.tolist()]
    assert removed == [int(np.argmin(g))]
    (q2, k2, v2), (o2,) = orc.coupled_group_compact([q, k, v], row_per, [o], col_per, kept)
    assert q2.shape == ((n_groups - r) * m * d, hidden) and o2.shape == (hidden, (n_groups - r) * m * d)
    # removing a key/value head with its query heads equals zeroing their o columns in the full block
    oz = o.copy()
    for grp in removed:
        oz[:, grp * m * d:(grp + 1) * m * d] = 0
    x = rng.standard_normal((5, hidden))
    np.testing.assert_allclose(_gqa_attention(q2, k2, v2, o2, x, n_groups - r, m, d),
                               _gqa_attention(q, k, v, oz, x, n_groups, m, d), rtol=1e-12, atol=1e-12)


def test_coupled_groups_reduce_to_mlp_channels():
    rng = np.random.default_rng(17)
    inter, hidden = 13, 6
    gate, up, down = rng.standard_normal((inter, hidden)), rng.standard_normal((inter, hidden)), rng.standard_normal((hidden, inter))
    np.testing.assert_allclose(orc.coupled_group_magnitude([gate, up], [1, 1], [down], [1], inter),
                               orc.group_magnitude(gate, up, down), rtol=1e-14)
    kept = np.array([0, 3, 4, 12])
    (g2, u2), (d2,) = orc.coupled_group_compact([gate, up], [1, 1], [down], [1], kept)
    wg, wu, wd = orc.struct_compact(gate, up, down, kept)
    assert np.array_equal(g2, wg) and np.array_equal(u2, wu) and np.array_equal(d2, wd)
