"""HIP path vs CPU oracle, element by element, through the C-ABI.

Floating-point outputs (sums of squares, norms, metric, metric sum, threshold,
group magnitudes) are compared within rel 1e-5 (float32 inputs) / 1e-2 (bf16
inputs).  Integer outputs (outlier count, masks, kept indices, gathers) are
compared bit-exactly: where a float decides an integer, both sides take the
decision in the kernel's precision -- the oracle's selection / count runs on
the kernel's own float32 metric bits (materialised, or recomputed on the host
as the single IEEE multiply float32(|w|) * float32(norm)).
"""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2504_06323_amd import prune, synth
from util import bits, rel_err, to_np, tol_for

pytestmark = pytest.mark.gpu
DEV = "cuda"
DTYPES = [torch.float32, torch.bfloat16]


def _sync():
    torch.cuda.synchronize()


def gpu_norms(x, chunks=1):
    c = x.shape[1]
    sumsq = torch.zeros(c, dtype=torch.float32, device=DEV)
    norms = torch.empty(c, dtype=torch.float32, device=DEV)
    step = (x.shape[0] + chunks - 1) // chunks if x.shape[0] else 1
    for t0 in range(0, max(x.shape[0], 1), step):
        prune.stats_accumulate(x[t0:t0 + step], sumsq)
    prune.stats_finalize(sumsq, norms)
    _sync()
    return sumsq, norms


def host_metric_f32(w, norms):
    """The kernel-precision metric recomputed on the host: one float32 multiply per element."""
    return np.abs(to_np(w).astype(np.float32)) * to_np(norms).astype(np.float32)[None, :]


# ----------------------------------------------------------------- stats

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(512, 256), (512, 688), (513, 2056), (1000, 4104), (77, 8), (301, 7), (260, 130),
                                   (1, 16), (4099, 24)])
def test_stats_vs_oracle(lib, dtype, shape):
    t, c = shape
    x = synth.random_matrix(t, c, dtype, seed=t * 31 + c, device=DEV, scale=1.0)
    x[:, c // 3] *= 20.0
    sumsq, norms = gpu_norms(x)
    want = orc.column_sumsq(to_np(x))
    assert rel_err(to_np(sumsq), want) < tol_for(dtype)
    assert rel_err(to_np(norms), np.sqrt(want)) < tol_for(dtype)
    assert rel_err(to_np(sumsq), want) < 2e-6      # what the float accumulation actually delivers


@pytest.mark.parametrize("dtype", DTYPES)
def test_stats_pitch_chunks_and_determinism(lib, dtype):
    big = synth.random_matrix(700, 1024, dtype, seed=5, device=DEV)
    x = big[:, 64:64 + 688]                               # pitch 1024, 16-byte aligned start
    y = big[:, 3:3 + 101]                                 # unaligned start, odd width: scalar path
    for view in (x, y):
        s1, n1 = gpu_norms(view)
        s2, n2 = gpu_norms(view)
        assert np.array_equal(bits(s1), bits(s2)) and np.array_equal(bits(n1), bits(n2))
        want = orc.column_sumsq(to_np(view))
        assert rel_err(to_np(s1), want) < 2e-6
        s3, _ = gpu_norms(view, chunks=3)                  # chunked accumulation into the same buffer
        assert rel_err(to_np(s3), want) < 2e-6


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(512, 688), (1000, 4104), (301, 7), (0, 64)])
def test_stats_norms_one_call(lib, dtype, shape):
    """The one-call form overwrites both outputs and equals accumulate + finalize bit for bit."""
    t, c = shape
    x = synth.random_matrix(max(t, 1), c, dtype, seed=t + c, device=DEV)[:t]
    sumsq = torch.full((c,), 123.0, dtype=torch.float32, device=DEV)      # stale contents must not leak in
    norms = torch.full((c,), -1.0, dtype=torch.float32, device=DEV)
    prune.stats_norms(x, sumsq, norms)
    _sync()
    want = orc.column_sumsq(to_np(x)) if t else np.zeros(c)
    if t:
        assert rel_err(to_np(sumsq), want) < 2e-6 and rel_err(to_np(norms), np.sqrt(want)) < 2e-6
        s2, n2 = gpu_norms(x)
        assert np.array_equal(bits(sumsq), bits(s2)) and np.array_equal(bits(norms), bits(n2))
    else:
        assert (to_np(sumsq) == 0).all() and (to_np(norms) == 0).all()


def test_stats_zero_tokens_and_closed_form(lib):
    x = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    sumsq = torch.full((64,), 3.0, dtype=torch.float32, device=DEV)
    prune.stats_accumulate(x, sumsq)
    _sync()
    assert (to_np(sumsq) == 3.0).all()
    x = torch.full((1024, 40), -1.5, dtype=torch.bfloat16, device=DEV)
    _, norms = gpu_norms(x)
    assert (to_np(norms) == np.float32(1.5 * 32.0)).all()   # |c| * sqrt(T), exact here


# ----------------------------------------------------------------- score + outliers

def _rank_inputs(rows, cols, dtype, seed):
    w = synth.random_matrix(rows, cols, dtype, seed=seed, device=DEV, scale=0.02, zero_frac=0.01)
    x = synth.random_matrix(300, cols, dtype, seed=seed + 1, device=DEV)
    x[:, cols // 2] *= 30.0
    return w, x


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(256, 256), (688, 256), (256, 688), (37, 2056), (129, 4104), (50, 7), (33, 130),
                                   (1, 8), (2000, 16)])
def test_score_and_outliers_vs_oracle(lib, dtype, shape):
    rows, cols = shape
    w, x = _rank_inputs(rows, cols, dtype, seed=rows * 7 + cols)
    _, norms = gpu_norms(x)
    scores = torch.empty((rows, cols), dtype=torch.float32, device=DEV)
    ssum = torch.zeros(1, dtype=torch.float64, device=DEV)
    ssum_hot = torch.zeros(1, dtype=torch.float64, device=DEV)
    prune.score(w, norms, ssum, scores=scores)
    prune.score(w, norms, ssum_hot)                         # hot mode: sum only
    _sync()
    tol = tol_for(dtype)
    # end to end against the float64 oracle (its own norms)
    onorms = orc.column_norms(to_np(x))
    omega = orc.weight_metric(to_np(w), onorms)
    got = to_np(scores)
    nz = omega > 0
    assert rel_err(got[nz], omega[nz]) < tol and (got[~nz] == 0).all()
    assert abs(ssum.item() - omega.sum()) <= tol * omega.sum()
    assert ssum.item() == ssum_hot.item()                   # materialising does not change the sum
    # kernel precision: the metric is exactly one float32 multiply
    assert np.array_equal(got, host_metric_f32(w, norms))
    assert abs(ssum.item() - got.astype(np.float64).sum()) <= 1e-6 * got.astype(np.float64).sum()

    for alpha in (0.0, 1.0, 5.0):
        count = torch.full((1,), -7, dtype=torch.int64, device=DEV)
        count2 = torch.full((1,), -7, dtype=torch.int64, device=DEV)
        tau = torch.zeros(1, dtype=torch.float32, device=DEV)
        prune.outlier_ratio(w, norms, alpha, ssum, count, tau=tau)            # recompute mode
        prune.outlier_ratio(None, None, alpha, ssum, count2, scores=scores)   # from materialised scores
        _sync()
        tau_h = np.float32(tau.item())
        assert tau_h == orc.threshold_f32(alpha, ssum.item(), rows * cols)
        # bit-exact protocol: the oracle counts on the kernel's score bits with the kernel's threshold
        assert count.item() == count2.item() == orc.count_above(got, tau_h)
        # end to end: oracle threshold within tolerance, counts differ at most by the near-threshold band
        c_o, o_o, r_o, mean_o = orc.outlier_stats(omega, alpha)
        assert abs(float(tau_h) - alpha * mean_o) <= tol * alpha * mean_o + 1e-30
        band = np.count_nonzero(np.abs(omega - alpha * mean_o) <= 2 * tol * alpha * mean_o)
        assert abs(count.item() - o_o) <= band


def test_outlier_strictness_and_planted_column(lib):
    # constant weights and activations: every metric equals the mean, nothing is strictly above it
    w = torch.full((64, 128), 0.5, dtype=torch.float32, device=DEV)
    x = torch.full((16, 128), 2.0, dtype=torch.float32, device=DEV)
    _, norms = gpu_norms(x)
    ssum = torch.zeros(1, dtype=torch.float64, device=DEV)
    count = torch.zeros(1, dtype=torch.int64, device=DEV)
    prune.score(w, norms, ssum)
    prune.outlier_ratio(w, norms, 1.0, ssum, count)
    _sync()
    assert ssum.item() == 64 * 128 * 0.5 * 8.0 and count.item() == 0
    # unit-magnitude weights, one channel with a huge norm: exactly that column's rows are outliers
    w = torch.ones((64, 128), dtype=torch.bfloat16, device=DEV)
    w[::2] *= -1
    x[:, 5] = 2.0e4
    _, norms = gpu_norms(x)
    prune.score(w, norms, ssum)
    prune.outlier_ratio(w, norms, 5.0, ssum, count)
    _sync()
    assert count.item() == 64


# ----------------------------------------------------------------- select + mask

def _check_select(w, norms, k, scores=None, in_place=False):
    rows, cols = w.shape
    w_in = w.clone() if in_place else w
    w_ref = to_np(w)
    out = w_in if in_place else torch.full_like(w, 7.0)
    mask = torch.full((rows, (cols + 31) // 32), -1, dtype=torch.int32, device=DEV)
    prune.select_mask(w_in, norms, k, w_out=None if in_place else out, mask_bits=mask, scores=scores)
    _sync()
    metric = to_np(scores) if scores is not None else host_metric_f32(w, norms)
    pruned = orc.select_smallest_per_row(metric, k)          # oracle selection on the kernel's metric bits
    want = orc.apply_mask(w_ref, pruned)
    got = to_np(out)
    assert np.array_equal(got, want), f"masked weights differ in {np.count_nonzero(got != want)} places"
    assert np.array_equal(to_np(mask).view(np.uint32), orc.pack_keep_bits(pruned))
    assert (pruned.sum(axis=1) == k).all()
    assert np.array_equal(got[~pruned].view(np.uint32), w_ref[~pruned].view(np.uint32))   # survivors bit-identical
    return out


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(256, 256), (688, 256), (256, 688), (19, 2056), (11, 4104), (9, 11008),
                                   (7, 14336), (5, 16384), (6, 16392), (50, 7), (33, 130), (3, 8), (4, 1000),
                                   (10, 8200), (6, 10240), (5, 13824), (5, 12296)])
def test_select_vs_oracle(lib, dtype, shape):
    rows, cols = shape
    w, x = _rank_inputs(rows, cols, dtype, seed=rows * 13 + cols)
    _, norms = gpu_norms(x)
    for k in sorted({0, 1, cols // 2, cols - 1, cols}):
        _check_select(w, norms, k)
    _check_select(w, norms, cols // 3, in_place=True)
    scores = torch.empty((rows, cols), dtype=torch.float32, device=DEV)
    ssum = torch.zeros(1, dtype=torch.float64, device=DEV)
    prune.score(w, norms, ssum, scores=scores)
    _check_select(w, norms, cols // 2, scores=scores)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("cols", [64, 688, 4096, 1001, 8200, 14336])
def test_select_ties(lib, dtype, cols):
    """Many equal metrics: zeros, constant rows, few distinct values -- the index decides."""
    rows = 12
    g = torch.Generator(device="cpu").manual_seed(cols)
    vals = torch.randint(-3, 4, (rows, cols), generator=g).to(torch.float32) * 0.25
    vals[0] = 0.0
    vals[1] = 0.5
    w = vals.to(dtype).to(DEV)
    norms = torch.ones(cols, dtype=torch.float32, device=DEV)
    norms[cols // 2:] = 2.0
    for k in (1, cols // 4, cols // 2, cols - 3):
        _check_select(w, norms, k)
    # an all-zero norm vector makes every metric zero
    _check_select(w, torch.zeros(cols, dtype=torch.float32, device=DEV), cols // 2)


def test_select_pitch_and_determinism(lib):
    big = synth.random_matrix(40, 2048, torch.bfloat16, seed=77, device=DEV, scale=0.02)
    w = big[:, 256:256 + 1024]                              # pitch 2048
    norms = (torch.arange(1024, device=DEV, dtype=torch.float32) % 17) + 0.5
    o1 = _check_select(w, norms, 400)
    o2 = _check_select(w, norms, 400)
    assert np.array_equal(bits(o1), bits(o2))
    assert np.array_equal(bits(big[:, :256]), bits(synth.random_matrix(40, 2048, torch.bfloat16, seed=77, device=DEV,
                                                                       scale=0.02)[:, :256]))


def test_select_is_magnitude_pruning_when_norms_are_one(lib):
    w = synth.random_matrix(64, 512, torch.float32, seed=3, device=DEV)
    norms = torch.ones(512, dtype=torch.float32, device=DEV)
    out = _check_select(w, norms, 256)
    kth = np.partition(np.abs(to_np(w)), 255, axis=1)[:, 255]          # library top-k special case
    got = to_np(out)
    assert (np.abs(to_np(w))[got == 0].reshape(64, -1).max(axis=1) <= kth).all()
    assert (np.count_nonzero(got == 0, axis=1) == 256).all()


# ----------------------------------------------------------------- structured

def _check_struct(gate, up, down, r, compact=True):
    inter, hidden = gate.shape
    g = torch.empty(inter, dtype=torch.float32, device=DEV)
    kept = torch.full((inter - r,), -1, dtype=torch.int32, device=DEV)
    outs = [None, None, None]
    if compact:
        outs = [torch.empty((inter - r, hidden), dtype=gate.dtype, device=DEV),
                torch.empty((inter - r, hidden), dtype=gate.dtype, device=DEV),
                torch.empty((hidden, inter - r), dtype=gate.dtype, device=DEV)]
    prune.struct_compact(gate, up, down, r, g, kept, *outs)
    _sync()
    want_g = orc.group_magnitude(to_np(gate), to_np(up), to_np(down))
    nz = want_g > 0
    assert rel_err(to_np(g)[nz], want_g[nz]) < tol_for(gate.dtype)
    assert rel_err(to_np(g)[nz], want_g[nz]) < 5e-6
    assert (to_np(g)[~nz] == 0).all()
    want_kept = orc.struct_rank(to_np(g), r)                # oracle ranking on the kernel's magnitudes
    assert np.array_equal(to_np(kept), want_kept)
    if compact:
        wg, wu, wd = orc.struct_compact(to_np(gate), to_np(up), to_np(down), want_kept)
        assert np.array_equal(to_np(outs[0]), wg) and np.array_equal(to_np(outs[1]), wu)
        assert np.array_equal(to_np(outs[2]), wd)
    return to_np(g), to_np(kept)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(688, 256), (2056, 264), (1500, 100), (37, 19), (4104, 512)])
def test_struct_vs_oracle(lib, dtype, shape):
    inter, hidden = shape
    gate = synth.random_matrix(inter, hidden, dtype, seed=inter + 1, device=DEV, scale=0.02, zero_frac=0.3)
    up = synth.random_matrix(inter, hidden, dtype, seed=inter + 2, device=DEV, scale=0.02, zero_frac=0.3)
    down = synth.random_matrix(hidden, inter, dtype, seed=inter + 3, device=DEV, scale=0.02, zero_frac=0.3)
    gate[5] = 0
    up[5] = 0
    down[:, 5] = 0                                          # an emptied channel: magnitude exactly zero
    gate[9] = 0
    up[9] = 0
    down[:, 9] = 0                                          # and a second one: a real tie
    for r in sorted({0, 1, 2, int(0.2 * inter), inter - 1}):
        _check_struct(gate, up, down, r)
    g1, k1 = _check_struct(gate, up, down, inter // 3, compact=False)
    g2, k2 = _check_struct(gate, up, down, inter // 3, compact=False)
    assert np.array_equal(g1.view(np.uint32), g2.view(np.uint32)) and np.array_equal(k1, k2)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(700, 64), (4104, 64), (9000, 32)])
def test_struct_rank_close_and_equal_magnitudes(lib, dtype, shape):
    """Channel magnitudes that share their leading bits, and magnitudes that are all the same (ties by index)."""
    inter, hidden = shape
    rng = np.random.default_rng(inter)
    sign = lambda *sh: torch.tensor(rng.choice([-0.5, 0.5], size=sh), dtype=dtype, device=DEV)
    gate, up, down = sign(inter, hidden), sign(inter, hidden), sign(hidden, inter)
    for r in (1, inter // 3, inter - 1):                    # every magnitude is 3 * hidden / 4: lowest indices go
        g, kept = _check_struct(gate, up, down, r, compact=False)
        assert np.all(g == 0.75 * hidden) and np.array_equal(kept, np.arange(r, inter))
    bump = torch.tensor(rng.choice([0.5, 0.53125, 0.5625, 0.625], size=inter), dtype=dtype, device=DEV)
    gate[:, 0] = bump                                       # now a handful of distinct, close values with many ties
    for r in (1, inter // 3, inter // 2, inter - 1):
        _check_struct(gate, up, down, r, compact=(r == inter // 3))


# ----------------------------------------------------------------- whole toy layer (configs[0])

def test_toy_layer_end_to_end(lib):
    """configs[0]: rank, plan, unstructured prune, structured removal; every output against the oracle."""
    from paper_2504_06323_amd import pipeline
    cfg = synth.CONFIGS["toy"]
    shapes = synth.projection_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 0, n, DEV) for n, _, _, _ in shapes}
    acts = {a: synth.make_activation(cfg, 0, a, DEV) for a in synth.activation_shapes(cfg)}
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, synth.activation_shapes(cfg),
                                    cfg.n_tokens)
    scores = {n: torch.empty((r, c), dtype=torch.float32, device=DEV) for n, r, c, _ in shapes}
    pipeline.rank_layer(st, acts, cfg.alpha, scores=scores)
    _sync()
    counts, numels, cols = st.count.tolist(), [r * c for _, r, c, _ in shapes], [c for _, _, c, _ in shapes]
    ratios = []
    for i, (n, r, c, a) in enumerate(shapes):
        norms, omega, C, O, R, mean = orc.rank_projection(to_np(acts[a]), to_np(weights[n]), cfg.alpha)
        assert rel_err(to_np(st.norms[a]), norms) < 1e-5
        assert rel_err(to_np(scores[n]), np.maximum(omega, 1e-300)) < 1e-5
        assert counts[i] == orc.count_above(to_np(scores[n]), np.float32(st.tau[i].item()))
        assert abs(counts[i] - O) <= np.count_nonzero(np.abs(omega - cfg.alpha * mean) <= 2e-5 * cfg.alpha * mean)
        assert 0.5 < R < 6.0                                  # planted outliers give a ratio of a few percent
        ratios.append(100.0 * counts[i] / numels[i])
    s, ks, clamped = pipeline.plan(counts, numels, cols, 1, len(shapes), cfg.p, cfg.lam)
    want_s, _ = orc.plan_sparsity(np.array(ratios).reshape(1, -1), cfg.p, cfg.lam, "global")
    assert np.allclose(s, want_s.reshape(-1), atol=1e-13) and not clamped
    assert ks == [orc.zeros_per_row(v, c) for v, c in zip(s, cols)]
    pipeline.plan_device(st, cfg.p, cfg.lam)                 # the same plan without the host round trip
    pipeline.prune_layer(st, None)                           # ... and the pruning takes its k from device memory
    _sync()
    assert st.ks_dev.tolist() == ks and st.plan_flags.tolist() == [0, 0]
    assert np.array_equal(to_np(st.sparsity_dev).view(np.uint64), np.array(s, dtype=np.float64).view(np.uint64))
    for i, (n, r, c, a) in enumerate(shapes):
        pruned = orc.select_smallest_per_row(to_np(scores[n]), ks[i])
        assert np.array_equal(to_np(st.pruned[n]), orc.apply_mask(to_np(weights[n]), pruned))
        assert np.array_equal(to_np(st.mask_bits[n]).view(np.uint32), orc.pack_keep_bits(pruned))
    r = int(cfg.struct_frac * cfg.inter)
    res = pipeline.alloc_struct(st, r)
    pipeline.struct_layer(st, r, res)
    _sync()
    masked = {n: to_np(st.pruned[n]) for n in ("gate", "up", "down")}
    want_g = orc.group_magnitude(masked["gate"], masked["up"], masked["down"])
    assert rel_err(to_np(res.group_mag), want_g) < 1e-5
    kept = orc.struct_rank(to_np(res.group_mag), r)
    assert np.array_equal(to_np(res.kept_idx), kept)
    wg, wu, wd = orc.struct_compact(masked["gate"], masked["up"], masked["down"], kept)
    assert np.array_equal(to_np(res.gate), wg) and np.array_equal(to_np(res.up), wu)
    assert np.array_equal(to_np(res.down), wd)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape,k", [((96, 4096), 2048), ((40, 5120), 3000), ((33, 1000), 400), ((64, 14336), 7000), ((30, 8200), 4100),
                                     ((50, 256), 0), ((20, 77), 30), ((9, 4096), 4096)])
def test_select_row_sums_of_squares(lib, dtype, shape, k):
    """The masking pass also hands out the sum of squares of every masked row (the row terms of the structured
    pass's group magnitude): against the oracle on the stored masked rows, for the packet kernels, the any-shape
    kernel and the copy-through path."""
    rows, cols = shape
    w = synth.random_matrix(rows, cols, dtype, seed=rows + cols, device=DEV, scale=0.02, zero_frac=0.1)
    norms = (torch.rand(cols, device=DEV) * 3 + 0.5).float()
    out = torch.full_like(w, 7.0)
    sums = torch.full((rows,), float("nan"), dtype=torch.float32, device=DEV)
    prune.select_mask_batch([w], [norms], [k], w_outs=[out], row_sumsq=[sums])
    _sync()
    masked = to_np(out).astype(np.float64)
    want = (masked * masked).sum(axis=1)
    got = to_np(sums).astype(np.float64)
    assert np.count_nonzero(masked == 0, axis=1).min() >= k
    assert np.max(np.abs(got - want)) <= 2e-6 * np.max(want) + 1e-30
    sums2 = torch.empty_like(sums)
    prune.select_mask_batch([w], [norms], [k], w_outs=[out], row_sumsq=[sums2])
    _sync()
    assert np.array_equal(to_np(sums).view(np.uint32), to_np(sums2).view(np.uint32))          # reproducible


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_struct_with_row_sums_from_the_masking_pass(lib, dtype):
    """prune_struct_compact given the row sums agrees with the call that forms them itself: magnitudes to
    rounding, and -- ranking the magnitudes each call reports -- both with the oracle."""
    inter, hidden, r = 688, 256, 137
    gate, up = (synth.random_matrix(inter, hidden, dtype, seed=s, device=DEV, scale=0.02) for s in (1, 2))
    down = synth.random_matrix(hidden, inter, dtype, seed=3, device=DEV, scale=0.02)
    norms = torch.ones(hidden, dtype=torch.float32, device=DEV)
    mg, mu = torch.empty_like(gate), torch.empty_like(up)
    sg, su = (torch.empty(inter, dtype=torch.float32, device=DEV) for _ in range(2))
    prune.select_mask_batch([gate, up], [norms, norms], [hidden // 2, hidden // 2], w_outs=[mg, mu], row_sumsq=[sg, su])
    res = []
    for given in (False, True):
        g = torch.empty(inter, dtype=torch.float32, device=DEV)
        kept = torch.empty(inter - r, dtype=torch.int32, device=DEV)
        outs = [torch.empty((inter - r, hidden), dtype=dtype, device=DEV), torch.empty((inter - r, hidden), dtype=dtype, device=DEV),
                torch.empty((hidden, inter - r), dtype=dtype, device=DEV)]
        prune.struct_compact(mg, mu, down, r, g, kept, *outs, gate_rowsq=sg if given else None, up_rowsq=su if given else None)
        _sync()
        want_g = orc.group_magnitude(to_np(mg), to_np(mu), to_np(down))
        assert rel_err(to_np(g), want_g) < 2e-6
        want_kept = orc.struct_rank(to_np(g), r)
        assert np.array_equal(to_np(kept), want_kept)
        wg, wu, wd = orc.struct_compact(to_np(mg), to_np(mu), to_np(down), want_kept)
        assert np.array_equal(to_np(outs[0]), wg) and np.array_equal(to_np(outs[1]), wu) and np.array_equal(to_np(outs[2]), wd)
        res.append(to_np(g))
    assert rel_err(res[0], res[1]) < 1e-6


# ----------------------------------------------------------------- planner on the device

@pytest.mark.parametrize("scope", ["global", "category", "layer"])
@pytest.mark.parametrize("n_layers,n_proj", [(1, 7), (32, 7), (3, 300), (40, 7), (300, 3)])
def test_plan_device_vs_host_and_oracle(lib, scope, n_layers, n_proj):
    """Same bits as the host planner, same plan as the oracle; clamping, equal ratios and bad input flagged."""
    rng = np.random.default_rng(n_layers * 1000 + n_proj)
    n = n_layers * n_proj
    cols = rng.choice([256, 688, 4096, 11008, 14336], size=n).astype(np.int64)
    numels = cols * rng.integers(8, 4096, size=n)
    counts = (numels * rng.uniform(0.001, 0.06, size=n)).astype(np.int64)
    code = {"global": prune.SCOPE_GLOBAL, "category": prune.SCOPE_CATEGORY, "layer": prune.SCOPE_LAYER}[scope]
    dev = lambda a, dt: torch.tensor(np.asarray(a), dtype=dt, device=DEV)
    for p, lam, cnt in ((0.5, 0.08, counts), (0.7, 0.08, counts), (0.05, 0.6, counts),      # the third clamps at 0
                        (0.5, 0.08, numels // 16)):                                          # equal ratios: s == p
        s_dev = torch.full((n,), -1.0, dtype=torch.float64, device=DEV)
        k_dev = torch.full((n,), -1, dtype=torch.int32, device=DEV)
        flags = torch.full((2,), -1, dtype=torch.int32, device=DEV)
        prune.plan_sparsity_device(dev(cnt, torch.int64), dev(numels, torch.int64), dev(cols, torch.int64), n_layers,
                                   n_proj, p, lam, s_dev, k_dev, flags, scope=code)
        _sync()
        s_host, k_host, clamped = prune.plan_sparsity(cnt.tolist(), numels.tolist(), n_layers, n_proj, p, lam, code,
                                                      cols=cols.tolist())
        assert np.array_equal(to_np(s_dev).view(np.uint64), np.array(s_host).view(np.uint64))
        assert k_dev.tolist() == k_host and flags.tolist() == [int(clamped), 0]
        ratios = (100.0 * cnt / numels).reshape(n_layers, n_proj)
        if scope == "layer":
            want, want_clamped = orc.plan_sparsity_layerwise(cnt.reshape(n_layers, n_proj),
                                                             numels.reshape(n_layers, n_proj), p, lam,
                                                             cols=cols.reshape(n_layers, n_proj))
        else:
            want, want_clamped = orc.plan_sparsity(ratios, p, lam, scope, cols=cols.reshape(n_layers, n_proj))
        assert np.allclose(to_np(s_dev), want.reshape(-1), atol=1e-12) and bool(want_clamped) == clamped
        exact = [orc.zeros_per_row(v, c) for v, c in zip(want.reshape(-1), cols)]
        near_integer = np.abs(want.reshape(-1) * cols - np.round(want.reshape(-1) * cols)) < 1e-6
        assert all(a == b or t for a, b, t in zip(k_dev.tolist(), exact, near_integer))
    # the last case: every ratio is 6.25 (cols divide numels, so a layer's pooled ratio is 6.25 too)
    assert np.all(to_np(s_dev) == 0.5)
    bad = counts.copy()
    bad[n // 2] = numels[n // 2] + 1
    prune.plan_sparsity_device(dev(bad, torch.int64), dev(numels, torch.int64), dev(cols, torch.int64), n_layers,
                               n_proj, 0.5, 0.08, s_dev, k_dev, flags, scope=code)
    _sync()
    assert flags.tolist()[1] == 1


# ----------------------------------------------------------------- batched ranking

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("case", ["layer", "many", "ragged"])
def test_score_outlier_batch_vs_oracle(lib, dtype, case):
    """One call for several projections: per projection the same sums, thresholds and counts as the oracle."""
    if case == "layer":
        shapes = [(256, 256), (64, 256), (64, 256), (256, 256), (688, 256), (688, 256), (256, 688)]
    elif case == "many":                       # more projections than one launch table holds
        shapes = [(8 + 3 * i, 64 + 8 * (i % 5)) for i in range(37)]
    else:                                      # widths that rule out 128-bit accesses: per-projection kernels
        shapes = [(33, 130), (50, 7), (129, 2056)]
    ws_, norms = [], []
    for i, (rows, cols) in enumerate(shapes):
        w, x = _rank_inputs(rows, cols, dtype, seed=1000 + i)
        ws_.append(w)
        norms.append(gpu_norms(x)[1])
    n = len(shapes)
    alpha = 3.0
    sums = torch.zeros(n, dtype=torch.float64, device=DEV)
    counts = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    taus = torch.zeros(n, dtype=torch.float32, device=DEV)
    prune.score_outlier_batch(ws_, norms, alpha, sums, counts, taus=taus)
    sums2, counts2 = torch.zeros_like(sums), torch.zeros_like(counts)
    prune.score_outlier_batch(ws_, norms, alpha, sums2, counts2)            # again, without the optional output
    _sync()
    assert np.array_equal(bits(sums.view(torch.int64)), bits(sums2.view(torch.int64)))   # reproducible
    assert counts.tolist() == counts2.tolist()
    for i, (rows, cols) in enumerate(shapes):
        m32 = host_metric_f32(ws_[i], norms[i])
        ref = m32.astype(np.float64).sum()
        assert abs(sums[i].item() - ref) <= 1e-6 * ref
        tau = np.float32(taus[i].item())
        assert tau == orc.threshold_f32(alpha, sums[i].item(), rows * cols)
        assert counts[i].item() == orc.count_above(m32, tau)
        single = torch.zeros(1, dtype=torch.float64, device=DEV)
        prune.score(ws_[i], norms[i], single)
        _sync()
        assert abs(single.item() - sums[i].item()) <= 1e-7 * ref      # float32 groups of 32 vs 64 metrics before widening


@pytest.mark.parametrize("k_source", ["host", "device"])
@pytest.mark.parametrize("dtype", DTYPES)
def test_select_mask_batch_vs_oracle(lib, dtype, k_source):
    """Several projections per call: equal-width ones share a launch, odd ones take the single path.
    k comes from the host array or is read by the kernels from device memory (0, cols and beyond included)."""
    shapes = [(40, 1024), (16, 1024), (9, 688), (25, 1024), (7, 4104), (5, 130), (12, 1024), (3, 16392)] + \
             [(4 + i, 512) for i in range(20)]                     # more than one launch table of one width
    ws_, norms, ks, outs, masks = [], [], [], [], []
    for i, (rows, cols) in enumerate(shapes):
        w, x = _rank_inputs(rows, cols, dtype, seed=2000 + i)
        ws_.append(w)
        norms.append(gpu_norms(x)[1])
        ks.append([cols // 2, 0, cols // 3, cols, 1][i % 5])
        outs.append(None if i % 4 == 3 else torch.full_like(w, 7.0))
        masks.append(None if i % 3 == 2 else torch.full((rows, (cols + 31) // 32), -1, dtype=torch.int32, device=DEV))
    originals = [to_np(w).copy() for w in ws_]
    metrics = [host_metric_f32(w, n) for w, n in zip(ws_, norms)]
    if k_source == "host":
        prune.select_mask_batch(ws_, norms, ks, w_outs=outs, mask_bits=masks)
    else:
        over = [k + 5 if k == c else k for k, (_, c) in zip(ks, shapes)]          # above cols counts as cols
        ks_dev = torch.tensor(over, dtype=torch.int32, device=DEV)
        prune.select_mask_batch(ws_, norms, None, w_outs=outs, mask_bits=masks, ks_dev=ks_dev)
    _sync()
    for i, (rows, cols) in enumerate(shapes):
        pruned = orc.select_smallest_per_row(metrics[i], ks[i])
        got = to_np(outs[i] if outs[i] is not None else ws_[i])
        assert np.array_equal(got, orc.apply_mask(originals[i], pruned)), f"item {i} {shapes[i]} k={ks[i]}"
        if masks[i] is not None:
            assert np.array_equal(to_np(masks[i]).view(np.uint32), orc.pack_keep_bits(pruned)), f"item {i}"
        if outs[i] is not None:
            assert np.array_equal(to_np(ws_[i]), originals[i])          # the input is untouched when out of place


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("aligned", [True, False])
def test_layer_scope_outliers_vs_oracle(lib, dtype, aligned):
    """Layer-level rule (Eq. 3, Eq. 4): one threshold from the mean over all projections of the batch."""
    shapes = [(256, 256), (64, 256), (688, 256), (256, 688)] if aligned else [(33, 130), (50, 7), (129, 2056)]
    ws_, norms = [], []
    for i, (rows, cols) in enumerate(shapes):
        w, x = _rank_inputs(rows, cols, dtype, seed=3000 + i)
        ws_.append(w * (1.0 + 3.0 * i))                  # different scales: layer and projection rules differ
        norms.append(gpu_norms(x)[1])
    n = len(shapes)
    alpha = 4.0
    sums = torch.zeros(n, dtype=torch.float64, device=DEV)
    counts = torch.zeros(n, dtype=torch.int64, device=DEV)
    taus = torch.zeros(n, dtype=torch.float32, device=DEV)
    prune.score_outlier_batch(ws_, norms, alpha, sums, counts, taus=taus, outlier_scope=prune.OUTLIERS_PER_LAYER)
    _sync()
    m32 = [host_metric_f32(w, nr) for w, nr in zip(ws_, norms)]
    numel = sum(r * c for r, c in shapes)
    tau = np.float32(taus[0].item())
    assert (to_np(taus) == tau).all()
    assert tau == orc.threshold_f32(alpha, float(np.sum(sums.tolist())), numel)
    assert counts.tolist() == [orc.count_above(m, tau) for m in m32]            # bit-exact, kernel precision
    omegas = [orc.weight_metric(to_np(w), to_np(nr).astype(np.float64)) for w, nr in zip(ws_, norms)]
    c, o, r, mean, per_proj = orc.layer_outlier_stats(omegas, alpha)
    assert abs(float(tau) - alpha * mean) <= 1e-6 * alpha * mean
    band = sum(np.count_nonzero(np.abs(om - alpha * mean) <= 1e-5 * alpha * mean) for om in omegas)
    assert abs(sum(counts.tolist()) - o) <= band
    per = torch.zeros(n, dtype=torch.int64, device=DEV)
    prune.score_outlier_batch(ws_, norms, alpha, sums, per, outlier_scope=prune.OUTLIERS_PER_PROJECTION)
    _sync()
    assert per.tolist() != counts.tolist()                                     # the two rules really differ here


def test_layer_pruning_ranked_planned_and_masked_on_the_device(lib):
    """Layer pruning (Section 4.1.3, Pruning Methods, item 2) without a host round trip: outliers against each
    layer's mean, one target per layer from the pooled layer ratios, every projection of a layer masked to it."""
    shapes = [(256, 256), (64, 256), (688, 256), (256, 688)]
    n_layers, n_proj, alpha, p, lam = 3, len(shapes), 4.0, 0.5, 0.08
    n = n_layers * n_proj
    counts = torch.zeros(n, dtype=torch.int64, device=DEV)
    sums = torch.zeros(n, dtype=torch.float64, device=DEV)
    layers = []
    for l in range(n_layers):
        ws_, norms = [], []
        for i, (rows, cols) in enumerate(shapes):
            w, x = _rank_inputs(rows, cols, torch.bfloat16, seed=4000 + 10 * l + i)
            x[:, : 3 * (l + 1)] *= 12.0                  # more planted outlier channels in later layers
            ws_.append(w)
            norms.append(gpu_norms(x)[1])
        layers.append((ws_, norms))
        prune.score_outlier_batch(ws_, norms, alpha, sums[l * n_proj:(l + 1) * n_proj],
                                  counts[l * n_proj:(l + 1) * n_proj], outlier_scope=prune.OUTLIERS_PER_LAYER)
    numels = torch.tensor([r * c for r, c in shapes] * n_layers, dtype=torch.int64, device=DEV)
    cols = torch.tensor([c for _, c in shapes] * n_layers, dtype=torch.int64, device=DEV)
    s_dev = torch.empty(n, dtype=torch.float64, device=DEV)
    k_dev = torch.empty(n, dtype=torch.int32, device=DEV)
    flags = torch.empty(2, dtype=torch.int32, device=DEV)
    prune.plan_sparsity_device(counts, numels, cols, n_layers, n_proj, p, lam, s_dev, k_dev, flags,
                               scope=prune.SCOPE_LAYER)
    outs = []
    for l, (ws_, norms) in enumerate(layers):
        o = [torch.empty_like(w) for w in ws_]
        prune.select_mask_batch(ws_, norms, None, w_outs=o, ks_dev=k_dev[l * n_proj:(l + 1) * n_proj])
        outs.append(o)
    _sync()
    assert flags.tolist() == [0, 0]
    c2 = to_np(counts).reshape(n_layers, n_proj)
    want, _ = orc.plan_sparsity_layerwise(c2, to_np(numels).reshape(n_layers, n_proj), p, lam,
                                          cols=to_np(cols).reshape(n_layers, n_proj))
    got = to_np(s_dev).reshape(n_layers, n_proj)
    assert np.allclose(got, want, atol=1e-13) and (got == got[:, :1]).all()
    assert got[:, 0].mean() == pytest.approx(p, abs=1e-12) and len(set(got[:, 0])) == n_layers
    ratios = orc.layer_ratios(c2, to_np(numels).reshape(n_layers, n_proj))
    assert (np.diff(got[np.argsort(ratios), 0]) < 0).all()                   # more outliers => pruned less
    ks = k_dev.tolist()
    for l in range(n_layers):
        for i, (rows, cols_i) in enumerate(shapes):
            k = ks[l * n_proj + i]
            assert k == orc.zeros_per_row(got[l, i], cols_i)
            w_in, w_out = to_np(layers[l][0][i]), to_np(outs[l][i])
            omega = host_metric_f32(layers[l][0][i], layers[l][1][i])
            pruned = orc.select_smallest_per_row(omega, k)
            assert np.array_equal(w_out, orc.apply_mask(w_in, pruned))


# ----------------------------------------------------------------- coupled groups (attention heads, grouped queries)

def _check_groups(row_mats, row_per, col_mats, col_per, n_groups, r, compact=True):
    g = torch.empty(n_groups, dtype=torch.float32, device=DEV)
    kept = torch.full((n_groups - r,), -1, dtype=torch.int32, device=DEV)
    row_outs = col_outs = None
    if compact:
        row_outs = [torch.full(((n_groups - r) * p, m.shape[1]), 7.0, dtype=m.dtype, device=DEV)
                    for m, p in zip(row_mats, row_per)]
        col_outs = [torch.full((m.shape[0], (n_groups - r) * p), 7.0, dtype=m.dtype, device=DEV)
                    for m, p in zip(col_mats, col_per)]
    prune.struct_groups(row_mats, row_per, col_mats, col_per, n_groups, r, g, kept, row_outs, col_outs)
    _sync()
    rm, cm = [to_np(m) for m in row_mats], [to_np(m) for m in col_mats]
    want_g = orc.coupled_group_magnitude(rm, row_per, cm, col_per, n_groups)
    nz = want_g > 0
    assert rel_err(to_np(g)[nz], want_g[nz]) < tol_for(row_mats[0].dtype if row_mats else col_mats[0].dtype)
    assert rel_err(to_np(g)[nz], want_g[nz]) < 5e-6 and (to_np(g)[~nz] == 0).all()
    want_kept = orc.struct_rank(to_np(g), r)                      # oracle ranking on the kernel's magnitudes
    assert np.array_equal(to_np(kept), want_kept)
    if compact:
        wr, wc = orc.coupled_group_compact(rm, row_per, cm, col_per, want_kept)
        for got, want in zip(row_outs + col_outs, wr + wc):
            assert np.array_equal(to_np(got), want)
    return to_np(g), to_np(kept)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("case", ["gqa", "mha_ragged", "mlp", "rows_only", "cols_only"])
def test_struct_groups_vs_oracle(lib, dtype, case):
    mk = lambda r, c, s: synth.random_matrix(r, c, dtype, seed=s, device=DEV, scale=0.02, zero_frac=0.2)
    if case == "gqa":            # 8 key/value heads, 4 query heads each, head width 16, hidden 256
        n_groups, m, d, hidden = 8, 4, 16, 256
        rows, row_per = [mk(n_groups * m * d, hidden, 1), mk(n_groups * d, hidden, 2), mk(n_groups * d, hidden, 3)], [m * d, d, d]
        cols, col_per = [mk(hidden, n_groups * m * d, 4)], [m * d]
    elif case == "mha_ragged":   # head width 5, hidden 37: nothing is packet-aligned
        n_groups, d, hidden = 6, 5, 37
        rows, row_per = [mk(n_groups * d, hidden, 5), mk(n_groups * d, hidden, 6), mk(n_groups * d, hidden, 7)], [d, d, d]
        cols, col_per = [mk(hidden, n_groups * d, 8)], [d]
    elif case == "mlp":          # one row / one column per group: the feed-forward channel case
        n_groups, hidden = 688, 256
        rows, row_per = [mk(n_groups, hidden, 9), mk(n_groups, hidden, 10)], [1, 1]
        cols, col_per = [mk(hidden, n_groups, 11)], [1]
    elif case == "rows_only":
        n_groups = 10
        rows, row_per, cols, col_per = [mk(n_groups * 3, 64, 12)], [3], [], []
    else:
        n_groups = 10
        rows, row_per, cols, col_per = [], [], [mk(48, n_groups * 8, 13)], [8]
    if rows:
        rows[0][:row_per[0]] = 0     # make group 0 weaker so the ranking is not trivial
    for r in sorted({0, 1, n_groups // 4, n_groups - 1}):
        _check_groups(rows, row_per, cols, col_per, n_groups, r)
    g1, k1 = _check_groups(rows, row_per, cols, col_per, n_groups, n_groups // 2, compact=False)
    g2, k2 = _check_groups(rows, row_per, cols, col_per, n_groups, n_groups // 2, compact=False)
    assert np.array_equal(g1.view(np.uint32), g2.view(np.uint32)) and np.array_equal(k1, k2)
    if case == "mlp":            # the dedicated feed-forward entry point agrees with the generic one
        gm = torch.empty(n_groups, dtype=torch.float32, device=DEV)
        kp = torch.empty(n_groups - n_groups // 2, dtype=torch.int32, device=DEV)
        prune.struct_compact(rows[0], rows[1], cols[0], n_groups // 2, gm, kp)
        _sync()
        assert np.array_equal(to_np(kp), k1) and rel_err(to_np(gm), g1) < 1e-6
