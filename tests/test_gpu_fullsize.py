"""Full-size parity: the workloads of the benchmark and of the larger configurations, in the launch
configuration bench.py times (hot mode: no materialised scores, shared workspace, out-of-place masking).

At these sizes the float64 oracle is applied to sampled outputs (channels of the activation
statistics, rows of the masks) and in full where NumPy finishes in seconds (metric sums, outlier
counts, group magnitudes, gathers); integer results are compared bit-exactly in the kernel's
precision as in test_gpu_parity.py, and properties that hold at any size (exactly k pruned per row,
survivors untouched, keep-bits consistent with the zeros) are checked over every row.
"""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2504_06323_amd import pipeline, prune, synth
from util import rel_err, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _sample(n, count, seed):
    rng = np.random.default_rng(seed)
    idx = set(rng.choice(n, size=min(count, n), replace=False).tolist()) | {0, n - 1}
    return np.array(sorted(idx))


def _metric_f32(w_np, norms_np):
    """Kernel-precision metric on the host: one float32 multiply per element."""
    return np.abs(w_np.astype(np.float32)) * norms_np.astype(np.float32)[None, :]


def _popcount32(a):
    a = a.astype(np.uint32)
    a = a - ((a >> 1) & 0x55555555)
    a = (a & 0x33333333) + ((a >> 2) & 0x33333333)
    a = (a + (a >> 4)) & 0x0F0F0F0F
    return (a * 0x01010101 >> 24) & 0xFF


def _check_norms(x, norms_gpu, seed, n_channels=24):
    """Sampled channels (plus the largest-norm ones, i.e. the planted outliers) against the oracle."""
    c = x.shape[1]
    idx = np.union1d(_sample(c, n_channels, seed), np.argsort(to_np(norms_gpu))[-4:])
    cols = to_np(x[:, torch.as_tensor(idx, device=x.device)])
    want = orc.column_norms(cols)
    got = to_np(norms_gpu)[idx]
    assert rel_err(got, want) < 1e-2            # the stated bf16 tolerance
    assert rel_err(got, want) < 5e-6            # what fp32 stripes + fp64 cross-stripe sums deliver


def _check_rank(w, norms, alpha, ssum, count, tau):
    w_np, n_np = to_np(w), to_np(norms)
    m32 = _metric_f32(w_np, n_np)
    assert tau == orc.threshold_f32(alpha, ssum, w_np.size)
    assert count == orc.count_above(m32, tau)                         # bit-exact in the kernel's precision
    omega = orc.weight_metric(w_np, n_np.astype(np.float64))          # float64 oracle on the same norms
    c, o, ratio, mean = orc.outlier_stats(omega, alpha)
    assert abs(ssum - omega.sum()) <= 1e-6 * omega.sum()
    band = np.count_nonzero(np.abs(omega - alpha * mean) <= 1e-5 * alpha * mean)
    assert abs(count - o) <= band
    return m32


def _check_mask(w, m32, k, w_out, mask_bits, seed, n_rows=12):
    w_np, out, bits = to_np(w), to_np(w_out), to_np(mask_bits).view(np.uint32)
    rows, cols = w_np.shape
    # every row: exactly k pruned, keep-bits consistent, survivors bit-identical, pruned entries zero
    assert (_popcount32(bits).sum(axis=1) == cols - k).all()
    keep = ((bits[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(rows, -1)[:, :cols].astype(bool)
    assert np.array_equal(out.view(np.uint32)[keep], w_np.view(np.uint32)[keep])
    assert (out[~keep] == 0).all()
    # pruned metrics never exceed kept metrics (row by row)
    hi_pruned = np.where(keep, -np.inf, m32).max(axis=1)
    lo_kept = np.where(keep, m32, np.inf).min(axis=1)
    assert (hi_pruned <= lo_kept).all()
    # sampled rows: the oracle's stable-sort selection on the kernel's metric bits
    idx = _sample(rows, n_rows, seed)
    pruned = orc.select_smallest_per_row(m32[idx], k)
    assert np.array_equal(~keep[idx], pruned)
    assert np.array_equal(out[idx], orc.apply_mask(w_np[idx], pruned))


def _check_sampled_rows(w, norms, k, w_out, mask_bits, seed, n_rows):
    """Sampled rows only: the oracle's stable-sort selection on the kernel-precision metric of those rows."""
    rows, cols = w.shape
    idx = _sample(rows, n_rows, seed)
    sel = torch.as_tensor(idx, device=w.device)
    w_np, out = to_np(w[sel]), to_np(w_out[sel])
    m32 = _metric_f32(w_np, to_np(norms))
    pruned = orc.select_smallest_per_row(m32, k)
    assert np.array_equal(out, orc.apply_mask(w_np, pruned))
    assert np.array_equal(to_np(mask_bits[sel]).view(np.uint32), orc.pack_keep_bits(pruned))


def _run_layer(cfg_name, check_struct=True, layer=0):
    cfg = synth.CONFIGS[cfg_name]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    print(f"[fullsize] {cfg_name}: generating inputs of layer {layer}", flush=True)
    weights = {n: synth.make_weight(cfg, layer, n, DEV) for n, _, _, _ in shapes}
    acts = {a: synth.make_activation(cfg, layer, a, DEV) for a in act_shapes}
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, cfg.n_tokens)
    print(f"[fullsize] {cfg_name}: phase 1", flush=True)
    pipeline.rank_layer(st, acts, cfg.alpha)
    torch.cuda.synchronize()
    for i, a in enumerate(act_shapes):
        _check_norms(acts[a], st.norms[a], seed=100 + i)
    del acts
    torch.cuda.empty_cache()
    counts, ssums, taus = st.count.tolist(), st.score_sum.tolist(), to_np(st.tau)
    metrics = {}
    for i, (n, r, c, a) in enumerate(shapes):
        metrics[n] = _check_rank(weights[n], st.norms[a], cfg.alpha, ssums[i], counts[i], taus[i])
    numels, cols = [r * c for _, r, c, _ in shapes], [c for _, _, c, _ in shapes]
    s, ks, clamped = pipeline.plan(counts, numels, cols, 1, len(shapes), cfg.p, cfg.lam)
    ratios = 100.0 * np.array(counts) / np.array(numels)
    want_s, _ = orc.plan_sparsity(ratios.reshape(1, -1), cfg.p, cfg.lam, "global", cols=np.array(cols).reshape(1, -1))
    assert np.allclose(s, want_s.reshape(-1), atol=1e-13) and not clamped
    assert ks == [orc.zeros_per_row(v, c) for v, c in zip(s, cols)]
    assert abs(np.mean(s) - cfg.p) < 1e-12
    print(f"[fullsize] {cfg_name}: phase 2, zeros per row {ks}", flush=True)
    pipeline.prune_layer(st, ks)
    torch.cuda.synchronize()
    for i, (n, r, c, a) in enumerate(shapes):
        _check_mask(weights[n], metrics[n], ks[i], st.pruned[n], st.mask_bits[n], seed=200 + i)
    del metrics
    if not check_struct:
        return
    r = int(cfg.struct_frac * cfg.inter)
    print(f"[fullsize] {cfg_name}: structured removal of {r} channels", flush=True)
    res = pipeline.alloc_struct(st, r)
    pipeline.struct_layer(st, r, res)
    torch.cuda.synchronize()
    masked = {n: to_np(st.pruned[n]) for n in ("gate", "up", "down")}
    want_g = orc.group_magnitude(masked["gate"], masked["up"], masked["down"])
    assert rel_err(to_np(res.group_mag), want_g) < 1e-2 and rel_err(to_np(res.group_mag), want_g) < 5e-6
    kept = orc.struct_rank(to_np(res.group_mag), r)
    assert np.array_equal(to_np(res.kept_idx), kept)
    assert len(kept) == cfg.inter - r
    wg, wu, wd = orc.struct_compact(masked["gate"], masked["up"], masked["down"], kept)
    assert np.array_equal(to_np(res.gate), wg) and np.array_equal(to_np(res.up), wu)
    assert np.array_equal(to_np(res.down), wd)
    # attention block: one group per key/value head (head width 128) with the query heads that share it
    d = 128
    n_groups, m = cfg.kv_out // d, cfg.q_out // cfg.kv_out
    r_att = max(1, int(cfg.struct_frac * n_groups))
    print(f"[fullsize] {cfg_name}: removing {r_att} of {n_groups} key/value heads ({m} query heads each)", flush=True)
    rows = [st.pruned["q"], st.pruned["k"], st.pruned["v"]]
    row_per, cols, col_per = [m * d, d, d], [st.pruned["o"]], [m * d]
    gm = torch.empty(n_groups, dtype=torch.float32, device=DEV)
    kp = torch.empty(n_groups - r_att, dtype=torch.int32, device=DEV)
    row_outs = [torch.empty(((n_groups - r_att) * p, t.shape[1]), dtype=t.dtype, device=DEV) for t, p in zip(rows, row_per)]
    col_outs = [torch.empty((cols[0].shape[0], (n_groups - r_att) * m * d), dtype=cols[0].dtype, device=DEV)]
    prune.struct_groups(rows, row_per, cols, col_per, n_groups, r_att, gm, kp, row_outs, col_outs)
    torch.cuda.synchronize()
    rm, cm = [to_np(t) for t in rows], [to_np(t) for t in cols]
    want = orc.coupled_group_magnitude(rm, row_per, cm, col_per, n_groups)
    assert rel_err(to_np(gm), want) < 1e-2 and rel_err(to_np(gm), want) < 5e-6
    kept_att = orc.struct_rank(to_np(gm), r_att)
    assert np.array_equal(to_np(kp), kept_att)
    wr, wc = orc.coupled_group_compact(rm, row_per, cm, col_per, kept_att)
    for got, ref in zip(row_outs + col_outs, wr + wc):
        assert np.array_equal(to_np(got), ref)


def test_llama7b_layer_bench_configuration(lib):
    """configs[1], exactly what bench.py runs."""
    _run_layer("llama7b_layer")


def test_llama3_8b_layer_gqa_composite(lib):
    """configs[2]: grouped-query shapes (k/v 1024 x 4096), 14336-wide MLP, 50 % unstructured + 20 % structured."""
    _run_layer("llama3_8b_layer")


@pytest.mark.timeout(600)
def test_llama2_13b_stress_layer(lib):
    """configs[4], layers 0 and 39: 256 x 4096 calibration tokens, x100 outlier channels, 60 % + 30 %."""
    _run_layer("llama2_13b_stress")
    _run_layer("llama2_13b_stress", layer=39, check_struct=False)


def test_long_calibration_statistic_error_does_not_grow(lib):
    """One million tokens, a channel a hundred times larger than the rest: single-precision sums are folded into
    doubles every 1024 rows, so the statistic of the large channel stays within 2e-6 of the float64 oracle."""
    cfg = synth.CONFIGS["llama2_13b_stress"]
    x = synth.make_activation(cfg, 1, "attn_in", DEV)                  # [1048576, 5120]
    c = x.shape[1]
    sumsq, norms = (torch.empty(c, dtype=torch.float32, device=DEV) for _ in range(2))
    prune.stats_norms(x, sumsq, norms)
    torch.cuda.synchronize()
    big = np.argsort(to_np(norms))[-5:]                                # the planted x100 channels
    idx = np.union1d(big, _sample(c, 16, 7))
    cols = to_np(x[:, torch.as_tensor(idx, device=x.device)])
    want = orc.column_sumsq(cols)
    got = to_np(sumsq)[idx].astype(np.float64)
    err = np.abs(got - want) / want
    assert err.max() < 2e-6, err.max()
    assert (to_np(norms)[big] > 50 * np.median(to_np(norms))).all()     # these are the planted ones


def _popcount_rows(bits):
    """Keep-bits per row, counted on the device (int32 words)."""
    b = bits.to(torch.int64) & 0xFFFFFFFF
    b = b - ((b >> 1) & 0x55555555)
    b = (b & 0x33333333) + ((b >> 2) & 0x33333333)
    b = (b + (b >> 4)) & 0x0F0F0F0F
    return ((b * 0x01010101) >> 24 & 0xFF).sum(dim=1)


def _check_mask_on_device(w, w_out, mask_bits, k):
    """Properties that hold at any size, evaluated on the GPU for every row of a projection: exactly k entries
    pruned (by the keep-bits), pruned entries zero, survivors bit-identical."""
    rows, cols = w.shape
    assert bool((_popcount_rows(mask_bits) == cols - k).all())
    shifts = torch.arange(32, device=w.device, dtype=torch.int32)
    keep = ((mask_bits[:, :, None] >> shifts) & 1).reshape(rows, -1)[:, :cols].bool()
    a, b = w.view(torch.int16), w_out.view(torch.int16)
    assert bool((b[~keep] == 0).all())
    assert bool((a[keep] == b[keep]).all())


@pytest.mark.timeout(900)
def test_full_model_llama3_8b_sweep(lib):
    """configs[3]: 32 layers, 224 projections ranked once, pruned at 30 / 50 / 70 % reusing the ranking.

    Every layer: norms on sampled channels, threshold and bit-exact outlier count of all seven projections
    (the host forms the kernel-precision metric), and at every target the any-size mask properties on the device
    for every row of every projection.  Sampled-row oracle selection on every layer at one target (p = 0.5) and
    on layers 0 and 31 at all three."""
    cfg = synth.CONFIGS["llama3_8b_full"]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    proj_inputs = {n: a for n, _, _, a in shapes}
    n_proj = len(shapes)
    end_layers = (0, cfg.n_layers - 1)
    states, counts = [], []
    for layer in range(cfg.n_layers):
        if layer % 8 == 0:
            print(f"[fullsize] full model: ranking layer {layer}", flush=True)
        weights = {n: synth.make_weight(cfg, layer, n, DEV) for n, _, _, _ in shapes}
        acts = {a: synth.make_activation(cfg, layer, a, DEV) for a in act_shapes}
        st = pipeline.LayerState.create(weights, proj_inputs, act_shapes, cfg.n_tokens,
                                        share_outputs_with=states[0] if states else None)
        pipeline.rank_layer(st, acts, cfg.alpha)
        torch.cuda.synchronize()
        for i, a in enumerate(act_shapes):
            _check_norms(acts[a], st.norms[a], seed=1000 * layer + i, n_channels=24 if layer in end_layers else 6)
        ssums, taus, cnts = st.score_sum.tolist(), to_np(st.tau), st.count.tolist()
        for i, (n, r, c, a) in enumerate(shapes):
            if layer in end_layers:                       # the float64 oracle as well
                _check_rank(weights[n], st.norms[a], cfg.alpha, ssums[i], cnts[i], taus[i])
            else:                                         # threshold and bit-exact count in the kernel's precision
                m32 = _metric_f32(to_np(weights[n]), to_np(st.norms[a]))
                assert taus[i] == orc.threshold_f32(cfg.alpha, ssums[i], m32.size)
                assert cnts[i] == orc.count_above(m32, taus[i])
                assert abs(ssums[i] - float(m32.sum(dtype=np.float64))) <= 1e-6 * ssums[i]
        del acts
        states.append(st)
        counts += st.count.tolist()
    assert len(counts) == 224
    numels = [r * c for _, r, c, _ in shapes] * cfg.n_layers
    cols = [c for _, _, c, _ in shapes] * cfg.n_layers
    ratios = (100.0 * np.array(counts) / np.array(numels)).reshape(cfg.n_layers, n_proj)
    assert ratios.std() > 0                                   # layers differ, so the targets are non-uniform
    for p in cfg.p_sweep:
        s, ks, clamped = pipeline.plan(counts, numels, cols, cfg.n_layers, n_proj, p, cfg.lam)
        want_s, _ = orc.plan_sparsity(ratios, p, cfg.lam, "global", cols=np.array(cols).reshape(cfg.n_layers, n_proj))
        assert np.allclose(np.array(s).reshape(cfg.n_layers, n_proj), want_s, atol=1e-13) and not clamped
        assert abs(np.mean(s) - p) < 1e-12 and max(s) - min(s) == pytest.approx(2 * cfg.lam, rel=1e-9)
        print(f"[fullsize] full model: pruning at p = {p}", flush=True)
        for layer, st in enumerate(states):
            lk = ks[layer * n_proj:(layer + 1) * n_proj]
            pipeline.prune_layer(st, lk)                      # phase 2 only: the ranking is reused
            for i, (n, r, c, a) in enumerate(shapes):
                _check_mask_on_device(st.weights[n], st.pruned[n], st.mask_bits[n], lk[i])
            if layer in end_layers or p == 0.5:
                torch.cuda.synchronize()
                for i, (n, r, c, a) in enumerate(shapes):
                    if layer in end_layers:
                        m32 = _metric_f32(to_np(st.weights[n]), to_np(st.norms[a]))
                        _check_mask(st.weights[n], m32, lk[i], st.pruned[n], st.mask_bits[n], seed=layer * 10 + i, n_rows=6)
                    else:
                        _check_sampled_rows(st.weights[n], st.norms[a], lk[i], st.pruned[n], st.mask_bits[n],
                                            seed=layer * 10 + i, n_rows=3)
        torch.cuda.synchronize()


def test_scaling_the_activations_by_two_changes_nothing_that_is_counted(lib):
    """A power-of-two factor on the activations scales every norm and metric exactly, so outlier counts, zeros per
    row and masks must be bit-identical (the norm needs no normalisation by tokens or samples)."""
    cfg = synth.CONFIGS["llama3_8b_layer"]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 3, n, DEV) for n, _, _, _ in shapes}
    results = []
    for factor in (1.0, 2.0):
        acts = {a: synth.make_activation(cfg, 3, a, DEV, n_seqs=8) * factor for a in act_shapes}
        st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, 8 * cfg.seq_len)
        pipeline.rank_layer(st, acts, cfg.alpha)
        pipeline.plan_device(st, cfg.p, cfg.lam)
        pipeline.prune_layer(st, None)
        torch.cuda.synchronize()
        results.append((st.count.tolist(), st.ks_dev.tolist(), {n: st.mask_bits[n].clone() for n in st.names},
                        {a: to_np(st.norms[a]) for a in act_shapes}))
        del acts
    (c1, k1, m1, n1), (c2, k2, m2, n2) = results
    assert c1 == c2 and k1 == k2
    for n in m1:
        assert torch.equal(m1[n], m2[n])
    for a in n1:
        assert np.array_equal(n2[a], 2.0 * n1[a])
