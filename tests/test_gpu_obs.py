"""GPU parity of the Hessian-based pruner's stages against oracle/obs_oracle.py, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from oracle import obs_oracle as obs
from paper_2504_06323_amd import prune, synth
from util import to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sync():
    torch.cuda.synchronize()


def _acts(tokens, channels, dtype, seed):
    x = synth.random_matrix(tokens, channels, dtype, seed=seed, device=DEV, scale=1.0)
    if channels >= 8:
        x[:, 3] *= 20.0                                    # an outlier channel, as in the synthetic activations
    return x


def _scaled_err(got, want):
    """max |got - want| / sqrt(H_ii H_jj): the natural scale of entry (i, j) (Cauchy-Schwarz bounds |H_ij| by it)."""
    d = np.sqrt(np.maximum(np.diag(want), 1e-300))
    return float(np.max(np.abs(got - want) / np.outer(d, d))) if want.size else 0.0


# fp32 sums of exact products over at most 64 k-steps of 16 tokens per share of the tokens here: the worst-case
# bound is (64 + 16) * 2^-24 = 5e-6 of sum |x_i x_j| <= sqrt(H_ii H_jj); fp32 input adds one rounding per product
HESSIAN_TOL = {torch.bfloat16: 5e-6, torch.float32: 2e-5}


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape", [(1000, 512), (300, 688), (70, 100), (33, 8), (2050, 256), (5, 1048)])
def test_hessian_vs_oracle(lib, dtype, shape):
    tokens, channels = shape
    x = _acts(tokens, channels, dtype, seed=tokens + channels)
    h = torch.zeros((channels, channels), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    _sync()
    want = obs.gram_matrix(to_np(x))
    got = to_np(h).astype(np.float64)
    assert _scaled_err(got, want) < HESSIAN_TOL[dtype]
    assert np.array_equal(to_np(h), to_np(h).T)                               # bitwise symmetric
    h2 = torch.zeros_like(h)
    prune.hessian_accumulate(x, h2)
    _sync()
    assert np.array_equal(to_np(h).view(np.uint32), to_np(h2).view(np.uint32))   # reproducible


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_hessian_chunks_pitch_and_empty(lib, dtype):
    tokens, channels = 777, 520
    wide = _acts(tokens, channels + 24, dtype, seed=9)
    x = wide[:, 8:8 + channels]                                               # a view with a pitch: still 16-byte aligned
    h = torch.zeros((channels, channels + 40), dtype=torch.float32, device=DEV)[:, :channels]   # pitched output
    prune.hessian_accumulate(x[:300], h)
    prune.hessian_accumulate(x[300:300], h)                                   # zero tokens: nothing happens
    prune.hessian_accumulate(x[300:], h)
    _sync()
    want = obs.gram_matrix(to_np(x))
    assert _scaled_err(to_np(h).astype(np.float64), want) < HESSIAN_TOL[dtype]
    odd = wide[:, 3:3 + channels]                                             # not 16-byte aligned: the plain kernel
    h3 = torch.zeros((channels, channels), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(odd, h3)
    _sync()
    assert _scaled_err(to_np(h3).astype(np.float64), obs.gram_matrix(to_np(odd))) < 2e-5


def test_hessian_diagonal_is_the_metric_path_statistic(lib):
    """diag(H) is the sum of squares that the weight metric's norms come from: both paths must agree."""
    x = _acts(4096, 768, torch.bfloat16, seed=11)
    h = torch.zeros((768, 768), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    sumsq = torch.zeros(768, dtype=torch.float32, device=DEV)
    prune.stats_accumulate(x, sumsq)
    _sync()
    want = orc.column_sumsq(to_np(x))
    assert np.max(np.abs(to_np(h).diagonal() - want) / want) < 1e-5
    assert np.max(np.abs(to_np(sumsq) - want) / want) < 1e-5


# ----------------------------------------------------------------- full size (the benchmark's launch configuration)

@pytest.mark.parametrize("act", ["attn_in", "down_in"])
def test_hessian_fullsize_sampled(lib, act):
    """One activation tensor of the LLaMA-7B-shaped layer (262144 tokens x 4096 or 11008 channels): sampled
    rows of H against the oracle (whole rows would need teraflops on the host), symmetry over the whole matrix,
    and the diagonal against the metric path's sums of squares."""
    cfg = synth.CONFIGS["llama7b_layer"]
    x = synth.make_activation(cfg, 0, act, DEV)
    tokens, channels = x.shape
    h = torch.zeros((channels, channels), dtype=torch.float32, device=DEV)
    ws = torch.empty(prune.hessian_workspace_bytes(tokens, channels), dtype=torch.uint8, device=DEV)
    prune.hessian_accumulate(x, h, ws=ws)
    _sync()
    assert bool(torch.equal(h, h.t()))
    rng = np.random.default_rng(channels)
    hot = torch.argsort(torch.diagonal(h))[-2:].cpu().numpy()                 # planted outlier channels
    rows = np.unique(np.concatenate([rng.choice(channels, size=6, replace=False), hot, [0, 255, 256, channels - 1]]))
    cols = np.unique(np.concatenate([rng.choice(channels, size=40, replace=False), rows]))
    xr = to_np(x[:, torch.as_tensor(rows, device=DEV)]).astype(np.float64)
    xc = to_np(x[:, torch.as_tensor(cols, device=DEV)]).astype(np.float64)
    want = xr.T @ xc                                                          # the oracle's definition on the sample
    got = to_np(h)[np.ix_(rows, cols)].astype(np.float64)
    diag = to_np(torch.diagonal(h)).astype(np.float64)
    scale = np.sqrt(np.outer(diag[rows], diag[cols]))
    # worst case for fp32 sums over a split of the tokens: (k-steps per split + 16) * 2^-24 of sum |x_i x_j|;
    # 262144 tokens in >= 4 splits of <= 4096 k-steps: 2.5e-4; the sums behave like random walks, far below that
    assert np.max(np.abs(got - want) / scale) < 2.5e-4
    assert np.max(np.abs(got - want) / scale) < 5e-6
    sumsq = torch.zeros(channels, dtype=torch.float32, device=DEV)
    prune.stats_accumulate(x, sumsq)
    _sync()
    assert np.max(np.abs(diag / to_np(sumsq).astype(np.float64) - 1.0)) < 1e-5


# ----------------------------------------------------------------- damping and factorisation

def _factor_err(r_gpu, r_ref):
    """max |R_gpu - R_ref| over the upper triangle, relative to the largest entry of R."""
    iu = np.triu_indices_from(r_ref)
    return float(np.max(np.abs(r_gpu[iu] - r_ref[iu])) / np.max(np.abs(r_ref)))


@pytest.mark.parametrize("n,tokens,dead_cols", [(256, 1024, ()), (688, 2048, (5, 300)), (132, 400, ()), (1540, 4096, (0,)),
                                                (8, 32, ())])
def test_factor_vs_oracle(lib, n, tokens, dead_cols):
    """Damped Hessian and its factor R (R R^T = H', R = U^-1 with U the oracle's inverse factor)."""
    x = _acts(tokens, n, torch.bfloat16, seed=n)
    for c in dead_cols:
        x[:, c] = 0
    h = torch.zeros((n, n), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    _sync()
    h0 = to_np(h).astype(np.float64)                        # the factorisation is checked on the kernel's own Hessian
    dead = torch.full((n,), 7, dtype=torch.uint8, device=DEV)
    info = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    prune.hessian_factor(h, 0.01, dead=dead, info=info)
    _sync()
    want_h, want_dead = obs.damped_hessian(h0, 0.01)
    assert info.item() == 0 and np.array_equal(to_np(dead).astype(bool), want_dead)
    assert sorted(np.nonzero(want_dead)[0].tolist()) == sorted(dead_cols)
    r_gpu = np.triu(to_np(h).astype(np.float64))
    r_ref = obs.reverse_factor(want_h)
    # fp32 factorisation of a matrix with condition number about 40 here (the x20 outlier channel squared over the
    # damped bulk): errors of a few 2^-24 * condition * sqrt(n)
    assert _factor_err(r_gpu, r_ref) < 2e-5
    assert np.max(np.abs(r_gpu @ r_gpu.T - want_h)) / np.max(np.abs(want_h)) < 1e-5
    u_ref = obs.inverse_factor(want_h)
    assert np.max(np.abs(np.linalg.inv(r_gpu) - u_ref)) / np.max(np.abs(u_ref)) < 1e-4
    assert (np.diag(r_gpu) > 0).all()


def test_factor_reports_a_bad_pivot(lib):
    h = torch.eye(64, dtype=torch.float32, device=DEV)
    h[40, 40] = -3.0                                        # not positive definite (and the damping cannot fix it)
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    prune.hessian_factor(h, 0.01, info=info)
    _sync()
    assert info.item() == 41


# ----------------------------------------------------------------- compensated sweep

def _sweep_case(rows, cols, tokens, dtype, sparsity, seed, zero_frac=0.0, dead_cols=(), mix=0.1):
    """Run the sweep one 128-column block at a time and record the saliencies every block's selection was taken on.

    The selection is an integer decision taken on fp32 saliencies, so the oracle takes it on the very saliencies
    the kernel computed -- after checking that they are the oracle's own float64 saliencies at that moment, to
    rounding; everything else of the oracle runs in float64 on the factor the kernel was given.  The activation
    channels are correlated (mix), so that compensation between columns and blocks matters."""
    rng = np.random.default_rng(seed)
    x = _acts(tokens, cols, torch.float32, seed=seed)
    mixer = torch.tensor(np.eye(cols) + mix * rng.standard_normal((cols, cols)) / np.sqrt(cols) * 8, dtype=torch.float32,
                         device=DEV)
    x = (x @ mixer).to(torch.bfloat16)
    for c in dead_cols:
        x[:, c] = 0
    w = synth.random_matrix(rows, cols, dtype, seed=seed + 1, device=DEV, scale=0.05, zero_frac=zero_frac)
    h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    dead = torch.zeros(cols, dtype=torch.uint8, device=DEV)
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    prune.hessian_factor(h, 0.01, dead=dead, info=info)
    _sync()
    assert info.item() == 0 and sorted(np.nonzero(to_np(dead))[0].tolist()) == sorted(dead_cols)
    r64 = np.triu(to_np(h).astype(np.float64))
    g = torch.full((rows, cols), float("nan"), dtype=torch.float32, device=DEV)
    sal = torch.full((rows, cols), float("nan"), dtype=torch.float32, device=DEV)
    w_out = torch.full_like(w, 7.0)
    bits = torch.full((rows, (cols + 31) // 32), -1, dtype=torch.int32, device=DEV)
    n_blocks = (cols + 127) // 128
    w0 = to_np(w).astype(np.float64)
    w0[:, to_np(dead).astype(bool)] = 0.0
    ws = None
    for b in range(n_blocks):
        ws = prune.obs_sweep(w, h, sparsity, w_out=w_out, dead=dead, first_block=b, n_blocks=1, v=g, mask_bits=bits,
                             ws=ws, saliency=sal)
    _sync()
    seen = to_np(sal)
    assert np.isfinite(seen).all()
    calls = iter(range(n_blocks))
    worst = [0.0]

    def kernel_saliency(w_block, u_diag):
        b = next(calls)
        mine = obs.block_saliency(w_block, u_diag)                       # the oracle's own, float64, at this moment
        theirs = seen[:, 128 * b:128 * b + w_block.shape[1]].astype(np.float64)
        worst[0] = max(worst[0], float(np.max(np.abs(theirs - mine)) / np.max(mine)))
        return theirs

    want_w, want_pruned = obs.obs_sweep(w0, np.linalg.inv(r64), sparsity, block=128, saliency_fn=kernel_saliency)
    assert worst[0] < 2e-5, worst[0]                                     # fp32 saliencies against float64 ones
    got_w = to_np(w_out).astype(np.float64)
    assert np.array_equal(to_np(bits).view(np.uint32), orc.pack_keep_bits(want_pruned))      # the same entries go
    assert (got_w[want_pruned] == 0).all()
    quota = sum(obs.block_quota(sparsity, rows, min(128, cols - c)) for c in range(0, cols, 128))
    assert want_pruned.sum() == quota
    scale = np.max(np.abs(w0))
    err = np.max(np.abs(got_w - want_w)) / scale
    # fp32 sweep against float64 on the same masks; bf16 storage adds half an ulp (2^-9) of the largest weights
    assert err < (6e-3 if dtype == torch.bfloat16 else 2e-4), err
    # one call for all blocks, in place, gives the same bits as the block-by-block run
    w2 = w.clone()
    prune.obs_sweep(w2, h, sparsity, dead=dead)
    _sync()
    assert np.array_equal(to_np(w2).view(np.uint16 if dtype == torch.bfloat16 else np.uint32),
                          to_np(w_out).view(np.uint16 if dtype == torch.bfloat16 else np.uint32))
    return w0, got_w, want_w, r64


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("rows,cols,tokens,sparsity", [(64, 256, 1024, 0.5), (37, 200, 800, 0.3), (130, 388, 2000, 0.7),
                                                       (16, 128, 512, 0.0), (5, 8, 64, 0.5)])
def test_sweep_vs_oracle(lib, dtype, rows, cols, tokens, sparsity):
    _sweep_case(rows, cols, tokens, dtype, sparsity, seed=rows + cols)


def test_sweep_ties_dead_channels_and_compensation(lib):
    """Many exact zeros (equal saliencies, split by position), channels that never fire, and the point of it all:
    the compensated weights reproduce the layer output better than the same mask without compensation."""
    w0, got_w, _, _ = _sweep_case(48, 384, 1500, torch.float32, 0.5, seed=77, zero_frac=0.6, dead_cols=(9, 200))
    assert (got_w[:, [9, 200]] == 0).all()
    first = slice(0, 128)                                                  # in the first block the quota falls inside the zeros:
    assert (got_w[:, first][w0[:, first] != 0] != 0).all()                 # equal saliencies are split and no weight is lost
    w0, got_w, want_w, r64 = _sweep_case(48, 384, 1500, torch.float32, 0.5, seed=78, zero_frac=0.2, dead_cols=(17,))
    h = r64 @ r64.T
    plain = np.where(got_w == 0, 0.0, w0)
    assert obs.reconstruction_error(w0, got_w, h) < 0.97 * obs.reconstruction_error(w0, plain, h)   # (nearly independent channels: a few percent)
    assert obs.reconstruction_error(w0, got_w, h) <= 1.001 * obs.reconstruction_error(w0, want_w, h)
    # the same splitting of equal saliencies in bf16 storage, with more rows than one workgroup of the walk takes
    w0, got_w, _, _ = _sweep_case(70, 256, 1200, torch.bfloat16, 0.5, seed=79, zero_frac=0.6, dead_cols=(5,))
    assert (got_w[:, 5] == 0).all() and (got_w[:, :128][w0[:, :128] != 0] != 0).all()


def test_sweep_resumed_with_a_fresh_workspace_at_a_group_boundary(lib):
    """What must survive between the calls of a split sweep: the working matrix v always, and the workspace only
    while a group of four blocks is unfinished.  A caller that owns v and resumes at a multiple of four blocks may
    hand over a different (here: poisoned) workspace and must get the bits of the one-call sweep."""
    rows, cols, tokens, sparsity = 40, 1280, 2048, 0.5                    # ten blocks: groups 0-3, 4-7, 8-9
    x = _acts(tokens, cols, torch.bfloat16, seed=5)
    w = synth.random_matrix(rows, cols, torch.float32, seed=6, device=DEV, scale=0.05)
    h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    prune.hessian_factor(h, 0.01)
    whole = torch.empty_like(w)
    prune.obs_sweep(w, h, sparsity, w_out=whole)
    need = int(prune.load().prune_obs_sweep_workspace_bytes(rows, cols, 0))
    v = torch.full((rows, cols), float("nan"), dtype=torch.float32, device=DEV)
    split = torch.full_like(w, 7.0)
    for first, count in ((0, 4), (4, 4), (8, 2)):
        fresh = torch.full((need,), 0xA5, dtype=torch.uint8, device=DEV)
        prune.obs_sweep(w, h, sparsity, w_out=split, first_block=first, n_blocks=count, v=v, ws=fresh)
    _sync()
    assert np.array_equal(to_np(split).view(np.uint32), to_np(whole).view(np.uint32))


def _popcount32(a):
    a = a.astype(np.uint32)
    a = a - ((a >> 1) & 0x55555555)
    a = (a & 0x33333333) + ((a >> 2) & 0x33333333)
    a = (a + (a >> 4)) & 0x0F0F0F0F
    return (a * 0x01010101 >> 24) & 0xFF


def test_obs_fullsize_q_projection(lib):
    """The q projection of the LLaMA-7B-shaped layer (4096 x 4096, 262144 calibration tokens) through all three
    stages, in the shapes the benchmark times.  Sampled entries of R R^T against the damped Hessian; for sampled
    column blocks the selection against the oracle's on the kernel's fp32 saliencies and the new weights against a
    float64 replay of the block; the per-block quota over every block; and the reconstruction error of the whole
    projection against plain masking with the same mask."""
    cfg = synth.CONFIGS["llama7b_layer"]
    x = synth.make_activation(cfg, 0, "attn_in", DEV)
    w = synth.make_weight(cfg, 0, "q", DEV)
    rows, cols = w.shape
    h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    del x
    h_plain = to_np(h).astype(np.float64)
    dead = torch.zeros(cols, dtype=torch.uint8, device=DEV)
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    prune.hessian_factor(h, 0.01, dead=dead, info=info)
    _sync()
    assert info.item() == 0 and not to_np(dead).any()
    h_damped, _ = obs.damped_hessian(h_plain, 0.01)
    r64 = np.triu(to_np(h).astype(np.float64))
    rng = np.random.default_rng(5)
    ii, jj = rng.integers(0, cols, 400), rng.integers(0, cols, 400)
    rrt = np.einsum("nk,nk->n", r64[ii], r64[jj])
    scale = np.sqrt(np.diag(h_damped)[ii] * np.diag(h_damped)[jj])
    assert np.max(np.abs(rrt - h_damped[ii, jj]) / scale) < 1e-5
    sparsity = 0.53
    g = torch.zeros((rows, cols), dtype=torch.float32, device=DEV)
    sal = torch.zeros((rows, cols), dtype=torch.float32, device=DEV)
    w_out = torch.empty_like(w)
    bits = torch.zeros((rows, cols // 32), dtype=torch.int32, device=DEV)
    w0 = to_np(w).astype(np.float64)
    ws, watch, snaps = None, (0, 1, 17, 31), {}
    for b in range(cols // 128):
        if b in watch:
            snaps[b] = np.zeros((rows, 128), dtype=np.float32) if b == 0 else to_np(g[:, 128 * b:128 * b + 128]).copy()
        ws = prune.obs_sweep(w, h, sparsity, w_out=w_out, first_block=b, n_blocks=1, v=g, mask_bits=bits, ws=ws,
                             saliency=sal)
    _sync()
    got = to_np(w_out).astype(np.float64)
    keep = to_np(bits).view(np.uint32)
    quota = obs.block_quota(sparsity, rows, 128)
    per_block = _popcount32(keep).reshape(rows, cols // 128, 4).sum(axis=(0, 2))
    assert (per_block == rows * 128 - quota).all()                          # every block prunes exactly its quota
    pruned_all = ~np.unpackbits(keep.view(np.uint8), axis=1, bitorder="little").astype(bool)
    assert (got[pruned_all] == 0).all()
    for b in watch:
        c0 = 128 * b
        gb = snaps[b].astype(np.float64)                                    # the kernel's state when the block started
        rb = r64[c0:c0 + 128, c0:c0 + 128]
        # the published sweep's weights at that moment, W + G inv(R_bb), and their saliencies (w / U_jj)^2 = (w R_jj)^2
        current = w0[:, c0:c0 + 128] + gb @ np.linalg.inv(rb)
        sal64 = (current * np.diag(rb)[None, :]) ** 2
        sal32 = to_np(sal[:, c0:c0 + 128])
        assert np.max(np.abs(sal32 - sal64)) / np.max(sal64) < 5e-5, b
        want_mask = obs.select_block(sal32, quota)                          # the oracle's selection on the kernel's saliencies
        assert np.array_equal(pruned_all[:, c0:c0 + 128], want_mask), b
        # float64 replay of the block: V_j = w_j R_jj + G_j; kept w' = V_j / R_jj, D_j = w_j - w'_j spreads with R
        cur = w0[:, c0:c0 + 128] * np.diag(rb)[None, :] + gb
        want = np.zeros((rows, 128))
        for j in range(128):
            want[:, j] = np.where(want_mask[:, j], 0.0, cur[:, j] / rb[j, j])
            d = w0[:, c0 + j] - want[:, j]
            cur[:, j + 1:] += np.outer(d, rb[j, j + 1:])
        err = np.max(np.abs(got[:, c0:c0 + 128] - want)) / np.max(np.abs(w0))
        assert err < 6e-3, (b, err)                                         # half a bf16 ulp of the largest weights
    delta = w0 - got
    plain = np.where(pruned_all, w0, 0.0)                                    # what plain masking with this mask removes
    e_obs = float(np.einsum("ij,ij->", delta @ h_damped, delta))
    e_plain = float(np.einsum("ij,ij->", plain @ h_damped, plain))
    assert e_obs < e_plain


@pytest.mark.parametrize("fused", [False, True])
def test_pipeline_streams_give_the_same_bits(lib, fused):
    """The layer-level helpers spread factorisations and sweeps over several streams (fused: as one schedule in which
    sweeps run beside the Hessians still to come): the results must be those of plain one-after-the-other calls on
    the current stream, bit for bit, also when a step is repeated."""
    from paper_2504_06323_amd import pipeline
    cfg = synth.CONFIGS["toy"]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 0, n, DEV) for n, _, _, _ in shapes}
    acts = {a: synth.make_activation(cfg, 0, a, DEV) for a in act_shapes}
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, cfg.n_tokens)
    ob = pipeline.ObsState.create(st, act_shapes, cfg.n_tokens)
    targets = [0.3 + 0.05 * i for i in range(len(shapes))]
    for _ in range(2):
        if fused:
            pipeline.obs_layer(st, ob, acts, targets)
        else:
            pipeline.hessian_layer(ob, acts)
            pipeline.obs_prune_layer(st, ob, targets)
    _sync()
    assert ob.info.tolist() == [0] * len(acts)
    for i, (n, rows, cols, a) in enumerate(shapes):
        h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
        prune.hessian_accumulate(acts[a], h)
        dead = torch.zeros(cols, dtype=torch.uint8, device=DEV)
        prune.hessian_factor(h, 0.01, dead=dead)
        out = torch.empty_like(weights[n])
        bits = torch.zeros_like(st.mask_bits[n])
        prune.obs_sweep(weights[n], h, targets[i], w_out=out, dead=dead, mask_bits=bits)
        _sync()
        assert torch.equal(out, st.pruned[n]) and torch.equal(bits, st.mask_bits[n]), n
        quota = sum(obs.block_quota(targets[i], rows, min(128, cols - c)) for c in range(0, cols, 128))
        assert int((~np.unpackbits(to_np(bits).view(np.uint8), axis=1, bitorder="little").astype(bool))[:, :cols].sum()) == quota


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_whole_pruner_against_the_float64_oracle(lib, dtype):
    """All three stages on the GPU against obs_prune in float64 with its own decisions.  Near-equal saliencies may
    be taken in a different order, so a few individual weights may differ; what must agree is what the method is
    for: the same number of weights goes in every block and the layer output on the calibration data is reproduced
    equally well."""
    rows, cols, tokens, sparsity = 96, 512, 3000, 0.6
    rng = np.random.default_rng(3)
    mix = torch.tensor(np.eye(cols) + 0.15 * rng.standard_normal((cols, cols)), dtype=torch.float32, device=DEV)
    x = (synth.random_matrix(tokens, cols, torch.float32, seed=5, device=DEV) @ mix).to(torch.bfloat16)   # correlated channels
    w = synth.random_matrix(rows, cols, dtype, seed=6, device=DEV, scale=0.05)
    h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    dead = torch.zeros(cols, dtype=torch.uint8, device=DEV)
    prune.hessian_factor(h, 0.01, dead=dead)
    out = torch.empty_like(w)
    bits = torch.zeros((rows, cols // 32), dtype=torch.int32, device=DEV)
    prune.obs_sweep(w, h, sparsity, w_out=out, dead=dead, mask_bits=bits)
    _sync()
    x64, w64 = to_np(x).astype(np.float64), to_np(w).astype(np.float64)
    want_w, want_pruned = obs.obs_prune(x64, w64, sparsity)
    got_w = to_np(out).astype(np.float64)
    got_pruned = ~np.unpackbits(to_np(bits).view(np.uint8), axis=1, bitorder="little").astype(bool)
    assert np.array_equal(got_pruned.reshape(rows, -1, 128).sum(axis=(0, 2)), want_pruned.reshape(rows, -1, 128).sum(axis=(0, 2)))
    assert np.mean(got_pruned != want_pruned) < 2e-3                         # only near-ties may be decided differently
    hd, _ = obs.damped_hessian(obs.gram_matrix(x64))
    e_gpu, e_ref = obs.reconstruction_error(w64, got_w, hd), obs.reconstruction_error(w64, want_w, hd)
    e_plain = obs.reconstruction_error(w64, np.where(want_pruned, 0.0, w64), hd)
    assert e_ref < 0.8 * e_plain                                             # correlated channels: compensation matters here
    assert abs(e_gpu / e_ref - 1.0) < (2e-2 if dtype == torch.bfloat16 else 2e-3)


@pytest.mark.parametrize("channels", [5120, 13824, 14336])
def test_obs_other_model_widths(lib, channels):
    """Input widths of the other configurations (LLaMA-2-13B: 5120 / 13824, LLaMA-3-8B: 14336) through all three
    stages with fewer tokens and rows: tile counts and splits that the 7B layer does not reach.  Sampled entries
    of H and of R R^T against the oracle, exact quotas, and a better reconstruction than plain masking."""
    tokens, rows, sparsity = 16384, 256, 0.5
    x = _acts(tokens, channels, torch.bfloat16, seed=channels)
    w = synth.random_matrix(rows, channels, torch.bfloat16, seed=channels + 1, device=DEV, scale=0.02)
    h = torch.zeros((channels, channels), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    _sync()
    rng = np.random.default_rng(channels)
    idx = np.unique(np.concatenate([rng.choice(channels, size=48, replace=False), [0, 3, 255, 256, channels - 1]]))
    xs = to_np(x[:, torch.as_tensor(idx, device=DEV)]).astype(np.float64)
    want = xs.T @ xs
    got = to_np(h)[np.ix_(idx, idx)].astype(np.float64)
    d = np.sqrt(np.diag(want))
    assert np.max(np.abs(got - want) / np.outer(d, d)) < 5e-6
    assert bool(torch.equal(h, h.t()))
    diag = to_np(torch.diagonal(h)).astype(np.float64)
    damped = got + np.diag(np.full(len(idx), 0.01 * diag.mean()))
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    prune.hessian_factor(h, 0.01, info=info)
    _sync()
    assert info.item() == 0
    r_rows = to_np(torch.triu(h)[torch.as_tensor(idx, device=DEV)]).astype(np.float64)
    assert np.max(np.abs(r_rows @ r_rows.T - damped) / np.outer(d, d)) < 2e-5
    out = torch.empty_like(w)
    bits = torch.zeros((rows, channels // 32), dtype=torch.int32, device=DEV)
    prune.obs_sweep(w, h, sparsity, w_out=out, mask_bits=bits)
    _sync()
    keep = to_np(bits).view(np.uint32)
    per_block = _popcount32(keep).reshape(rows, channels // 128, 4).sum(axis=(0, 2))
    assert (per_block == rows * 128 - obs.block_quota(sparsity, rows, 128)).all()
    pruned = ~np.unpackbits(keep.view(np.uint8), axis=1, bitorder="little").astype(bool)
    got_w, w0 = to_np(out).astype(np.float64), to_np(w).astype(np.float64)
    assert (got_w[pruned] == 0).all()
    # reconstruction error through R: ||(W - W') X^T||^2 + damping = ||(W - W') R||_F^2
    r64 = to_np(torch.triu(h)).astype(np.float64)
    e_obs = np.sum(((w0 - got_w) @ r64) ** 2)
    e_plain = np.sum((np.where(pruned, w0, 0.0) @ r64) ** 2)
    assert e_obs < e_plain


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_sweep_in_place_with_pitch(lib, dtype):
    """Weights that are a view into a wider buffer, pruned in place: the same bits as the contiguous out-of-place
    call, and nothing outside the view is touched."""
    rows, cols, tokens, sparsity = 70, 264, 1200, 0.4
    x = _acts(tokens, cols, torch.bfloat16, seed=21)
    w = synth.random_matrix(rows, cols, dtype, seed=22, device=DEV, scale=0.05)
    h = torch.zeros((cols, cols), dtype=torch.float32, device=DEV)
    prune.hessian_accumulate(x, h)
    prune.hessian_factor(h, 0.01)
    want = torch.empty_like(w)
    prune.obs_sweep(w, h, sparsity, w_out=want)
    wide = torch.full((rows, cols + 24), 3.0, dtype=dtype, device=DEV)
    view = wide[:, 8:8 + cols]
    view.copy_(w)
    prune.obs_sweep(view, h, sparsity)                       # in place, pitch cols + 24
    _sync()
    assert torch.equal(view, want)
    assert bool((wide[:, :8] == 3.0).all()) and bool((wide[:, 8 + cols:] == 3.0).all())
