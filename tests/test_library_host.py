"""Host-side checks of the C-ABI library: it loads, exports what the header declares,
rejects bad arguments before any launch, and its planner agrees with the oracle's."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

from oracle import mosaic_oracle as orc
from paper_2504_06323_amd import prune

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mosaic_prune.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(prune_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_functions()
    assert {"prune_stats_accumulate", "prune_score", "prune_outlier_ratio", "prune_select_mask",
            "prune_struct_compact"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert sorted(prune.exported_symbols()) == names
    assert prune.version() >= 100
    assert prune.status_string(0) == "ok" and "workspace" in prune.status_string(-5)


def test_workspace_sizes(lib):
    assert prune.workspace_bytes(prune.OP_STATS, 262144, 4096) >= 4096 * 4
    assert prune.workspace_bytes(prune.OP_STATS, 262144, 4096) <= 64 << 20
    assert prune.workspace_bytes(prune.OP_SCORE, 4096, 4096) >= 8
    assert prune.workspace_bytes(prune.OP_OUTLIER, 4096, 4096) == 0
    assert prune.workspace_bytes(prune.OP_STRUCT, 14336, 4096) >= 14336 * 4
    assert prune.workspace_bytes(prune.OP_STATS, 0, 4096) == 0 and prune.workspace_bytes(99, 8, 8) == 0
    for op in range(5):
        assert prune.workspace_bytes(op, 1000, 1000) % 256 == 0


def test_error_paths_return_before_any_launch(lib):
    """Every rejected call returns its status without touching a device (runs without a GPU)."""
    fake = ctypes.c_void_p(0x1000)        # aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1001)
    E = dict(null=-1, shape=-2, dtype=-3, align=-4, ws=-5, rng=-6)
    sa = lib.prune_stats_accumulate
    assert sa(fake, 7, 8, 8, 8, fake, fake, 1 << 20, None) == E["dtype"]
    assert sa(fake, 1, 8, 0, 8, fake, fake, 1 << 20, None) == E["shape"]
    assert sa(fake, 1, 8, 16, 8, fake, fake, 1 << 20, None) == E["shape"]      # ld < channels
    assert sa(fake, 1, 8, 8, 8, None, fake, 1 << 20, None) == E["null"]
    assert sa(None, 1, 8, 8, 8, fake, fake, 1 << 20, None) == E["null"]
    assert sa(odd, 1, 8, 8, 8, fake, fake, 1 << 20, None) == E["align"]
    assert sa(fake, 1, 8, 8, 8, fake, fake, 4, None) == E["ws"]
    assert sa(None, 1, 0, 8, 8, fake, None, 0, None) == 0                       # zero tokens: valid no-op
    sn = lib.prune_stats_norms
    assert sn(fake, 1, 8, 8, 8, fake, None, fake, 1 << 20, None) == E["null"]
    assert sn(None, 1, 8, 8, 8, fake, fake, fake, 1 << 20, None) == E["null"]
    assert sn(fake, 1, 8, 8, 4, fake, fake, fake, 1 << 20, None) == E["shape"]
    assert sn(fake, 3, 8, 8, 8, fake, fake, fake, 1 << 20, None) == E["dtype"]
    assert sn(fake, 1, 8, 8, 8, fake, fake, fake, 4, None) == E["ws"]
    ss = lib.prune_stats_norms_static                                           # the variant with built-in scratch
    assert ss(fake, 3, 8, 8, 8, fake, fake, None) == E["dtype"]
    assert ss(fake, 1, 8, 8, 4, fake, fake, None) == E["shape"]
    assert ss(None, 1, 8, 8, 8, fake, fake, None) == E["null"]
    assert ss(fake, 1, 8, 8, 8, fake, None, None) == E["null"]
    assert ss(odd, 1, 8, 8, 8, fake, fake, None) == E["align"]
    assert ss(fake, 1, 8, 600000, 600000, fake, fake, None) == E["ws"]          # partial sums beyond the 2 MiB array
    assert prune.workspace_bytes(prune.OP_STATS, 1 << 20, 524288) <= 2 << 20 < prune.workspace_bytes(prune.OP_STATS, 8, 600000)
    assert lib.prune_stats_finalize(None, 8, fake, None) == E["null"]
    assert lib.prune_stats_finalize(fake, 0, fake, None) == E["shape"]
    sc = lib.prune_score
    assert sc(fake, 1, 8, 8, 8, fake, None, None, fake, 1 << 20, None) == E["null"]
    assert sc(fake, 1, 0, 8, 8, fake, None, fake, fake, 1 << 20, None) == E["shape"]
    assert sc(fake, 1, 8, 8, 8, fake, None, fake, fake, 0, None) == E["ws"]
    assert sc(fake, 5, 8, 8, 8, fake, None, fake, fake, 1 << 20, None) == E["dtype"]
    orr = lib.prune_outlier_ratio
    assert orr(fake, 1, 8, 8, 8, fake, None, -1.0, fake, fake, None, None) == E["rng"]
    assert orr(None, 1, 8, 8, 8, None, None, 5.0, fake, fake, None, None) == E["null"]
    assert orr(fake, 1, 8, 8, 8, fake, None, 5.0, fake, None, None, None) == E["null"]
    sb = lib.prune_score_outlier_batch
    good = prune.Projection(0x1000, 8, 8, 8, 0x1000)
    arr = (prune.Projection * 1)(good)
    assert sb(arr, 0, 1, 5.0, 0, fake, fake, None, fake, 1 << 20, None) == E["shape"]
    assert sb(None, 1, 1, 5.0, 0, fake, fake, None, fake, 1 << 20, None) == E["null"]
    assert sb(arr, 1, 1, -1.0, 0, fake, fake, None, fake, 1 << 20, None) == E["rng"]
    assert sb(arr, 1, 9, 5.0, 0, fake, fake, None, fake, 1 << 20, None) == E["dtype"]
    assert sb(arr, 1, 1, 5.0, 0, fake, fake, None, fake, 8, None) == E["ws"]
    assert sb(arr, 1, 1, 5.0, 7, fake, fake, None, fake, 1 << 20, None) == E["rng"]      # unknown outlier scope
    many = (prune.Projection * 17)(*([good] * 17))
    assert sb(many, 17, 1, 5.0, 1, fake, fake, None, fake, 1 << 20, None) == E["rng"]    # a layer has at most 16
    bad = (prune.Projection * 1)(prune.Projection(0x1000, 8, 8, 4, 0x1000))
    assert sb(bad, 1, 1, 5.0, 0, fake, fake, None, fake, 1 << 20, None) == E["shape"]
    bad = (prune.Projection * 1)(prune.Projection(0x1000, 8, 8, 8, None))
    assert sb(bad, 1, 1, 5.0, 0, fake, fake, None, fake, 1 << 20, None) == E["null"]
    sm = lib.prune_select_mask
    assert sm(fake, fake, 1, 8, 8, 8, 8, fake, None, 9, None, None, 0, None) == E["rng"]   # k > cols
    assert sm(fake, fake, 1, 8, 8, 4, 8, fake, None, 1, None, None, 0, None) == E["shape"]
    assert sm(fake, fake, 1, 8, 8, 8, 16, fake, None, 1, None, None, 0, None) == E["shape"]  # in place, other pitch
    assert sm(fake, None, 1, 8, 8, 8, 8, fake, None, 1, None, None, 0, None) == E["null"]
    assert sm(fake, fake, 1, 8, 8, 8, 8, None, None, 1, None, None, 0, None) == E["null"]
    assert sm(fake, ctypes.c_void_p(0x1010), 1, 8, 8, 8, 8, fake, None, 1, None, None, 0, None) == E["rng"]  # overlap
    smb = lib.prune_select_mask_batch
    item = lambda **kw: prune.SelectItem(**{**dict(w=0x1000, w_out=0x1000, rows=8, cols=8, ld_w=8, ld_out=8,
                                                   norms=0x1000, k=1, mask_bits=None), **kw})
    one = lambda **kw: (prune.SelectItem * 1)(item(**kw))
    assert smb(one(), 0, 1, None, 0, None) == E["shape"]
    assert smb(None, 1, 1, None, 0, None) == E["null"]
    assert smb(one(), 1, 4, None, 0, None) == E["dtype"]
    assert smb(one(k=9), 1, 1, None, 0, None) == E["rng"]
    assert smb(one(norms=None), 1, 1, None, 0, None) == E["null"]
    assert smb(one(ld_w=4), 1, 1, None, 0, None) == E["shape"]
    assert smb(one(w_out=0x1010), 1, 1, None, 0, None) == E["rng"]
    assert smb(one(k_dev=0x1002), 1, 1, None, 0, None) == E["align"]     # k in device memory: a 4-byte pointer
    two = (prune.SelectItem * 2)(item(), item(w_out=None))          # a bad second item rejects the whole batch
    assert smb(two, 2, 1, None, 0, None) == E["null"]
    pd = lib.prune_plan_sparsity_device
    assert pd(None, fake, fake, 1, 7, 0.5, 0.08, 0, fake, fake, fake, None) == E["null"]
    assert pd(fake, fake, None, 1, 7, 0.5, 0.08, 0, fake, fake, fake, None) == E["null"]      # cols are required here
    assert pd(fake, fake, fake, 1, 7, 0.5, 0.08, 0, fake, fake, None, None) == E["null"]
    assert pd(fake, fake, fake, 0, 7, 0.5, 0.08, 0, fake, fake, fake, None) == E["shape"]
    assert pd(fake, fake, fake, 1 << 12, 1 << 12, 0.5, 0.08, 0, fake, fake, fake, None) == E["shape"]
    assert pd(fake, fake, fake, 1, 7, 1.0, 0.08, 0, fake, fake, fake, None) == E["rng"]
    assert pd(fake, fake, fake, 1, 7, 0.5, -1.0, 0, fake, fake, fake, None) == E["rng"]
    assert pd(fake, fake, fake, 1, 7, 0.5, 0.08, 9, fake, fake, fake, None) == E["rng"]
    assert pd(ctypes.c_void_p(0x1004), fake, fake, 1, 7, 0.5, 0.08, 0, fake, fake, fake, None) == E["align"]
    assert pd(fake, fake, fake, 1, 7, 0.5, 0.08, 0, fake, odd, fake, None) == E["align"]
    ha = lib.prune_hessian_accumulate
    assert ha(fake, 9, 8, 8, 8, fake, 8, fake, 1 << 30, None) == E["dtype"]
    assert ha(fake, 1, 8, 0, 8, fake, 8, fake, 1 << 30, None) == E["shape"]
    assert ha(fake, 1, 8, 16, 8, fake, 16, fake, 1 << 30, None) == E["shape"]     # ld_x < channels
    assert ha(fake, 1, 8, 16, 16, fake, 8, fake, 1 << 30, None) == E["shape"]     # ld_h < channels
    assert ha(fake, 1, 8, 8, 8, None, 8, fake, 1 << 30, None) == E["null"]
    assert ha(None, 1, 8, 8, 8, fake, 8, fake, 1 << 30, None) == E["null"]
    assert ha(odd, 1, 8, 8, 8, fake, 8, fake, 1 << 30, None) == E["align"]
    assert ha(fake, 1, 8, 8, 8, fake, 8, fake, 16, None) == E["ws"]               # bf16, aligned: the tiled path needs room
    assert ha(fake, 1, 8, 8, 8, fake, 8, None, 0, None) == E["null"]
    assert ha(None, 1, 0, 8, 8, fake, 8, None, 0, None) == 0                      # zero tokens: valid no-op
    assert lib.prune_hessian_workspace_bytes(262144, 4096) >= 136 * 256 * 256 * 4
    assert lib.prune_hessian_workspace_bytes(0, 4096) == 0
    hf = lib.prune_hessian_factor
    assert hf(fake, 0, 8, 0.01, None, None, fake, 1 << 20, None) == E["shape"]
    assert hf(fake, 8, 4, 0.01, None, None, fake, 1 << 20, None) == E["shape"]       # ld_h < n
    assert hf(fake, 6, 8, 0.01, None, None, fake, 1 << 20, None) == E["shape"]       # n must be a multiple of 4
    assert hf(None, 8, 8, 0.01, None, None, fake, 1 << 20, None) == E["null"]
    assert hf(fake, 8, 8, 0.01, None, None, None, 0, None) == E["null"]
    assert hf(fake, 8, 8, -1.0, None, None, fake, 1 << 20, None) == E["rng"]
    assert hf(ctypes.c_void_p(0x1004), 8, 8, 0.01, None, None, fake, 1 << 20, None) == E["align"]
    assert hf(fake, 8, 8, 0.01, None, None, fake, 16, None) == E["ws"]
    assert lib.prune_hessian_factor_workspace_bytes(4096) >= 128 * 128 * 4
    sw = lib.prune_obs_sweep
    big = ctypes.c_void_p(0x10000)
    ok = lambda **kw: sw(*[{**dict(w=big, o=big, dt=1, rows=8, cols=8, ldw=8, ldo=8, r=big, ldr=8, dead=None, s=0.5, fb=0,
                                  nb=-1, v=None, sal=None, mb=None, ws=big, wsb=1 << 30, st=None), **kw}[k]
                           for k in ("w", "o", "dt", "rows", "cols", "ldw", "ldo", "r", "ldr", "dead", "s", "fb", "nb", "v",
                                     "sal", "mb", "ws", "wsb", "st")])
    assert ok(dt=5) == E["dtype"]
    assert ok(rows=0) == E["shape"]
    assert ok(cols=6, ldw=6, ldo=6) == E["shape"]                                  # cols must be a multiple of 4
    assert ok(ldr=4) == E["shape"]
    assert ok(r=None) == E["null"]
    assert ok(ws=None) == E["null"]
    assert ok(s=1.0) == E["rng"]
    assert ok(fb=2) == E["rng"]                                                    # only one block of columns
    assert ok(fb=1) == 0                                                           # an empty range of blocks: nothing to do
    assert ok(nb=2) == E["rng"]
    assert ok(r=ctypes.c_void_p(0x10004)) == E["align"]
    assert ok(wsb=64) == E["ws"]
    assert lib.prune_obs_sweep_workspace_bytes(4096, 4096, 1) >= 4096 * 4096 * 4 + 4096 * 128 * 4
    assert lib.prune_obs_sweep_workspace_bytes(4096, 4096, 0) < 4096 * 4096 * 4
    ln = lib.prune_linear
    assert ln(fake, fake, fake, 9, 8, 8, 8, 8, 8, 8, None) == E["dtype"]
    assert ln(fake, fake, fake, 1, 0, 8, 8, 8, 8, 8, None) == E["shape"]
    assert ln(fake, fake, fake, 1, 8, 8, 8, 4, 8, 8, None) == E["shape"]              # ld_x < k
    assert ln(fake, fake, fake, 1, 8, 16, 8, 8, 8, 8, None) == E["shape"]             # ld_y < n
    assert ln(None, fake, fake, 1, 8, 8, 8, 8, 8, 8, None) == E["null"]
    assert ln(odd, fake, fake, 1, 8, 8, 8, 8, 8, 8, None) == E["align"]
    gu = lib.prune_mlp_gate_up
    assert gu(fake, fake, None, fake, 1, 8, 8, 8, 8, 8, 8, None, None, 0, None) == E["null"]
    assert gu(fake, fake, fake, fake, 1, 8, 8, 8, 8, 8, 4, None, None, 0, None) == E["shape"]   # ld_h < inter
    assert gu(fake, fake, fake, fake, 1, 256, 32, 128, 32, 32, 128, fake, None, 0, None) == E["null"]   # statistic wanted, no workspace
    assert gu(fake, fake, fake, fake, 1, 256, 32, 128, 32, 32, 128, fake, fake, 16, None) == E["ws"]
    assert lib.prune_mlp_workspace_bytes(16384, 11008) >= 2 * 64 * 11008 * 4
    F = ctypes.c_float
    rn = lib.prune_rmsnorm
    assert rn(fake, fake, fake, 5, 8, 8, 8, 8, F(1e-5), None) == E["dtype"]
    assert rn(fake, fake, fake, 1, 8, 8, 4, 8, F(1e-5), None) == E["shape"]
    assert rn(fake, None, fake, 1, 8, 8, 8, 8, F(1e-5), None) == E["null"]
    assert rn(fake, fake, fake, 1, 8, 8, 8, 8, F(-1.0), None) == E["rng"]
    ro = lib.prune_rotary
    assert ro(fake, 1, 8, 2, 7, 14, 8, F(10000.0), None) == E["shape"]                 # odd head width
    assert ro(fake, 1, 8, 2, 8, 8, 8, F(10000.0), None) == E["shape"]                  # pitch < heads * head_dim
    assert ro(None, 1, 8, 2, 8, 16, 8, F(10000.0), None) == E["null"]
    assert ro(fake, 1, 8, 2, 8, 16, 8, F(1.0), None) == E["rng"]
    at = lib.prune_causal_attention
    assert at(fake, fake, fake, fake, 1, 1, 8, 3, 2, 8, 24, 16, 16, 24, None) == E["shape"]   # heads not a multiple of kv heads
    assert at(fake, fake, fake, fake, 1, 1, 8, 2, 1, 512, 1024, 512, 512, 1024, None) == E["shape"]   # head too wide
    assert at(fake, fake, None, fake, 1, 1, 8, 2, 1, 8, 16, 8, 8, 16, None) == E["null"]
    assert at(odd, fake, fake, fake, 1, 1, 8, 2, 1, 8, 16, 8, 8, 16, None) == E["align"]
    ad = lib.prune_add
    assert ad(fake, fake, fake, 1, 8, 8, 8, 4, 8, None) == E["shape"]
    assert ad(fake, None, fake, 1, 8, 8, 8, 8, 8, None) == E["null"]
    st = lib.prune_struct_compact
    assert st(fake, fake, fake, 1, 8, 8, 8, None, None, fake, fake, None, None, None, fake, 1 << 20, None) == E["rng"]  # r >= inter
    assert st(fake, fake, fake, 1, 8, 8, 1, None, None, fake, fake, fake, None, None, fake, 1 << 20, None) == E["null"]  # 1 of 3 outs
    assert st(fake, fake, fake, 1, 8, 8, 1, None, None, fake, fake, None, None, None, fake, 0, None) == E["ws"]
    assert st(fake, fake, None, 1, 8, 8, 1, None, None, fake, fake, None, None, None, fake, 1 << 20, None) == E["null"]
    assert st(fake, fake, fake, 1, 8, 8, 1, fake, None, fake, fake, None, None, None, fake, 1 << 20, None) == E["null"]  # one row-sum vector of two
    assert st(fake, fake, fake, 1, 8, 8, 1, odd, fake, fake, fake, None, None, None, fake, 1 << 20, None) == E["align"]
    sg = lib.prune_struct_groups
    P = lambda *v: (ctypes.c_void_p * len(v))(*v)
    I = lambda *v: (ctypes.c_int64 * len(v))(*v)
    ok = dict(rm=P(0x1000), rp=I(2), rw=I(8), nr=1, cm=P(0x1000), cp=I(2), ch=I(8), nc=1)
    call = lambda dt=1, ng=4, r=1, gm=fake, kp=fake, ro=None, co=None, w=fake, wb=1 << 20, **kw: sg(
        *[{**ok, **kw}[k] for k in ("rm", "rp", "rw", "nr", "cm", "cp", "ch", "nc")], dt, ng, r, gm, kp, ro, co, w, wb,
        None)
    assert call(dt=6) == E["dtype"]
    assert call(ng=0) == E["shape"]
    assert call(nr=9) == E["shape"]
    assert call(nr=0, nc=0) == E["shape"]
    assert call(r=4) == E["rng"]
    assert call(gm=None) == E["null"]
    assert call(rm=P(None)) == E["null"]
    assert call(rp=I(0)) == E["shape"]
    assert call(ro=P(0x2000)) == E["null"]                                        # row outputs without column outputs
    assert call(wb=16) == E["ws"]
    assert lib.prune_struct_groups_workspace_bytes(I(2), I(8), 1, I(2), I(8), 1, 4) >= (8 + 8) * 4
    assert lib.prune_struct_groups_workspace_bytes(I(0), I(8), 1, None, None, 0, 4) == 0
    with pytest.raises(prune.PruneError):
        prune.plan_sparsity([1], [10], 1, 1, 1.0, 0.08)                         # p must be < 1
    with pytest.raises(prune.PruneError):
        prune.plan_sparsity([11], [10], 1, 1, 0.5, 0.08)                        # count > numel


def test_planner_matches_hand_example(lib):
    ex = json.load(open(os.path.join(ROOT, "tests", "golden", "hand_examples.json")))["planner"]
    numels = [1000] * 4
    counts = [int(round(r * 10)) for row in ex["R"] for r in row]              # R = count / numel * 100
    s, k, clamped = prune.plan_sparsity(counts, numels, 2, 2, ex["p"], ex["lam"], cols=[100] * 4)
    np.testing.assert_allclose(np.array(s).reshape(2, 2), ex["s"], rtol=1e-14)
    assert k == [60, 40, 50, 50] and not clamped


def test_layer_planner_matches_hand_example(lib):
    ex = json.load(open(os.path.join(ROOT, "tests", "golden", "hand_examples.json")))["layer_planner"]
    counts = [c for row in ex["counts"] for c in row]
    numels = [e for row in ex["numels"] for e in row]
    s, k, clamped = prune.plan_sparsity(counts, numels, 3, 2, ex["p"], ex["lam"], prune.SCOPE_LAYER, cols=[100] * 6)
    np.testing.assert_allclose(np.array(s).reshape(3, 2), np.repeat(np.array(ex["s_layer"])[:, None], 2, axis=1),
                               rtol=1e-14)
    assert k == [60, 60, 40, 40, 50, 50] and not clamped


@pytest.mark.parametrize("p", [0.3, 0.5, 0.7])
def test_layer_planner_matches_oracle(lib, p):
    rng = np.random.default_rng(22)
    n_layers, n_proj = 32, 7
    numels = rng.integers(1 << 20, 1 << 26, size=(n_layers, n_proj))
    counts = (numels * rng.uniform(0, 0.05, size=numels.shape)).astype(np.int64)
    cols = rng.choice([4096, 11008, 14336], size=numels.shape)
    s, k, clamped = prune.plan_sparsity(counts.reshape(-1).tolist(), numels.reshape(-1).tolist(), n_layers, n_proj, p,
                                        0.08, prune.SCOPE_LAYER, cols=cols.reshape(-1).tolist())
    want, want_clamped = orc.plan_sparsity_layerwise(counts, numels, p, 0.08, cols=cols)
    np.testing.assert_allclose(np.array(s).reshape(n_layers, n_proj), want, rtol=0, atol=1e-13)
    assert clamped == want_clamped
    assert k == [orc.zeros_per_row(v, c) for v, c in zip(np.array(s), cols.reshape(-1))]
    # the three pruning methods side by side (Section 4.1.3): one target, one per layer, one per projection
    uniform, _, _ = prune.plan_sparsity(counts.reshape(-1).tolist(), numels.reshape(-1).tolist(), n_layers, n_proj, p,
                                        0.0, prune.SCOPE_GLOBAL)
    per_proj, _, _ = prune.plan_sparsity(counts.reshape(-1).tolist(), numels.reshape(-1).tolist(), n_layers, n_proj, p,
                                         0.08, prune.SCOPE_GLOBAL)
    assert uniform == [p] * (n_layers * n_proj)
    assert len(set(np.array(s).round(15))) == n_layers and len(set(per_proj)) == n_layers * n_proj
    for plan in (uniform, s, per_proj):
        assert np.mean(plan) == pytest.approx(p, abs=1e-12)


@pytest.mark.parametrize("scope", [prune.SCOPE_GLOBAL, prune.SCOPE_CATEGORY])
@pytest.mark.parametrize("p", [0.3, 0.5, 0.7])
def test_planner_matches_oracle(lib, scope, p):
    rng = np.random.default_rng(21)
    n_layers, n_proj = 32, 7
    numels = rng.integers(1 << 20, 1 << 26, size=n_layers * n_proj)
    counts = (numels * rng.uniform(0, 0.05, size=numels.shape)).astype(np.int64)
    cols = rng.choice([4096, 11008, 14336], size=numels.shape)
    s, k, clamped = prune.plan_sparsity(counts.tolist(), numels.tolist(), n_layers, n_proj, p, 0.08, scope,
                                        cols=cols.tolist())
    ratios = (100.0 * counts / numels).reshape(n_layers, n_proj)
    want, want_clamped = orc.plan_sparsity(ratios, p, 0.08, "global" if scope == prune.SCOPE_GLOBAL else "category",
                                           cols=cols.reshape(n_layers, n_proj))
    np.testing.assert_allclose(np.array(s).reshape(n_layers, n_proj), want, rtol=0, atol=1e-13)
    assert clamped == want_clamped
    assert np.mean(s) == pytest.approx(p, abs=1e-12)
    want_k = [orc.zeros_per_row(v, c) for v, c in zip(np.array(s), cols)]
    assert k == want_k


def test_planner_uniform_when_ranks_equal(lib):
    s, k, _ = prune.plan_sparsity([5] * 14, [100] * 14, 2, 7, 0.5, 0.08, cols=[256] * 14)
    assert s == [0.5] * 14 and k == [128] * 14
