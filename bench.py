"""Benchmark of the projection-pruning hot path on one MI355X.

Default workload: the layers of the full 32-layer LLaMA-3-8B-shaped model (grouped-query k / v of 1024 x 4096,
14336-wide feed-forward block, 128 x 2048 calibration tokens per layer).  A step is one pass of the whole path
over one layer: activation statistics of its four distinct projection inputs, metric sums and outlier counts of
its seven projections (the ranking, done once), then for every target of the sweep (30 / 50 / 70 %) the planner
over the whole model's table of counts, per-row selection and masking of the seven projections, and structured
ranking and compaction of the feed-forward block on the masked weights.  Successive steps take successive
layers out of a ring of distinct layers resident in HBM (inputs are generated before the timed region).
One JSON line goes to stdout; everything else to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import mmap
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def storage_name(cfg):
    return "bf16" if str(cfg.dtype).endswith("bfloat16") else "f32"


def algorithmic_bytes(cfg, shapes, act_shapes, r, n_targets):
    """Bytes the method itself must move per step (what the roofline is priced on)."""
    es = 2 if str(cfg.dtype).endswith("bfloat16") else 4
    numel = sum(rw * c for _, rw, c, _ in shapes)
    stats = sum(cfg.n_tokens * ch * es + ch * 4 for ch in act_shapes.values())
    score = numel * es
    count = numel * es
    select = numel * (2 * es) + numel // 8
    mlp = 3 * cfg.inter * cfg.hidden
    struct_rank = mlp * es if r > 0 else 0
    kept_frac = (cfg.inter - r) / cfg.inter
    compact = mlp * es + int(mlp * es * kept_frac) if r > 0 else 0
    return dict(stats=stats, score=score, count=count, select=select, struct_rank=struct_rank, compact=compact,
                total=stats + score + count + n_targets * (select + struct_rank + compact))


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", f"stats_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":", 1)[1]))
    except OSError:
        pass
    return None


def mean_sigma(xs):
    m = sum(xs) / len(xs)
    return m, math.sqrt(sum((x - m) ** 2 for x in xs) / max(1, len(xs) - 1))


# ---------------------------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands on a sample of the same layer, once on one core and once with the same
# calls dealt to all host cores (a plain parallel loop over channel slices, projections and row blocks).  The
# worker processes are forked before the GPU is touched and sit idle until the GPU part is over; the sample is
# handed to them through shared memory.

_CPU = {}


def _shared_array(shape, dtype="float32"):
    import numpy as np
    count = 1
    for d in shape:
        count *= int(d)
    buf = mmap.mmap(-1, max(16, count * np.dtype(dtype).itemsize))      # anonymous and shared: survives fork
    return np.frombuffer(buf, dtype=dtype, count=count).reshape(shape)


def cpu_prepare(cfg, shapes, act_shapes, den, workers):
    """Allocate the shared sample buffers and fork the worker pool (call before the GPU is initialised)."""
    import multiprocessing as mp
    n_seqs = max(1, cfg.n_seqs // den)
    t_rows = n_seqs * cfg.seq_len
    _CPU.update(cfg=cfg, shapes=shapes, den=den, n_seqs=n_seqs,
                x={a: _shared_array((t_rows, ch)) for a, ch in act_shapes.items()},
                norms={a: _shared_array((ch,), "float64") for a, ch in act_shapes.items()},
                w={n: _shared_array((len(range(0, rw, den)), c)) for n, rw, c, _ in shapes},
                masked={n: _shared_array((len(range(0, rw, den)), c)) for n, rw, c, _ in shapes},
                down_cols=_shared_array((cfg.hidden, len(range(0, cfg.inter, den)))))
    pool = mp.get_context("fork").Pool(workers) if workers > 1 else None
    _CPU.update(pool=pool, workers=workers)


def _cpu_task(task):
    from oracle import mosaic_oracle as orc
    kind = task[0]
    if kind == "norms":
        _, a, c0, c1 = task
        _CPU["norms"][a][c0:c1] = orc.column_norms(_CPU["x"][a][:, c0:c1])
        return None
    if kind == "rank":
        _, n, a, alpha = task
        omega = orc.weight_metric(_CPU["w"][n], _CPU["norms"][a])
        return orc.outlier_stats(omega, alpha)[2]
    if kind == "prune":
        _, n, a, r0, r1, k = task
        w = _CPU["w"][n][r0:r1]
        _CPU["masked"][n][r0:r1] = orc.prune_projection(w, orc.weight_metric(w, _CPU["norms"][a]), k)[0]
        return None
    raise ValueError(kind)


def _cpu_leg(run_map, slices):
    """The whole path on the sample through run_map (the builtin map, or a pool's)."""
    import numpy as np
    from oracle import mosaic_oracle as orc
    cfg, shapes = _CPU["cfg"], _CPU["shapes"]
    t0 = time.perf_counter()
    tasks = []
    for a, x in _CPU["x"].items():
        step = max(1, -(-x.shape[1] // slices))
        tasks += [("norms", a, c0, min(c0 + step, x.shape[1])) for c0 in range(0, x.shape[1], step)]
    list(run_map(_cpu_task, tasks))
    ratios = list(run_map(_cpu_task, [("rank", n, a, cfg.alpha) for n, _, _, a in shapes]))
    s, _ = orc.plan_sparsity(np.array(ratios).reshape(1, -1), cfg.p, cfg.lam, "global")
    tasks = []
    for i, (n, _, c, a) in enumerate(shapes):
        rows = _CPU["w"][n].shape[0]
        step = max(1, -(-rows // slices))
        tasks += [("prune", n, a, r0, min(r0 + step, rows), orc.zeros_per_row(s[0, i], c)) for r0 in range(0, rows, step)]
    list(run_map(_cpu_task, tasks))
    # structured part on the sample: every den-th feed-forward channel forms the sampled block
    gate, up, down = _CPU["masked"]["gate"], _CPU["masked"]["up"], _CPU["down_cols"]
    g = orc.group_magnitude(gate, up, down)
    kept = orc.struct_rank(g, int(cfg.struct_frac * g.shape[0]))
    orc.struct_compact(gate, up, down, kept)
    return time.perf_counter() - t0


def cpu_baseline(weights, acts):
    """Fill the shared sample from the tensors the GPU path ran on, then time the two legs."""
    import torch
    cfg, den = _CPU["cfg"], _CPU["den"]
    for a, x in acts.items():
        dst = _CPU["x"][a]
        for r0 in range(0, dst.shape[0], 8192):          # piecewise: no second full-size float32 copy on the device
            dst[r0:r0 + 8192] = x[r0:min(r0 + 8192, dst.shape[0])].to(torch.float32).cpu().numpy()
    for n, w in weights.items():
        _CPU["w"][n][:] = w[::den].to(torch.float32).cpu().numpy()
    _CPU["down_cols"][:] = weights["down"][:, ::den].to(torch.float32).cpu().numpy()
    sampled = sum(w.size for w in _CPU["w"].values())
    workers, pool = _CPU["workers"], _CPU["pool"]
    t_one = _cpu_leg(map, 1)
    t_all = _cpu_leg(pool.map, 2 * workers) if pool is not None else t_one
    if pool is not None:
        pool.close()
        pool.join()
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": sampled / t_all, "unit": "weights/s", "cores": workers, "kind": "oracle",
            "sample": f"1/{den} of one layer of the workload: {_CPU['n_seqs']} of {cfg.n_seqs} calibration sequences "
                      f"for the activation statistics, every {den}th output row of each projection ({sampled} "
                      f"weights), one target sparsity; NumPy float64; {t_all:.1f} s on {workers} worker processes "
                      f"(the same oracle calls dealt out over channel slices, projections and row blocks), "
                      f"{t_one:.1f} s on one core",
            "single_core": {"value": sampled / t_one, "unit": "weights/s", "cores": 1, "seconds": round(t_one, 2)},
            "seconds": round(t_all, 2), "nproc": os.cpu_count(), "affinity": len(os.sched_getaffinity(0)),
            "cpu_model": model}


def run_hessian_stage(args):
    """--stage hessian: the matrix-core stage of the Hessian-based pruner on the workload's activation tensors.

    A step is H += X^T X for each of the layer's four distinct projection inputs.  Prints its own JSON line."""
    import numpy as np
    import torch
    from paper_2504_06323_amd import prune, synth

    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    act_shapes = synth.activation_shapes(cfg)
    acts = {a: synth.make_activation(cfg, 0, a, dev) for a in act_shapes}
    hs = {a: torch.zeros((c, c), dtype=torch.float32, device=dev) for a, c in act_shapes.items()}
    need = max(prune.hessian_workspace_bytes(x.shape[0], x.shape[1]) for x in acts.values())
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    flops = {a: x.shape[0] * x.shape[1] * (x.shape[1] + 1) for a, x in acts.items()}   # the upper triangle, 2 per MAC
    big = max(act_shapes, key=lambda a: act_shapes[a])
    ev = lambda: torch.cuda.Event(enable_timing=True)
    events = []

    def step(record):
        for a, x in acts.items():
            if record and a == big:
                e0, e1 = ev(), ev()
                e0.record()
            prune.hessian_accumulate(x, hs[a], ws=ws)
            if record and a == big:
                e1.record()
                events.append((e0, e1))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = 1e3 * elapsed / args.steps
    launch_ms = sum(a.elapsed_time(b) for a, b in events) / len(events)
    achieved = flops[big] / (launch_ms * 1e-3) / 1e12
    out = {"metric": "Hessian accumulation H += X^T X for the four projection inputs of a layer (algorithmic TFLOP/s)",
           "value": sum(flops.values()) / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: activation tensors {[list(x.shape) for x in acts.values()]}, bf16, "
                                  f"fp32 accumulation, symmetric: T * C * (C + 1) flops per tensor"},
           "roofline": {"bound": "mfma", "kernel": f"gram_tiles_bf16 + gram_reduce on [{acts[big].shape[0]}, {acts[big].shape[1]}]",
                        "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": round(achieved / 2500.0, 4), "traffic": None,
                        "avg_launch_ms": round(launch_ms, 4), "launches": len(events)}}
    if not args.no_cpu_baseline:
        from oracle import obs_oracle as obs
        sample = acts[big][:2048].detach().cpu().to(torch.float32).numpy()
        t0 = time.perf_counter()
        obs.gram_matrix(sample)
        dt = time.perf_counter() - t0
        c = sample.shape[1]
        out["cpu_baseline"] = {"value": sample.shape[0] * c * (c + 1) / dt / 1e12, "unit": "TFLOP/s",
                               "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
                               "sample": f"2048 tokens of the [{acts[big].shape[0]}, {c}] tensor, NumPy float64 matmul, {dt:.1f} s"}
    log(f"hessian stage: {ms:.3f} ms per layer; {big} {launch_ms:.3f} ms = {achieved:.0f} TFLOP/s algorithmic")
    print(json.dumps(out), flush=True)


def run_obs_stage(args):
    """--stage obs: the whole Hessian-based path on the workload's layer, with the planner's targets.

    A step is: activation statistics, metric sums and outlier counts, planner (host), then one Hessian and one
    factor per distinct projection input and one compensated sweep per projection.  Prints its own JSON line."""
    import torch
    from paper_2504_06323_amd import pipeline, prune, synth

    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 0, n, dev) for n, _, _, _ in shapes}
    acts = {a: synth.make_activation(cfg, 0, a, dev) for a in act_shapes}
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, cfg.n_tokens)
    ob = pipeline.ObsState.create(st, act_shapes, cfg.n_tokens)
    numels = [rw * c for _, rw, c, _ in shapes]
    cols = [c for _, _, c, _ in shapes]
    big = max(act_shapes, key=lambda a: act_shapes[a])
    flops_big = acts[big].shape[0] * acts[big].shape[1] * (acts[big].shape[1] + 1)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks_all, gram_events = [], []

    def step(record):
        m = [ev() for _ in range(4)] if record else None
        if record:
            m[0].record()
        pipeline.rank_layer(st, acts, cfg.alpha)
        s, _, _ = pipeline.plan(st.count.tolist(), numels, cols, 1, len(shapes), cfg.p, cfg.lam)
        if record:
            m[1].record()
        if args.obs_two_phases:
            pipeline.hessian_layer(ob, acts, on_big=(lambda e: gram_events.append(e)) if record else None, big=big)
            if record:
                m[2].record()
            pipeline.obs_prune_layer(st, ob, s)
        else:
            if record:
                m[2].record()
            pipeline.obs_layer(st, ob, acts, s, on_big=(lambda e: gram_events.append(e)) if record else None, big=big)
        if record:
            m[3].record()
            marks_all.append(m)
        return s

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        s = step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if ob.info.tolist() != [0] * len(acts):
        raise RuntimeError(f"a Hessian factorisation met a pivot that was not positive: {ob.info.tolist()}")
    ms = 1e3 * elapsed / args.steps
    seg = [sum(m[i].elapsed_time(m[i + 1]) for m in marks_all) / len(marks_all) for i in range(3)]
    launch_ms = sum(a.elapsed_time(b) for a, b in gram_events) / len(gram_events)
    achieved = flops_big / (launch_ms * 1e-3) / 1e12
    numel = synth.layer_numel(cfg)
    zeros = sum(int((st.pruned[n] == 0).sum().item()) for n in st.names)
    out = {"metric": "projection weights pruned/s through the Hessian-based pruner with per-projection targets, 1 GPU",
           "value": numel / (ms * 1e-3), "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: one layer, {numel} weights in bf16, {cfg.n_tokens} calibration tokens, "
                                  f"target sparsity {cfg.p}, planner targets {[round(v, 4) for v in s]}, "
                                  f"achieved sparsity {zeros / numel:.4f}"},
           "ms_rank_and_plan": round(seg[0], 3),
           **({"ms_hessians_and_factors": round(seg[1], 3), "ms_sweeps": round(seg[2], 3)} if args.obs_two_phases
              else {"ms_hessians_factors_and_sweeps_as_one_schedule": round(seg[2], 3)}),
           "roofline": {"bound": "mfma", "kernel": f"gram_tiles_bf16 + gram_reduce on [{acts[big].shape[0]}, {acts[big].shape[1]}]",
                        "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": round(achieved / 2500.0, 4), "traffic": None, "avg_launch_ms": round(launch_ms, 4),
                        "launches": len(gram_events)}}
    if not args.no_cpu_baseline:
        from oracle import obs_oracle as obs
        name, a = st.names[0], st.proj_inputs[st.names[0]]
        xs = acts[a][:8192].detach().cpu().to(torch.float32).numpy()
        wsamp = weights[name][:256].detach().cpu().to(torch.float32).numpy()
        t0 = time.perf_counter()
        obs.obs_prune(xs, wsamp, float(s[0]))
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": wsamp.size / dt, "unit": "weights/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle",
                               "sample": f"projection {name}: 256 of {weights[name].shape[0]} rows, 8192 of {cfg.n_tokens} "
                                         f"calibration tokens (the Hessian and its factor cost the same for any number "
                                         f"of rows); NumPy float64, {dt:.1f} s"}
    log(f"obs stage: {ms:.2f} ms per layer | rank+plan {seg[0]:.2f} | " + (f"hessians+factors {seg[1]:.2f} | sweeps {seg[2]:.2f}"
        if args.obs_two_phases else f"hessians, factors and sweeps as one schedule {seg[2]:.2f}"))
    print(json.dumps(out), flush=True)


def run_mlp_stage(args):
    """--stage mlp: forward pass of the layer's feed-forward block on calibration tokens, at full size and after
    the composite pruning of the headline path has removed MLP channels; the first product also accumulates the
    statistic of the down projection's input.  Prints its own JSON line."""
    import numpy as np
    import torch
    from paper_2504_06323_amd import pipeline, prune, synth

    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 0, n, dev) for n, _, _, _ in shapes}
    n_seqs = min(cfg.n_seqs, 32)
    acts = {a: synth.make_activation(cfg, 0, a, dev, n_seqs=n_seqs) for a in act_shapes}
    tokens = n_seqs * cfg.seq_len
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, tokens)
    # the pruned block: rank, plan, mask, remove channels (the headline path), then pad the kept channels to a
    # multiple of 32 with zero rows / columns (they contribute silu(0) * 0 = 0)
    r = int(cfg.struct_frac * cfg.inter)
    pipeline.rank_layer(st, acts, cfg.alpha)
    _, ks, _ = pipeline.plan(st.count.tolist(), [rw * c for _, rw, c, _ in shapes], [c for _, _, c, _ in shapes], 1,
                             len(shapes), cfg.p, cfg.lam)
    pipeline.prune_layer(st, ks)
    res = pipeline.alloc_struct(st, r)
    pipeline.struct_layer(st, r, res)
    kept = cfg.inter - r
    padded = (kept + 31) // 32 * 32
    small = {"gate": torch.zeros((padded, cfg.hidden), dtype=res.gate.dtype, device=dev),
             "up": torch.zeros((padded, cfg.hidden), dtype=res.gate.dtype, device=dev),
             "down": torch.zeros((cfg.hidden, padded), dtype=res.gate.dtype, device=dev)}
    small["gate"][:kept] = res.gate
    small["up"][:kept] = res.up
    small["down"][:, :kept] = res.down
    full = {n: st.pruned[n] for n in ("gate", "up", "down")}
    x = acts["mlp_in"]
    bufs = {}
    for tag, ws_ in (("full", full), ("pruned", small)):
        inter = ws_["gate"].shape[0]
        bufs[tag] = (torch.empty((tokens, inter), dtype=x.dtype, device=dev),
                     torch.empty((tokens, cfg.hidden), dtype=x.dtype, device=dev),
                     torch.zeros(inter, dtype=torch.float32, device=dev),
                     torch.empty(int(prune.load().prune_mlp_workspace_bytes(tokens, inter)), dtype=torch.uint8, device=dev))
    ev = lambda: torch.cuda.Event(enable_timing=True)
    events = {"full": [], "pruned": [], "gate_up": []}

    def block(tag, ws_, record):
        h, y, sq, wsb = bufs[tag]
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        prune.mlp_gate_up(x, ws_["gate"], ws_["up"], h=h, sumsq=sq, ws=wsb)
        e1.record()
        prune.linear(h, ws_["down"], y=y)
        e2.record()
        if record:
            events[tag].append((e0, e2))
            if tag == "full":
                events["gate_up"].append((e0, e1))

    for _ in range(args.warmup):
        block("full", full, False)
        block("pruned", small, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        block("full", full, True)
        block("pruned", small, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    mean = lambda k: sum(a.elapsed_time(b) for a, b in events[k]) / len(events[k])
    ms_full, ms_small, ms_gu = mean("full"), mean("pruned"), mean("gate_up")
    flops_gu = 4.0 * tokens * cfg.hidden * cfg.inter
    achieved = flops_gu / (ms_gu * 1e-3) / 1e12
    out = {"metric": "feed-forward block forward pass on calibration tokens, full and after composite pruning (tokens/s)",
           "value": tokens / (ms_full * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(1e3 * elapsed / args.steps, 3), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: feed-forward block, hidden {cfg.hidden}, intermediate {cfg.inter} -> {kept} "
                                  f"kept channels (padded to {padded}), {tokens} tokens, bf16, fp32 accumulation; a step "
                                  f"runs the full and the pruned block once each"},
           "ms_full_block": round(ms_full, 3), "ms_pruned_block": round(ms_small, 3),
           "speedup_from_removed_channels": round(ms_full / ms_small, 3),
           "tflops_full_block": round(6.0 * tokens * cfg.hidden * cfg.inter / (ms_full * 1e-3) / 1e12, 1),
           "roofline": {"bound": "mfma", "kernel": f"linear_tiles_bf16<gate / up pair> on [{tokens}, {cfg.hidden}] x 2 x [{cfg.inter}, {cfg.hidden}]",
                        "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": round(achieved / 2500.0, 4), "traffic": None, "avg_launch_ms": round(ms_gu, 4),
                        "launches": len(events["gate_up"])}}
    if not args.no_cpu_baseline:
        from oracle import mlp_oracle as mlp
        rows = 512
        xs = x[:rows].detach().cpu().to(torch.float32).numpy()
        ws64 = {n: full[n].detach().cpu().to(torch.float32).numpy() for n in full}
        t0 = time.perf_counter()
        mlp.mlp_forward(xs, ws64["gate"], ws64["up"], ws64["down"])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": rows / dt, "unit": "tokens/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"{rows} tokens through the full block, NumPy float64, {dt:.1f} s"}
    log(f"mlp stage: full block {ms_full:.3f} ms, pruned block {ms_small:.3f} ms (x{ms_full / ms_small:.2f}); "
        f"gate/up pair {ms_gu:.3f} ms = {achieved:.0f} TFLOP/s")
    print(json.dumps(out), flush=True)


def run_layer_stage(args):
    """--stage layer: forward pass of one randomly initialised layer of the workload's shape on calibration
    sequences (the activations of all seven projections come out of it), followed once, outside the timing, by
    the headline ranking on those activations.  Prints its own JSON line."""
    import torch
    from paper_2504_06323_amd import pipeline, prune, synth

    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    weights = {n: synth.make_weight(cfg, 0, n, dev) for n, _, _, _ in shapes}
    head_dim = 128
    heads, kv_heads = cfg.q_out // head_dim, cfg.kv_out // head_dim
    n_seqs = min(cfg.n_seqs, 32)
    tokens = n_seqs * cfg.seq_len
    x = synth.make_activation(cfg, 0, "attn_in", dev, n_seqs=n_seqs)          # the layer's input (residual stream)
    norms = {n: torch.ones(cfg.hidden, dtype=x.dtype, device=dev) for n in ("attn_norm", "mlp_norm")}
    sumsq = torch.zeros(cfg.inter, dtype=torch.float32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    spans = []

    def step(record):
        e0, e1 = ev(), ev()
        e0.record()
        out = pipeline.layer_forward(weights, norms, x, n_seqs, cfg.seq_len, heads, kv_heads, head_dim, down_sumsq=sumsq)
        e1.record()
        if record:
            spans.append((e0, e1))
        return out

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        acts_out = step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = sum(a.elapsed_time(b) for a, b in spans) / len(spans)
    proj_flops = 2.0 * tokens * sum(rw * c for _, rw, c, _ in shapes)
    attn_flops = 4.0 * cfg.seq_len * cfg.seq_len * head_dim * heads * n_seqs / 2
    # the headline ranking on the activations that came out of the forward pass
    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, tokens)
    pipeline.rank_layer(st, {a: acts_out[a] for a in act_shapes}, cfg.alpha)
    counts = st.count.tolist()
    out = {"metric": "forward pass of one layer on calibration sequences (tokens/s); its activations feed the ranking",
           "value": tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(1e3 * elapsed / args.steps, 3), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: hidden {cfg.hidden}, {heads} query / {kv_heads} key-value heads of "
                                  f"{head_dim}, intermediate {cfg.inter}, {n_seqs} sequences of {cfg.seq_len} tokens, "
                                  f"random weights, unit norm weights; outlier counts on the real activations {counts}"},
           "tflops": round((proj_flops + attn_flops) / (ms * 1e-3) / 1e12, 1),
           "roofline": {"bound": "mfma", "kernel": "whole layer (seven projections and causal attention)",
                        "achieved": round((proj_flops + attn_flops) / (ms * 1e-3) / 1e12, 1), "peak": 2500.0,
                        "unit": "TFLOP/s", "frac": round((proj_flops + attn_flops) / (ms * 1e-3) / 1e12 / 2500.0, 4),
                        "traffic": None, "avg_launch_ms": round(ms, 3), "launches": len(spans)}}
    if not args.no_cpu_baseline:
        from oracle import layer_oracle as lay
        rows = 256
        host = lambda t: t.detach().cpu().to(torch.float32).numpy()
        w64 = {**{n: host(t) for n, t in weights.items()}, **{n: host(t) for n, t in norms.items()}}
        t0 = time.perf_counter()
        lay.layer_forward(host(x[:rows]), w64, 1, rows, heads, kv_heads, head_dim)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": rows / dt, "unit": "tokens/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"one sequence of {rows} tokens, NumPy float64, {dt:.1f} s"}
    log(f"layer stage: forward {ms:.2f} ms for {tokens} tokens ({(proj_flops + attn_flops) / (ms * 1e-3) / 1e12:.0f} TFLOP/s)")
    print(json.dumps(out), flush=True)


def measure_ceilings(torch, prune, dev, n_bytes=2 << 30, trials=5):
    """Streaming rates of the plainest kernels on this card, in this run: read-only and copy, best grid of a few."""
    src = torch.empty(n_bytes // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    out = {}
    for mode, name, moved in ((prune.PROBE_READ, "read", n_bytes), (prune.PROBE_COPY, "copy", 2 * n_bytes)):
        best = (0.0, 0.0, 0)
        for blocks in (256, 512, 1024, 2048, 4096, 8192):
            for _ in range(2):
                prune.bandwidth_probe(src, dst, mode, blocks)
            ts = []
            for _ in range(trials):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                prune.bandwidth_probe(src, dst, mode, blocks)
                e1.record()
                e1.synchronize()
                ts.append(e0.elapsed_time(e1))
            m, sd = mean_sigma(ts)
            gbps = moved / (m * 1e-3) / 1e9
            if gbps > best[0]:
                best = (gbps, moved / ((m + sd) * 1e-3) / 1e9, blocks)
        out[name] = {"gbps": round(best[0], 1), "blocks": best[2], "bytes_moved": moved}
    del src, dst
    return out


def run_prune_stage(args):
    import torch
    from paper_2504_06323_amd import pipeline, prune, synth

    cfg = synth.CONFIGS[args.workload]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    n_proj = len(shapes)
    numel = synth.layer_numel(cfg)
    struct_frac = cfg.struct_frac if cfg.struct_frac > 0 else args.struct_frac
    r = int(struct_frac * cfg.inter)
    targets = list(cfg.p_sweep) if cfg.p_sweep else [cfg.p]
    resident = max(1, min(args.resident_layers, cfg.n_layers))
    table_layers = cfg.n_layers if args.table_layers < 0 else max(resident, min(args.table_layers, cfg.n_layers))

    if not args.no_cpu_baseline:       # fork the oracle's workers while this process has not touched the GPU
        cpu_prepare(cfg, shapes, act_shapes, args.cpu_sample_den, min(16, len(os.sched_getaffinity(0))))

    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(2)
    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    # the whole model's table of outlier counts (Algorithm 1's R_LLM), the planner's inputs and outputs: on the device
    n_table = table_layers * n_proj
    t_count = torch.zeros(n_table, dtype=torch.int64, device=dev)
    t_numel = torch.tensor([rw * c for _, rw, c, _ in shapes] * table_layers, dtype=torch.int64, device=dev)
    t_cols = torch.tensor([c for _, _, c, _ in shapes] * table_layers, dtype=torch.int64, device=dev)
    t_sparsity = torch.zeros(n_table, dtype=torch.float64, device=dev)
    t_ks = torch.zeros(n_table, dtype=torch.int32, device=dev)
    t_flags = torch.zeros(2, dtype=torch.int32, device=dev)
    proj_inputs = {n: a for n, _, _, a in shapes}

    # Inputs: `resident` distinct layers stay in HBM (weights and all four activation tensors); the other layers of
    # the table are generated, ranked once for their row of counts, and dropped again.
    t0 = time.perf_counter()
    ring, first = [], None
    for layer in range(table_layers):
        weights = {n: synth.make_weight(cfg, layer, n, dev) for n, _, _, _ in shapes}
        acts = {a: synth.make_activation(cfg, layer, a, dev) for a in act_shapes}
        st = pipeline.LayerState.create(weights, proj_inputs, act_shapes, cfg.n_tokens, share_outputs_with=first)
        first = first or st
        st.count = t_count[layer * n_proj:(layer + 1) * n_proj]
        pipeline.rank_layer(st, acts, cfg.alpha)
        if layer < resident:
            ring.append((layer, st, acts))
        else:
            torch.cuda.synchronize()
            del weights, acts, st
    torch.cuda.synchronize()
    log(f"inputs generated in {time.perf_counter() - t0:.1f} s: {table_layers} layers ranked for the table of counts, "
        f"{resident} resident ({numel} weights and {sum(cfg.n_tokens * c for c in act_shapes.values())} activation "
        f"elements each)")
    res = pipeline.alloc_struct(first, r) if r > 0 else None
    names = list(act_shapes)
    stats_bytes = sum(cfg.n_tokens * c * (2 if storage_name(cfg) == "bf16" else 4) + c * 8 for c in act_shapes.values())
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stats_events = []   # (start, stop) around the statistics launches of every timed step
    pass_events = []    # marks between the passes, recorded in extra steps after the timed region

    def step(i: int, record: bool, breakdown: bool = False):
        """One pass of the whole path over the next layer of the ring.  record: one HIP-event pair around the
        statistics launches (the roofline figure).  breakdown: marks between all passes; every event costs the
        stream a few microseconds, so these steps run after the timed region, not inside it."""
        layer, st, acts = ring[i % len(ring)]
        marks = [] if breakdown else None
        mark = (lambda: (marks.append(ev()), marks[-1].record())) if breakdown else (lambda: None)
        mark()
        # ranking (independent of the target): done once per layer
        if record:
            e0, e1 = ev(), ev()
            e0.record()
        for a in names:
            prune.stats_norms(acts[a], st.sumsq[a], st.norms[a], ws=st.ws)
        if record:
            e1.record()
            stats_events.append((e0, e1))
        mark()
        prune.score_outlier_batch([st.weights[n] for n in st.names], [st.norms[proj_inputs[n]] for n in st.names],
                                  cfg.alpha, st.score_sum, st.count, taus=st.tau, ws=st.ws)
        mark()
        # pruning, once per target of the sweep, reusing the ranking
        for p in targets:
            if args.host_plan:          # the step waits for the table of counts on the host
                _, ks_all, _ = pipeline.plan(t_count.tolist(), t_numel.tolist(), t_cols.tolist(), table_layers, n_proj,
                                             p, cfg.lam)
                ks = ks_all[layer * n_proj:(layer + 1) * n_proj]
                mark()
                pipeline.prune_layer(st, ks)
            else:                       # the planner runs on the device over the whole table, behind the ranking
                prune.plan_sparsity_device(t_count, t_numel, t_cols, table_layers, n_proj, p, cfg.lam, t_sparsity,
                                           t_ks, t_flags)
                mark()
                pipeline.prune_layer(st, None, ks_dev=t_ks[layer * n_proj:(layer + 1) * n_proj])
            mark()
            if r > 0:
                pipeline.struct_layer(st, r, res)
            mark()
        if breakdown:
            pass_events.append(marks)

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib * (1 << 20) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            prune.bandwidth_probe(src, dst, prune.PROBE_COPY, 2048)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # after the clock has stopped: the device planner against the host planner on the same table, for every target
    counts = t_count.tolist()
    for p in targets:
        prune.plan_sparsity_device(t_count, t_numel, t_cols, table_layers, n_proj, p, cfg.lam, t_sparsity, t_ks, t_flags)
        _, ks_host, _ = pipeline.plan(counts, t_numel.tolist(), t_cols.tolist(), table_layers, n_proj, p, cfg.lam)
        if t_ks.tolist() != ks_host or t_flags.tolist()[1] != 0:
            raise RuntimeError(f"device plan differs from host plan at p = {p}")
    ks_last = ks_host

    ms_per_step = 1e3 * elapsed / args.steps
    ab = algorithmic_bytes(cfg, shapes, act_shapes, r, len(targets))
    n_break = max(5, min(args.steps, 10))
    for i in range(n_break):      # the per-pass breakdown, outside the timed region
        step(i, False, breakdown=True)
    torch.cuda.synchronize()
    ceilings = measure_ceilings(torch, prune, dev)

    # The timed region above is a few tens of milliseconds.  The same steps are run once more for a couple of seconds
    # (not part of `value`), so that the rate can be cross-checked against a clock or a utilisation sampler outside
    # this process.
    sustained = None
    if args.sustain_seconds > 0:
        n_sus = max(args.steps, int(1e3 * args.sustain_seconds / ms_per_step))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(n_sus):
            step(i, False)
        torch.cuda.synchronize()
        sus = time.perf_counter() - t1
        sustained = {"steps": n_sus, "seconds": round(sus, 3), "ms_per_step": round(1e3 * sus / n_sus, 4),
                     "value": numel * n_sus / sus}

    spans = [a.elapsed_time(b) / len(names) for a, b in stats_events]
    avg_ms, sd_ms = mean_sigma(spans)
    avg_bytes = stats_bytes / len(names)
    achieved = avg_bytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "colsumsq_partial_vec (activation statistics)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(cfg.name),
                "avg_launch_ms": round(avg_ms, 4), "avg_launch_ms_sigma": round(sd_ms, 4),
                "avg_launch_bytes": int(avg_bytes), "launches": len(stats_events) * len(names),
                "frac_of_read_ceiling": round(achieved / ceilings["read"]["gbps"], 4)}

    # per-pass figures from the marked steps: [start | stats | score+outlier | (plan | select | struct) per target]
    samples = {"stats": [], "score_outlier": [], "plan": [], "select": [], "struct": [], "step": []}
    for m in pass_events:
        d = [m[j].elapsed_time(m[j + 1]) for j in range(len(m) - 1)]
        samples["stats"].append(d[0])
        samples["score_outlier"].append(d[1])
        for t in range(len(targets)):
            samples["plan"].append(d[2 + 3 * t])
            samples["select"].append(d[3 + 3 * t])
            samples["struct"].append(d[4 + 3 * t])
        samples["step"].append(m[0].elapsed_time(m[-1]))
    pass_bytes = {"stats": ab["stats"], "score_outlier": ab["score"] + ab["count"], "plan": 0, "select": ab["select"],
                  "struct": ab["struct_rank"] + ab["compact"]}
    pass_ceiling = {"stats": "read", "score_outlier": "read", "select": "copy", "struct": "copy"}
    passes = {}
    for name, xs in samples.items():
        if name == "step" or (name == "struct" and r == 0):
            continue
        m, sd = mean_sigma(xs)
        entry = {"ms": round(m, 4), "ms_sigma": round(sd, 4), "trials": len(xs), "bytes": pass_bytes[name]}
        if pass_bytes[name]:
            gbps = pass_bytes[name] / (m * 1e-3) / 1e9
            entry.update(gbps=round(gbps, 1), frac_of_peak=round(gbps / HBM_PEAK_GBPS, 4),
                         frac_of_ceiling=round(gbps / ceilings[pass_ceiling[name]]["gbps"], 4),
                         ceiling=pass_ceiling[name])
        passes[name] = entry
    step_m, step_sd = mean_sigma(samples["step"])
    log(f"step {ms_per_step:.3f} ms (marked steps {step_m:.3f} +- {step_sd:.3f}) | " +
        " | ".join(f"{k} {v['ms']:.3f} ms" + (f" ({v['gbps']:.0f} GB/s)" if "gbps" in v else "") for k, v in passes.items()))
    log(f"ceilings: read {ceilings['read']['gbps']:.0f} GB/s, copy {ceilings['copy']['gbps']:.0f} GB/s")
    log(f"outlier counts of layer 0 {counts[:n_proj]}; zeros per row at p = {targets[-1]}: {ks_last[:n_proj]}; "
        f"removed MLP channels {r}")

    out = {
        "metric": "projection weights pruned/s (GB/s scored+masked) and % of HBM peak, 1 GPU",
        "value": numel * args.steps / elapsed,
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_sigma": round(step_sd, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: layers of the {cfg.n_layers}-layer model, {storage_name(cfg)} storage, hidden "
                               f"{cfg.hidden}, q/o {cfg.q_out}, k/v {cfg.kv_out}, intermediate {cfg.inter}, "
                               f"{cfg.n_seqs} x {cfg.seq_len} calibration tokens per layer, {len(names)} distinct activation "
                               f"tensors; a step = one layer: ranking once, then for each target in {targets}: "
                               f"planner over the {table_layers} x {n_proj} table, select + mask, "
                               f"{r} of {cfg.inter} MLP channels removed structurally; {resident} distinct layers "
                               f"resident and cycled, alpha {cfg.alpha}, lambda {cfg.lam}",
                   "weights_per_step": numel,
                   "algorithmic_bytes_per_step": ab["total"],
                   "storage_dtype": storage_name(cfg),
                   "targets": targets,
                   "layers_resident": resident,
                   "layers_in_table": table_layers},
        "algorithmic_gbps": round(ab["total"] / elapsed * args.steps / 1e9, 1),
        "hbm_frac_whole_step": round(ab["total"] / elapsed * args.steps / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
        "passes": passes,
        "ceilings": ceilings,
    }
    if sustained:
        out["sustained"] = sustained
    if not args.no_cpu_baseline:
        layer0, st0, acts0 = ring[0]
        out["cpu_baseline"] = cpu_baseline(st0.weights, acts0)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stage", default="prune", choices=["prune", "hessian", "obs", "mlp", "layer"],
                    help="prune (default): the scoring / masking / structured path the headline metric is quoted on; "
                         "hessian: the matrix-core stage of the Hessian-based pruner, its own JSON line; "
                         "obs: the whole Hessian-based path of one layer, its own JSON line; "
                         "mlp: forward pass of the feed-forward block, full and pruned, its own JSON line; "
                         "layer: forward pass of a whole layer, its own JSON line")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    help="default: llama3_8b_full for the prune stage, llama7b_layer for the other stages")
    ap.add_argument("--resident-layers", type=int, default=8,
                    help="distinct layers kept in HBM and cycled through by the steps (capped at the model's layers)")
    ap.add_argument("--table-layers", type=int, default=-1,
                    help="layers in the planner's table of counts (default: all layers of the model); the ones that "
                         "are not resident are generated and ranked once before the timed region")
    ap.add_argument("--struct-frac", type=float, default=0.2,
                    help="fraction of MLP channels removed structurally when the workload itself names none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sustain-seconds", type=float, default=2.0,
                    help="default stage: after the timed steps, run the same steps for about this long and report "
                         "their rate as `sustained` (0: skip)")
    ap.add_argument("--obs-two-phases", action="store_true",
                    help="obs stage: all Hessians and factors, then all sweeps (two timed segments) instead of one "
                         "schedule in which the sweeps of a projection input start as soon as its factor is there")
    ap.add_argument("--host-plan", action="store_true",
                    help="run the projection planner on the host (the step then waits for the outlier counts)")
    ap.add_argument("--cpu-sample-den", type=int, default=4)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the warm-up, run the plain copy kernel (read N MiB, write N MiB) three times so "
                         "that a rocprofv3 --pmc run of this command carries a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: every box of this build has one MI355X and the path has no "
            "multi-GPU leg. Run with --gpus 1.")
        sys.exit(2)
    if args.workload is None:
        args.workload = "llama3_8b_full" if args.stage == "prune" else "llama7b_layer"

    if args.stage == "hessian":
        run_hessian_stage(args)
    elif args.stage == "obs":
        run_obs_stage(args)
    elif args.stage == "mlp":
        run_mlp_stage(args)
    elif args.stage == "layer":
        run_layer_stage(args)
    else:
        run_prune_stage(args)


if __name__ == "__main__":
    main()
