#!/usr/bin/env python3
"""Benchmark of the projection-pruning hot path on one MI355X.

A step is one pass of the whole path over one synthetic LLaMA-7B-shaped layer
(the workload the headline metric is quoted on): activation statistics for the
four distinct projection inputs (128 x 2048 calibration tokens), metric sum and
outlier count for the seven projections, the host planner, per-row selection
and masking of the seven projections, then structured ranking and compaction
of the MLP on the masked weights.  All inputs are resident in HBM before the
timed region starts.  One JSON line goes to stdout; everything else to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(cfg, shapes, act_shapes, r):
    """Bytes the method itself must move per step (what the roofline is priced on)."""
    es = 2 if str(cfg.dtype).endswith("bfloat16") else 4
    numel = sum(rw * c for _, rw, c, _ in shapes)
    stats = sum(cfg.n_tokens * ch * es + ch * 4 for ch in act_shapes.values())
    score = numel * es
    count = numel * es
    select = numel * (2 * es) + numel // 8
    mlp = 3 * cfg.inter * cfg.hidden
    struct_rank = mlp * es
    kept_frac = (cfg.inter - r) / cfg.inter
    compact = mlp * es + int(mlp * es * kept_frac)
    return dict(stats=stats, score=score, count=count, select=select, struct_rank=struct_rank, compact=compact,
                total=stats + score + count + select + struct_rank + compact)


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


def cpu_baseline(cfg, shapes, weights, acts, frac_den=8):
    """Time the CPU oracle, as it stands, on a 1/frac_den sample of the same layer."""
    import numpy as np
    import torch
    from oracle import mosaic_oracle as orc

    n_seqs = max(1, cfg.n_seqs // frac_den)
    t_rows = n_seqs * cfg.seq_len
    host = lambda t: t.detach().cpu().to(torch.float32).numpy()
    xs = {a: host(x[:t_rows]) for a, x in acts.items()}
    ws = {n: host(w[::frac_den]) for n, w in weights.items()}
    sampled = sum(w.size for w in ws.values())
    t0 = time.perf_counter()
    norms = {a: orc.column_norms(x) for a, x in xs.items()}
    ratios, omegas = [], {}
    for n, rw, c, a in shapes:
        omega = orc.weight_metric(ws[n], norms[a])
        _, _, ratio, _ = orc.outlier_stats(omega, cfg.alpha)
        ratios.append(ratio)
        omegas[n] = omega
    s, _ = orc.plan_sparsity(np.array(ratios).reshape(1, -1), cfg.p, cfg.lam, "global")
    masked = {}
    for i, (n, rw, c, a) in enumerate(shapes):
        masked[n], _ = orc.prune_projection(ws[n], omegas[n], orc.zeros_per_row(s[0, i], c))
    # structured part on the sample: every frac_den-th MLP channel forms the sampled MLP
    gate, up = masked["gate"], masked["up"]
    down = host(weights["down"][:, ::frac_den])
    g = orc.group_magnitude(gate, up, down)
    kept = orc.struct_rank(g, int(cfg.struct_frac * g.shape[0]))
    orc.struct_compact(gate, up, down, kept)
    dt = time.perf_counter() - t0
    return {"value": sampled / dt, "unit": "weights/s", "cores": 1, "kind": "oracle",
            "sample": f"1/{frac_den} of the layer: {n_seqs} of {cfg.n_seqs} calibration sequences for the activation "
                      f"statistics, every {frac_den}th output row of each projection ({sampled} weights); "
                      f"NumPy float64, {dt:.1f} s"}


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
        pipeline.hessian_layer(ob, acts, on_big=(lambda e: gram_events.append(e)) if record else None, big=big)
        if record:
            m[2].record()
        pipeline.obs_prune_layer(st, ob, s)
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
           "ms_rank_and_plan": round(seg[0], 3), "ms_hessians_and_factors": round(seg[1], 3), "ms_sweeps": round(seg[2], 3),
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
    log(f"obs stage: {ms:.2f} ms per layer | rank+plan {seg[0]:.2f} | hessians+factors {seg[1]:.2f} | sweeps {seg[2]:.2f}")
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
    ap.add_argument("--workload", default="llama7b_layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--host-plan", action="store_true",
                    help="run the projection planner on the host (the step then waits for the outlier counts)")
    ap.add_argument("--cpu-sample-den", type=int, default=2)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the warm-up, run a plain float32 copy kernel (read N MiB, write N MiB) three "
                         "times so that a rocprofv3 --pmc run of this command carries a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: every box of this build has one MI355X and the path has no "
            "multi-GPU leg. Run with --gpus 1.")
        sys.exit(2)

    if args.stage == "hessian":
        run_hessian_stage(args)
        return
    if args.stage == "obs":
        run_obs_stage(args)
        return
    if args.stage == "mlp":
        run_mlp_stage(args)
        return
    if args.stage == "layer":
        run_layer_stage(args)
        return

    import torch
    from paper_2504_06323_amd import pipeline, prune, synth

    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(2)
    prune.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    shapes = synth.projection_shapes(cfg)
    act_shapes = synth.activation_shapes(cfg)
    numel = synth.layer_numel(cfg)
    r = int(cfg.struct_frac * cfg.inter)

    t0 = time.perf_counter()
    weights = {n: synth.make_weight(cfg, 0, n, dev) for n, _, _, _ in shapes}
    acts = {a: synth.make_activation(cfg, 0, a, dev) for a in act_shapes}
    torch.cuda.synchronize()
    log(f"inputs generated in {time.perf_counter() - t0:.1f} s: {numel} weights, "
        f"{sum(x.numel() for x in acts.values())} activation elements")

    st = pipeline.LayerState.create(weights, {n: a for n, _, _, a in shapes}, act_shapes, cfg.n_tokens)
    res = pipeline.alloc_struct(st, r)
    numels = [rw * c for _, rw, c, _ in shapes]
    cols = [c for _, _, c, _ in shapes]
    names = list(act_shapes)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stats_events = []   # (start, stop, bytes, launches) around the statistics launches of every timed step
    pass_events = []    # per-step boundaries for the stderr breakdown

    def step(record: bool, breakdown: bool = False):
        """One pass of the whole path.  record: one HIP-event pair around the statistics launches (the
        roofline figure).  breakdown: marks between the passes as well; each event costs the stream a few
        microseconds, so these steps are run after the timed region, not inside it."""
        marks = [ev() for _ in range(5)] if breakdown else None
        if breakdown:
            marks[0].record()
        # phase 1: ranking (independent of p)
        if record:
            e0, e1 = ev(), ev()
            e0.record()
        for a in names:
            prune.stats_norms(acts[a], st.sumsq[a], st.norms[a], ws=st.ws)
        if record:
            e1.record()
            stats_events.append((e0, e1, sum(acts[a].numel() * acts[a].element_size() + acts[a].shape[1] * 8
                                             for a in names), len(names)))
        if breakdown:
            marks[1].record()
        prune.score_outlier_batch([st.weights[n] for n in st.names],
                                  [st.norms[st.proj_inputs[n]] for n in st.names], cfg.alpha, st.score_sum,
                                  st.count, taus=st.tau, ws=st.ws)
        if breakdown:
            marks[2].record()
        if args.host_plan:
            counts = st.count.tolist()      # 7 integers cross to the host, the step waits for them
            _, ks, _ = pipeline.plan(counts, numels, cols, 1, len(shapes), cfg.p, cfg.lam)
        else:
            counts = ks = None              # the planner runs on the device, behind the ranking
            pipeline.plan_device(st, cfg.p, cfg.lam)
        # phase 2: pruning
        pipeline.prune_layer(st, ks)
        if breakdown:
            marks[3].record()
        pipeline.struct_layer(st, r, res)
        if breakdown:
            marks[4].record()
            pass_events.append(marks)
        return counts, ks

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib * (1 << 20) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        counts, ks = step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    if not args.host_plan:   # read the plan back once, after the clock has stopped, and hold it against the host planner
        counts, ks = st.count.tolist(), st.ks_dev.tolist()
        _, ks_host, _ = pipeline.plan(counts, numels, cols, 1, len(shapes), cfg.p, cfg.lam)
        if ks != ks_host or st.plan_flags.tolist()[1] != 0:
            raise RuntimeError(f"device plan {ks} differs from host plan {ks_host}")

    ms_per_step = 1e3 * elapsed / args.steps
    ab = algorithmic_bytes(cfg, shapes, act_shapes, r)
    for _ in range(min(args.steps, 10)):     # the per-pass breakdown for stderr, outside the timed region
        step(False, breakdown=True)
    torch.cuda.synchronize()
    n_launches = sum(n for _, _, _, n in stats_events)
    avg_ms = sum(a.elapsed_time(b) for a, b, _, _ in stats_events) / n_launches
    avg_bytes = sum(n for _, _, n, _ in stats_events) / n_launches
    achieved = avg_bytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "colsumsq_partial_vec (activation statistics)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(cfg.name),
                "avg_launch_ms": round(avg_ms, 4), "avg_launch_bytes": int(avg_bytes),
                "launches": n_launches}

    seg = [[m[i].elapsed_time(m[i + 1]) for i in range(4)] for m in pass_events]
    mean = lambda j: sum(s[j] for s in seg) / len(seg)
    gb = lambda key: ab[key] / 1e9
    log(f"step {ms_per_step:.3f} ms | stats {mean(0):.3f} ms ({gb('stats') / mean(0) * 1e3:.0f} GB/s) | "
        f"score+count {mean(1):.3f} ms ({(gb('score') + gb('count')) / mean(1) * 1e3:.0f} GB/s) | "
        f"plan+select {mean(2):.3f} ms ({gb('select') / mean(2) * 1e3:.0f} GB/s) | "
        f"struct {mean(3):.3f} ms ({(gb('struct_rank') + gb('compact')) / mean(3) * 1e3:.0f} GB/s)")
    log(f"outlier counts {counts}; zeros per row {ks}; removed MLP channels {r}")

    out = {
        "metric": "projection weights pruned/s (GB/s scored+masked) and % of HBM peak, 1 GPU",
        "value": numel * args.steps / elapsed,
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: one LLaMA-7B-shaped layer, bf16 storage, hidden {cfg.hidden}, "
                               f"intermediate {cfg.inter}, {cfg.n_seqs} x {cfg.seq_len} calibration tokens, "
                               f"4 distinct activation tensors, alpha {cfg.alpha}, target sparsity {cfg.p}, "
                               f"{r} of {cfg.inter} MLP channels removed structurally",
                   "weights_per_step": numel,
                   "algorithmic_bytes_per_step": ab["total"],
                   "storage_dtype": "bf16"},
        "algorithmic_gbps": round(ab["total"] / elapsed * args.steps / 1e9, 1),
        "hbm_frac_whole_step": round(ab["total"] / elapsed * args.steps / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, shapes, weights, acts, args.cpu_sample_den)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
