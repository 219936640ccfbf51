"""Call sequencing for one LLaMA-style layer: which entry point runs on which tensor, in what order.

Nothing is computed here.  The two phases mirror the paper's two controllers:

  rank_layer   Parameter Ranking Controller (Algorithm 1): activation norms per
               distinct projection input, then metric sum and outlier count per
               projection.  Independent of the pruning target p, so it runs once.
  plan         Projection Planner (Section 3.3): counts -> zeros per row, on the host
               (plan) or on the device without a host round trip (plan_device).
  prune_layer  Parameter Pruning Controller, unstructured category, then (for
               the composite category) structured removal of MLP channels on
               the masked weights.

Device buffers are allocated once per LayerState and reused across steps.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import prune


@dataclass
class LayerState:
    """Device buffers of one layer.  proj_inputs maps projection name -> activation name."""

    weights: Dict[str, torch.Tensor]
    proj_inputs: Dict[str, str]
    device: torch.device
    sumsq: Dict[str, torch.Tensor] = field(default_factory=dict)
    norms: Dict[str, torch.Tensor] = field(default_factory=dict)
    score_sum: torch.Tensor = None      # [n_proj] float64
    count: torch.Tensor = None          # [n_proj] int64
    tau: torch.Tensor = None            # [n_proj] float32
    pruned: Dict[str, torch.Tensor] = field(default_factory=dict)   # masked copies (phase 2 output)
    mask_bits: Dict[str, torch.Tensor] = field(default_factory=dict)
    rowsq: Dict[str, torch.Tensor] = field(default_factory=dict)    # gate / up: row sums of squares of the masked copies
    rowsq_valid: bool = False                                        # set by prune_layer, cleared by whoever rewrites pruned
    ws: torch.Tensor = None
    names: Tuple[str, ...] = ()
    numels_dev: torch.Tensor = None     # [n_proj] int64, constant
    cols_dev: torch.Tensor = None       # [n_proj] int64, constant
    sparsity_dev: torch.Tensor = None   # [n_proj] float64, written by plan_device
    ks_dev: torch.Tensor = None         # [n_proj] int32, written by plan_device
    plan_flags: torch.Tensor = None     # [2] int32: clamped, invalid input

    @classmethod
    def create(cls, weights: Dict[str, torch.Tensor], proj_inputs: Dict[str, str],
               act_channels: Dict[str, int], act_tokens: int, want_mask_bits: bool = True,
               share_outputs_with: Optional["LayerState"] = None) -> "LayerState":
        """share_outputs_with: another layer's state of the same shapes whose masked copies, keep-bits and
        workspace this one reuses (layers processed one after the other need only one set)."""
        dev = next(iter(weights.values())).device
        st = cls(weights=weights, proj_inputs=proj_inputs, device=dev)
        st.names = tuple(weights)
        n = len(st.names)
        for a, ch in act_channels.items():
            st.sumsq[a] = torch.zeros(ch, dtype=torch.float32, device=dev)
            st.norms[a] = torch.empty(ch, dtype=torch.float32, device=dev)
        st.score_sum = torch.zeros(n, dtype=torch.float64, device=dev)
        st.count = torch.zeros(n, dtype=torch.int64, device=dev)
        st.tau = torch.zeros(n, dtype=torch.float32, device=dev)
        st.numels_dev = torch.tensor([weights[k].numel() for k in st.names], dtype=torch.int64, device=dev)
        st.cols_dev = torch.tensor([weights[k].shape[1] for k in st.names], dtype=torch.int64, device=dev)
        st.sparsity_dev = torch.zeros(n, dtype=torch.float64, device=dev)
        st.ks_dev = torch.zeros(n, dtype=torch.int32, device=dev)
        st.plan_flags = torch.zeros(2, dtype=torch.int32, device=dev)
        if share_outputs_with is not None:
            o = share_outputs_with
            st.pruned, st.mask_bits, st.ws, st.rowsq = o.pruned, o.mask_bits, o.ws, o.rowsq
            return st
        need = 256
        for a, ch in act_channels.items():
            need = max(need, prune.workspace_bytes(prune.OP_STATS, max(act_tokens, 1), ch))
        for name, w in weights.items():
            need = max(need, prune.workspace_bytes(prune.OP_SCORE, w.shape[0], w.shape[1]),
                       prune.workspace_bytes(prune.OP_BATCH, w.shape[0], w.shape[1]))
            st.pruned[name] = torch.empty_like(w)
            if want_mask_bits:
                st.mask_bits[name] = torch.empty((w.shape[0], (w.shape[1] + 31) // 32), dtype=torch.int32, device=dev)
        if "gate" in weights:
            inter, hidden = weights["gate"].shape
            need = max(need, prune.workspace_bytes(prune.OP_STRUCT, inter, hidden))
            if "up" in weights:
                st.rowsq = {n: torch.empty(inter, dtype=torch.float32, device=dev) for n in ("gate", "up")}
        st.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        return st


def rank_layer(st: LayerState, acts: Dict[str, torch.Tensor], alpha: float,
               scores: Optional[Dict[str, torch.Tensor]] = None,
               outlier_scope: int = prune.OUTLIERS_PER_PROJECTION) -> None:
    """Phase 1: norms for every distinct input, then metric sum + outlier count for every projection.

    outlier_scope = prune.OUTLIERS_PER_LAYER measures outliers against the layer mean (the
    layer-level rule the paper starts from) instead of each projection's own mean."""
    for a, x in acts.items():        # each activation tensor is resident whole: one call gives sums and norms
        prune.stats_norms(x, st.sumsq[a], st.norms[a], ws=st.ws)
    if scores is None:      # hot mode: every projection of the layer in one batch
        prune.score_outlier_batch([st.weights[n] for n in st.names], [st.norms[st.proj_inputs[n]] for n in st.names],
                                  alpha, st.score_sum, st.count, taus=st.tau, ws=st.ws, outlier_scope=outlier_scope)
        return
    if outlier_scope != prune.OUTLIERS_PER_PROJECTION:
        raise ValueError("materialised scores are only offered with per-projection thresholds")
    for i, name in enumerate(st.names):     # parity mode: scores materialised, one projection at a time
        w = st.weights[name]
        nrm = st.norms[st.proj_inputs[name]]
        sc = scores.get(name)
        prune.score(w, nrm, st.score_sum[i:i + 1], scores=sc, ws=st.ws)
        prune.outlier_ratio(w, nrm, alpha, st.score_sum[i:i + 1], st.count[i:i + 1], tau=st.tau[i:i + 1], scores=sc)


def down_input_from_forward(st: LayerState, x_mlp: torch.Tensor, h: Optional[torch.Tensor] = None,
                            act: str = "down_in") -> torch.Tensor:
    """The down projection's input from a real forward pass of the feed-forward block, h = silu(x gate^T) * (x up^T),
    with its channel statistic accumulated where h is produced: fills st.sumsq[act] and st.norms[act] (instead of
    a statistics pass over an injected tensor) and returns h."""
    st.sumsq[act].zero_()
    h = prune.mlp_gate_up(x_mlp, st.weights["gate"], st.weights["up"], h=h, sumsq=st.sumsq[act])
    prune.stats_finalize(st.sumsq[act], st.norms[act])
    return h


def plan(counts: Sequence[int], numels: Sequence[int], cols: Sequence[int], n_layers: int, n_proj: int, p: float,
         lam: float, scope: int = prune.SCOPE_GLOBAL):
    """Host planner over all layers' counts: returns (sparsities, zeros per row, clamped)."""
    return prune.plan_sparsity(counts, numels, n_layers, n_proj, p, lam, scope, cols=cols)


def plan_device(st: LayerState, p: float, lam: float, scope: int = prune.SCOPE_GLOBAL) -> None:
    """The planner over this layer's counts, enqueued behind the ranking: st.count -> st.ks_dev, st.sparsity_dev."""
    prune.plan_sparsity_device(st.count, st.numels_dev, st.cols_dev, 1, len(st.names), p, lam, st.sparsity_dev,
                               st.ks_dev, st.plan_flags, scope=scope)


def prune_layer(st: LayerState, ks: Optional[Sequence[int]], in_place: bool = False,
                ks_dev: Optional[torch.Tensor] = None) -> None:
    """Phase 2, unstructured: zero the k lowest-metric entries per row of every projection.
    ks = None takes the zeros per row from ks_dev (default: what plan_device left in st.ks_dev).
    The masking pass also leaves the row sums of squares of the masked gate and up in st.rowsq, which
    struct_layer hands to the structured pass."""
    names = st.names
    if ks_dev is None and ks is None:
        ks_dev = st.ks_dev
    prune.select_mask_batch([st.weights[n] for n in names], [st.norms[st.proj_inputs[n]] for n in names],
                            None if ks is None else [int(k) for k in ks],
                            w_outs=None if in_place else [st.pruned[n] for n in names],
                            mask_bits=[st.mask_bits.get(n) for n in names], ks_dev=ks_dev if ks is None else None,
                            row_sumsq=[st.rowsq.get(n) for n in names])
    st.rowsq_valid = bool(st.rowsq) and not in_place     # the sums describe st.pruned


@dataclass
class StructResult:
    group_mag: torch.Tensor
    kept_idx: torch.Tensor
    gate: Optional[torch.Tensor]
    up: Optional[torch.Tensor]
    down: Optional[torch.Tensor]


def alloc_struct(st: LayerState, r: int, compact: bool = True) -> StructResult:
    gate = st.weights["gate"]
    inter, hidden = gate.shape
    kept = inter - r
    mk = lambda *shape: torch.empty(shape, dtype=gate.dtype, device=st.device)
    return StructResult(torch.empty(inter, dtype=torch.float32, device=st.device),
                        torch.empty(kept, dtype=torch.int32, device=st.device),
                        mk(kept, hidden) if compact else None, mk(kept, hidden) if compact else None,
                        mk(hidden, kept) if compact else None)


def struct_layer(st: LayerState, r: int, out: StructResult, masked: bool = True) -> None:
    """Phase 2, structured: rank MLP channels on the (masked) weights, drop r, compact."""
    src = st.pruned if masked else st.weights
    have = masked and st.rowsq_valid
    prune.struct_compact(src["gate"], src["up"], src["down"], r, out.group_mag, out.kept_idx,
                         out.gate, out.up, out.down, ws=st.ws, gate_rowsq=st.rowsq["gate"] if have else None,
                         up_rowsq=st.rowsq["up"] if have else None)


# ----------------------------------------------------------------------------------------------------------------
# The Hessian-based pruner the paper's experiments run with the planner's targets (Section 4.1.3, "Pruning
# Methods"): one Hessian and one factor per distinct projection input, one compensated sweep per projection.

@dataclass
class ObsState:
    """Device buffers of the Hessian-based path of one layer (on top of a LayerState).

    The factorisations of the different projection inputs, and the sweeps of the different projections, are
    independent and each has phases that occupy a single compute unit or are bound by launch latency, so they are
    spread over a few HIP streams (default priority), each with its own workspace."""

    hessian: Dict[str, torch.Tensor]        # per activation: [C, C] float32; after hessian_layer its upper triangle is R
    dead: Dict[str, torch.Tensor]           # per activation: [C] uint8
    info: torch.Tensor                      # [n_activations] int32, 0 = factorisation went through
    ws: List[torch.Tensor]                  # one workspace per stream
    factor_ws: torch.Tensor                 # scratch of the factorisations on stream 0 (ws[0] belongs to the Hessian kernel)
    gram_ws: torch.Tensor                   # the Hessian kernel's partial sums when sweeps run beside it (obs_layer)
    streams: List["torch.cuda.Stream"]
    factored: Dict[str, "torch.cuda.Event"] = field(default_factory=dict)

    @classmethod
    def create(cls, st: LayerState, act_channels: Dict[str, int], act_tokens: int, n_streams: int = 4) -> "ObsState":
        dev = st.device
        need = 256
        for a, ch in act_channels.items():
            need = max(need, prune.hessian_workspace_bytes(act_tokens, ch),
                       int(prune.load().prune_hessian_factor_workspace_bytes(ch)))
        for name, w in st.weights.items():
            need = max(need, int(prune.load().prune_obs_sweep_workspace_bytes(w.shape[0], w.shape[1], 1)))
        return cls(hessian={a: torch.zeros((ch, ch), dtype=torch.float32, device=dev) for a, ch in act_channels.items()},
                   dead={a: torch.zeros(ch, dtype=torch.uint8, device=dev) for a, ch in act_channels.items()},
                   info=torch.zeros(len(act_channels), dtype=torch.int32, device=dev),
                   ws=[torch.empty(need, dtype=torch.uint8, device=dev) for _ in range(n_streams)],
                   factor_ws=torch.empty(int(prune.load().prune_hessian_factor_workspace_bytes(128)),
                                         dtype=torch.uint8, device=dev),
                   gram_ws=torch.empty(max(prune.hessian_workspace_bytes(act_tokens, ch) for ch in act_channels.values()),
                                       dtype=torch.uint8, device=dev),
                   streams=[torch.cuda.Stream(device=dev) for _ in range(n_streams)])


def hessian_layer(ob: ObsState, acts: Dict[str, torch.Tensor], damp: float = 0.01, on_big=None, big: str = "") -> None:
    """H = X^T X for every distinct projection input (one after the other: each fills the chip), each followed by
    damping and factorisation in place on a stream of its own."""
    main = torch.cuda.current_stream()
    wait_factored(ob, main)     # a factorisation of an earlier call may still be running on these buffers
    order = sorted(range(len(acts)), key=lambda i: -list(acts.values())[i].shape[1])   # widest first: its
    names = list(acts)                                   # factorisation is the longest and overlaps the other Hessians
    for slot, i in enumerate(order):
        a, x = names[i], acts[names[i]]
        side = ob.streams[slot % len(ob.streams)]
        ob.hessian[a].zero_()
        timed = on_big is not None and a == big        # a benchmark's event pair around one accumulation
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
        prune.hessian_accumulate(x, ob.hessian[a], ws=ob.ws[0])
        if timed:
            e1.record(main)
            on_big((e0, e1))
        ready = torch.cuda.Event()
        ready.record(main)
        side.wait_event(ready)
        prune.hessian_factor(ob.hessian[a], damp, dead=ob.dead[a], info=ob.info[i:i + 1],
                             ws=ob.ws[slot % len(ob.streams)] if slot % len(ob.streams) else ob.factor_ws, stream=side)
        done = torch.cuda.Event()
        done.record(side)
        ob.factored[a] = done


def wait_factored(ob: ObsState, stream=None) -> None:
    """Order `stream` (default: the current one) behind every factorisation hessian_layer has enqueued on its side
    streams: needed before that stream reads or overwrites ob.hessian, ob.dead or ob.info."""
    stream = torch.cuda.current_stream() if stream is None else stream
    for done in ob.factored.values():
        stream.wait_event(done)


def obs_prune_layer(st: LayerState, ob: ObsState, sparsities: Sequence[float], in_place: bool = False) -> None:
    """Compensated sweep of every projection with its own sparsity target (the planner's p_{n,m}), the
    projections dealt round robin to the streams; the calling stream waits for all of them at the end."""
    main = torch.cuda.current_stream()
    start = torch.cuda.Event()
    start.record(main)
    order = sorted(range(len(st.names)), key=lambda i: -st.weights[st.names[i]].numel())   # longest sweeps first
    for slot, i in enumerate(order):
        name, a = st.names[i], st.proj_inputs[st.names[i]]
        side = ob.streams[slot % len(ob.streams)]
        side.wait_event(start)
        if a in ob.factored:
            side.wait_event(ob.factored[a])
        prune.obs_sweep(st.weights[name], ob.hessian[a], float(sparsities[i]),
                        w_out=None if in_place else st.pruned[name], dead=ob.dead[a], mask_bits=st.mask_bits.get(name),
                        ws=ob.ws[slot % len(ob.streams)], stream=side)
    for side in ob.streams:
        done = torch.cuda.Event()
        done.record(side)
        main.wait_event(done)
    st.rowsq_valid = False      # st.pruned no longer holds what the masking pass summed


def obs_layer(st: LayerState, ob: ObsState, acts: Dict[str, torch.Tensor], sparsities: Sequence[float],
              damp: float = 0.01, in_place: bool = False, on_big=None, big: str = "") -> None:
    """hessian_layer and obs_prune_layer as one schedule.  The Hessians are accumulated on the calling stream one
    after the other; an accumulation fills the chip and next to nothing else runs beside it, so what matters is
    what waits behind the last one.  The widest Hessian comes first (its factorisation and sweep are the longest
    chain of the layer and get the head start), the others in the order of the sweep work that waits for them.
    Each factorisation is queued on a side stream of its own as soon as its Hessian is there, all of them before any
    sweep, so that no factorisation waits behind a sweep of another input.  The largest sweep of an input follows
    its factorisation on the same stream; the others go, largest first, to the stream with the least work queued
    (by a rough cost: panels of 128 columns times a factor for the rows).  The calling stream waits for all side
    streams at the end."""
    main = torch.cuda.current_stream()
    wait_factored(ob, main)
    n_side = len(ob.streams)

    def sweep_cost(name: str) -> float:
        w = st.weights[name]
        return (w.shape[1] / 128.0) * (1.0 + w.shape[0] / 8192.0)

    readers = {a: sorted((n for n in st.names if st.proj_inputs[n] == a), key=lambda n: -sweep_cost(n)) for a in acts}
    widest = max(acts, key=lambda a: acts[a].shape[1])
    names = [widest] + sorted((a for a in acts if a != widest), key=lambda a: -sum(sweep_cost(n) for n in readers[a]))
    load = [0.0] * n_side
    slot_of, done = {}, {}
    for i, a in enumerate(names):
        x = acts[a]
        ch = x.shape[1]
        ob.hessian[a].zero_()
        timed = on_big is not None and a == big
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
        prune.hessian_accumulate(x, ob.hessian[a], ws=ob.gram_ws)
        if timed:
            e1.record(main)
            on_big((e0, e1))
        ready = torch.cuda.Event()
        ready.record(main)
        slot = i % n_side if i < n_side else min(range(n_side), key=lambda j: load[j])
        side = ob.streams[slot]
        side.wait_event(ready)
        i_info = list(acts).index(a)
        prune.hessian_factor(ob.hessian[a], damp, dead=ob.dead[a], info=ob.info[i_info:i_info + 1], ws=ob.ws[slot],
                             stream=side)
        done[a] = torch.cuda.Event()
        done[a].record(side)
        ob.factored[a] = done[a]
        slot_of[a] = slot
        load[slot] += (ch / 128.0) * 1.6 * (ch / 4096.0) ** 0.5

    def sweep_on(name: str, a: str, slot: int) -> None:
        side = ob.streams[slot]
        if slot != slot_of[a]:
            side.wait_event(done[a])
        prune.obs_sweep(st.weights[name], ob.hessian[a], float(sparsities[st.names.index(name)]),
                        w_out=None if in_place else st.pruned[name], dead=ob.dead[a],
                        mask_bits=st.mask_bits.get(name), ws=ob.ws[slot], stream=side)
        load[slot] += sweep_cost(name)

    for a in names:                                   # the largest reader of an input stays with its factorisation
        if readers[a]:
            sweep_on(readers[a][0], a, slot_of[a])
    rest = sorted(((n, a) for a in names for n in readers[a][1:]), key=lambda na: -sweep_cost(na[0]))
    for name, a in rest:
        sweep_on(name, a, min(range(n_side), key=lambda j: load[j]))
    for i in range(n_side):
        fin = torch.cuda.Event()
        fin.record(ob.streams[i])
        main.wait_event(fin)
    st.rowsq_valid = False


# ----------------------------------------------------------------------------------------------------------------
# Forward pass of one layer: the four activation tensors the projections' statistics are taken from come out of the
# layer itself instead of being injected.

def layer_forward(weights: Dict[str, torch.Tensor], norms: Dict[str, torch.Tensor], x: torch.Tensor, n_seqs: int,
                  seq_len: int, heads: int, kv_heads: int, head_dim: int, eps: float = 1e-5, base: float = 10000.0,
                  down_sumsq: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """x [n_seqs * seq_len, hidden] -> {"attn_in", "o_in", "mlp_in", "down_in", "out"}.

    weights: the seven projections; norms: {"attn_norm", "mlp_norm"} weight vectors.  down_sumsq (fp32 [inter])
    receives the channel sums of squares of down_in from the epilogue of the product that creates it."""
    attn_in = prune.rmsnorm(x, norms["attn_norm"], eps)
    q, k, v = (prune.linear(attn_in, weights[n]) for n in ("q", "k", "v"))
    prune.rotary(q, heads, head_dim, seq_len, base)
    prune.rotary(k, kv_heads, head_dim, seq_len, base)
    o_in = prune.causal_attention(q, k, v, n_seqs, seq_len, heads, kv_heads, head_dim)
    x1 = prune.add(x, prune.linear(o_in, weights["o"]))
    mlp_in = prune.rmsnorm(x1, norms["mlp_norm"], eps)
    down_in = prune.mlp_gate_up(mlp_in, weights["gate"], weights["up"], sumsq=down_sumsq)
    out = prune.add(x1, prune.linear(down_in, weights["down"]))
    return {"attn_in": attn_in, "o_in": o_in, "mlp_in": mlp_in, "down_in": down_in, "out": out,
            "q": q, "k": k, "v": v, "x1": x1}
