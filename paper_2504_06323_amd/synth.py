"""Seeded synthetic inputs: LLaMA-shaped projection weights and calibration activations.

This module only manufactures input bytes.  It holds none of the pruning
method's arithmetic (no norms, scores, thresholds, selections) so that both the
HIP path and the CPU oracle can be fed from it without sharing any method code.

Shapes follow the model table of the paper (Table 2: layers / attention dim /
feed-forward dim) and its calibration set shape (128 samples x 2048 tokens,
Section 4.1.4 "Calibration").  The trained checkpoints and the calibration
corpus are not available, so random tensors with planted heavy-tailed outlier
channels stand in for them.

Every tensor is a pure function of (SEED_BASE, config id, layer, tensor id,
chunk id) and of the device kind it is generated on; a test always hands the
*same bytes* to both sides, so generator arithmetic never enters parity.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import torch

SEED_BASE = 250406323

_MASK64 = (1 << 64) - 1


def _mix64(x: int) -> int:
    """splitmix64 finaliser on a Python int (seed derivation only)."""
    x = (x + 0x9E3779B97F4A7C15) & _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def stream_seed(config_id: int, layer: int, tensor_id: int, chunk: int = 0) -> int:
    """Seed of one tensor (or one chunk of it): a hash of the five integers."""
    h = _mix64(SEED_BASE)
    for v in (config_id, layer, tensor_id, chunk):
        h = _mix64(h ^ (v & _MASK64))
    return h & ((1 << 63) - 1)


@dataclass(frozen=True)
class LayerConfig:
    """One synthetic workload: shapes, distributions and pruning parameters."""

    config_id: int
    name: str
    dtype: torch.dtype
    hidden: int
    q_out: int           # rows of q (and columns of o)
    kv_out: int          # rows of k and v (smaller than q_out with grouped-query attention)
    inter: int           # MLP intermediate width
    n_layers: int
    n_seqs: int
    seq_len: int
    w_outlier_frac: float
    w_outlier_kind: str  # "scale10" (columns x10) or "student_t3" (columns redrawn heavy-tailed)
    x_outlier_frac: float
    x_outlier_scale: float
    p: float             # unstructured target sparsity
    alpha: float = 5.0   # outlier threshold multiplier of Eq. 6
    lam: float = 0.08    # planner spread (free parameter, not a value from the paper)
    struct_frac: float = 0.0  # fraction of MLP channels removed structurally (composite mode)
    p_sweep: Tuple[float, ...] = field(default_factory=tuple)

    @property
    def n_tokens(self) -> int:
        return self.n_seqs * self.seq_len


_BF16 = torch.bfloat16
_F32 = torch.float32

CONFIGS: Dict[str, LayerConfig] = {
    # configs[0]: toy layer, fp32, the oracle finishes it in well under a second
    "toy": LayerConfig(0, "toy", _F32, 256, 256, 256, 688, 1, 4, 128,
                       0.02, "scale10", 0.01, 20.0, 0.5, struct_frac=0.2),
    # configs[1]: one LLaMA-7B-shaped layer, the workload the headline metric is quoted on
    "llama7b_layer": LayerConfig(1, "llama7b_layer", _BF16, 4096, 4096, 4096, 11008, 1, 128, 2048,
                                 0.005, "student_t3", 0.001, 50.0, 0.5, struct_frac=0.2),
    # configs[2]: one LLaMA-3-8B-shaped layer with grouped-query attention, composite mode
    "llama3_8b_layer": LayerConfig(2, "llama3_8b_layer", _BF16, 4096, 4096, 1024, 14336, 1, 128, 2048,
                                   0.005, "student_t3", 0.001, 50.0, 0.5, struct_frac=0.2),
    # configs[3]: the full 32-layer 8B-shaped model, sparsity sweep reusing the ranking phase
    "llama3_8b_full": LayerConfig(3, "llama3_8b_full", _BF16, 4096, 4096, 1024, 14336, 32, 128, 2048,
                                  0.005, "student_t3", 0.001, 50.0, 0.5, struct_frac=0.0,
                                  p_sweep=(0.3, 0.5, 0.7)),
    # configs[4]: LLaMA-2-13B-shaped stress layers, long calibration, x100 activation outliers
    "llama2_13b_stress": LayerConfig(4, "llama2_13b_stress", _BF16, 5120, 5120, 5120, 13824, 40, 256, 4096,
                                     0.005, "student_t3", 0.001, 100.0, 0.6, struct_frac=0.3),
}

# tensor ids inside a layer (used only for seeding)
_PROJ_IDS = {"q": 0, "k": 1, "v": 2, "o": 3, "gate": 4, "up": 5, "down": 6}
_INPUT_IDS = {"attn_in": 16, "o_in": 17, "mlp_in": 18, "down_in": 19}

PROJ_NAMES: Tuple[str, ...] = ("q", "k", "v", "o", "gate", "up", "down")


def projection_shapes(cfg: LayerConfig) -> List[Tuple[str, int, int, str]]:
    """(name, rows=out features, cols=in features, name of the activation it multiplies).

    q/k/v read the same tensor and so do gate/up, hence four distinct
    activation tensors per layer for seven projections.
    """
    h, qo, kvo, it = cfg.hidden, cfg.q_out, cfg.kv_out, cfg.inter
    return [
        ("q", qo, h, "attn_in"),
        ("k", kvo, h, "attn_in"),
        ("v", kvo, h, "attn_in"),
        ("o", h, qo, "o_in"),
        ("gate", it, h, "mlp_in"),
        ("up", it, h, "mlp_in"),
        ("down", h, it, "down_in"),
    ]


def activation_shapes(cfg: LayerConfig) -> Dict[str, int]:
    """Channel count of each distinct activation tensor of a layer."""
    return {"attn_in": cfg.hidden, "o_in": cfg.q_out, "mlp_in": cfg.hidden, "down_in": cfg.inter}


def _generator(device: torch.device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def outlier_count(frac: float, n: int) -> int:
    return max(1, int(round(frac * n)))


def _outlier_indices(n: int, frac: float, seed: int) -> torch.Tensor:
    """First entries of a seeded permutation (always drawn on the host)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randperm(n, generator=g)[: outlier_count(frac, n)]


def make_weight(cfg: LayerConfig, layer: int, proj: str, device="cpu") -> torch.Tensor:
    """Projection weight [rows, cols], iid N(0, 0.02^2) with planted outlier input channels."""
    device = torch.device(device)
    rows, cols = {n: (r, c) for n, r, c, _ in projection_shapes(cfg)}[proj]
    tid = _PROJ_IDS[proj]
    g = _generator(device, stream_seed(cfg.config_id, layer, tid, 0))
    w = torch.empty((rows, cols), dtype=torch.float32, device=device)
    w.normal_(0.0, 0.02, generator=g)
    idx = _outlier_indices(cols, cfg.w_outlier_frac, stream_seed(cfg.config_id, layer, tid, 1)).to(device)
    if cfg.w_outlier_kind == "scale10":
        w[:, idx] *= 10.0
    elif cfg.w_outlier_kind == "student_t3":
        z = torch.empty((4, rows, idx.numel()), dtype=torch.float32, device=device)
        z.normal_(0.0, 1.0, generator=g)
        t3 = z[0] / torch.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0)
        w[:, idx] = 0.02 * t3
    else:
        raise ValueError(cfg.w_outlier_kind)
    return w.to(cfg.dtype).contiguous()


def make_activation(cfg: LayerConfig, layer: int, which: str, device="cpu",
                    n_seqs: Optional[int] = None, seqs_per_chunk: int = 16) -> torch.Tensor:
    """Calibration activation [n_seqs * seq_len, channels], iid N(0,1) with scaled outlier channels.

    Generated chunk by chunk (a chunk is `seqs_per_chunk` sequences) so the
    temporary footprint stays small for multi-GB tensors.
    """
    device = torch.device(device)
    ch = activation_shapes(cfg)[which]
    tid = _INPUT_IDS[which]
    n_seqs = cfg.n_seqs if n_seqs is None else n_seqs
    t_total = n_seqs * cfg.seq_len
    x = torch.empty((t_total, ch), dtype=cfg.dtype, device=device)
    idx = _outlier_indices(ch, cfg.x_outlier_frac, stream_seed(cfg.config_id, layer, tid, 1 << 20)).to(device)
    for c, s0 in enumerate(range(0, n_seqs, seqs_per_chunk)):
        s1 = min(n_seqs, s0 + seqs_per_chunk)
        g = _generator(device, stream_seed(cfg.config_id, layer, tid, c))
        blk = x[s0 * cfg.seq_len: s1 * cfg.seq_len]
        blk.normal_(0.0, 1.0, generator=g)
        blk[:, idx] *= cfg.x_outlier_scale
    return x


def layer_numel(cfg: LayerConfig) -> int:
    return sum(r * c for _, r, c, _ in projection_shapes(cfg))


def random_matrix(rows: int, cols: int, dtype: torch.dtype, seed: int, device="cpu",
                  scale: float = 1.0, zero_frac: float = 0.0) -> torch.Tensor:
    """Free-form seeded matrix for edge-case tests (ragged shapes, planted zeros)."""
    device = torch.device(device)
    g = _generator(device, stream_seed(99, 0, seed, 0))
    m = torch.empty((rows, cols), dtype=torch.float32, device=device)
    m.normal_(0.0, scale, generator=g)
    if zero_frac > 0.0:
        u = torch.empty((rows, cols), dtype=torch.float32, device=device)
        u.uniform_(0.0, 1.0, generator=g)
        m[u < zero_frac] = 0.0
    return m.to(dtype).contiguous()
