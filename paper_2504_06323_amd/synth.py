"""Seeded synthetic inputs: LLaMA-shaped projection weights and calibration activations.

This module only manufactures input bytes.  It holds none of the pruning
method's arithmetic (no norms, scores, thresholds, selections) so that both the
HIP path and the CPU oracle can be fed from it without sharing any method code.

Shapes follow the model table of the paper (Table 2: layers / attention dim /
feed-forward dim) and its calibration set shape (128 samples x 2048 tokens,
Section 4.1.4 "Calibration").  The trained checkpoints and the calibration
corpus are not available, so random tensors with planted heavy-tailed outlier
channels stand in for them.

Every tensor is a pure function of (SEED_BASE, config id, layer, tensor id):
the random numbers come from the counter-based generator of counter_rng.py,
which exists as NumPy code (tensors asked for on the host) and as a HIP kernel
(tensors asked for on the GPU) with identical results, so the same call gives
the same bytes wherever it runs.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

from . import counter_rng

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


def outlier_count(frac: float, n: int) -> int:
    return max(1, int(round(frac * n)))


def _outlier_indices(n: int, frac: float, seed: int) -> np.ndarray:
    """The first entries of a seeded permutation of 0 .. n-1 (a partial Fisher-Yates shuffle, always on the host)."""
    m = outlier_count(frac, n)
    draws = counter_rng.bits32(m, 0, seed)
    perm = np.arange(n, dtype=np.int64)
    for j in range(m):
        t = j + int(draws[j]) % (n - j)
        perm[j], perm[t] = perm[t], perm[j]
    return perm[:m].copy()


_HOST_CHUNK_ROWS_ELEMS = 1 << 22   # elements generated per NumPy pass on the host (bounds the float64 temporaries)


def _fill(rows: int, cols: int, dtype: torch.dtype, device: torch.device, seed: int, scale: float,
          col_scale: Optional[np.ndarray], kind: Optional[np.ndarray]) -> torch.Tensor:
    """[rows, cols] tensor of the generator's values (see counter_rng.fill_normal_host for the element rule)."""
    if dtype not in (torch.float32, torch.bfloat16):
        raise ValueError(f"unsupported dtype {dtype}")
    if device.type == "cpu":
        out = torch.empty((rows, cols), dtype=dtype)
        step = max(1, _HOST_CHUNK_ROWS_ELEMS // max(cols, 1))
        for r0 in range(0, rows, step):
            r1 = min(rows, r0 + step)
            blk = counter_rng.fill_normal_host(r1 - r0, cols, seed, 0, scale, col_scale, kind, first_row=r0)
            out[r0:r1] = torch.from_numpy(blk).to(dtype)   # float32 -> bfloat16 rounds to nearest even, as the kernel does
        return out
    lib = counter_rng.device_lib()
    with torch.cuda.device(device):
        out = torch.empty((rows, cols), dtype=dtype, device=device)
        cs = None if col_scale is None else torch.from_numpy(np.ascontiguousarray(col_scale, dtype=np.float32)).to(device)
        kd = None if kind is None else torch.from_numpy(np.ascontiguousarray(kind, dtype=np.uint8)).to(device)
        rc = lib.synth_fill_normal(out.data_ptr(), 1 if dtype == torch.bfloat16 else 0, rows, cols, cols, seed, 0,
                                   None if cs is None else cs.data_ptr(), None if kd is None else kd.data_ptr(),
                                   float(scale), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError("synth_fill_normal refused its arguments or the launch failed")
        if cs is not None:
            cs.record_stream(torch.cuda.current_stream())
        if kd is not None:
            kd.record_stream(torch.cuda.current_stream())
    return out


def make_weight(cfg: LayerConfig, layer: int, proj: str, device="cpu") -> torch.Tensor:
    """Projection weight [rows, cols], iid N(0, 0.02^2) with planted outlier input channels: columns ten times
    larger ("scale10") or drawn from a Student-t law with three degrees of freedom ("student_t3")."""
    device = torch.device(device)
    rows, cols = {n: (r, c) for n, r, c, _ in projection_shapes(cfg)}[proj]
    tid = _PROJ_IDS[proj]
    idx = _outlier_indices(cols, cfg.w_outlier_frac, stream_seed(cfg.config_id, layer, tid, 1))
    col_scale = kind = None
    if cfg.w_outlier_kind == "scale10":
        col_scale = np.ones(cols, dtype=np.float32)
        col_scale[idx] = 10.0
    elif cfg.w_outlier_kind == "student_t3":
        kind = np.zeros(cols, dtype=np.uint8)
        kind[idx] = 1
    else:
        raise ValueError(cfg.w_outlier_kind)
    return _fill(rows, cols, cfg.dtype, device, stream_seed(cfg.config_id, layer, tid, 0), 0.02, col_scale, kind)


def make_activation(cfg: LayerConfig, layer: int, which: str, device="cpu",
                    n_seqs: Optional[int] = None) -> torch.Tensor:
    """Calibration activation [n_seqs * seq_len, channels], iid N(0,1) with scaled outlier channels.  A tensor of
    fewer sequences is a prefix of the full one."""
    device = torch.device(device)
    ch = activation_shapes(cfg)[which]
    tid = _INPUT_IDS[which]
    n_seqs = cfg.n_seqs if n_seqs is None else n_seqs
    idx = _outlier_indices(ch, cfg.x_outlier_frac, stream_seed(cfg.config_id, layer, tid, 1))
    col_scale = np.ones(ch, dtype=np.float32)
    col_scale[idx] = cfg.x_outlier_scale
    return _fill(n_seqs * cfg.seq_len, ch, cfg.dtype, device, stream_seed(cfg.config_id, layer, tid, 0), 1.0,
                 col_scale, None)


def layer_numel(cfg: LayerConfig) -> int:
    return sum(r * c for _, r, c, _ in projection_shapes(cfg))


def random_matrix(rows: int, cols: int, dtype: torch.dtype, seed: int, device="cpu",
                  scale: float = 1.0, zero_frac: float = 0.0) -> torch.Tensor:
    """Free-form seeded matrix for edge-case tests (ragged shapes, planted zeros): N(0, scale^2) entries, each
    replaced by zero when its 32-bit draw from a second seed falls below zero_frac * 2^32."""
    device = torch.device(device)
    if rows == 0 or cols == 0:
        return torch.zeros((rows, cols), dtype=dtype, device=device)
    m = _fill(rows, cols, dtype, device, stream_seed(99, 0, seed, 0), scale, None, None)
    if zero_frac > 0.0:
        limit = min(int(zero_frac * 4294967296.0), 4294967295)
        zseed = stream_seed(99, 0, seed, 1)
        if device.type == "cpu":
            draws = torch.from_numpy(counter_rng.bits32(rows * cols, 0, zseed).astype(np.int64))
        else:
            with torch.cuda.device(device):
                raw = torch.empty(rows * cols, dtype=torch.int32, device=device)
                if counter_rng.device_lib().synth_fill_bits(raw.data_ptr(), rows * cols, zseed, 0,
                                                            torch.cuda.current_stream().cuda_stream) != 0:
                    raise RuntimeError("synth_fill_bits refused its arguments or the launch failed")
                draws = raw.to(torch.int64) & 0xFFFFFFFF
        m[(draws < limit).view(rows, cols)] = 0.0
    return m
