"""GPU parity of the attention-half kernels (rmsnorm, rotary embedding, causal attention) against oracle/layer_oracle.py."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as lay
from paper_2504_06323_amd import prune, synth
from util import to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ULP = {torch.bfloat16: 2.0 ** -8, torch.float32: 2.0 ** -22}


def _sync():
    torch.cuda.synchronize()


def _mat(rows, cols, dtype, seed, scale=1.0):
    return synth.random_matrix(rows, cols, dtype, seed=seed, device=DEV, scale=scale)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape", [(37, 256), (512, 4096), (5, 100)])
def test_rmsnorm_vs_oracle(lib, dtype, shape):
    tokens, channels = shape
    x = _mat(tokens, channels, dtype, 1, 3.0)
    w = _mat(1, channels, dtype, 2, 1.0).reshape(-1).contiguous()
    y = prune.rmsnorm(x, w, eps=1e-5)
    _sync()
    want = lay.rmsnorm(to_np(x), to_np(w), 1e-5)
    assert np.max(np.abs(to_np(y).astype(np.float64) - want) / (ULP[dtype] * np.abs(want) + 1e-6)) < 1.0


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_rotary_vs_oracle(lib, dtype):
    n_seqs, seq_len, heads, d = 3, 200, 4, 64
    x = _mat(n_seqs * seq_len, heads * d, dtype, 3)
    x0 = to_np(x).astype(np.float64).reshape(n_seqs * seq_len, heads, d)
    prune.rotary(x, heads, d, seq_len)
    _sync()
    pos = np.tile(np.arange(seq_len), n_seqs)
    want = lay.rotary(x0, pos).reshape(n_seqs * seq_len, heads * d)
    # fp32 angles up to 199 rad (relative error 2^-24 of the angle), then one rounding to dtype
    assert np.max(np.abs(to_np(x).astype(np.float64) - want)) <= (ULP[dtype] + 5e-5) * np.max(np.abs(want))


def _attention_case(dtype, n_seqs, seq_len, heads, kv_heads, d, seed, elem_ulp=2.0 ** -8):
    tokens = n_seqs * seq_len
    q, k, v = _mat(tokens, heads * d, dtype, seed), _mat(tokens, kv_heads * d, dtype, seed + 1), _mat(tokens, kv_heads * d, dtype, seed + 2)
    o = prune.causal_attention(q, k, v, n_seqs, seq_len, heads, kv_heads, d)
    _sync()
    got = to_np(o).astype(np.float64).reshape(n_seqs, seq_len, heads, d)
    q64, k64, v64 = (to_np(t).astype(np.float64) for t in (q, k, v))
    worst, worst_elem = 0.0, 0.0
    for b in range(n_seqs):
        sl = slice(b * seq_len, (b + 1) * seq_len)
        q3, k3 = q64[sl].reshape(seq_len, heads, d), k64[sl].reshape(seq_len, kv_heads, d)
        want = lay.causal_attention(q3, k3, v64[sl].reshape(seq_len, kv_heads, d))
        # the same probabilities applied to |v|: the scale of what was added up for each output element
        mix = lay.causal_attention(q3, k3, np.abs(v64[sl]).reshape(seq_len, kv_heads, d))
        err = np.abs(got[b] - want)
        worst = max(worst, float(np.max(err)))
        worst_elem = max(worst_elem, float(np.max(err / (elem_ulp * (np.abs(want) + mix) + 1e-30))))
    return worst, float(np.max(np.abs(v64))), worst_elem


@pytest.mark.parametrize("dtype,case", [(torch.bfloat16, (2, 100, 4, 2, 64)), (torch.float32, (2, 100, 4, 2, 64)),
                                        (torch.bfloat16, (1, 70, 3, 3, 40)), (torch.float32, (1, 70, 3, 3, 40)),
                                        (torch.float32, (2, 64, 2, 1, 128))])
def test_attention_plain_kernel_vs_oracle(lib, dtype, case):
    """Shapes that take the any-shape kernel (fp32, or heads that are not 128 wide)."""
    worst, vmax, _ = _attention_case(dtype, *case, seed=10)
    assert worst <= (ULP[dtype] + 2e-5) * vmax * 4


@pytest.mark.parametrize("case", [(2, 256, 4, 2, 128), (1, 384, 2, 2, 128), (3, 200, 4, 1, 128), (1, 128, 1, 1, 128),
                                  (2, 2048, 2, 1, 128), (3, 1024, 8, 2, 128), (1, 1000, 4, 4, 128)])
def test_attention_matrix_core_kernel_vs_oracle(lib, case):
    """bf16, 128-wide heads.  Probabilities enter the second product as bf16 (half an ulp each, averaging out over
    the keys of a query) and the output is rounded to bf16."""
    worst, vmax, worst_elem = _attention_case(torch.bfloat16, *case, seed=20)
    assert worst <= 2.0 ** -7 * vmax
    # element by element: the rounding of the output (half a bf16 ulp of its value) plus the rounding of the
    # probabilities that entered the second product as bf16 (half an ulp each, of sum_t p_t |v_t|), 2^-8 for both
    assert worst_elem <= 1.0, worst_elem
    q = _mat(case[0] * case[1], case[2] * 128, torch.bfloat16, 30)
    k = _mat(case[0] * case[1], case[3] * 128, torch.bfloat16, 31)
    v = _mat(case[0] * case[1], case[3] * 128, torch.bfloat16, 32)
    a = prune.causal_attention(q, k, v, *case)
    b = prune.causal_attention(q, k, v, *case)
    _sync()
    assert torch.equal(a, b)


@pytest.mark.parametrize("dtype,dims", [(torch.float32, (2, 96, 4, 2, 64, 256, 688)),       # the toy layer's widths: plain kernels
                                        (torch.bfloat16, (2, 256, 4, 2, 128, 512, 1024))])  # matrix-core kernels throughout
def test_layer_forward_stage_by_stage(lib, dtype, dims):
    """pipeline.layer_forward against the oracle, stage by stage: every stage is checked on the previous stage's
    stored output (so roundings to the storage type do not pile up in the comparison), and the fused statistic of
    the down projection's input against the oracle's column sums of squares."""
    from oracle import mlp_oracle as mlp
    from oracle import mosaic_oracle as orc
    from paper_2504_06323_amd import pipeline
    n_seqs, seq_len, heads, kv_heads, d, hidden, inter = dims
    tokens = n_seqs * seq_len
    w = {"q": _mat(heads * d, hidden, dtype, 40, 0.05), "k": _mat(kv_heads * d, hidden, dtype, 41, 0.05),
         "v": _mat(kv_heads * d, hidden, dtype, 42, 0.05), "o": _mat(hidden, heads * d, dtype, 43, 0.05),
         "gate": _mat(inter, hidden, dtype, 44, 0.05), "up": _mat(inter, hidden, dtype, 45, 0.05),
         "down": _mat(hidden, inter, dtype, 46, 0.05)}
    norms = {"attn_norm": (1.0 + 0.1 * _mat(1, hidden, torch.float32, 47)).to(dtype).reshape(-1).contiguous(),
             "mlp_norm": (1.0 + 0.1 * _mat(1, hidden, torch.float32, 48)).to(dtype).reshape(-1).contiguous()}
    x = _mat(tokens, hidden, dtype, 49)
    sumsq = torch.zeros(inter, dtype=torch.float32, device=DEV)
    got = pipeline.layer_forward(w, norms, x, n_seqs, seq_len, heads, kv_heads, d, down_sumsq=sumsq)
    _sync()
    f = lambda t: to_np(t).astype(np.float64)
    tol = 2.0 ** -7 if dtype == torch.bfloat16 else 2e-5

    def check(name, want):
        err = np.max(np.abs(f(got[name]) - want)) / np.max(np.abs(want))
        assert err < tol, (name, err)

    pos = np.tile(np.arange(seq_len), n_seqs)
    check("attn_in", lay.rmsnorm(f(x), f(norms["attn_norm"])))
    a = f(got["attn_in"])
    check("q", lay.rotary((a @ f(w["q"]).T).reshape(tokens, heads, d), pos).reshape(tokens, -1))
    check("k", lay.rotary((a @ f(w["k"]).T).reshape(tokens, kv_heads, d), pos).reshape(tokens, -1))
    check("v", a @ f(w["v"]).T)
    q3, k3, v3 = f(got["q"]).reshape(tokens, heads, d), f(got["k"]).reshape(tokens, kv_heads, d), f(got["v"]).reshape(tokens, kv_heads, d)
    check("o_in", np.concatenate([lay.causal_attention(q3[b * seq_len:(b + 1) * seq_len], k3[b * seq_len:(b + 1) * seq_len],
                                                       v3[b * seq_len:(b + 1) * seq_len]) for b in range(n_seqs)]).reshape(tokens, -1))
    check("x1", f(x) + f(got["o_in"]) @ f(w["o"]).T)
    check("mlp_in", lay.rmsnorm(f(got["x1"]), f(norms["mlp_norm"])))
    check("down_in", mlp.mlp_hidden(f(got["mlp_in"]), f(w["gate"]), f(w["up"])))
    check("out", f(got["x1"]) + f(got["down_in"]) @ f(w["down"]).T)
    want_sq = orc.column_sumsq(f(got["down_in"]))
    assert np.max(np.abs(to_np(sumsq) - want_sq) / np.maximum(want_sq, 1e-30)) < 1e-5
    # and the whole layer at once against the oracle's own forward pass (roundings accumulate: looser)
    whole = lay.layer_forward(f(x), {**{n: f(t) for n, t in w.items()}, **{n: f(t) for n, t in norms.items()}}, n_seqs,
                              seq_len, heads, kv_heads, d)
    for name in ("attn_in", "o_in", "mlp_in", "down_in", "out"):
        err = np.max(np.abs(f(got[name]) - whole[name])) / np.max(np.abs(whole[name]))
        assert err < 8 * tol, (name, err)
