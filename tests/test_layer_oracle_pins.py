"""Pins for the attention-half oracle."""
import numpy as np
import pytest

from oracle import layer_oracle as lay


def test_rmsnorm_hand_example_and_scale_invariance():
    x = np.array([[3.0, 4.0]])                                   # mean of squares 12.5
    got = lay.rmsnorm(x, np.array([2.0, 0.5]), eps=0.0)
    assert np.allclose(got, [[3.0 / np.sqrt(12.5) * 2.0, 4.0 / np.sqrt(12.5) * 0.5]], rtol=1e-15)
    rng = np.random.default_rng(0)
    x, w = rng.standard_normal((5, 16)), rng.standard_normal(16)
    assert np.allclose(lay.rmsnorm(7.0 * x, w, eps=0.0), lay.rmsnorm(x, w, eps=0.0), rtol=1e-12)
    assert np.allclose(np.mean(lay.rmsnorm(x, np.ones(16), eps=0.0) ** 2, axis=1), 1.0, rtol=1e-12)


def test_rotary_identity_norm_and_relative_position():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((6, 2, 8)), rng.standard_normal((6, 2, 8))
    pos = np.arange(6)
    rq, rk = lay.rotary(q, pos), lay.rotary(k, pos)
    assert np.allclose(rq[0], q[0], rtol=1e-15)                                     # position 0: no turn
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    # the score of a (query, key) pair depends on the positions only through their difference
    shifted_q, shifted_k = lay.rotary(q, pos + 11), lay.rotary(k, pos + 11)
    assert np.allclose(np.einsum("shd,thd->hst", rq, rk), np.einsum("shd,thd->hst", shifted_q, shifted_k), rtol=1e-10)
    # hand value: d = 2, one pair, angle = position (base^0 = 1): (1, 0) at position 1 -> (cos 1, sin 1)
    assert np.allclose(lay.rotary(np.array([[[1.0, 0.0]]]), np.array([1.0])), [[[np.cos(1.0), np.sin(1.0)]]], rtol=1e-15)


def test_causal_attention_brute_force_and_special_cases():
    rng = np.random.default_rng(2)
    q, k, v = rng.standard_normal((5, 4, 8)), rng.standard_normal((5, 2, 8)), rng.standard_normal((5, 2, 8))
    got = lay.causal_attention(q, k, v)
    for s in range(5):
        for h in range(4):
            g = h // 2
            e = [np.exp(np.dot(q[s, h], k[t, g]) / np.sqrt(8.0)) for t in range(s + 1)]
            want = sum(e[t] * v[t, g] for t in range(s + 1)) / sum(e)
            assert np.allclose(got[s, h], want, rtol=1e-12)
    assert np.allclose(got[0], v[0][[0, 0, 1, 1]], rtol=1e-14)                     # the first token sees only itself
    flat = lay.causal_attention(np.zeros_like(q), k, v)                          # equal scores: the running mean of v
    assert np.allclose(flat[3, 0], v[:4, 0].mean(axis=0), rtol=1e-13)
    assert np.allclose(got, lay.causal_attention(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)), rtol=1e-14)


def test_layer_forward_composition():
    from oracle import mlp_oracle as mlp
    rng = np.random.default_rng(3)
    n_seqs, seq_len, heads, kv_heads, d, hidden, inter = 2, 5, 2, 1, 4, 8, 12
    w = {"attn_norm": rng.standard_normal(hidden), "mlp_norm": rng.standard_normal(hidden),
         "q": rng.standard_normal((heads * d, hidden)), "k": rng.standard_normal((kv_heads * d, hidden)),
         "v": rng.standard_normal((kv_heads * d, hidden)), "o": rng.standard_normal((hidden, heads * d)),
         "gate": rng.standard_normal((inter, hidden)), "up": rng.standard_normal((inter, hidden)),
         "down": rng.standard_normal((hidden, inter))}
    x = rng.standard_normal((n_seqs * seq_len, hidden))
    out = lay.layer_forward(x, w, n_seqs, seq_len, heads, kv_heads, d)
    assert np.allclose(out["attn_in"], lay.rmsnorm(x, w["attn_norm"]))
    # the feed-forward part is the feed-forward oracle on the normalised residual stream
    x1 = x + out["o_in"] @ w["o"].T
    assert np.allclose(out["mlp_in"], lay.rmsnorm(x1, w["mlp_norm"]), rtol=1e-13)
    assert np.allclose(out["down_in"], mlp.mlp_hidden(out["mlp_in"], w["gate"], w["up"]), rtol=1e-13)
    assert np.allclose(out["out"], x1 + mlp.mlp_forward(out["mlp_in"], w["gate"], w["up"], w["down"]), rtol=1e-12)
    # sequences do not see each other: the second sequence alone gives the same rows
    alone = lay.layer_forward(x[seq_len:], w, 1, seq_len, heads, kv_heads, d)
    assert np.allclose(alone["out"], out["out"][seq_len:], rtol=1e-12)
    # with the o and down projections zeroed the residual stream passes through
    w0 = dict(w, o=np.zeros_like(w["o"]), down=np.zeros_like(w["down"]))
    assert np.allclose(lay.layer_forward(x, w0, n_seqs, seq_len, heads, kv_heads, d)["out"], x, rtol=1e-15)
