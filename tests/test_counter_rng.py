"""The counter-based generator of the synthetic inputs (host side): the published known-answer vectors of
Philox-4x32-10, the accuracy of the hand-written logarithm / sine / cosine, the law of the normals, and the
properties the input recipe relies on (prefixes, chunks, distinct outlier channels)."""
import ctypes
import os

import numpy as np
import pytest
import torch
from scipy import stats

from paper_2504_06323_amd import counter_rng as cr
from paper_2504_06323_amd import synth


def _one(v):
    return np.array([v], dtype=np.uint64)


# counter, key, output: the three test vectors published with the Random123 library for philox4x32 with 10 rounds
KAT = [
    ((0x00000000, 0x00000000, 0x00000000, 0x00000000), (0x00000000, 0x00000000),
     (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
    ((0xffffffff, 0xffffffff, 0xffffffff, 0xffffffff), (0xffffffff, 0xffffffff),
     (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
    ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
     (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)),
]


@pytest.mark.parametrize("ctr,key,want", KAT)
def test_philox_known_answers(ctr, key, want):
    got = cr.philox4x32_10_words(*[_one(c) for c in ctr], *key)
    assert tuple(int(g[0]) for g in got) == want


def test_stream_layout_is_counter_block_stream_zero():
    # element i of stream s with seed k: output i % 4 of counter (i // 4 low, i // 4 high, s, 0), key (k low, k high)
    seed, stream = 0x299f31d0a4093822, 0x13198a2e
    blocks = np.array([0x85a308d3243f6a88], dtype=np.uint64)
    got = cr.philox4x32_10(blocks, stream, seed)
    want = cr.philox4x32_10_words(_one(0x243f6a88), _one(0x85a308d3), _one(0x13198a2e), _one(0), 0xa4093822, 0x299f31d0)
    assert [int(g[0]) for g in got] == [int(w[0]) for w in want]
    bits = cr.bits32(10, 5, 77)
    four = cr.philox4x32_10(np.array([2], dtype=np.uint64), 5, 77)
    assert int(bits[9]) == int(four[1][0])


def test_logarithm_and_turn_functions_are_accurate():
    rng = np.random.default_rng(1)
    x = np.concatenate([np.array([0, 1, 2, 2 ** 31, 2 ** 32 - 1, 2 ** 30, 3 * 2 ** 30, 2 ** 30 - 1], dtype=np.uint64),
                        rng.integers(0, 2 ** 32, 200000, dtype=np.uint64)])
    ln = cr._ln_unit(x)
    ref = np.log((x.astype(np.float64) + 0.5) / 4294967296.0)
    assert np.max(np.abs(ln - ref) / np.maximum(np.abs(ref), 1e-300)) < 1e-15 or np.max(np.abs(ln - ref)) < 4e-16
    c, s = cr._cos_sin_turn(x)
    ang = 2.0 * np.pi * x.astype(np.float64) / 4294967296.0
    assert np.max(np.abs(c - np.cos(ang))) < 1e-15
    assert np.max(np.abs(s - np.sin(ang))) < 1e-15
    assert np.max(np.abs(c * c + s * s - 1.0)) < 1e-15


def test_normals_follow_the_standard_normal_law():
    z = cr.normals(1 << 21, 3, 12345)
    assert abs(z.mean()) < 4.0 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / z.size)
    assert abs(np.mean(z ** 4) - 3.0) < 0.03
    assert stats.kstest(z[:200000], "norm").pvalue > 1e-3
    # the four lanes of a block and neighbouring streams are uncorrelated
    q = z.reshape(-1, 4)
    assert np.max(np.abs(np.corrcoef(q.T) - np.eye(4))) < 0.01
    z2 = cr.normals(1 << 21, 4, 12345)
    assert abs(np.corrcoef(z, z2)[0, 1]) < 0.005


def test_prefix_chunk_and_gather_give_the_same_numbers():
    full = cr.normals(1000, 2, 9)
    assert np.array_equal(cr.normals(123, 2, 9, first=77), full[77:200])
    idx = np.array([[0, 999], [5, 6], [402, 3]])
    assert np.array_equal(cr.normals_at(idx, 2, 9), full[idx])
    kind = np.zeros(37, dtype=np.uint8)
    kind[[3, 30, 36]] = 1
    scale = np.linspace(0.5, 2.0, 37).astype(np.float32)
    whole = cr.fill_normal_host(10, 37, 5, 0, 0.02, scale, kind)
    parts = [cr.fill_normal_host(n, 37, 5, 0, 0.02, scale, kind, first_row=r0) for r0, n in ((0, 3), (3, 6), (9, 1))]
    assert np.array_equal(whole, np.concatenate(parts))


def test_student_t_columns_are_heavy_tailed_and_the_rest_normal():
    kind = np.zeros(8, dtype=np.uint8)
    kind[5] = 1
    m = cr.fill_normal_host(200000, 8, 4242, 0, 1.0, None, kind).astype(np.float64)
    assert stats.kstest(m[:, 5], "t", args=(3,)).pvalue > 1e-3
    assert stats.kstest(m[:, 2], "norm").pvalue > 1e-3
    assert np.abs(m[:, 5]).max() > 3.0 * np.abs(m[:, 2]).max()


def test_bf16_rounding_matches_the_tensor_library():
    f = cr.fill_normal_host(64, 333, 1, 0, 3.0)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(cr.to_bf16_bits(f), want)


def test_outlier_channels_are_distinct_and_seeded():
    for n, frac in ((256, 0.02), (4096, 0.005), (14336, 0.001), (7, 0.9)):
        idx = synth._outlier_indices(n, frac, 99)
        assert len(idx) == synth.outlier_count(frac, n) and len(set(idx.tolist())) == len(idx)
        assert idx.min() >= 0 and idx.max() < n
        assert np.array_equal(idx, synth._outlier_indices(n, frac, 99))
    assert not np.array_equal(synth._outlier_indices(4096, 0.005, 1), synth._outlier_indices(4096, 0.005, 2))


def test_toy_tensors_have_the_planted_structure():
    cfg = synth.CONFIGS["toy"]
    w = synth.make_weight(cfg, 0, "gate").double()
    col = w.pow(2).mean(0).sqrt()
    big = torch.nonzero(col > 0.1).flatten()
    assert big.numel() == synth.outlier_count(cfg.w_outlier_frac, cfg.hidden)
    assert torch.all((col[big] - 0.2).abs() < 0.03) and abs(float(col.median()) - 0.02) < 0.003
    x = synth.make_activation(cfg, 0, "mlp_in").double()
    colx = x.pow(2).mean(0).sqrt()
    assert int((colx > 5).sum()) == synth.outlier_count(cfg.x_outlier_frac, cfg.hidden)
    assert torch.equal(synth.make_activation(cfg, 0, "mlp_in", n_seqs=2), synth.make_activation(cfg, 0, "mlp_in")[: 2 * cfg.seq_len])
    assert not torch.equal(synth.make_weight(cfg, 0, "gate"), synth.make_weight(cfg, 1, "gate"))
    m = synth.random_matrix(50, 41, torch.float32, 7, zero_frac=0.3)
    assert 0.25 < float((m == 0).double().mean()) < 0.35
    assert synth.random_matrix(0, 5, torch.float32, 1).shape == (0, 5)


def test_device_generator_library_exports_its_entry_points():
    path = os.path.join(os.path.dirname(cr.__file__), "csrc", "libmosaic_synth.so")
    if not os.path.exists(path):
        pytest.skip("library not built")
    lib = ctypes.CDLL(path)
    for name in ("synth_fill_normal", "synth_fill_bits"):
        assert hasattr(lib, name)
