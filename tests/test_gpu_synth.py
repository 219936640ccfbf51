"""The synthetic-input generator on the GPU gives the bytes its NumPy twin gives on the host."""
import numpy as np
import pytest
import torch

from paper_2504_06323_amd import counter_rng as cr
from paper_2504_06323_amd import synth

pytestmark = pytest.mark.gpu


def _bytes(t):
    return t.detach().cpu().contiguous().view(torch.uint8).numpy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 5), (257, 1023), (1024, 4096)])
def test_plain_normals_host_and_device_agree(dtype, rows, cols):
    dev = torch.device("cuda:0")
    seed = synth.stream_seed(7, rows, cols, 0)
    a = synth._fill(rows, cols, dtype, torch.device("cpu"), seed, 0.02, None, None)
    b = synth._fill(rows, cols, dtype, dev, seed, 0.02, None, None)
    torch.cuda.synchronize()
    assert np.array_equal(_bytes(a), _bytes(b))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_column_scales_and_student_t_columns_agree(dtype):
    dev = torch.device("cuda:0")
    rows, cols = 777, 1030
    rng = np.random.default_rng(5)
    scale = rng.uniform(0.5, 50.0, cols).astype(np.float32)
    kind = (rng.uniform(size=cols) < 0.05).astype(np.uint8)
    kind[[0, cols - 1]] = 1
    seed = synth.stream_seed(8, 0, 0, 0)
    a = synth._fill(rows, cols, dtype, torch.device("cpu"), seed, 0.3, scale, kind)
    b = synth._fill(rows, cols, dtype, dev, seed, 0.3, scale, kind)
    torch.cuda.synchronize()
    assert np.array_equal(_bytes(a), _bytes(b))


def test_uniform_bits_agree():
    n = 100003
    raw = torch.empty(n, dtype=torch.int32, device="cuda:0")
    assert cr.device_lib().synth_fill_bits(raw.data_ptr(), n, 1234567, 9, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert np.array_equal(raw.cpu().numpy().view(np.uint32), cr.bits32(n, 9, 1234567))


def test_workload_tensors_are_the_same_bytes_on_both_sides():
    cfg = synth.CONFIGS["toy"]
    for proj in ("q", "gate", "down"):
        assert np.array_equal(_bytes(synth.make_weight(cfg, 1, proj, "cpu")), _bytes(synth.make_weight(cfg, 1, proj, "cuda:0")))
    assert np.array_equal(_bytes(synth.make_activation(cfg, 1, "down_in", "cpu")),
                          _bytes(synth.make_activation(cfg, 1, "down_in", "cuda:0")))
    big = synth.CONFIGS["llama3_8b_layer"]          # bf16, Student-t outlier columns, 4096 x 1024 rows of k
    assert np.array_equal(_bytes(synth.make_weight(big, 0, "k", "cpu")), _bytes(synth.make_weight(big, 0, "k", "cuda:0")))
    a = synth.random_matrix(129, 515, torch.bfloat16, 3, "cpu", scale=2.0, zero_frac=0.2)
    b = synth.random_matrix(129, 515, torch.bfloat16, 3, "cuda:0", scale=2.0, zero_frac=0.2)
    assert np.array_equal(_bytes(a), _bytes(b))


def test_bad_arguments_are_refused():
    lib = cr.device_lib()
    out = torch.empty(16, dtype=torch.float32, device="cuda:0")
    assert lib.synth_fill_normal(None, 0, 4, 4, 4, 1, 0, None, None, 1.0, None) == -1
    assert lib.synth_fill_normal(out.data_ptr(), 0, 4, 4, 3, 1, 0, None, None, 1.0, None) == -1
    assert lib.synth_fill_normal(out.data_ptr(), 2, 4, 4, 4, 1, 0, None, None, 1.0, None) == -1
    assert lib.synth_fill_normal(out.data_ptr(), 0, 0, 4, 4, 1, 0, None, None, 1.0, None) == 0
    assert lib.synth_fill_bits(None, 4, 1, 0, None) == -1
