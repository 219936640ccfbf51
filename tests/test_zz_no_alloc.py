"""prune_stats_norms_static (scratch built into the library, nothing allocated) against prune_stats_norms
(caller's workspace): the same kernels on a different scratch address, so the outputs must agree bit for bit.
Two calls in a row, the second on a smaller input, so that what the first call left in the shared array is there
when the second runs."""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2504_06323_amd import prune, synth
from util import rel_err, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(x):
    c = x.shape[1]
    want_s, want_n = (torch.full((c,), float("nan"), dtype=torch.float32, device=DEV) for _ in range(2))
    got_s, got_n = (torch.full((c,), float("nan"), dtype=torch.float32, device=DEV) for _ in range(2))
    prune.stats_norms(x, want_s, want_n)
    prune.stats_norms_static(x, got_s, got_n)
    torch.cuda.synchronize()
    return (to_np(got_s), to_np(got_n)), (to_np(want_s), to_np(want_n))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_matches_workspace_variant_twice(lib, dtype):
    big = synth.random_matrix(5000, 4096, dtype, seed=41, device=DEV)
    big[:, 7] *= 50.0
    small = synth.random_matrix(333, 1000, dtype, seed=42, device=DEV)       # ragged, scalar path, fewer stripes
    for x in (big, small):
        (got_s, got_n), (want_s, want_n) = _both(x)
        assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32))
        assert np.array_equal(got_n.view(np.uint32), want_n.view(np.uint32))
        assert rel_err(got_n, orc.column_norms(to_np(x))) < (1e-5 if dtype == torch.float32 else 1e-2)
    # no tokens: zeros, whatever the array holds
    empty = big[:0]
    (got_s, got_n), _ = _both(empty)
    assert (got_s == 0).all() and (got_n == 0).all()


def test_static_scratch_rejects_what_does_not_fit(lib):
    x = torch.zeros((1, 8), dtype=torch.float32, device=DEV)
    out = torch.zeros(600000, dtype=torch.float32, device=DEV)
    st = lib.prune_stats_norms_static(x.data_ptr(), prune.F32, 1, 600000, 600000, out.data_ptr(), out.data_ptr(), None)
    assert st == -5 and "workspace" in prune.status_string(st)
