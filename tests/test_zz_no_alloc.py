"""The entry point that allocates nothing: dw_overlap_partition_static against dw_overlap_partition.

Index work, so the two must agree in every entry.  Both calls of the static variant share the one scratch array the
library holds on the GPU; the second, smaller call finds the first call's keys and ranks in it."""
import numpy as np
import pytest
import torch

from paper_2409_09242_amd import binding as B

pytestmark = pytest.mark.gpu


def _static(n, o, k, seed):
    m = o + (n - o) // k
    index = torch.full((k, m), -7, dtype=torch.int32, device="cuda:0")
    before = torch.cuda.memory_allocated()
    s = B.overlap_partition_static(n, o, k, seed, index)
    assert torch.cuda.memory_allocated() == before
    assert s == (n - o) // k
    torch.cuda.synchronize()
    return index.cpu().numpy()


def test_static_partition_matches_the_scratch_argument_form_on_two_calls_in_a_row():
    torch.cuda.set_device(0)
    for n, o, k, seed in ((60000, 7500, 8, 12345), (9001, 1200, 5, 12345)):      # the second call is smaller
        got = _static(n, o, k, seed)
        want = B.overlap_partition(n, o, k, seed, "cuda:0").cpu().numpy()
        np.testing.assert_array_equal(got, want)
        # a valid partition whatever the reference says: O shared, the S_j disjoint, every index in range
        assert all((got[j, :o] == got[0, :o]).all() for j in range(k))
        own = got[:, o:].reshape(-1)
        assert len(set(own.tolist()) | set(got[0, :o].tolist())) == own.size + o
        assert got.min() >= 0 and got.max() < n
    # the largest size the fixed array takes, then one point more
    n = B.DW_STATIC_MAX_POINTS
    got = _static(n, 1024, 64, 3)
    np.testing.assert_array_equal(got, B.overlap_partition(n, 1024, 64, 3, "cuda:0").cpu().numpy())
    index = torch.zeros((2, 8), dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.DwError) as err:
        B.overlap_partition_static(n + 1, 0, 2, 3, index)
    assert err.value.status == -8 and "capacity" in str(err.value)
    # and a small call after the largest one
    np.testing.assert_array_equal(_static(300, 40, 4, 7), B.overlap_partition(300, 40, 4, 7, "cuda:0").cpu().numpy())
