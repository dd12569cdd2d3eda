"""The allocation-free distortion entry point (moshpit_dist_to_mean_static) against
moshpit_dist_to_mean through the C ABI: same kernels, same order of additions, so
the two must agree to the bit (which is within the parity bar of the distortion by
a wide margin); the existing entry point itself is held to the oracle here too.
Two calls in a row, the second on a smaller input (the shared scratch keeps the
first call's partial sums)."""
import numpy as np
import pytest
import torch

from oracle import moshpit_oracle as orc
from paper_2103_03239_amd import binding, inputs
from parity_util import TOL, dist_floor

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _pair(w, stride=None):
    X = inputs.make_state(w, DEV, row_stride=stride)
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    binding.dist_to_mean_static(X, out)
    torch.cuda.synchronize()
    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(X)
        want = m.dist_to_mean()
    return float(out.item()), want, X


@pytest.mark.parametrize("dtype", [0, 1])
def test_static_scratch_matches_the_allocating_entry_point(dtype):
    big = inputs.Workload("noalloc-big", 256, 16, 2, 300_001, dtype, "peer_offset", 0, 0.0, 0, 0, 11, 12)
    small = inputs.Workload("noalloc-small", 16, 4, 2, 1_000, dtype, "normal", 0, 0.0, 0, 0, 13, 14)
    for w, stride in ((big, 300_008), (small, None), (big, None)):
        print(f"no-alloc {w.name} dtype={dtype} stride={stride}", flush=True)
        got, want, X = _pair(w, stride)
        assert got == want, (got, want)
        ref = orc.dist_to_mean(X.cpu().to(torch.float64).numpy())
        assert abs(got - ref) <= TOL[dtype] * ref + dist_floor(w.P, dtype, 1.5)


def test_static_scratch_rejects_what_does_not_fit():
    lib = binding.load_library()
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    X = torch.zeros(4, 64, device=DEV)
    # more partial sums than the static array holds: 16-byte-aligned rows of 2^25 + 256 columns
    rc = lib.moshpit_dist_to_mean_static(X.data_ptr(), 4, 2 ** 25 + 256, 2 ** 25 + 256, 0, None, out.data_ptr())
    assert rc == -1 and b"static scratch" in lib.moshpit_last_error(None)
    for args in ((None, 4, 64, 64, 0, None, out.data_ptr()), (X.data_ptr(), 4, 64, 32, 0, None, out.data_ptr()),
                 (X.data_ptr(), 4, 64, 64, 5, None, out.data_ptr()), (X.data_ptr(), 4, 64, 64, 0, None, None)):
        assert lib.moshpit_dist_to_mean_static(*args) == -1
    torch.cuda.synchronize()
    assert float(out.item()) == 0.0
