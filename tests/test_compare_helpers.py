"""The comparison helper that the GPU parity tests use for results stored in bf16: what it forgives (an element
rounded to the other neighbour when the exact value sits at the midpoint) and what it does not."""
import numpy as np

from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U


def _bf16(x):
    return np.asarray(W.round_storage(np.asarray(x, np.float64), "bf16"), np.float64)


def test_storage_err_rows_forgives_only_midpoint_neighbours():
    g = np.random.default_rng(0)
    ref = g.standard_normal((4, 64)) * 2
    lo, hi = 2.078125, 2.09375                      # neighbouring bf16 values
    assert _bf16(lo) == lo and _bf16(hi) == hi and _bf16(0.5 * (lo + hi) + 1e-7) == hi
    ref[0, 3] = 0.5 * (lo + hi) + 1e-6              # exact value a hair above the midpoint: rounds to hi
    got = _bf16(ref)
    assert U.storage_err_rows(got, ref, "bf16").max() == 0.0
    got[0, 3] = lo                                  # the other neighbour: an error of the size of the arithmetic's
    plain = U.rel_err_rows(got, _bf16(ref))
    assert plain[0] > 1e-3                          # one bf16 ulp of a large element, seen by the plain comparison
    assert U.storage_err_rows(got, ref, "bf16").max() == 0.0
    # the same neighbour when the exact value is NOT at the midpoint is an error
    ref2 = ref.copy()
    ref2[0, 3] = hi - 1e-4
    got2 = _bf16(ref2)
    got2[0, 3] = lo
    assert U.storage_err_rows(got2, ref2, "bf16")[0] > 1e-3
    # ... and so is an exact value 2e-4 from the midpoint (1e-5 of this vector's norm: beyond the arithmetic's error)
    ref4 = ref.copy()
    ref4[0, 3] = 0.5 * (lo + hi) + 2e-4
    assert 2e-4 > 5e-6 * np.linalg.norm(ref4[0])
    got4 = _bf16(ref4)
    got4[0, 3] = lo
    err4, n4 = U.storage_err_rows(got4, ref4, "bf16", return_forgiven=True)
    assert err4[0] > 1e-3 and n4 == 0
    assert U.storage_err_rows(got, ref, "bf16", return_forgiven=True)[1] == 1
    # two ulps away is never forgiven, midpoint or not
    got3 = _bf16(ref)
    got3[0, 3] = lo - (hi - lo)
    assert U.storage_err_rows(got3, ref, "bf16")[0] > 1e-3
    # f32 storage: no forgiveness rule, plain comparison with the rounded reference
    ref32 = ref.astype(np.float32).astype(np.float64)
    assert U.storage_err_rows(ref32, ref, "f32").max() < 1e-7
