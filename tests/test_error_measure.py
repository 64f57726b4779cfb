"""The error measure the GPU parity tests gate on, checked on the CPU with a
mistake planted in the oracle's own output: a light row of a sum aggregation on
a power-law pattern loses one neighbour.  The pooled maximum over the tensor
does not see it at the bf16 tolerance; the per-row measure must."""
import numpy as np

from oracle import ops as oops
from tests.util import max_rel_err, row_rel_err, node_rel_err


def _hub_and_light_rows(n_light=200, hub_len=3000, F=32, seed=5):
    r = np.random.default_rng(seed)
    lens = np.concatenate([[hub_len], r.integers(1, 6, n_light)])
    ptr = np.zeros(lens.size + 1, dtype=np.int32)
    ptr[1:] = np.cumsum(lens)
    n_cols = 4000
    col = np.concatenate([np.sort(r.choice(n_cols, l, replace=False)) for l in lens]).astype(np.int32)
    x = np.abs(r.standard_normal((n_cols, F))).astype(np.float32) + 0.5     # positive: the hub row's sum is large
    return ptr, col, x


def test_a_dropped_neighbour_of_a_light_row_fails_the_per_row_gate():
    ptr, col, x = _hub_and_light_rows()
    want = oops.spmm(ptr, col, None, x)
    victim = 7                                            # a light row
    k = ptr[victim]                                       # drop its first entry
    bad = want.copy()
    bad[victim] -= x[col[k]]
    assert max_rel_err(bad, want) <= 2e-2                 # the pooled measure is blind to it
    assert row_rel_err(bad, want) > 0.1
    assert node_rel_err(bad, want) > 0.1
    assert node_rel_err(want, want) == 0.0


def test_rows_of_zeros_do_not_divide_by_nothing():
    b = np.zeros((4, 8))
    b[0, 0] = 100.0
    a = b.copy()
    a[2, 3] = 1e-6                                        # noise in an all-zero row (e.g. after a ReLU)
    assert row_rel_err(a, b) == 1e-6 / (1e-3 * 100.0)
    assert row_rel_err(np.zeros((0, 8)), np.zeros((0, 8))) == 0.0
