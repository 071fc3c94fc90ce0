"""The regrouping through the entry point that allocates nothing (its staging lives in a
file-scope device array) against the allocating entry point, bit for bit, and against the
oracle: two calls in a row, the second with a smaller input, then a sweep."""
import numpy as np
import pytest

import oracle
from paper_2007_00433_amd import binding as se

pytestmark = pytest.mark.gpu


def _same(n, m, it):
    print(f"se_plan_noalloc n={n} group_size={m} iter={it}", flush=True)
    g0, mem0 = se.se_plan(n, m, it)
    g1, mem1 = se.se_plan_noalloc(n, m, it)
    assert g1.dtype == np.int32 and np.array_equal(g1, g0), (n, m, it)
    assert np.array_equal(mem1, mem0), (n, m, it)
    want = oracle.plan(n, m, it, seed=se.se_get_seed())
    assert np.array_equal(g1, want["group_of"]) and np.array_equal(mem1, want["members"])


def test_no_alloc_plan_equals_the_allocating_plan_twice_in_a_row():
    se.se_set_seed(0)
    _same(64, 8, 3)            # fills the whole array
    _same(12, 4, 3)            # smaller: the array still holds the larger call's tail
    g, mem = se.se_plan_noalloc(12, 4, 3, want_members=False)
    assert mem is None and np.array_equal(g, oracle.plan(12, 4, 3)["group_of"])


def test_no_alloc_plan_sweep_and_limits():
    for seed in (0, 2 ** 63 + 11):
        se.se_set_seed(seed)
        for n, m in [(64, 64), (1, 1), (63, 7), (16, 4), (5, 1), (48, 16), (2, 2)]:
            for it in (0, 1, 2 ** 40 + 3):
                _same(n, m, it)
    se.se_set_seed(0)
    out = np.full(80, -7, np.int32)
    assert se.se_plan_noalloc_raw(65, 5, 0, out.ctypes.data, None) == se.SE_ERR_UNSUPPORTED
    assert se.se_plan_noalloc_raw(12, 5, 0, out.ctypes.data, None) == se.SE_ERR_DIVISIBILITY
    assert se.se_plan_noalloc_raw(12, 4, -1, out.ctypes.data, None) == se.SE_ERR_ARG
    assert se.se_plan_noalloc_raw(12, 4, 0, None, None) == se.SE_ERR_NULL
    assert (out == -7).all()
