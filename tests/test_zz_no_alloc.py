"""knng_graph_recall_static (the entry point that allocates nothing) against knng_graph_recall."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_27691_amd import knng

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _graphs(rows, k, seed):
    rng = np.random.default_rng(seed)
    ref_i = np.argsort(rng.random((rows, 4 * k), dtype=np.float32), axis=1)[:, :k].astype(np.int32)   # distinct ids per row
    test_i = ref_i.copy()
    swap = rng.random((rows, k)) < 0.3
    test_i[swap] = (4 * k + rng.integers(0, 1000, swap.sum())).astype(np.int32)   # misses
    test_i[rng.random((rows, k)) < 0.02] = -1                                      # padding
    ref_d = np.sort(rng.random((rows, k)).astype(np.float32), axis=1)
    test_d = np.sort((ref_d * rng.uniform(0.8, 1.3, (rows, k))).astype(np.float32), axis=1)
    g = lambda a: torch.from_numpy(a).to(DEV)
    return g(test_i), g(test_d), g(ref_i), g(ref_d)


def test_recall_without_allocation_equals_the_allocating_entry_point_twice_in_a_row():
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    # the second call is smaller: it must not see what the first left in the library's array
    for rows, k, at_k, seed in ((300_000, 32, 32, 1), (777, 16, 10, 2)):
        t_i, t_d, r_i, r_d = _graphs(rows, k, seed)
        for mode in (0, 1):
            want = knng.knng_graph_recall(t_i, t_d, r_i, r_d, at_k, mode)
            got = knng.knng_graph_recall_static(t_i, t_d, r_i, r_d, at_k, mode, out=out)
            torch.cuda.synchronize()
            assert float(got.item()) == want and 0.0 < want < 1.0, (rows, mode, float(got.item()), want)


def test_recall_without_allocation_rejects_what_its_scratch_cannot_take():
    lib = knng.load()
    t_i, t_d, r_i, r_d = _graphs(64, 8, 3)
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    args = lambda rows: (ctypes.c_void_p(t_i.data_ptr()), None, 8, ctypes.c_void_p(r_i.data_ptr()), None, 8, rows, 8, 0,
                         ctypes.c_void_p(out.data_ptr()), None)
    assert lib.knng_graph_recall_static(*args((1 << 36) // 8 + 1)) == -4       # KNNG_ETOOLARGE, nothing enqueued
    assert b"scratch" in lib.knng_strerror(-4)
    assert lib.knng_graph_recall_static(*args(0)) == -1
    torch.cuda.synchronize()
    assert float(out.item()) == -1.0
