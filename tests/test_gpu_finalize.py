"""GPU parity of the last step of a build (rank by exact distance, cut to k, split into ids / distances).

With no refinement iteration (max_iters = -1) a build is: random rows, then finalize.  What comes
back must then be a valid graph whose every distance equals the oracle's recomputation bit for bit
(the fp64 recipe in index order, or the exact integer for uint8), rows ascending by (distance, id).
The shapes walk the row lengths around the 128-byte steps of the staged kernel (one piece, a ragged
last step, many steps), the list lengths around the lane groups (K = 1, 5, 17, 33, 64), the rows
that are not made of aligned 16-byte pieces (the lane-per-row kernel), and all three element types.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_27691_amd import knng

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _gpu(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _check(values, ids, dists, metric, k):
    ids, dists = ids.cpu().numpy(), dists.cpu().numpy()
    assert ids.shape == (values.shape[0], k) and dists.shape == ids.shape
    viol = oracle.check_graph(values, ids, dists, metric, rel_tol=0.0)
    assert sum(viol.values()) == 0, viol


@pytest.mark.parametrize("d", [4, 8, 20, 32, 36, 60, 64, 100, 128, 132, 260, 1000, 3, 33, 50, 129])
@pytest.mark.parametrize("k,kb", [(1, 1), (5, 5), (16, 17), (20, 33), (32, 64)])
def test_finalize_fp32_random_rows(d, k, kb):
    rng = np.random.default_rng(d * 100 + kb)
    n = 300 + d % 7
    x = (rng.standard_normal((n, d)) * 3.0 + rng.standard_normal(d)).astype(np.float32)
    ids, dists, _ = knng.knng_build_knn_graph(_gpu(x), k, oracle.L2SQ, k_build=kb, max_iters=-1, seed=d)
    _check(x, ids, dists, oracle.L2SQ, k)
    if d >= 8:
        xn = x / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
        ids, dists, _ = knng.knng_build_knn_graph(_gpu(xn), k, oracle.IP_UNIT, k_build=kb, max_iters=-1, seed=d)
        _check(xn, ids, dists, oracle.IP_UNIT, k)


def test_finalize_fp32_rows_not_16_byte_aligned():
    # d % 4 == 0 but the first row starts 4 bytes into an allocation: the lane-per-row kernel
    rng = np.random.default_rng(5)
    n, d, k = 257, 64, 9
    flat = _gpu(rng.standard_normal(n * d + 1).astype(np.float32))
    x = flat[1:].view(n, d)
    assert x.data_ptr() % 16 != 0
    ids, dists, _ = knng.knng_build_knn_graph(x, k, oracle.L2SQ, max_iters=-1, seed=1)
    _check(x.cpu().numpy(), ids, dists, oracle.L2SQ, k)


@pytest.mark.parametrize("d", [2, 8, 24, 64, 72, 200, 960, 6, 34])
@pytest.mark.parametrize("k,kb", [(3, 3), (16, 17), (32, 64)])
def test_finalize_fp16_random_rows(d, k, kb):
    rng = np.random.default_rng(d * 100 + kb + 1)
    n = 280
    x16 = (rng.standard_normal((n, d)) * 2.0).astype(np.float16)
    ids, dists, _ = knng.knng_build_knn_graph_f16(_gpu(x16), k, oracle.L2SQ, k_build=kb, max_iters=-1, seed=d)
    _check(x16.astype(np.float32), ids, dists, oracle.L2SQ, k)


@pytest.mark.parametrize("d", [4, 16, 48, 128, 144, 400, 2048, 20, 132])
@pytest.mark.parametrize("k,kb", [(3, 3), (16, 17), (32, 64)])
def test_finalize_uint8_random_rows(d, k, kb):
    rng = np.random.default_rng(d * 100 + kb + 2)
    n = 280
    x8 = rng.integers(0, 256, (n, d)).astype(np.uint8)
    x8[::9] = 255
    x8[1::9] = 0                                      # largest differences: sums above 2^24 for long rows
    ids, dists, _ = knng.knng_build_knn_graph_u8(_gpu(x8), k, oracle.L2SQ, k_build=kb, max_iters=-1, seed=d)
    _check(x8, ids, dists, oracle.L2SQ, k)
