"""GPU parity of knng_optimize_graph (k-NN graph -> search graph) against the CPU oracle.

Index work: the bar is bit-exact, at every size including the benchmark's.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_27691_amd import knng, workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _gpu(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def _both(ids, d_out):
    got = knng.knng_optimize_graph(_gpu(ids), d_out).cpu().numpy()
    want = oracle.optimize_graph(ids, d_out)
    return got, want


def _exact_graph(n, d, k, seed):
    rng = np.random.default_rng(seed)
    c = rng.standard_normal((12, d)) * 4.0
    x = (c[rng.integers(0, 12, n)] + rng.standard_normal((n, d))).astype(np.float32)
    return oracle.brute_knn(x, k, oracle.L2SQ)[0]


@pytest.mark.parametrize("n,k,d_out", [(3000, 32, 32), (3000, 32, 16), (3000, 32, 7), (3000, 32, 1),
                                        (1500, 64, 64), (1500, 64, 33), (2000, 10, 10), (2000, 3, 2),
                                        (500, 1, 1), (4097, 17, 9)])
def test_optimize_exact_graphs_bit_exact(n, k, d_out):
    ids = _exact_graph(n, 8, k, seed=n + k)
    got, want = _both(ids, d_out)
    assert np.array_equal(got, want)
    if d_out > 1:
        assert not np.array_equal(got, ids[:, :d_out])       # something was pruned or reversed


def test_optimize_an_approximate_graph_from_the_build():
    x, w = workloads.make(1)
    ids, _, _ = knng.knng_build_knn_graph(_gpu(x), 16, w.metric, k_build=32, seed=2)
    for d_out in (16, 8):
        got = knng.knng_optimize_graph(ids, d_out).cpu().numpy()
        assert np.array_equal(got, oracle.optimize_graph(ids.cpu().numpy(), d_out))


def test_optimize_padding_self_loops_and_repeats():
    rng = np.random.default_rng(5)
    for n, k, d_out in [(700, 12, 12), (700, 12, 5), (64, 40, 40), (33, 64, 20)]:
        ids = rng.integers(-3, n + 3, (n, k)).astype(np.int32)
        ids[::7, :] = -1                                     # whole rows of padding
        ids[1::7, 1:] = ids[1::7, :1]                        # rows that repeat one id
        got, want = _both(ids, d_out)
        assert np.array_equal(got, want)
        assert (got == -1).any()


def test_optimize_hubs_with_long_reverse_lists():
    # every point's nearest neighbour is point 7, the second one of 64 points: reverse lists of
    # n - 1 and of about n / 64 entries, far more than a wavefront holds, in arbitrary order
    n, k = 9000, 24
    ids = _exact_graph(n, 6, k, seed=4)
    hub = np.full(n, 7, np.int32)
    second = (np.arange(n) % 64 + 100).astype(np.int32)
    keep = np.array([[x for x in row if x not in (7, second[u])][:k - 2] for u, row in enumerate(ids)], np.int32)
    g = np.concatenate([hub[:, None], second[:, None], keep], axis=1)
    g[7, 0] = 8
    for d_out in (24, 12, 3):
        got, want = _both(g, d_out)
        assert np.array_equal(got, want)


def test_optimize_ring_closed_form_and_tiny_inputs():
    n, k, d_out = 1001, 12, 8
    ids = ((np.arange(n)[:, None] + np.arange(1, k + 1)[None, :]) % n).astype(np.int32)
    got = knng.knng_optimize_graph(_gpu(ids), d_out).cpu().numpy()
    h = d_out // 2
    want = np.concatenate([(np.arange(n)[:, None] + np.arange(1, d_out - h + 1)[None, :]) % n,
                           (np.arange(n)[:, None] - np.arange(1, h + 1)[None, :]) % n], axis=1)
    assert np.array_equal(got, want)
    for ids in (np.array([[0]], np.int32), np.array([[1], [0]], np.int32), np.array([[1, 2], [2, 0], [0, 1]], np.int32)):
        for d_out in range(1, ids.shape[1] + 1):
            got, want = _both(ids, d_out)
            assert np.array_equal(got, want)


def test_optimize_argument_errors():
    ids = _gpu(_exact_graph(300, 4, 8, seed=1))
    out = torch.full((300, 8), -5, dtype=torch.int32, device=DEV)
    for d_out in (0, 9):
        with pytest.raises(knng.KnngError):
            knng.knng_optimize_graph(ids, d_out, ids_out=out)
    with pytest.raises(knng.KnngError):
        knng.knng_optimize_graph(ids, 4, workspace=torch.empty(256, dtype=torch.uint8, device=DEV), ids_out=out)
    assert bool((out == -5).all())
    assert knng.knng_optimize_workspace_bytes(300, 65, 8) == 0


def test_optimize_full_size_config2_graph_bit_exact():
    # the graph the benchmark's build produces (1,000,000 x 32), optimised to degree 32 and 16
    x, w = workloads.make(2, device=DEV)
    ids, _, _ = knng.knng_build_knn_graph(x, w.k, w.metric, seed=0)
    del x
    ids_h = ids.cpu().numpy()
    for d_out in (32, 16):
        got = knng.knng_optimize_graph(ids, d_out)
        assert np.array_equal(got.cpu().numpy(), oracle.optimize_graph(ids_h, d_out))
        # properties on every row: valid ids, no self loops, no repeats
        assert int(got.min()) >= 0 and int(got.max()) < w.n
        assert not bool((got == torch.arange(w.n, device=DEV, dtype=torch.int32)[:, None]).any())
        srt = got.sort(dim=1).values
        assert not bool((srt[:, 1:] == srt[:, :-1]).any())


def test_optimize_random_sizes_and_graphs_against_the_oracle():
    rng = np.random.default_rng(2024)
    for t in range(24):
        n = int(rng.integers(2, 3000))
        k = int(rng.integers(1, min(64, n - 1) + 1))
        d_out = int(rng.integers(1, k + 1))
        if t % 3 == 0:
            ids = rng.integers(-2, n + 2, (n, k)).astype(np.int32)          # arbitrary entries
        else:
            x = rng.standard_normal((n, int(rng.integers(1, 6)))).astype(np.float32)
            ids = oracle.brute_knn(x, k, oracle.L2SQ)[0]
            if t % 3 == 2:
                ids[rng.random(ids.shape) < 0.1] = -1
        got, want = _both(ids, d_out)
        assert np.array_equal(got, want), (n, k, d_out)
