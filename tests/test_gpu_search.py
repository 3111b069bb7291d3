"""GPU parity of knng_graph_search against the CPU oracle.

Both sides evaluate distances with the fp64 recipe and order by (fp32 distance, id), so every
decision is the same: ids, distances and iteration counts are compared bit for bit.
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


def _both(x, g, q, st, k_s, L, width, cap, metric=0):
    gi, gd, git, gev = knng.knng_graph_search(_gpu(x), _gpu(g), _gpu(q), _gpu(st), k_s, L, width, cap, metric,
                                              want_iters=True)
    oi, od, oit, oev = oracle.graph_search(x, g, q, st, k_s, L, width, cap, metric, want_evals=True)
    return (gi.cpu().numpy(), gd.cpu().numpy(), git.cpu().numpy(), gev.cpu().numpy()), (oi, od, oit, oev)


def _assert_same(a, b):
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
    assert np.array_equal(a[2], b[2])
    # distances evaluated: the kernel offers a row at once and so may skip a repeat inside the
    # row or an id the row itself has just pushed out, which offering one id at a time evaluates
    # again; it never evaluates more, and every listed id was evaluated at least once
    assert np.all(a[3] <= b[3]) and np.all(a[3] >= (a[0] >= 0).sum(1))


def _data(n, d, nq, metric, seed):
    rng = np.random.default_rng(seed)
    c = rng.standard_normal((10, d)) * 3.0
    x = (c[rng.integers(0, 10, n)] + rng.standard_normal((n, d))).astype(np.float32)
    q = (c[rng.integers(0, 10, nq)] + rng.standard_normal((nq, d))).astype(np.float32)
    if metric == 1:
        x = (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)
        q = (q / np.linalg.norm(q, axis=1, keepdims=True)).astype(np.float32)
    return x, q, rng


@pytest.mark.parametrize("n,d,deg,nq,k_s,L,width,cap,ns,metric", [
    (4000, 32, 16, 300, 10, 32, 1, 100, 8, 0),
    (4000, 32, 16, 300, 16, 64, 2, 100, 16, 0),
    (3000, 96, 32, 200, 32, 64, 1, 100, 32, 1),
    (2000, 13, 8, 150, 5, 8, 3, 100, 1, 0),          # odd d: scalar loads
    (2500, 128, 64, 101, 1, 1, 1, 100, 64, 0),       # a list of one entry, the widest rows and starts
    (2000, 20, 12, 100, 12, 12, 64, 3, 5, 0),        # capped at three iterations, every entry a parent
    (1500, 960, 24, 40, 8, 24, 1, 100, 4, 0),        # long vectors
    (3000, 8, 10, 130, 4, 16, 1, 0, 6, 1),           # no iteration: the best of the start points
])
def test_search_bit_exact_against_the_oracle(n, d, deg, nq, k_s, L, width, cap, ns, metric):
    x, q, rng = _data(n, d, nq, metric, seed=n + d + deg)
    g = oracle.brute_knn(x, deg, metric)[0]
    st = rng.integers(0, n, (nq, ns)).astype(np.int32)
    got, want = _both(x, g, q, st, k_s, L, width, cap, metric)
    _assert_same(got, want)


def test_search_graph_with_padding_repeats_and_bad_starts():
    x, q, rng = _data(1200, 16, 120, 0, seed=9)
    g = oracle.brute_knn(x, 12, 0)[0]
    g[rng.random(g.shape) < 0.15] = -1
    g[rng.random(g.shape) < 0.05] = 1200 + 7
    g[:, 3] = np.where(rng.random(1200) < 0.3, g[:, 2], g[:, 3])
    st = rng.integers(-2, 1202, (120, 7)).astype(np.int32)
    st[5] = -1                                                   # nothing to start from
    st[6] = st[6, 0]                                             # the same start seven times
    got, want = _both(x, g, q, st, 9, 20, 2, 100)
    _assert_same(got, want)
    assert got[0][5].tolist() == [-1] * 9 and np.all(np.isinf(got[1][5]))


def test_search_on_the_search_graph_of_a_built_graph_two_partitions():
    # one level of the paper's scheme without the network: the points of partition B search
    # the optimised graph of partition A
    x, w = workloads.make(1)
    a, b = x[:12_000], x[12_000:]
    ids, _, _ = knng.knng_build_knn_graph(_gpu(a), 16, w.metric, k_build=32, seed=3)
    gs = knng.knng_optimize_graph(ids, 16).cpu().numpy()
    rng = np.random.default_rng(4)
    # the workload's 16 clusters are islands of the graph: enough starts to land in the right one
    st = rng.integers(0, len(a), (len(b), 64)).astype(np.int32)
    got, want = _both(a, gs, b, st, 16, 64, 1, 100, w.metric)
    _assert_same(got, want)
    rows = (np.arange(2000) + len(a)).astype(np.int32)       # the first 2000 points of B, as rows of x
    ex_i, ex_d = knng.knng_brute_knn(_gpu(x), 16, w.metric, _gpu(rows), n_base=len(a))
    rec = knng.knng_graph_recall(_gpu(got[0][:2000]), _gpu(got[1][:2000]), ex_i, ex_d, 16, 0)
    assert rec >= 0.95, rec


def test_search_argument_errors():
    x, q, rng = _data(500, 8, 10, 0, seed=1)
    g = oracle.brute_knn(x, 8, 0)[0]
    st = rng.integers(0, 500, (10, 4)).astype(np.int32)
    for kw in (dict(k_s=9, itopk=8), dict(k_s=4, itopk=65), dict(k_s=4, itopk=8, width=0),
               dict(k_s=4, itopk=8, max_iters=-1), dict(k_s=4, itopk=8, metric=2)):
        with pytest.raises(knng.KnngError):
            knng.knng_graph_search(_gpu(x), _gpu(g), _gpu(q), _gpu(st), **kw)
    with pytest.raises(knng.KnngError):
        knng.knng_graph_search(_gpu(x), _gpu(g), _gpu(q[:, :7].copy()), _gpu(st), 4, 8)
    ids, dists = knng.knng_graph_search(_gpu(x), _gpu(g), _gpu(q[:0]), _gpu(st[:0]), 4, 8)
    assert ids.shape == (0, 4)


def test_one_refinement_level_on_one_gpu_build_optimise_search_merge():
    # Two partitions A and B of one point set, the way the paper's scheme treats two ranks
    # (Sec. 4.3, 4.4), with the exchange left out: each builds its own graph, B's points search
    # A's search graph and A's search B's, each updates its rows with what it found.  The
    # result is compared with the exact graph of the whole set.
    x, w = workloads.make(6, n=24_000)
    k = 16
    half = len(x) // 2
    parts = [x[:half], x[half:]]
    dev = [_gpu(p) for p in parts]
    local, search_graph = [], []
    for p in dev:
        ids, dists, _ = knng.knng_build_knn_graph(p, k, w.metric, k_build=32, seed=6)
        local.append((ids, dists))
        search_graph.append(knng.knng_optimize_graph(ids, k))
    rng = np.random.default_rng(8)
    merged = []
    for me, other in ((0, 1), (1, 0)):
        st = _gpu(rng.integers(0, half, (half, 16)).astype(np.int32))
        r_ids, r_dists = knng.knng_graph_search(dev[other], search_graph[other], dev[me], st, k, 48, 1, 100, w.metric)
        # global ids: partition 0 keeps its ids, partition 1 is shifted by `half`
        own = local[me][0] + me * half
        found = torch.where(r_ids >= 0, r_ids + other * half, r_ids)
        merged.append(knng.knng_merge_graphs(own, local[me][1], found, r_dists, k))
    g_ids = torch.cat([m[0] for m in merged]).cpu().numpy()
    g_dists = torch.cat([m[1] for m in merged]).cpu().numpy()
    viol = oracle.check_graph(x, g_ids, g_dists, w.metric, rel_tol=0.0)
    assert sum(viol.values()) == 0, viol
    ex = knng.knng_brute_knn(_gpu(x), k, w.metric)
    rec = knng.knng_graph_recall(_gpu(g_ids), _gpu(g_dists), ex[0], ex[1], k, 0)
    before = knng.knng_graph_recall(torch.cat([local[0][0], local[1][0] + half]), torch.cat([local[0][1], local[1][1]]),
                                    ex[0], ex[1], k, 0)
    assert before < 0.7 and rec >= 0.95, (before, rec)


# ------------------------------------------------------------------ uint8 points and queries
def _both_u8(x8, g, q8, st, k_s, L, width, cap):
    gi, gd, git, gev = knng.knng_graph_search_u8(_gpu(x8), _gpu(g), _gpu(q8), _gpu(st), k_s, L, width, cap, 0,
                                                 want_iters=True)
    oi, od, oit, oev = oracle.graph_search(x8, g, q8, st, k_s, L, width, cap, 0, want_evals=True)
    return (gi.cpu().numpy(), gd.cpu().numpy(), git.cpu().numpy(), gev.cpu().numpy()), (oi, od, oit, oev)


@pytest.mark.parametrize("n,d,deg,nq,k_s,L,width,cap,ns", [
    (4000, 128, 16, 300, 10, 32, 1, 100, 8),         # 16-byte pieces
    (3000, 64, 32, 200, 32, 64, 2, 100, 32),
    (2000, 20, 8, 150, 5, 8, 3, 100, 1),             # d % 16 != 0: 4-byte words
    (1500, 960, 24, 40, 8, 24, 1, 100, 4),           # distances above 2^24
    (2000, 4, 12, 100, 12, 12, 64, 3, 5),            # one word per row, capped iterations
])
def test_search_u8_bit_exact_against_the_oracle(n, d, deg, nq, k_s, L, width, cap, ns):
    rng = np.random.default_rng(n + d)
    c = rng.integers(0, 256, (10, d)).astype(np.float64)
    x8 = np.clip(np.rint(c[rng.integers(0, 10, n)] + 25.0 * rng.standard_normal((n, d))), 0, 255).astype(np.uint8)
    q8 = np.clip(np.rint(c[rng.integers(0, 10, nq)] + 25.0 * rng.standard_normal((nq, d))), 0, 255).astype(np.uint8)
    g = oracle.brute_knn(x8, deg, 0)[0]
    st = rng.integers(0, n, (nq, ns)).astype(np.int32)
    got, want = _both_u8(x8, g, q8, st, k_s, L, width, cap)
    _assert_same(got, want)
    # and the same answer as the fp32 search of the same values
    f = knng.knng_graph_search(_gpu(x8.astype(np.float32)), _gpu(g), _gpu(q8.astype(np.float32)), _gpu(st), k_s, L,
                               width, cap, 0)
    assert np.array_equal(f[0].cpu().numpy(), got[0]) and np.array_equal(f[1].cpu().numpy(), got[1])


def test_search_u8_argument_errors():
    rng = np.random.default_rng(2)
    x8 = rng.integers(0, 256, (400, 32), dtype=np.uint8)
    g = oracle.brute_knn(x8, 8, 0)[0]
    st = rng.integers(0, 400, (10, 4)).astype(np.int32)
    xg, qg, gg, sg = _gpu(x8), _gpu(x8[:10]), _gpu(g), _gpu(st)
    with pytest.raises(knng.KnngError):
        knng.knng_graph_search_u8(xg, gg, qg, sg, 4, 8, metric=1)
    with pytest.raises(knng.KnngError):
        knng.knng_graph_search_u8(xg[:, :30].contiguous(), gg, qg[:, :30].contiguous(), sg, 4, 8)


def test_search_random_parameters_against_the_oracle():
    rng = np.random.default_rng(2025)
    for t in range(24):
        n = int(rng.integers(2, 4000))
        d = int(rng.choice([1, 3, 4, 8, 13, 32, 100]))
        deg = int(rng.integers(1, min(64, n - 1) + 1))
        nq = int(rng.integers(1, 200))
        L = int(rng.integers(1, 65))
        k_s = int(rng.integers(1, L + 1))
        width = int(rng.integers(1, 6))
        cap = int(rng.integers(0, 80))
        ns = int(rng.integers(1, 65))
        metric = int(rng.integers(0, 2))
        x = rng.standard_normal((n, d)).astype(np.float32)
        q = rng.standard_normal((nq, d)).astype(np.float32)
        if metric == 1:
            x /= np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-6)
            q /= np.maximum(np.linalg.norm(q, axis=1, keepdims=True), 1e-6)
        g = oracle.brute_knn(x, deg, metric)[0] if t % 2 == 0 else rng.integers(-1, n + 1, (n, deg)).astype(np.int32)
        st = rng.integers(-1, n + 1, (nq, ns)).astype(np.int32)
        got, want = _both(x, g, q, st, k_s, L, width, cap, metric)
        _assert_same(got, want)
