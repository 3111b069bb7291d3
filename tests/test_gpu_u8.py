"""GPU parity of the uint8 build (knng_build_knn_graph_u8) against the CPU oracle.

The oracle takes uint8 points at their values, so the bars are those of the fp32 build: every
written distance equal to the oracle's recomputation (here an exact integer rounded once), row
invariants, recall@k >= 0.95 against the exact graph; and, where fp32 arithmetic is exact on
these values as well (d * 255^2 < 2^24), the same graph bit for bit as the fp32 build.
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


def _clustered_u8(n, d, seed, centres=16, sigma=20.0):
    rng = np.random.default_rng(seed)
    c = rng.integers(0, 256, (centres, d)).astype(np.float64)
    x = c[rng.integers(0, centres, n)] + sigma * rng.standard_normal((n, d))
    return np.clip(np.rint(x), 0, 255).astype(np.uint8)


def _check(x8, k, ids, dists, min_recall=0.95):
    ids, dists = ids.cpu().numpy(), dists.cpu().numpy()
    viol = oracle.check_graph(x8, ids, dists, 0, rel_tol=0.0)          # distances: exact
    assert sum(viol.values()) == 0, viol
    ex = oracle.brute_knn(x8, k, 0)
    rec = oracle.graph_recall(ids, dists, ex[0], ex[1], k, 0)
    assert rec >= min_recall, rec
    return rec


@pytest.mark.parametrize("n,d,k,kb,rho", [
    (3000, 128, 16, 32, 0.5),      # one 128-byte slab per row, 16-byte pieces
    (5000, 64, 32, 32, 0.5),       # half a slab
    (2000, 20, 10, 16, 1.0),       # d % 16 != 0: 4-byte words, predicated loads
    (1500, 960, 16, 32, 0.5),      # 7.5 slabs, distances above 2^24
    (600, 4, 5, 8, 0.5),           # one word per row, wavefront kernel with <= 32 members
    (100, 16, 32, 32, 0.5),        # K close to n
    (2, 4, 1, 1, 1.0),             # smallest
    (3001, 128, 32, 64, 0.5),      # samples of 32: the workgroup kernel with 128 member slots
    (3003, 128, 32, 48, 0.5),      # samples of 24: the workgroup kernel with 96 member slots
    (2500, 36, 16, 64, 0.36),      # samples of 24, 4-byte words
    (2000, 64, 16, 64, 1.0),       # samples of 64: 256 member slots
    (1500, 20, 10, 48, 0.8),       # the same kernel on 4-byte words
])
def test_u8_build_against_the_oracle(n, d, k, kb, rho):
    x8 = _clustered_u8(n, d, seed=n + d)
    ids, dists, st = knng.knng_build_knn_graph_u8(_gpu(x8), k, 0, k_build=kb, rho=rho, seed=5)
    _check(x8, k, ids, dists)


def test_u8_extreme_values_and_duplicates():
    # only 0 and 255: the signed bytes are -128 and 127, sums of squares at their largest;
    # many exact duplicates (distance 0, ties on the id)
    rng = np.random.default_rng(8)
    proto = (rng.integers(0, 2, (40, 192)) * 255).astype(np.uint8)
    x8 = proto[rng.integers(0, 40, 2500)].copy()
    flip = rng.integers(0, 192, 2500)
    x8[np.arange(2500), flip] ^= 255
    ids, dists, _ = knng.knng_build_knn_graph_u8(_gpu(x8), 12, 0, k_build=32, seed=1)
    ids, dists = ids.cpu().numpy(), dists.cpu().numpy()
    viol = oracle.check_graph(x8, ids, dists, 0, rel_tol=0.0)
    assert sum(viol.values()) == 0, viol
    assert np.all(dists % 65025.0 == 0.0)
    ex = oracle.brute_knn(x8, 12, 0)
    # ties everywhere: compare distances (unique), not ids
    assert oracle.graph_recall(ids, dists, ex[0], ex[1], 12, 1) >= 0.95


@pytest.mark.parametrize("n,d,k,kb", [(20_000, 128, 32, 32), (6000, 256, 16, 16), (4000, 36, 24, 24),
                                      (8000, 128, 32, 64)])
def test_u8_build_is_the_fp32_build_bit_for_bit_where_fp32_is_exact(n, d, k, kb):
    x8 = _clustered_u8(n, d, seed=d, centres=64)
    xd = _gpu(x8)
    a = knng.knng_build_knn_graph_u8(xd, k, 0, k_build=kb, seed=11)
    b = knng.knng_build_knn_graph(xd.float(), k, 0, k_build=kb, seed=11)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))
    assert a[2]["iterations"] == b[2]["iterations"] and a[2]["updates"] == b[2]["updates"]


def test_u8_pointer_alignment_paths():
    x8 = _clustered_u8(3000, 64, seed=2)
    flat = torch.zeros(3000 * 64 + 64, dtype=torch.uint8, device=DEV)
    ref = knng.knng_build_knn_graph_u8(_gpu(x8), 10, 0, k_build=16, seed=4)
    for off in (4, 16):                     # 4: word path (same graph, different loads); 16: pieces
        view = flat[off:off + 3000 * 64].view(3000, 64)
        view.copy_(_gpu(x8))
        got = knng.knng_build_knn_graph_u8(view, 10, 0, k_build=16, seed=4)
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
    bad = flat[1:1 + 3000 * 64].view(3000, 64)
    with pytest.raises(knng.KnngError):
        knng.knng_build_knn_graph_u8(bad, 10, 0, k_build=16, seed=4)


def test_u8_argument_errors_leave_outputs_untouched():
    x8 = _gpu(_clustered_u8(500, 32, seed=3))
    ids = torch.full((500, 8), -7, dtype=torch.int32, device=DEV)
    dists = torch.full((500, 8), -7.0, dtype=torch.float32, device=DEV)
    cases = [
        dict(points=x8, metric=1),                                   # inner product: fp32 build only
        dict(points=x8[:, :30].contiguous(), metric=0),              # d % 4 != 0
        dict(points=x8, metric=0, k_build=4),                        # K < k
    ]
    for c in cases:
        pts = c.pop("points")
        metric = c.pop("metric")
        with pytest.raises(knng.KnngError):
            knng.knng_build_knn_graph_u8(pts, 8, metric, ids_out=ids, dists_out=dists, **c)
    assert bool((ids == -7).all()) and bool((dists == -7.0).all())


def test_u8_full_size_config2_sift_shape():
    # config 2's values are 8-bit by construction: the same workload stored as uint8, in the
    # launch configuration the benchmark times; sampled rows against the oracle
    x, w = workloads.make(2, device=DEV)
    x8 = x.to(torch.uint8)
    assert torch.equal(x8.float(), x)
    n, k = w.n, w.k
    rows = workloads.sample_rows(n, 10_000)
    rows_d = torch.from_numpy(rows).to(DEV)
    ex_i, ex_d = knng.knng_brute_knn(x, k, 0, rows_d)
    ids, dists, st = knng.knng_build_knn_graph_u8(x8, k, 0, seed=0)
    sel = rows_d.long()
    t_i, t_d = ids[sel].contiguous(), dists[sel].contiguous()
    rec = knng.knng_graph_recall(t_i, t_d, ex_i, ex_d, k, 0)
    assert rec >= 0.95, rec
    assert st["converged"] and st["iterations"] < 100
    xh = x8.cpu().numpy()
    sub = np.linspace(0, len(rows) - 1, 48).astype(np.int64)
    o_i, o_d = oracle.brute_knn(xh, k, 0, query_rows=rows[sub])
    assert np.array_equal(o_i, ex_i[sub].cpu().numpy()) and np.array_equal(o_d, ex_d[sub].cpu().numpy())
    viol = oracle.check_graph(xh, t_i[sub].cpu().numpy(), t_d[sub].cpu().numpy(), 0, rel_tol=0.0, rows=rows[sub])
    assert sum(viol.values()) == 0, viol
    assert int(ids.min()) >= 0 and int(ids.max()) < n
    assert not bool((ids == torch.arange(n, device=DEV, dtype=torch.int32)[:, None]).any())
    assert bool((dists[:, 1:] >= dists[:, :-1]).all()) and bool((dists >= 0).all())
    srt = ids.sort(dim=1).values
    assert not bool((srt[:, 1:] == srt[:, :-1]).any())
