"""CPU oracle for the k-NN-graph path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to oracle/knn_oracle.c (plain C, fp64 accumulation).  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do, and this package
imports nothing from them.
"""
import ctypes
import numpy as np

from .build import build as _build

L2SQ, IP_UNIT, COSINE = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build())
        c_i32, c_i64, c_f32, c_f64, c_u64 = (ctypes.c_int32, ctypes.c_int64, ctypes.c_float,
                                             ctypes.c_double, ctypes.c_uint64)
        P = ctypes.c_void_p
        L.oracle_distance.restype = c_f32
        L.oracle_distance.argtypes = [P, P, c_i32, c_i32]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_brute_knn.restype = ctypes.c_int
        L.oracle_brute_knn.argtypes = [P, c_i64, c_i32, c_i32, c_i32, P, c_i64, P, P]
        L.oracle_brute_knn_base.restype = ctypes.c_int
        L.oracle_brute_knn_base.argtypes = [P, c_i64, c_i64, c_i32, c_i32, c_i32, P, c_i64, P, P]
        L.oracle_graph_recall.restype = c_f64
        L.oracle_graph_recall.argtypes = [P, P, c_i32, P, P, c_i32, c_i64, c_i32, c_i32]
        L.oracle_check_graph.restype = c_i64
        L.oracle_check_graph.argtypes = [P, c_i64, c_i32, c_i32, P, P, c_i32, c_f64, P]
        L.oracle_nn_descent.restype = ctypes.c_int
        L.oracle_nn_descent.argtypes = [P, c_i64, c_i32, c_i32, c_i32, c_i32, c_f64, c_f64,
                                        c_i32, c_i32, c_u64, P, P, P]
        L.oracle_nn_descent_trace.restype = ctypes.c_int
        L.oracle_nn_descent_trace.argtypes = [P, c_i64, c_i32, c_i32, c_i32, c_i32, c_f64, c_f64,
                                              c_i32, c_i32, c_u64, P, P, P, P, P, P, P, P, P, P]
        L.oracle_merge_rows.restype = ctypes.c_int
        L.oracle_merge_rows.argtypes = [P, P, c_i32, P, P, c_i32, c_i64, c_i32, P, P]
        L.oracle_optimize_graph.restype = ctypes.c_int
        L.oracle_optimize_graph.argtypes = [P, c_i64, c_i32, c_i32, P]
        L.oracle_graph_search.restype = ctypes.c_int
        L.oracle_graph_search.argtypes = [P, c_i64, c_i32, c_i32, P, c_i32, P, c_i64, P, c_i32,
                                          c_i32, c_i32, c_i32, c_i32, P, P, P, P]
        _lib = L
    return _lib


def _f32(a):
    # Compact element types (uint8 / float16 point storage) are taken at their values: both
    # convert to fp32 without rounding, so the functions below define the result for them too.
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def distance(a, b, metric=L2SQ) -> np.float32:
    a, b = _f32(a), _f32(b)
    assert a.ndim == 1 and a.shape == b.shape
    return np.float32(lib().oracle_distance(_p(a), _p(b), a.shape[0], metric))


def brute_knn(points, k, metric=L2SQ, query_rows=None, n_base=None):
    """Exact k-NN rows for all points (or for query_rows), among all points or the first n_base.
    -> (ids i32, dists f32)."""
    x = _f32(points)
    n, d = x.shape
    q = None if query_rows is None else _i32(query_rows)
    nq = n if q is None else q.shape[0]
    ids = np.empty((nq, k), dtype=np.int32)
    dists = np.empty((nq, k), dtype=np.float32)
    rc = lib().oracle_brute_knn_base(_p(x), n, n if n_base is None else n_base, d, k, metric, _p(q), nq,
                                     _p(ids), _p(dists))
    if rc != 0:
        raise ValueError(f"oracle_brute_knn: bad arguments (rc={rc})")
    return ids, dists


def graph_recall(test_ids, test_dists, ref_ids, ref_dists, at_k, mode=0) -> float:
    ti = None if test_ids is None else _i32(test_ids)
    td = None if test_dists is None else _f32(test_dists)
    ri = None if ref_ids is None else _i32(ref_ids)
    rd = None if ref_dists is None else _f32(ref_dists)
    shape_t = (ti if ti is not None else td).shape
    shape_r = (ri if ri is not None else rd).shape
    assert shape_t[0] == shape_r[0]
    r = lib().oracle_graph_recall(_p(ti), _p(td), shape_t[1], _p(ri), _p(rd), shape_r[1],
                                  shape_t[0], at_k, mode)
    if r < 0:
        raise ValueError("oracle_graph_recall: bad arguments")
    return float(r)


def merge_rows(ids_a, dists_a, ids_b, dists_b, k_out):
    """Rows of graph A updated with the candidates B (same number of rows).  -> (ids i32, dists f32)."""
    ia, da, ib, db = _i32(ids_a), _f32(dists_a), _i32(ids_b), _f32(dists_b)
    n = ia.shape[0]
    assert ia.shape == da.shape and ib.shape == db.shape and ib.shape[0] == n
    ids = np.empty((n, k_out), dtype=np.int32)
    dists = np.empty((n, k_out), dtype=np.float32)
    rc = lib().oracle_merge_rows(_p(ia), _p(da), ia.shape[1], _p(ib), _p(db), ib.shape[1], n, k_out,
                                 _p(ids), _p(dists))
    if rc != 0:
        raise ValueError("oracle_merge_rows: bad arguments")
    return ids, dists


VIOLATION_NAMES = ("id_range", "self_loop", "duplicate_id", "not_ascending",
                   "distance_mismatch", "bad_distance")


def optimize_graph(ids, d_out):
    """Search graph G^s of a k-NN graph given as ids [n][k], nearest first.  -> ids [n][d_out]."""
    ids = _i32(ids)
    assert ids.ndim == 2
    n, k = ids.shape
    out = np.empty((n, d_out), dtype=np.int32)
    rc = lib().oracle_optimize_graph(_p(ids), n, k, d_out, _p(out))
    if rc != 0:
        raise ValueError(f"oracle_optimize_graph: bad arguments (rc={rc})")
    return out


def graph_search(points, graph, queries, starts, k_s, itopk, width=1, max_iters=64, metric=L2SQ, want_evals=False):
    """Greedy search of `queries` over `graph` ([n][deg] ids).
    -> (ids, dists, iterations per query[, distance evaluations per query])."""
    x, qv = _f32(points), _f32(queries)
    g, st = _i32(graph), _i32(starts)
    n, d = x.shape
    nq = qv.shape[0]
    assert qv.shape[1] == d and g.shape[0] == n and st.shape[0] == nq
    ids = np.empty((nq, k_s), dtype=np.int32)
    dists = np.empty((nq, k_s), dtype=np.float32)
    iters = np.empty(nq, dtype=np.int32)
    evals = np.empty(nq, dtype=np.int32)
    rc = lib().oracle_graph_search(_p(x), n, d, metric, _p(g), g.shape[1], _p(qv), nq, _p(st), st.shape[1],
                                   k_s, itopk, width, max_iters, _p(ids), _p(dists), _p(iters), _p(evals))
    if rc != 0:
        raise ValueError(f"oracle_graph_search: bad arguments (rc={rc})")
    return (ids, dists, iters, evals) if want_evals else (ids, dists, iters)


def check_graph(points, ids, dists, metric=L2SQ, rel_tol=1e-5, rows=None):
    """Row invariants of a graph; `rows` = source point of each graph row (default 0..n-1).

    Returns a dict name -> violation count.
    """
    x = _f32(points)
    ids, dists = _i32(ids), _f32(dists)
    n, d = x.shape
    if rows is not None:
        # graph rows belong to a subset of the points: check each against its own source
        rows = np.asarray(rows, dtype=np.int64)
        out = dict.fromkeys(VIOLATION_NAMES, 0)
        for q, r in enumerate(rows):
            sub = _check_one(x, int(r), ids[q], dists[q], metric, rel_tol)
            for kname, v in sub.items():
                out[kname] += v
        return out
    assert ids.shape[0] == n
    viol = np.zeros(6, dtype=np.int64)
    rc = lib().oracle_check_graph(_p(x), n, d, metric, _p(ids), _p(dists), ids.shape[1],
                                  rel_tol, _p(viol))
    if rc < 0:
        raise ValueError("oracle_check_graph: bad arguments")
    return dict(zip(VIOLATION_NAMES, (int(v) for v in viol)))


def _check_one(x, r, ids_row, dists_row, metric, rel_tol):
    n = x.shape[0]
    out = dict.fromkeys(VIOLATION_NAMES, 0)
    seen = set()
    for a, (i, l) in enumerate(zip(ids_row.tolist(), dists_row.tolist())):
        if not (l >= 0.0) or l == float("inf"):
            out["bad_distance"] += 1
        if i < 0 or i >= n:
            out["id_range"] += 1
            continue
        if i == r:
            out["self_loop"] += 1
        if i in seen:
            out["duplicate_id"] += 1
        seen.add(i)
        if a > 0:
            pl, pi = float(dists_row[a - 1]), int(ids_row[a - 1])
            if not (pl < l or (pl == l and pi < i)):
                out["not_ascending"] += 1
        s = float(distance(x[r], x[i], metric))
        if abs(l - s) > rel_tol * s + 1e-30:
            out["distance_mismatch"] += 1
    return out


def nn_descent(points, k, metric=L2SQ, k_build=None, rho=0.5, delta=1e-4, max_iters=100,
               cand_cap=0, seed=0):
    """CPU reference NN-Descent.  -> (ids, dists, stats dict)."""
    x = _f32(points)
    n, d = x.shape
    K = k if k_build is None else k_build
    ids = np.empty((n, k), dtype=np.int32)
    dists = np.empty((n, k), dtype=np.float32)
    stats = np.zeros(3 + max(max_iters, 1), dtype=np.int64)
    rc = lib().oracle_nn_descent(_p(x), n, d, k, metric, K, rho, delta, max_iters, cand_cap,
                                 seed, _p(ids), _p(dists), _p(stats))
    if rc != 0:
        raise ValueError(f"oracle_nn_descent failed (rc={rc})")
    it = int(stats[0])
    return ids, dists, {"iterations": it, "distance_evals": int(stats[1]),
                        "dropped": int(stats[2]), "updates": stats[3:3 + it].tolist()}


def nn_descent_trace(points, metric=L2SQ, k_build=8, rho=0.5, max_iters=1, cand_cap=0, seed=0):
    """The reference NN-Descent run for exactly max_iters iterations (no stop rule), with the
    lists of its last iteration written out.  -> dict: rows [n][K] ids, dists [n][K], flags
    [n][K] (new-flags of the final rows), s, distance_evals, updates, and for the last iteration
    fwd_new / fwd_old / rev_new / rev_old / NEW / OLD as lists of Python lists per point."""
    x = _f32(points)
    n, d = x.shape
    K = k_build
    smax = K                                               # room for any reading of the sample size
    ids = np.empty((n, K), dtype=np.int32)
    dists = np.empty((n, K), dtype=np.float32)
    stats = np.zeros(3 + max(max_iters, 1), dtype=np.int64)
    # the C side lays the traces out with its own s; find it from the counts it reports
    fwd = np.full((2, n, smax), -1, np.int32)
    rev = np.full((2, n, smax), -1, np.int32)
    cnt = np.zeros((n, 4), np.int32)
    full = np.full((2, n, 2 * smax), -1, np.int32)
    fcnt = np.zeros((n, 2), np.int32)
    flags = np.zeros((n, K), np.uint8)
    rows = np.empty((n, K), np.int32)
    rc = lib().oracle_nn_descent_trace(_p(x), n, d, K, metric, K, rho, 0.0, max_iters, cand_cap, seed,
                                       _p(ids), _p(dists), _p(stats), _p(fwd), _p(rev), _p(cnt),
                                       _p(full), _p(fcnt), _p(flags), _p(rows))
    if rc != 0:
        raise ValueError(f"oracle_nn_descent_trace failed (rc={rc})")
    return {"ids": rows, "dists": dists, "flags": flags.astype(bool), "cnt": cnt, "fcnt": fcnt,
            "raw_fwd": fwd.reshape(-1), "raw_rev": rev.reshape(-1), "raw_full": full.reshape(-1),
            "distance_evals": int(stats[1]), "updates": stats[3:3 + int(stats[0])].tolist(),
            "iterations": int(stats[0])}


def trace_lists(tr, n, s):
    """Unpack the flat trace buffers of nn_descent_trace for sample size s.
    -> dict of lists of lists: fwd_new, fwd_old, rev_new, rev_old, NEW, OLD."""
    cnt, fcnt = tr["cnt"], tr["fcnt"]
    f = tr["raw_fwd"][:2 * n * s].reshape(2, n, s)
    r = tr["raw_rev"][:2 * n * s].reshape(2, n, s)
    u = tr["raw_full"][:2 * n * 2 * s].reshape(2, n, 2 * s)
    return {"fwd_new": [f[0, v, :cnt[v, 0]].tolist() for v in range(n)],
            "fwd_old": [f[1, v, :cnt[v, 1]].tolist() for v in range(n)],
            "rev_new": [r[0, v, :cnt[v, 2]].tolist() for v in range(n)],
            "rev_old": [r[1, v, :cnt[v, 3]].tolist() for v in range(n)],
            "NEW": [u[0, v, :fcnt[v, 0]].tolist() for v in range(n)],
            "OLD": [u[1, v, :fcnt[v, 1]].tolist() for v in range(n)]}
