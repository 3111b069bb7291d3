"""ctypes binding over libknng.so: argument marshalling only.

Every step of the path runs in the HIP library; torch is used for device
memory (inputs, outputs, workspace) and for the current stream.  If the
library is missing and cannot be built, calls raise: there is no fallback.
Function names and argument meaning follow include/knng.h.
"""
import ctypes
import os
import threading

import torch

from . import build as _build

L2SQ, IP_UNIT, COSINE = 0, 1, 2
MAX_K = 64
STATS_MAX_ITERS = 128

_P = ctypes.c_void_p


class Stats(ctypes.Structure):
    _fields_ = [("iterations", ctypes.c_int32),
                ("converged", ctypes.c_int32),
                ("updates", ctypes.c_uint64 * STATS_MAX_ITERS),
                ("join_ms", ctypes.c_float * STATS_MAX_ITERS),
                ("join_rows", ctypes.c_uint64 * STATS_MAX_ITERS),
                ("ms_init", ctypes.c_float), ("ms_sample", ctypes.c_float),
                ("ms_join", ctypes.c_float), ("ms_merge", ctypes.c_float),
                ("ms_finalize", ctypes.c_float), ("ms_total", ctypes.c_float),
                ("offers", ctypes.c_uint64),
                ("pairs", ctypes.c_uint64),
                ("cand_kept", ctypes.c_uint64),
                ("joined", ctypes.c_uint64),
                ("rejoined", ctypes.c_uint64),
                ("row_violations", ctypes.c_uint64)]


class Params(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32),
                ("k_build", ctypes.c_int32),
                ("rho", ctypes.c_float),
                ("delta", ctypes.c_float),
                ("max_iters", ctypes.c_int32),
                ("cand_cap", ctypes.c_int32),
                ("seed", ctypes.c_uint64),
                ("init_ids_dev", _P),
                ("stream", _P),
                ("workspace_dev", _P),
                ("workspace_bytes", ctypes.c_uint64),
                ("stats_host", ctypes.POINTER(Stats)),
                ("pinned_host", _P),
                ("check_rows", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


EXPORTS = ("knng_build_workspace_bytes", "knng_build_cosine_extra_bytes", "knng_build_knn_graph", "knng_build_knn_graph_u8", "knng_build_knn_graph_f16",
           "knng_brute_workspace_bytes",
           "knng_brute_knn", "knng_brute_knn_base", "knng_graph_recall", "knng_graph_recall_static", "knng_merge_graphs", "knng_optimize_workspace_bytes",
           "knng_optimize_graph", "knng_graph_search", "knng_graph_search_u8", "knng_strerror", "knng_version")

_lib = None


def lib_path() -> str:
    return _build.LIB


def load():
    """Load libknng.so (building it once if no built library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    # KNNG_LIBRARY: another build of the library (a tuning variant) instead of the in-tree one
    path = os.environ.get("KNNG_LIBRARY") or _build.LIB
    if path == _build.LIB and not os.path.exists(path):
        _build.build(force=True)
    L = ctypes.CDLL(path)
    i32, i64, u64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    L.knng_build_workspace_bytes.restype = u64
    L.knng_build_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(Params)]
    L.knng_build_cosine_extra_bytes.restype = u64
    L.knng_build_cosine_extra_bytes.argtypes = [i64, i32]
    L.knng_build_knn_graph.restype = ctypes.c_int
    L.knng_build_knn_graph.argtypes = [_P, i64, i32, i32, i32, ctypes.POINTER(Params), _P, _P]
    L.knng_build_knn_graph_f16.restype = ctypes.c_int
    L.knng_build_knn_graph_f16.argtypes = [_P, i64, i32, i32, i32, ctypes.POINTER(Params), _P, _P]
    L.knng_build_knn_graph_u8.restype = ctypes.c_int
    L.knng_build_knn_graph_u8.argtypes = [_P, i64, i32, i32, i32, ctypes.POINTER(Params), _P, _P]
    L.knng_brute_workspace_bytes.restype = u64
    L.knng_brute_workspace_bytes.argtypes = [i64, i32, i32, i64]
    L.knng_brute_knn.restype = ctypes.c_int
    L.knng_brute_knn.argtypes = [_P, i64, i32, i32, i32, _P, i64, _P, _P, _P, u64, _P]
    L.knng_brute_knn_base.restype = ctypes.c_int
    L.knng_brute_knn_base.argtypes = [_P, i64, i64, i32, i32, i32, _P, i64, _P, _P, _P, u64, _P]
    L.knng_graph_recall.restype = ctypes.c_int
    L.knng_graph_recall.argtypes = [_P, _P, i32, _P, _P, i32, i64, i32, i32,
                                    ctypes.POINTER(ctypes.c_double), _P]
    L.knng_graph_recall_static.restype = ctypes.c_int
    L.knng_graph_recall_static.argtypes = [_P, _P, i32, _P, _P, i32, i64, i32, i32, _P, _P]
    L.knng_merge_graphs.restype = ctypes.c_int
    L.knng_merge_graphs.argtypes = [_P, _P, i32, _P, _P, i32, i64, i32, _P, _P, _P]
    L.knng_optimize_workspace_bytes.restype = u64
    L.knng_optimize_workspace_bytes.argtypes = [i64, i32, i32]
    L.knng_optimize_graph.restype = ctypes.c_int
    L.knng_optimize_graph.argtypes = [_P, i64, i32, i32, _P, _P, u64, _P]
    L.knng_graph_search.restype = ctypes.c_int
    L.knng_graph_search.argtypes = [_P, i64, i32, i32, _P, i32, _P, i64, _P, i32, i32, i32, i32, i32, _P, _P, _P, _P, _P]
    L.knng_graph_search_u8.restype = ctypes.c_int
    L.knng_graph_search_u8.argtypes = L.knng_graph_search.argtypes
    L.knng_strerror.restype = ctypes.c_char_p
    L.knng_strerror.argtypes = [ctypes.c_int]
    L.knng_version.restype = ctypes.c_int
    L.knng_version.argtypes = []
    _lib = L
    return L


class KnngError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"libknng error {code}: {load().knng_strerror(code).decode()}")


def _check(code: int):
    if code != 0:
        raise KnngError(code)


def _dev(t, dtype, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _shape(t, shape, name):
    """The library takes sizes as scalars and cannot see how much memory stands behind a pointer:
    an array of another shape than those scalars say would be read or written past its end."""
    if t is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _room(t, shape, name):
    """An output array: at least as many elements as the library writes."""
    need = 1
    for e in shape:
        need *= int(e)
    if t is not None and t.numel() < need:
        raise ValueError(f"{name}: room for {t.numel()} elements, {need} ({tuple(shape)}) are written")
    return t


def _matrix(t, name):
    if t is not None and t.dim() != 2:
        raise ValueError(f"{name}: expected a 2-D tensor, got {tuple(t.shape)}")
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_tls = threading.local()


def _pinned_counter():
    """64 bytes of page-locked host memory per calling thread (the build's convergence counter)."""
    t = getattr(_tls, "pinned", None)
    if t is None:
        t = _tls.pinned = torch.empty(64, dtype=torch.uint8, pin_memory=True)
    return t


def knng_version() -> int:
    return int(load().knng_version())


def make_params(k_build=0, rho=0.0, delta=0.0, max_iters=0, cand_cap=0, seed=0, check_rows=False) -> Params:
    p = Params()
    p.struct_size = ctypes.sizeof(Params)
    p.k_build, p.rho, p.delta, p.max_iters, p.cand_cap, p.seed = (
        int(k_build), float(rho), float(delta), int(max_iters), int(cand_cap), int(seed))
    p.check_rows = 1 if check_rows else 0
    return p


def knng_build_workspace_bytes(n, d, k, params=None) -> int:
    return int(load().knng_build_workspace_bytes(n, d, k, ctypes.byref(params) if params else None))


def _build_graph(entry, dtype, points, k, metric, k_build, rho, delta, max_iters, cand_cap, seed,
                 init_ids, workspace, want_stats, ids_out, dists_out, check_rows=False):
    L = load()
    points = _matrix(_dev(points, dtype, "points"), "points")
    n, d = points.shape
    p = make_params(k_build, rho, delta, max_iters, cand_cap, seed, check_rows)
    need = int(L.knng_build_workspace_bytes(n, d, k, ctypes.byref(p)))
    if need == 0:
        raise KnngError(-1)
    if metric == COSINE:
        need += int(L.knng_build_cosine_extra_bytes(n, d))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=points.device)
    workspace = _dev(workspace, torch.uint8, "workspace")
    init_ids = _shape(_dev(init_ids, torch.int32, "init_ids"), (n, int(k_build) or int(k)), "init_ids")   # [n][K]
    if ids_out is None:
        ids_out = torch.empty((n, k), dtype=torch.int32, device=points.device)
    if dists_out is None:
        dists_out = torch.empty((n, k), dtype=torch.float32, device=points.device)
    ids_out = _room(_dev(ids_out, torch.int32, "ids_out"), (n, k), "ids_out")
    dists_out = _room(_dev(dists_out, torch.float32, "dists_out"), (n, k), "dists_out")
    st = Stats() if want_stats else None
    p.init_ids_dev = _ptr(init_ids)
    p.stream = _stream()
    p.workspace_dev = _ptr(workspace)
    p.workspace_bytes = workspace.numel()
    if st is not None:
        p.stats_host = ctypes.pointer(st)
    p.pinned_host = ctypes.c_void_p(_pinned_counter().data_ptr())
    _check(getattr(L, entry)(_ptr(points), n, d, k, metric, ctypes.byref(p), _ptr(ids_out), _ptr(dists_out)))
    stats = None
    if st is not None:
        it = min(st.iterations, STATS_MAX_ITERS)
        stats = {"iterations": st.iterations, "converged": bool(st.converged),
                 "updates": list(st.updates[:it]), "join_ms": list(st.join_ms[:it]),
                 "join_rows": list(st.join_rows[:it]), "ms_init": st.ms_init,
                 "ms_sample": st.ms_sample, "ms_join": st.ms_join, "ms_merge": st.ms_merge,
                 "ms_finalize": st.ms_finalize, "ms_total": st.ms_total,
                 "offers": int(st.offers), "pairs": int(st.pairs), "cand_kept": int(st.cand_kept), "joined": int(st.joined), "rejoined": int(st.rejoined),
                 "row_violations": int(st.row_violations)}
    return ids_out, dists_out, stats


def knng_build_knn_graph(points, k, metric=L2SQ, *, k_build=0, rho=0.0, delta=0.0, max_iters=0,
                         cand_cap=0, seed=0, init_ids=None, workspace=None, want_stats=True,
                         ids_out=None, dists_out=None, check_rows=False):
    """Approximate k-NN graph of `points` ([n][d] fp32, GPU).  -> (ids, dists, stats | None).

    Zero-valued keyword parameters select the library defaults; max_iters=-1 runs
    no refinement iteration (random graph).  `workspace` (uint8 GPU tensor) is
    allocated here when not given.
    """
    return _build_graph("knng_build_knn_graph", torch.float32, points, k, metric, k_build, rho, delta,
                        max_iters, cand_cap, seed, init_ids, workspace, want_stats, ids_out, dists_out, check_rows)


def knng_build_knn_graph_u8(points, k, metric=L2SQ, *, k_build=0, rho=0.0, delta=0.0, max_iters=0,
                            cand_cap=0, seed=0, init_ids=None, workspace=None, want_stats=True,
                            ids_out=None, dists_out=None, check_rows=False):
    """The same for `points` stored as [n][d] uint8 (GPU): squared L2 only, d % 4 == 0."""
    return _build_graph("knng_build_knn_graph_u8", torch.uint8, points, k, metric, k_build, rho, delta,
                        max_iters, cand_cap, seed, init_ids, workspace, want_stats, ids_out, dists_out, check_rows)


def knng_build_knn_graph_f16(points, k, metric=L2SQ, *, k_build=0, rho=0.0, delta=0.0, max_iters=0,
                             cand_cap=0, seed=0, init_ids=None, workspace=None, want_stats=True,
                             ids_out=None, dists_out=None, check_rows=False):
    """The same for `points` stored as [n][d] float16 (GPU): squared L2 only, d % 2 == 0."""
    return _build_graph("knng_build_knn_graph_f16", torch.float16, points, k, metric, k_build, rho, delta,
                        max_iters, cand_cap, seed, init_ids, workspace, want_stats, ids_out, dists_out, check_rows)


def knng_brute_workspace_bytes(n, d, k, nq) -> int:
    return int(load().knng_brute_workspace_bytes(n, d, k, nq))


def knng_brute_knn(points, k, metric=L2SQ, query_rows=None, workspace=None, n_base=None):
    """Exact k-NN rows of all points, or of `query_rows` (int32 GPU tensor), among all points or
    (knng_brute_knn_base) the first `n_base`.  -> (ids, dists)."""
    L = load()
    points = _matrix(_dev(points, torch.float32, "points"), "points")
    n, d = points.shape
    query_rows = _dev(query_rows, torch.int32, "query_rows")
    nq = n if query_rows is None else query_rows.numel()
    if query_rows is not None and nq > 0 and not (int(query_rows.min()) >= 0 and int(query_rows.max()) < n):
        raise ValueError("query_rows: row numbers must lie in [0, n)")   # the kernels index the points with them
    need = int(L.knng_brute_workspace_bytes(n, d, k, nq))
    if need == 0:
        raise KnngError(-1)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=points.device)
    workspace = _dev(workspace, torch.uint8, "workspace")
    ids = torch.empty((nq, k), dtype=torch.int32, device=points.device)
    dists = torch.empty((nq, k), dtype=torch.float32, device=points.device)
    if n_base is None:
        _check(L.knng_brute_knn(_ptr(points), n, d, k, metric, _ptr(query_rows), nq, _ptr(ids), _ptr(dists),
                                _ptr(workspace), workspace.numel(), _stream()))
    else:
        _check(L.knng_brute_knn_base(_ptr(points), n, n_base, d, k, metric, _ptr(query_rows), nq, _ptr(ids),
                                     _ptr(dists), _ptr(workspace), workspace.numel(), _stream()))
    return ids, dists


def knng_graph_recall(test_ids, test_dists, ref_ids, ref_dists, at_k, mode=0) -> float:
    """Recall of a test graph against a reference graph over the nearest at_k entries."""
    L = load()
    test_ids = _dev(test_ids, torch.int32, "test_ids")
    ref_ids = _dev(ref_ids, torch.int32, "ref_ids")
    test_dists = _dev(test_dists, torch.float32, "test_dists")
    ref_dists = _dev(ref_dists, torch.float32, "ref_dists")
    t = test_ids if test_ids is not None else test_dists
    r = ref_ids if ref_ids is not None else ref_dists
    if t is None or r is None or t.dim() != 2 or r.dim() != 2 or t.shape[0] != r.shape[0]:
        raise KnngError(-1)
    _shape(test_dists, t.shape, "test_dists")
    _shape(ref_dists, r.shape, "ref_dists")
    out = ctypes.c_double(0.0)
    _check(L.knng_graph_recall(_ptr(test_ids), _ptr(test_dists), t.shape[1], _ptr(ref_ids),
                               _ptr(ref_dists), r.shape[1], t.shape[0], at_k, mode,
                               ctypes.byref(out), _stream()))
    return float(out.value)


def knng_graph_recall_static(test_ids, test_dists, ref_ids, ref_dists, at_k, mode=0, out=None):
    """The same recall without allocation, host copy or synchronisation inside the library.
    -> `out`, a float64 GPU tensor of one element, valid once the current stream has run."""
    L = load()
    test_ids = _dev(test_ids, torch.int32, "test_ids")
    ref_ids = _dev(ref_ids, torch.int32, "ref_ids")
    test_dists = _dev(test_dists, torch.float32, "test_dists")
    ref_dists = _dev(ref_dists, torch.float32, "ref_dists")
    t = test_ids if test_ids is not None else test_dists
    r = ref_ids if ref_ids is not None else ref_dists
    if t is None or r is None or t.dim() != 2 or r.dim() != 2 or t.shape[0] != r.shape[0]:
        raise KnngError(-1)
    _shape(test_dists, t.shape, "test_dists")
    _shape(ref_dists, r.shape, "ref_dists")
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=t.device)
    out = _dev(out, torch.float64, "out")
    if out.numel() < 1:
        raise ValueError("out: expected one float64 element")
    _check(L.knng_graph_recall_static(_ptr(test_ids), _ptr(test_dists), t.shape[1], _ptr(ref_ids),
                                      _ptr(ref_dists), r.shape[1], t.shape[0], at_k, mode, _ptr(out), _stream()))
    return out


def knng_merge_graphs(ids_a, dists_a, ids_b, dists_b, k_out, ids_out=None, dists_out=None):
    """Rows of graph A updated with the candidates B: the k_out nearest distinct ids of both."""
    L = load()
    ids_a = _dev(ids_a, torch.int32, "ids_a")
    dists_a = _dev(dists_a, torch.float32, "dists_a")
    ids_b = _dev(ids_b, torch.int32, "ids_b")
    dists_b = _dev(dists_b, torch.float32, "dists_b")
    if ids_a is None or ids_b is None or dists_a is None or dists_b is None:
        raise KnngError(-1)
    if ids_a.dim() != 2 or ids_b.dim() != 2:
        raise KnngError(-1)
    if ids_a.shape != dists_a.shape or ids_b.shape != dists_b.shape or ids_a.shape[0] != ids_b.shape[0]:
        raise KnngError(-1)
    n = ids_a.shape[0]
    if ids_out is None:
        ids_out = torch.empty((n, k_out), dtype=torch.int32, device=ids_a.device)
    if dists_out is None:
        dists_out = torch.empty((n, k_out), dtype=torch.float32, device=ids_a.device)
    ids_out = _room(_dev(ids_out, torch.int32, "ids_out"), (n, k_out), "ids_out")
    dists_out = _room(_dev(dists_out, torch.float32, "dists_out"), (n, k_out), "dists_out")
    _check(L.knng_merge_graphs(_ptr(ids_a), _ptr(dists_a), ids_a.shape[1], _ptr(ids_b), _ptr(dists_b),
                               ids_b.shape[1], n, k_out, _ptr(ids_out), _ptr(dists_out), _stream()))
    return ids_out, dists_out


def knng_optimize_workspace_bytes(n, k, d_out) -> int:
    return int(load().knng_optimize_workspace_bytes(n, k, d_out))


def knng_optimize_graph(ids, d_out, workspace=None, ids_out=None):
    """Search graph of the k-NN graph `ids` ([n][k] int32, GPU, nearest first).  -> ids [n][d_out]."""
    L = load()
    ids = _matrix(_dev(ids, torch.int32, "ids"), "ids")
    n, k = ids.shape
    need = int(L.knng_optimize_workspace_bytes(n, k, d_out))
    if need == 0:
        raise KnngError(-1)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=ids.device)
    workspace = _dev(workspace, torch.uint8, "workspace")
    if ids_out is None:
        ids_out = torch.empty((n, d_out), dtype=torch.int32, device=ids.device)
    ids_out = _room(_dev(ids_out, torch.int32, "ids_out"), (n, max(int(d_out), 0)), "ids_out")
    _check(L.knng_optimize_graph(_ptr(ids), n, k, d_out, _ptr(ids_out), _ptr(workspace), workspace.numel(),
                                 _stream()))
    return ids_out


def _graph_search(entry, dtype, points, graph, queries, starts, k_s, itopk, width, max_iters, metric, want_iters):
    """Greedy search of `queries` ([nq][d] fp32) over `graph` ([n][deg] int32) from `starts`
    ([nq][n_starts] int32); all GPU tensors.
    -> (ids [nq][k_s], dists [nq][k_s][, iterations per query, distance evaluations per query])."""
    L = load()
    points = _matrix(_dev(points, dtype, "points"), "points")
    queries = _matrix(_dev(queries, dtype, "queries"), "queries")
    graph = _matrix(_dev(graph, torch.int32, "graph"), "graph")
    starts = _matrix(_dev(starts, torch.int32, "starts"), "starts")
    n, d = points.shape
    nq = queries.shape[0]
    if queries.shape[1] != d or graph.shape[0] != n or starts.shape[0] != nq:
        raise KnngError(-1)
    ids = torch.empty((nq, k_s), dtype=torch.int32, device=points.device)
    dists = torch.empty((nq, k_s), dtype=torch.float32, device=points.device)
    iters = torch.empty(nq, dtype=torch.int32, device=points.device) if want_iters else None
    evals = torch.empty(nq, dtype=torch.int32, device=points.device) if want_iters else None
    _check(getattr(L, entry)(_ptr(points), n, d, metric, _ptr(graph), graph.shape[1], _ptr(queries), nq,
                               _ptr(starts), starts.shape[1], k_s, itopk, width, max_iters, _ptr(ids),
                               _ptr(dists), _ptr(iters), _ptr(evals), _stream()))
    return (ids, dists, iters, evals) if want_iters else (ids, dists)


def knng_graph_search(points, graph, queries, starts, k_s, itopk, width=1, max_iters=64, metric=L2SQ,
                      want_iters=False):
    """Greedy search of `queries` ([nq][d] fp32) over `graph` ([n][deg] int32) from `starts`."""
    return _graph_search("knng_graph_search", torch.float32, points, graph, queries, starts, k_s, itopk, width,
                         max_iters, metric, want_iters)


def knng_graph_search_u8(points, graph, queries, starts, k_s, itopk, width=1, max_iters=64, metric=L2SQ,
                         want_iters=False):
    """The same for uint8 `points` and `queries` (squared L2, d % 4 == 0)."""
    return _graph_search("knng_graph_search_u8", torch.uint8, points, graph, queries, starts, k_s, itopk, width,
                         max_iters, metric, want_iters)
