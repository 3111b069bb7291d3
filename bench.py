#!/usr/bin/env python3
"""Benchmark of the single-GPU k-NN-graph build (one MI355X).

A step is one whole build (`knng_build_knn_graph`: init, all sample/join/merge
iterations until convergence, finalize) of the workload, with the points
already resident in HBM.  The default workload is the largest of the benchmark's
configurations that one GPU holds: number 5, 20,000,000 x 128 fp32, k = 32 (the
other configurations: `--config 1..4`, or a workload's name).  Workloads are
numbered as in the benchmark's own list, from 1; 6 is the connected set the graph
search uses.  Prints ONE JSON line:

  value      build throughput, points/s (n / seconds per build)
  roofline   the local-join kernel: algorithmic bytes of its launches in the
             timed region / their summed duration (HIP events recorded by the
             library on its stream), against 8 TB/s HBM
  cpu_baseline  the CPU oracle's NN-Descent timed on a bounded sample of the
             same recipe, on the host cores

  time_to_recall  outside the timed region: the smallest iteration cap whose
             graph reaches recall@k >= 0.95, its wall time and throughput

Recall@k is measured outside the timed region against the exact rows of a
seeded sample of points (GPU brute force, itself compared bit-for-bit with the
CPU oracle on a few rows); the run fails if recall@k < 0.95.

`--op optimize` times the search-graph optimisation (`knng_optimize_graph`) of
the graph that build produces instead (one step = one call; the graph is built
once, outside the timed region); the oracle runs on the same graph beside it
and the run fails unless the two results are identical.

`--op search` times the graph search (`knng_graph_search`): the workload's second
half searches the search graph of its first half (one level of the paper's
cross-partition refinement on one GPU; graph built and optimised once, outside
the timed region; one step = all queries); the oracle runs on a sample of the
queries beside it (identical results required), recall against exact neighbours
is measured on a sample outside the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
INT8_MFMA_PEAK_TOPS = 5000.0     # dense int8 MFMA (the uint8 build's Gram tiles)
FP16_MFMA_PEAK_TFLOPS = 2500.0   # dense fp16 MFMA (the fp16 build's Gram tiles)
SIG_BYTES = 32          # row signature read per gathered member
# HBM-side bytes per join launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE, each
# scaled by what a plain 1 GiB device copy reads: 2.0 and 1.0 KiB per count), averaged over the same
# launch mix as the timed region.  Only measured for the workloads and parameters listed
# (profiles/k_join_wave_u8gmm1024_1m_d128_hbm_traffic.txt: 17.28 GB fetched + 1.47 GB written).
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {("u8gmm1024_1m_d128_l2", "f32", 32, 0.5): 18.75e9,
                                     # profiles/k_join_wave_u8_u8gmm1024_1m_d128.txt: 7.92 GB + 1.47 GB
                                     ("u8gmm1024_1m_d128_l2", "u8", 32, 0.5): 9.39e9,
                                     # profiles/k_join_gmm4096_20m_d128_hbm_traffic.txt: 609.6 GB + 48.4 GB
                                     ("gmm4096_20m_d128_l2", "f32", 64, 0.375): 658.0e9}
BF16_MFMA_PEAK_TFLOPS = 2500.0   # dense bf16 MFMA (the split Gram pass of long fp32 rows: three per product)
SPLIT_MIN_D = 256                # fp32 rows from this length on take the bf16-split Gram pass (s <= 16; s > 16: from 64)
# Parameters a workload runs with when none are given: the cheapest set found that passes
# recall@k >= 0.95 (the paper's knobs, Sec. 5.3.1: a build degree above k, then cut to k).
# Everything else runs the paper's defaults K = k, rho = 0.5, delta = 1e-4.
PARAM_SETS = {"gmm4096_20m_d128_l2": dict(k_build=64, rho=0.375)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="",
                    help="workload number (1..6, as the benchmark's configurations are listed) or name; default 5 "
                         "(20M x 128), for --op optimize 2, for --op search 6 (a set whose graph a walk can cross)")
    ap.add_argument("--n", type=int, default=0, help="override the number of points")
    ap.add_argument("--elem", choices=("f32", "u8", "f16"), default="f32",
                    help="point storage; u8 (knng_build_knn_graph_u8) needs a workload with 8-bit values: config 2; "
                         "f16 (knng_build_knn_graph_f16) rounds the workload's values to fp16 first (squared L2 only)")
    ap.add_argument("--op", choices=("build", "optimize", "search"), default="build")
    ap.add_argument("--itopk", type=int, default=64, help="--op search: list length")
    ap.add_argument("--width", type=int, default=1, help="--op search: entries expanded per iteration")
    ap.add_argument("--n-starts", type=int, default=32, help="--op search: start points per query")
    ap.add_argument("--max-search-iters", type=int, default=100)
    ap.add_argument("--oracle-queries", type=int, default=20000, help="--op search: queries the oracle repeats")
    ap.add_argument("--d-out", type=int, default=0, help="--op optimize: degree of the search graph (default k)")
    ap.add_argument("--k-build", type=int, default=0)
    ap.add_argument("--rho", type=float, default=0.0)
    ap.add_argument("--delta", type=float, default=0.0)
    ap.add_argument("--max-iters", type=int, default=0)
    ap.add_argument("--recall-rows", type=int, default=20000)
    ap.add_argument("--oracle-rows", type=int, default=-1,
                    help="sampled rows the CPU oracle repeats (default 128; 64 above 2M points)")
    ap.add_argument("--cpu-n", type=int, default=-1,
                    help="points of the CPU-baseline sample (0 = skip; default 250000, fewer for K > 32 or long rows)")
    ap.add_argument("--time-to-recall", type=int, default=1,
                    help="also search the smallest iteration cap that reaches recall@k >= 0.95 (0 = skip)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (counter calibration under rocprofv3 --pmc)")
    return ap.parse_args()


def bench_optimize(a):
    """knng_optimize_graph on the k-NN graph of the workload (built once, untimed)."""
    import numpy as np
    import torch
    from paper_2605_27691_amd import knng, workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    x, w = workloads.make(a.config, n=(a.n or None), device=dev)
    n, k = w.n, w.k
    d_out = a.d_out or k
    g_ids, _, st = knng.knng_build_knn_graph(x, k, w.metric, seed=0, k_build=a.k_build, rho=a.rho, delta=a.delta)
    del x
    ws = torch.empty(knng.knng_optimize_workspace_bytes(n, k, d_out), dtype=torch.uint8, device=dev)
    out = torch.empty((n, d_out), dtype=torch.int32, device=dev)
    for _ in range(a.warmup):
        knng.knng_optimize_graph(g_ids, d_out, workspace=ws, ids_out=out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        knng.knng_optimize_graph(g_ids, d_out, workspace=ws, ids_out=out)
    e1.record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / max(a.steps, 1)
    dev_ms = e0.elapsed_time(e1) / max(a.steps, 1)
    # algorithmic bytes per point: own row + k neighbour rows (4k each); the pruned list with its
    # places (8 per entry) written once and read twice; the (p, u) words (8) written and read;
    # the result (4 per entry); in-degree counter, offsets
    alg_bytes = n * (4 * k * (k + 1) + (24 + 16 + 4) * d_out + 40)
    import oracle
    ids_h = g_ids.cpu().numpy()
    t1 = time.perf_counter()
    want = oracle.optimize_graph(ids_h, d_out)
    cpu_sec = time.perf_counter() - t1
    same = bool(np.array_equal(want, out.cpu().numpy()))
    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    res = {
        "metric": "search-graph optimisation points/sec (1 MI355X)",
        "value": n / sec, "unit": "points/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i32", "data": "synthetic",
        "config": {"workload": w.name + "_knn_graph", "n": n, "k": k, "d_out": d_out,
                   "graph_from": "knng_build_knn_graph, seed 0", "build_iterations": st["iterations"]},
        "oracle_check": {"identical_to_oracle": same, "rows": n},
        "roofline": {"kernel": "knng_optimize_graph (k_opt_prune, prefix sum, k_opt_fill, k_opt_merge)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "device_ms_per_call": dev_ms,
                     "alg_bytes_per_call": alg_bytes},
        "cpu_baseline": {"value": n / cpu_sec, "unit": "points/s", "cores": oracle.num_threads(), "kind": "oracle",
                         "sample": f"oracle_optimize_graph on the same {n} x {k} graph, {cpu_sec:.2f} s"},
    }
    print(json.dumps(res))
    if not same:
        print("bench.py: the search graph differs from the oracle's", file=sys.stderr)
        sys.exit(1)


def bench_search(a):
    """knng_graph_search: the second half of the workload searches the first half's search graph."""
    import numpy as np
    import torch
    from paper_2605_27691_amd import knng, workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    x, w = workloads.make(a.config, n=(a.n or None), device=dev)
    n, d, k = w.n // 2, w.d, w.k
    build, search, elem_bytes = knng.knng_build_knn_graph, knng.knng_graph_search, 4
    if a.elem == "u8":                      # the workload quantised to 8 bits: x -> round(24 x + 128), clipped
        if w.metric != 0:
            print("bench.py: --elem u8 needs squared L2", file=sys.stderr)
            sys.exit(2)
        x = (x * 24.0 + 128.0).round_().clamp_(0.0, 255.0)
        build, search, elem_bytes = knng.knng_build_knn_graph_u8, knng.knng_graph_search_u8, 1
    elif a.elem != "f32":
        print("bench.py: --op search takes --elem f32 or u8", file=sys.stderr)
        sys.exit(2)
    x = x[:2 * n].contiguous()                              # fp32 values: ground truth and the oracle use them
    pa, qb = x[:n], x[n:]
    sa, sq = (pa.to(torch.uint8), qb.to(torch.uint8)) if a.elem == "u8" else (pa, qb)
    nq = qb.shape[0]
    d_out = a.d_out or k
    g_ids, _, st = build(sa, k, w.metric, seed=0, k_build=a.k_build, rho=a.rho, delta=a.delta)
    gs = knng.knng_optimize_graph(g_ids, d_out)
    del g_ids
    gen = torch.Generator(device="cpu").manual_seed(12345)
    starts = torch.randint(0, n, (nq, a.n_starts), generator=gen, dtype=torch.int32).to(dev)
    args = (sa, gs, sq, starts, k, a.itopk, a.width, a.max_search_iters, w.metric)
    for _ in range(a.warmup):
        search(*args)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        ids, dists = search(*args)
    e1.record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / max(a.steps, 1)
    dev_ms = e0.elapsed_time(e1) / max(a.steps, 1)
    ids, dists, iters, evals = search(*args, want_iters=True)
    tot_iters, tot_evals = int(iters.sum()), int(evals.sum())
    # algorithmic bytes: every evaluated candidate's vector, every expanded row, per query its
    # vector, start ids and result
    alg_bytes = tot_evals * elem_bytes * d + tot_iters * a.width * 4 * d_out + nq * (elem_bytes * d + 4 * a.n_starts + 8 * k)
    gathered_rate = alg_bytes / (dev_ms * 1e-3) / 1e9
    # The whole-vector count above is not what the kernel must read: a lane stops reading a vector
    # once its partial sum rules the candidate out.  The bytes it did read are the measured fetch
    # (profiles/k_graph_search_manifold16_500k_d128.txt: FETCH_SIZE + WRITE_SIZE, default arguments
    # only); the fraction is of that, and stays null where no measurement exists.  The searched half
    # (256 MB) fits the Infinity Cache, which FETCH_SIZE does not tell from HBM: the kernel is bound by
    # the memory system below the L2, of which HBM's 8 TB/s is the slower part.
    traffic = 422.1e9 if (w.name, a.itopk, a.width, a.n_starts, d_out) == \
        ("manifold16_1m_d128_l2", 64, 1, 32, 32) and not a.n and a.elem == "f32" else None
    achieved = traffic / (dev_ms * 1e-3) / 1e9 if traffic else None
    # recall on a sample (outside the timed region): the exact neighbours, in the first half, of
    # sampled points of the second half
    ns = min(a.recall_rows, nq)
    rows_s = workloads.sample_rows(nq, ns)
    sel = torch.from_numpy(rows_s).to(dev).long()
    ex_i, ex_d = knng.knng_brute_knn(x, k, w.metric, (sel + n).int(), n_base=n)
    recall = knng.knng_graph_recall(ids[sel].contiguous(), dists[sel].contiguous(), ex_i, ex_d, k, 0)
    import oracle
    no = min(a.oracle_queries, nq)
    pa_h, gs_h = pa.cpu().numpy(), gs.cpu().numpy()
    chk = np.arange(0, ns, max(1, ns // 64))[:64]            # a few exact rows against the oracle's
    o_ei, o_ed = oracle.brute_knn(x.cpu().numpy(), k, w.metric, query_rows=(rows_s[chk] + n).astype(np.int32), n_base=n)
    brute_ok = bool(np.array_equal(o_ei, ex_i[chk].cpu().numpy()) and np.array_equal(o_ed, ex_d[chk].cpu().numpy()))
    t1 = time.perf_counter()
    o_i, o_d, o_it, o_ev = oracle.graph_search(pa_h, gs_h, qb[:no].cpu().numpy(), starts[:no].cpu().numpy(), k, a.itopk,
                                                a.width, a.max_search_iters, w.metric, want_evals=True)
    cpu_sec = time.perf_counter() - t1
    # ids, distances and iteration counts are the oracle's bit for bit; the kernel offers a row as a
    # batch and so evaluates at most as many distances as the oracle's one offer at a time
    same = bool(np.array_equal(o_i, ids[:no].cpu().numpy()) and
                np.array_equal(o_d.view(np.uint32), dists[:no].cpu().numpy().view(np.uint32)) and
                np.array_equal(o_it, iters[:no].cpu().numpy()) and np.all(evals[:no].cpu().numpy() <= o_ev))
    res = {
        "metric": "graph search queries/sec (1 MI355X)",
        "value": nq / sec, "unit": "queries/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if a.elem == "f32" else "u8 x u8 -> u32", "data": "synthetic",
        "config": {"workload": w.name + ("" if a.elem == "f32" else "_quantised_u8") + "_second_half_searches_first_half", "n": n, "nq": nq, "d": d, "k_s": k,
                   "graph_degree": d_out, "itopk": a.itopk, "width": a.width, "n_starts": a.n_starts,
                   "max_iters": a.max_search_iters, "metric": ["l2sq", "ip_unit"][w.metric]},
        "recall_at_k": recall, "recall_rows": ns,
        "mean_iterations": tot_iters / nq, "mean_distance_evaluations": tot_evals / nq,
        "oracle_check": {"identical_to_oracle": same, "queries": no, "exact_rows_bit_exact": brute_ok},
        "roofline": {"kernel": "k_graph_search", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": min(1.0, achieved / HBM_PEAK_GBS) if achieved else None,
                     "traffic": traffic,
                     "note": "achieved = measured L2-miss bytes (early abandon included) per call / time; the "
                             "searched half fits the Infinity Cache, so part of it is not HBM traffic",
                     "whole_vector_bytes_per_call": alg_bytes, "whole_vector_rate_gbs": gathered_rate,
                     "device_ms_per_call": dev_ms},
        "cpu_baseline": {"value": no / cpu_sec, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
                         "sample": f"oracle_graph_search on the first {no} queries, {cpu_sec:.1f} s"},
    }
    print(json.dumps(res))
    if not same or not brute_ok:
        print("bench.py: the search results or the exact rows differ from the oracle's", file=sys.stderr)
        sys.exit(1)


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (nothing here uses a second GPU)",
              file=sys.stderr)
        sys.exit(2)
    from paper_2605_27691_amd import workloads as _wl
    try:
        a.config = _wl.number_of(a.config or {"search": 6, "optimize": 2, "build": 5}[a.op])
    except ValueError as e:
        print(f"bench.py: {e}", file=sys.stderr)
        sys.exit(2)
    if a.op == "optimize":
        return bench_optimize(a)
    if a.op == "search":
        return bench_search(a)
    import numpy as np
    import torch
    from paper_2605_27691_amd import knng, workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    x, w = workloads.make(a.config, n=(a.n or None), device=dev)
    n, d, k = w.n, w.d, w.k
    if not (a.k_build or a.rho or a.delta):                 # nothing given: the workload's own set
        for key, val in PARAM_SETS.get(w.name, {}).items():
            setattr(a, key, val)
    kw = dict(k_build=a.k_build, rho=a.rho, delta=a.delta, max_iters=a.max_iters)
    K = a.k_build or k
    s_size = max(1, min(K, int(np.ceil(np.float32(a.rho or 0.5).astype(np.float64) * K))))
    if a.oracle_rows < 0:
        a.oracle_rows = 128 if n <= 2_000_000 else 64
    if a.cpu_n < 0:                                         # about 10-30 s of oracle work on 16 cores
        a.cpu_n = int(250000 * (0.5 if K > 32 else 1.0) * (0.4 if d > 384 else 1.0))
    p = knng.make_params(**kw)
    ws = torch.empty(knng.knng_build_workspace_bytes(n, d, k, p), dtype=torch.uint8, device=dev)
    ids = torch.empty((n, k), dtype=torch.int32, device=dev)
    dists = torch.empty((n, k), dtype=torch.float32, device=dev)

    build, xb, elem_bytes = knng.knng_build_knn_graph, x, 4
    if a.elem == "u8":
        xb = x.to(torch.uint8)
        if w.metric != 0 or not torch.equal(xb.float(), x):
            print("bench.py: --elem u8 needs 8-bit point values and squared L2 (config 2)", file=sys.stderr)
            sys.exit(2)
        build, elem_bytes = knng.knng_build_knn_graph_u8, 1
    if a.elem == "f16":
        if w.metric != 0:
            print("bench.py: --elem f16 needs squared L2", file=sys.stderr)
            sys.exit(2)
        xb = x.to(torch.float16)
        x = xb.float()                      # the values the build sees: ground truth and oracle use them
        build, elem_bytes = knng.knng_build_knn_graph_f16, 2

    def step(seed):
        return build(xb, k, w.metric, seed=seed, workspace=ws, ids_out=ids, dists_out=dists, **kw)[2]

    for i in range(a.warmup):
        step(1000 + i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = [step(i) for i in range(a.steps)]
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / max(a.steps, 1)

    if a.calib_copy_mib > 0:       # a copy kernel of known size: FETCH_SIZE / WRITE_SIZE should read this many MiB
        src = torch.empty(a.calib_copy_mib * 262144, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- what a plain device copy reaches on this machine (the practical HBM ceiling, same process)
    cp_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()      # 1 GiB
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        cp_dst.copy_(cp_src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * cp_src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del cp_src, cp_dst

    # ---- roofline of the dominant kernel (local join), over the timed region
    join_ms = sum(sum(s["join_ms"]) for s in stats)
    launches = sum(len(s["join_ms"]) for s in stats)
    rows = sum(sum(s["join_rows"]) for s in stats)
    alg_bytes = rows * (elem_bytes * d + 4 + 4 + SIG_BYTES) + launches * n * 16
    achieved = alg_bytes / (join_ms * 1e-3) / 1e9 if join_ms > 0 else 0.0
    pairs = sum(s["pairs"] for s in stats)                    # pairs the joins had to evaluate
    offers = sum(s["offers"] for s in stats)                  # atomic mins sent to candidate slots
    kept = sum(s["cand_kept"] for s in stats)                 # slots the merges found occupied
    needed_tflops = 2.0 * d * pairs / (join_ms * 1e-3) / 1e12 if join_ms > 0 else 0.0
    last = stats[-1]
    # the join is priced against HBM (a gather) unless its Gram blocks are the larger fraction of
    # their own peak (large samples: s = 32 does four times the pair work per gathered byte)
    mfma_peak = {"u8": INT8_MFMA_PEAK_TOPS, "f16": FP16_MFMA_PEAK_TFLOPS, "f32": FP32_MFMA_PEAK_TFLOPS}[a.elem]
    # long fp32 rows: the Gram pass runs on the bf16 matrix instruction, three instructions per product
    split = a.elem == "f32" and d % 4 == 0 and ((d >= SPLIT_MIN_D and s_size <= 16) or (d >= 64 and s_size > 16))
    mfma_work = needed_tflops
    if split:
        mfma_peak, mfma_work = BF16_MFMA_PEAK_TFLOPS, 3.0 * needed_tflops
    if mfma_work / mfma_peak > achieved / HBM_PEAK_GBS:
        bound = {"bound": "mfma", "achieved": mfma_work, "peak": mfma_peak, "unit": "TFLOP/s",
                 "frac": mfma_work / mfma_peak, "hbm_gbs": achieved, "frac_of_hbm_peak": achieved / HBM_PEAK_GBS}
    else:
        bound = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": achieved / HBM_PEAK_GBS}

    traffic = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get((w.name, a.elem, K, a.rho or 0.5))
    t_ratio = traffic / (alg_bytes / max(launches, 1)) if traffic else None
    t_frac = traffic / (join_ms / max(launches, 1) * 1e-3) / 1e9 / HBM_PEAK_GBS if traffic and join_ms > 0 else None

    # ---- quality, outside the timed region
    rows_s = workloads.sample_rows(n, a.recall_rows)
    rows_d = torch.from_numpy(rows_s).to(dev)
    ex_i, ex_d = knng.knng_brute_knn(x, k, w.metric, rows_d)
    sel = rows_d.long()
    t_i, t_d = ids[sel].contiguous(), dists[sel].contiguous()
    recall = knng.knng_graph_recall(t_i, t_d, ex_i, ex_d, k, 0)
    recall_dist = knng.knng_graph_recall(t_i, t_d, ex_i, ex_d, k, 1)

    # ---- time to recall (outside the timed region): the smallest iteration cap whose graph
    # reaches recall@k >= 0.95 on the same sample, everything else as in the timed builds
    ttr = None
    if a.time_to_recall and recall >= 0.95:
        ids2, dists2 = torch.empty_like(ids), torch.empty_like(dists)
        kw2 = dict(kw)
        kw2.pop("max_iters")

        def probe(cap):
            best = None
            for rep_ in range(2 if n <= 2_000_000 else 1):
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                st2 = build(xb, k, w.metric, seed=0, workspace=ws, ids_out=ids2, dists_out=dists2,
                            max_iters=cap, **kw2)[2]
                torch.cuda.synchronize()
                el = time.perf_counter() - t1
                best = el if best is None or el < best else best
            r2 = knng.knng_graph_recall(ids2[sel].contiguous(), dists2[sel].contiguous(), ex_i, ex_d, k, 0)
            return {"max_iters": cap, "iterations": st2["iterations"], "ms": best * 1e3,
                    "points_per_s": n / best, "recall_at_k": r2}

        # recall grows with the cap: bisect for the smallest cap that passes (the full run does)
        lo, hi = 1, stats[-1]["iterations"]
        while lo < hi:
            mid = (lo + hi) // 2
            got = probe(mid)
            if got["recall_at_k"] >= 0.95:
                hi, ttr = mid, got
            else:
                lo = mid + 1
        if ttr is None or ttr["max_iters"] != lo:
            ttr = probe(lo)
        del ids2, dists2

    # ---- the oracle: exact rows and row invariants on a few sampled rows, then the CPU baseline
    import oracle
    xh = x.cpu().numpy()
    sub = np.arange(0, len(rows_s), max(1, len(rows_s) // max(a.oracle_rows, 1)))[:a.oracle_rows]
    o_i, o_d = oracle.brute_knn(xh, k, w.metric, query_rows=rows_s[sub])
    brute_ok = bool(np.array_equal(o_i, ex_i[sub].cpu().numpy()) and
                    np.array_equal(o_d, ex_d[sub].cpu().numpy()))
    viol = oracle.check_graph(xh, t_i[sub].cpu().numpy(), t_d[sub].cpu().numpy(), w.metric,
                              rel_tol=1e-5, rows=rows_s[sub])
    cpu = None
    if a.cpu_n > 0:
        xs, wsml = workloads.make(a.config, n=min(a.cpu_n, n))
        t1 = time.perf_counter()
        _, _, ost = oracle.nn_descent(xs, k, w.metric, k_build=K, rho=(a.rho or 0.5),
                                      delta=(a.delta or 1e-4), max_iters=(a.max_iters or 100), seed=0)
        cpu_sec = time.perf_counter() - t1
        cpu = {"value": wsml.n / cpu_sec, "unit": "points/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"oracle NN-Descent (fp64 distances) on {wsml.n} points of the same recipe "
                         f"({wsml.n_centres} centres), {ost['iterations']} iterations, {cpu_sec:.1f} s"}

    out = {
        "metric": "kNN-graph build points/sec at recall@k>=0.95 (1 MI355X)",
        "value": n / sec, "unit": "points/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16x3-split -> f32" if split else
                  {"f32": "f32", "u8": "i8 x i8 -> i32", "f16": "f16 x f16 -> f32"}[a.elem]), "data": "synthetic",
        "config": {"workload": w.name + ("" if a.elem == "f32" else "_stored_" + a.elem), "n": n, "d": d, "k": k, "metric": ["l2sq", "ip_unit"][w.metric],
                   "config_number": a.config, "k_build": K, "rho": a.rho or 0.5, "sample_size": s_size,
                   "delta": a.delta or 1e-4, "join_kernel": "k_join_wave" if s_size <= 16 else "k_join",
                   "iterations": last["iterations"], "converged": last["converged"]},
        "recall_at_k": recall, "recall_at_k_distance": recall_dist, "recall_rows": int(len(rows_s)),
        "time_to_recall": ttr,
        "oracle_check": {"brute_rows_bit_exact": brute_ok, "rows": int(len(sub)),
                         "graph_violations": int(sum(viol.values()))},
        "kernel_ms": {"init": last["ms_init"], "sample": last["ms_sample"], "join": last["ms_join"],
                      "merge": last["ms_merge"], "finalize": last["ms_finalize"], "total": last["ms_total"]},
        "roofline": {"kernel": "k_join_wave" if s_size <= 16 else "k_join", **bound,
                     "traffic": traffic, "traffic_over_algorithmic": t_ratio, "hbm_frac_of_measured_traffic": t_frac,
                     "launches": launches, "avg_launch_ms": join_ms / max(launches, 1),
                     "alg_bytes_per_launch": alg_bytes / max(launches, 1),
                     "device_copy_gbs": copy_gbs, "frac_of_device_copy": achieved / copy_gbs,
                     # gathered rows repeat (neighbours of neighbours share members): above the copy rate
                     # part of them came from the L2 / Infinity Cache, not from HBM
                     "cache_reuse": bool(achieved > copy_gbs),
                     "needed_pair_tflops": needed_tflops, "mfma_peak_tflops": mfma_peak,
                     "frac_of_mfma_peak": mfma_work / mfma_peak,
                     "offers_per_launch": offers / max(launches, 1),
                     # offers that did not survive in their slot (a repeat of the same neighbour or a
                     # closer neighbour sharing the slot): upper bound of the candidates dropped
                     "offers_not_kept_share": (offers - kept) / max(offers, 1),
                     # joins repeated in fp32 because the bf16-split Gram pass chose a partner it could
                     # not be trusted with (share of the joins of the timed builds)
                     "rejoined_share": sum(s["rejoined"] for s in stats) / max(sum(s["joined"] for s in stats), 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    if recall < 0.95 or not brute_ok or sum(viol.values()) != 0:
        print(f"bench.py: quality gate failed (recall={recall:.4f}, brute_ok={brute_ok}, viol={viol})",
              file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
