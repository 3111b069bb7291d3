// knng_search.hip -- greedy graph search for query points (Sec. 3.2: start from given points of
// the graph, explore by visiting neighbours of points already visited, until nothing closer
// turns up; k_s results per query).
//
// Per query a list of at most L <= 64 entries is kept ascending by (fp32 distance, id), ids
// distinct, each entry expanded or not.  "Offer x": if x is a valid id not in the list, evaluate
// its distance and keep the L smallest of the list and x.  Start: offer the query's start ids.
// Iteration: the first `width` unexpanded entries are marked expanded, then the graph row of each
// is offered, in list order; stop when no entry is unexpanded or at the iteration cap.  Result:
// the first k_s entries.
//
// One wavefront per query.  Lane t holds list entry t as a packed word (distance bits, id,
// expanded flag in bit 0).  A batch (the start ids, or one graph row: at most 64 ids) has a lane
// per id: the lane drops ids that are invalid, repeat an earlier lane's or are in the list,
// evaluates the distance with the fp64 recipe (the query sits in LDS, the candidate's vector
// streams through the lane, and stops early where a partial sum already rules the candidate
// out), drops what cannot enter a full list, and the survivors are merged by counting ranks.
// Offering a batch at once gives the same list as offering its ids one by one: the L smallest
// of a union do not depend on the order of insertion.
//
// ELEM = 1: points and queries stored as uint8 (squared L2): the distance is the exact integer
// sum of squared differences (unsigned 8-bit dot products on packed words), rounded once to fp32
// -- what the fp64 recipe gives on the same values.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

__device__ __forceinline__ void wave_lds_sync_search() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// four packed uint8 pairs: sum of squared differences = a.a + b.b - 2 a.b
__device__ __forceinline__ uint32_t search_sqdiff4_u8(uint32_t a, uint32_t b)
{
    const uint32_t nn = __builtin_amdgcn_udot4(a, a, __builtin_amdgcn_udot4(b, b, 0u, false), false);
    return nn - 2u * __builtin_amdgcn_udot4(a, b, 0u, false);
}

// ELEM 1: pts / queries point at uint8 rows and d counts 32-bit words (4 coordinates)
template <int METRIC, bool VEC, int ELEM = 0>
__global__ void __launch_bounds__(256)
k_graph_search(const float* __restrict__ pts, int64_t n, int d, const int32_t* __restrict__ graph, int deg,
               const float* __restrict__ queries, int64_t nq, const int32_t* __restrict__ starts, int n_starts,
               int k_s, int L, int width, int max_iters, int32_t* __restrict__ ids_out,
               float* __restrict__ dists_out, int32_t* __restrict__ iters_out, int32_t* __restrict__ evals_out)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ u64 lbuf[4][WAVE];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 4 + w;
    if (q >= nq) return;
    const int dpad = (d + 3) & ~3;
    float* qs = reinterpret_cast<float*>(smem) + (size_t)w * dpad;
    u64* lb = lbuf[w];
    for (int t = lane; t < dpad; t += WAVE) qs[t] = t < d ? queries[q * d + t] : 0.0f;
    wave_lds_sync_search();

    u64 lk = EMPTY_KEY;                                         // list entry `lane`
    int len = 0;
    int evals = 0;                                              // distances evaluated

    // offer the ids held by lanes < cnt
    auto offer_batch = [&](int id, int cnt) {
        // one sweep over the batch: lane j's id is dropped if the list holds it, and later lanes
        // that repeat it are dropped (lanes >= cnt hold -1 and match nothing)
        const int lid = lane < len ? key_id(lk) : -1;
        u64 okm = __ballot(lane < cnt && id >= 0 && (int64_t)id < n);
        for (int j = 0; j < cnt; ++j) {
            if (!((okm >> j) & 1ull)) continue;                 // uniform
            const int idj = (int)bcast32((uint32_t)id, j);
            if (__ballot(lid == idj) != 0ull) { okm &= ~(1ull << j); continue; }
            okm &= ~__ballot(lane > j && id == idj);
        }
        bool ok = (okm >> lane) & 1ull;
        if (okm == 0ull) return;
        evals += __popcll(okm);
        float dist = 0.0f;
        // Squared L2 with a full list: the partial sums only grow, in fp64 and after rounding to
        // fp32 alike, so a lane whose partial sum already rounds above the list's last distance
        // stops reading its vector -- the candidate would be left out with the full sum too.
        const float worst_d = len == L ? key_dist(bcast64(lk, L - 1)) : __uint_as_float(0x7f800000u);
        if (ELEM == 1) {
            if (ok) {
                const uint32_t* __restrict__ b = reinterpret_cast<const uint32_t*>(pts) + (int64_t)id * d;
                const uint32_t* qw = reinterpret_cast<const uint32_t*>(qs);
                uint32_t acc = 0u;
                if (VEC) {
                    for (int t = 0; t < d; t += 4) {
                        if ((float)acc > worst_d) { ok = false; break; }
                        const uint4 bv = *reinterpret_cast<const uint4*>(b + t);
                        const uint4 av = *reinterpret_cast<const uint4*>(qw + t);
                        acc += search_sqdiff4_u8(av.x, bv.x) + search_sqdiff4_u8(av.y, bv.y) +
                               search_sqdiff4_u8(av.z, bv.z) + search_sqdiff4_u8(av.w, bv.w);
                    }
                } else {
                    for (int t = 0; t < d; ++t) acc += search_sqdiff4_u8(qw[t], b[t]);
                }
                dist = (float)acc;
            }
        } else if (ok) {
            const float* __restrict__ b = pts + (int64_t)id * d;
            double acc = 0.0;
            if (VEC) {
                int t = 0;
                for (; t + 16 <= d; t += 16) {
                    if (METRIC == 0 && (float)acc > worst_d) { ok = false; break; }
                    float4 bv[4], av[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) bv[u] = *reinterpret_cast<const float4*>(b + t + 4 * u);
#pragma unroll
                    for (int u = 0; u < 4; ++u) av[u] = *reinterpret_cast<const float4*>(qs + t + 4 * u);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        acc = exact_step<METRIC>(acc, av[u].x, bv[u].x);
                        acc = exact_step<METRIC>(acc, av[u].y, bv[u].y);
                        acc = exact_step<METRIC>(acc, av[u].z, bv[u].z);
                        acc = exact_step<METRIC>(acc, av[u].w, bv[u].w);
                    }
                }
                for (; ok && t < d; t += 4) {
                    const float4 bv = *reinterpret_cast<const float4*>(b + t);
                    const float4 av = *reinterpret_cast<const float4*>(qs + t);
                    acc = exact_step<METRIC>(acc, av.x, bv.x);
                    acc = exact_step<METRIC>(acc, av.y, bv.y);
                    acc = exact_step<METRIC>(acc, av.z, bv.z);
                    acc = exact_step<METRIC>(acc, av.w, bv.w);
                }
            } else {
                for (int t = 0; t < d; ++t) acc = exact_step<METRIC>(acc, qs[t], b[t]);
            }
            dist = exact_finish<METRIC>(acc);
        }
        u64 ck = ok ? pack_key(dist, id, 0) : EMPTY_KEY;
        if (len == L) {                                         // cannot enter a full list
            const u64 worst = bcast64(lk, L - 1);
            if (ck > worst) ck = EMPTY_KEY;
        }
        const u64 cm = __ballot(ck != EMPTY_KEY);
        if (cm == 0ull) return;
        // ranks in the union: list entries move up by the candidates before them; a candidate
        // lands after the list entries and the candidates before it
        lb[lane] = lk;
        wave_lds_sync_search();
        int rl = lane, rc = 0;
        for (u64 m = cm; m; m &= m - 1) {
            const int j = __ffsll((long long)m) - 1;
            const u64 kj = bcast64(ck, j);
            rl += kj < lk ? 1 : 0;
            rc += kj < ck ? 1 : 0;
        }
        {
            int lo = 0, hi = len;                               // list entries before the candidate
            while (__ballot(lo < hi) != 0ull) {
                const int mid = (lo + hi) >> 1;
                const u64 lm = lb[mid < WAVE ? mid : WAVE - 1];
                if (lo < hi) { if (lm < ck) lo = mid + 1; else hi = mid; }
            }
            rc += lo;
        }
        wave_lds_sync_search();
        if (lane < len && rl < L) lb[rl] = lk;
        if (ck != EMPTY_KEY && rc < L) lb[rc] = ck;
        wave_lds_sync_search();
        len += __popcll(cm);
        if (len > L) len = L;
        lk = lane < len ? lb[lane] : EMPTY_KEY;
        wave_lds_sync_search();
    };

    offer_batch(lane < n_starts ? starts[q * n_starts + lane] : -1, n_starts);

    int iters = 0;
    for (; iters < max_iters; ++iters) {
        u64 un = __ballot(lane < len && !(lk & 1ull));
        if (un == 0ull) break;
        int par = -1;                                           // lane a: the a-th parent
        int np = 0;
        for (; np < width && un; ++np, un &= un - 1) {
            const int t = __ffsll((long long)un) - 1;
            const int pid = key_id(bcast64(lk, t));
            if (lane == np) par = pid;
            if (lane == t) lk |= 1ull;
        }
        for (int a = 0; a < np; ++a) {
            const int pid = (int)bcast32((uint32_t)par, a);
            offer_batch(lane < deg ? graph[(int64_t)pid * deg + lane] : -1, deg);
        }
    }
    if (lane < k_s) {
        ids_out[q * k_s + lane] = lane < len ? key_id(lk) : -1;
        dists_out[q * k_s + lane] = lane < len ? key_dist(lk) : __uint_as_float(0x7f800000u);
    }
    if (iters_out && lane == 0) iters_out[q] = iters;
    if (evals_out && lane == 0) evals_out[q] = evals;
}

}  // namespace knng

using namespace knng;

// elem 0: fp32 points and queries; elem 1: uint8 (squared L2, d % 4 == 0, d <= 65536)
static int search_impl(const void* points_void, const void* queries_void, int elem, int64_t n, int32_t d, int32_t metric,
                                 const int32_t* graph_dev, int32_t deg, int64_t nq,
                                 const int32_t* starts_dev, int32_t n_starts, int32_t k_s, int32_t itopk,
                                 int32_t width, int32_t max_iters, int32_t* ids_out_dev, float* dists_out_dev,
                                 int32_t* iters_out_dev, int32_t* evals_out_dev, void* stream)
{
    const float* points_dev = static_cast<const float*>(points_void);   // the kernel casts back for elem 1
    const float* queries_dev = static_cast<const float*>(queries_void);
    if (!points_dev || !graph_dev || nq < 0) return KNNG_EINVAL;
    if (nq > 0 && (!queries_dev || !starts_dev || !ids_out_dev || !dists_out_dev)) return KNNG_EINVAL;
    if (elem == 1) {
        if (metric != KNNG_METRIC_L2SQ || (d & 3) || d > 65536 || (reinterpret_cast<uintptr_t>(points_void) & 3u) ||
            (reinterpret_cast<uintptr_t>(queries_void) & 3u))
            return KNNG_EINVAL;
        d /= 4;                                                 // words from here on
    }
    if (n < 1 || n > 2147483647LL || d < 1 || deg < 1 || deg > KNNG_MAX_K || n_starts < 1 || n_starts > KNNG_MAX_K)
        return KNNG_EINVAL;
    if (k_s < 1 || itopk < k_s || itopk > KNNG_MAX_K || width < 1 || width > KNNG_MAX_K || max_iters < 0)
        return KNNG_EINVAL;
    if (metric != KNNG_METRIC_L2SQ && metric != KNNG_METRIC_IP_UNIT) return KNNG_EINVAL;
    const size_t lds = (size_t)4 * ((d + 3) & ~3) * sizeof(float);
    if (lds > 128 * 1024) return KNNG_EINVAL;                   // d <= 8192
    if (nq == 0) return KNNG_OK;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(points_dev) & 15u) == 0);
    auto kern = elem == 1 ? (vec ? k_graph_search<0, true, 1> : k_graph_search<0, false, 1>)
              : metric == 0 ? (vec ? k_graph_search<0, true, 0> : k_graph_search<0, false, 0>)
                            : (vec ? k_graph_search<1, true, 0> : k_graph_search<1, false, 0>);
    hipError_t e;
    if (lds > 48 * 1024) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_graph_search)");
    }
    const unsigned blocks = (unsigned)((nq + 3) / 4);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, st, points_dev, n, d, graph_dev, deg, queries_dev, nq,
                       starts_dev, n_starts, k_s, itopk, width, max_iters, ids_out_dev, dists_out_dev, iters_out_dev, evals_out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_graph_search launch");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return set_hip_error(e, "hipStreamSynchronize");
    return KNNG_OK;
}

extern "C" __attribute__((visibility("default"))) int knng_graph_search(const float* points_dev, int64_t n, int32_t d, int32_t metric,
                                 const int32_t* graph_dev, int32_t deg, const float* queries_dev, int64_t nq,
                                 const int32_t* starts_dev, int32_t n_starts, int32_t k_s, int32_t itopk,
                                 int32_t width, int32_t max_iters, int32_t* ids_out_dev, float* dists_out_dev,
                                 int32_t* iters_out_dev, int32_t* evals_out_dev, void* stream)
{
    return search_impl(points_dev, queries_dev, 0, n, d, metric, graph_dev, deg, nq, starts_dev, n_starts, k_s, itopk,
                       width, max_iters, ids_out_dev, dists_out_dev, iters_out_dev, evals_out_dev, stream);
}

extern "C" __attribute__((visibility("default"))) int knng_graph_search_u8(const uint8_t* points_dev, int64_t n, int32_t d, int32_t metric,
                                    const int32_t* graph_dev, int32_t deg, const uint8_t* queries_dev, int64_t nq,
                                    const int32_t* starts_dev, int32_t n_starts, int32_t k_s, int32_t itopk,
                                    int32_t width, int32_t max_iters, int32_t* ids_out_dev, float* dists_out_dev,
                                    int32_t* iters_out_dev, int32_t* evals_out_dev, void* stream)
{
    return search_impl(points_dev, queries_dev, 1, n, d, metric, graph_dev, deg, nq, starts_dev, n_starts, k_s, itopk,
                       width, max_iters, ids_out_dev, dists_out_dev, iters_out_dev, evals_out_dev, stream);
}
