// knng_brute.hip -- exact k-NN rows by brute force on one MI355X (gfx950).
//
// The exact kNNG is the reference that recall is measured against (paper Sec. 2.1, 5.3.1).
// Every (query, base) distance is evaluated in the fp64 recipe of the C ABI -- coordinates in
// index order, fused multiply-add, one rounding to fp32 -- so the (distance, id) order, and
// with it every returned index, is reproducible bit for bit by a sequential CPU evaluation.
//
// k_brute: a 256-thread workgroup owns 64 queries and walks a range of base points in tiles of
// 64.  Slabs of 32 coordinates of both tiles are staged transposed in LDS; each thread keeps a
// 4x4 block of fp64 accumulators.  After the last slab the 16 distances are packed with their
// ids, filtered against the query's current k-th key and queued in LDS; one wavefront per 16
// queries merges the queues into the sorted per-query lists by rank counting.
// k_brute_reduce: merges the lists of the base ranges and writes ids / distances.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

constexpr int BT = 64;            // tile edge (queries and base points)
constexpr int BDC = 32;           // coordinates per slab
constexpr int BLD = BT + 4;       // row stride of a transposed slab (floats)

template <int METRIC>
__global__ void __launch_bounds__(256)
k_brute(const float* __restrict__ pts, int64_t n, int d, int k,
        const int32_t* __restrict__ query_rows, int64_t nq, int64_t base_chunk, int nsplit,
        u64* __restrict__ part)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* QT = reinterpret_cast<float*>(smem);            // [BDC][BLD]
    float* BTt = QT + BDC * BLD;                           // [BDC][BLD]
    u64* pend = reinterpret_cast<u64*>(BTt + BDC * BLD);   // [BT][BT]
    u64* list = pend + BT * BT;                            // [BT][k] ascending
    u64* thr = list + BT * k;                              // [BT] current k-th key
    int* pcnt = reinterpret_cast<int*>(thr + BT);          // [BT]
    int* qrow = pcnt + BT;                                 // [BT] source point of each query

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t q0 = (int64_t)blockIdx.x * BT;
    const int64_t b_begin = (int64_t)blockIdx.y * base_chunk;
    const int64_t b_end = (b_begin + base_chunk) < n ? (b_begin + base_chunk) : n;

    if (tid < BT) {
        int64_t q = q0 + tid;
        int r = -1;
        if (q < nq) r = query_rows ? query_rows[q] : (int)q;
        qrow[tid] = r;
        thr[tid] = EMPTY_KEY;
        pcnt[tid] = 0;
    }
    for (int i = tid; i < BT * k; i += 256) list[i] = EMPTY_KEY;
    __syncthreads();

    const bool vec = (d & 3) == 0;
    for (int64_t b0 = b_begin; b0 < b_end; b0 += BT) {
        double acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

        for (int k0 = 0; k0 < d; k0 += BDC) {
            const int len = (d - k0) < BDC ? (d - k0) : BDC;
            __syncthreads();
            // stage both slabs transposed: thread -> (row, 4 coordinates)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int row = (tid >> 3) + 32 * half, c4 = tid & 7, t = 4 * c4;
                const int qr = qrow[row];
                const int64_t br = b0 + row;
                float4 xq = float4{0, 0, 0, 0}, xb = float4{0, 0, 0, 0};
                if (qr >= 0) {
                    const float* p = pts + (int64_t)qr * d + k0 + t;
                    if (vec && t + 3 < len) xq = *reinterpret_cast<const float4*>(p);
                    else {
                        if (t < len) xq.x = p[0];
                        if (t + 1 < len) xq.y = p[1];
                        if (t + 2 < len) xq.z = p[2];
                        if (t + 3 < len) xq.w = p[3];
                    }
                }
                if (br < b_end) {
                    const float* p = pts + br * d + k0 + t;
                    if (vec && t + 3 < len) xb = *reinterpret_cast<const float4*>(p);
                    else {
                        if (t < len) xb.x = p[0];
                        if (t + 1 < len) xb.y = p[1];
                        if (t + 2 < len) xb.z = p[2];
                        if (t + 3 < len) xb.w = p[3];
                    }
                }
                QT[(t + 0) * BLD + row] = xq.x; QT[(t + 1) * BLD + row] = xq.y;
                QT[(t + 2) * BLD + row] = xq.z; QT[(t + 3) * BLD + row] = xq.w;
                BTt[(t + 0) * BLD + row] = xb.x; BTt[(t + 1) * BLD + row] = xb.y;
                BTt[(t + 2) * BLD + row] = xb.z; BTt[(t + 3) * BLD + row] = xb.w;
            }
            __syncthreads();
            for (int t = 0; t < len; ++t) {
                const float4 qf = *reinterpret_cast<const float4*>(QT + t * BLD + 4 * ty);
                const float4 bf = *reinterpret_cast<const float4*>(BTt + t * BLD + 4 * tx);
                const float qa[4] = {qf.x, qf.y, qf.z, qf.w};
                const float ba[4] = {bf.x, bf.y, bf.z, bf.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = exact_step<METRIC>(acc[i][j], qa[i], ba[j]);
            }
        }
        // queue the survivors of this tile
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int qi = 4 * ty + i;
            const int qr = qrow[qi];
            const u64 t = thr[qi];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t b = b0 + 4 * tx + j;
                if (qr >= 0 && b < b_end && b != (int64_t)qr) {
                    const u64 key = pack_key(exact_finish<METRIC>(acc[i][j]), (int)b, 0);
                    if (key < t) {
                        int pos = atomicAdd(&pcnt[qi], 1);
                        pend[qi * BT + pos] = key;
                    }
                }
            }
        }
        __syncthreads();
        // merge: wavefront w owns queries 16w .. 16w+15
        for (int qq = 0; qq < 16; ++qq) {
            const int qi = 16 * w + qq;
            const int pc = pcnt[qi];
            if (pc == 0) continue;
            const u64 ck = lane < pc ? pend[qi * BT + lane] : EMPTY_KEY;
            const u64 lk = lane < k ? list[qi * k + lane] : EMPTY_KEY;
            int rl = lane, rc = 0;
            for (int j = 0; j < pc; ++j) {
                const u64 cj = bcast64(ck, j);
                rl += (cj < lk) ? 1 : 0;
                rc += (cj < ck) ? 1 : 0;
            }
            for (int i = 0; i < k; ++i) rc += (bcast64(lk, i) < ck) ? 1 : 0;
            if (lane < k && rl < k) list[qi * k + rl] = lk;
            if (lane < pc && rc < k) list[qi * k + rc] = ck;
            if (lane == 0) pcnt[qi] = 0;
        }
        __syncthreads();
        if (tid < BT) thr[tid] = list[tid * k + (k - 1)];
    }
    __syncthreads();
    for (int i = tid; i < BT * k; i += 256) {
        const int qi = i / k, e = i - qi * k;
        const int64_t q = q0 + qi;
        if (q < nq) part[(q * nsplit + blockIdx.y) * k + e] = list[i];
    }
}

// one wavefront per query: fold the nsplit sorted partial lists, write ids and distances
__global__ void __launch_bounds__(256)
k_brute_reduce(int64_t nq, int k, int nsplit, const u64* __restrict__ part,
               int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    const int lane = lane_id();
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;
    u64 cur = lane < k ? part[(q * nsplit) * k + lane] : EMPTY_KEY;
    for (int sidx = 1; sidx < nsplit; ++sidx) {
        const u64 oth = lane < k ? part[(q * nsplit + sidx) * k + lane] : EMPTY_KEY;
        int rcur = lane, roth = lane;            // both lists ascending
        for (int j = 0; j < k; ++j) {
            rcur += (bcast64(oth, j) < cur) ? 1 : 0;
            roth += (bcast64(cur, j) < oth) ? 1 : 0;
        }
        // scatter the first k of the union back into lanes through a shuffle-free trick:
        // lane r wants the element of rank r; ranks are a permutation, so invert by search
        u64 next = EMPTY_KEY;
        for (int j = 0; j < k; ++j) {
            const u64 cj = bcast64(cur, j);
            const int rj = (int)bcast32((uint32_t)rcur, j);
            if (rj == lane) next = cj;
            const u64 oj = bcast64(oth, j);
            const int sj = (int)bcast32((uint32_t)roth, j);
            if (sj == lane && oj != EMPTY_KEY) next = oj;
        }
        cur = lane < k ? next : EMPTY_KEY;
    }
    if (lane < k) {
        ids_out[q * k + lane] = key_id(cur);
        dists_out[q * k + lane] = key_dist(cur);
    }
}

static int brute_nsplit(int64_t n, int64_t nq)
{
    const int64_t qtiles = (nq + BT - 1) / BT;
    if (qtiles <= 0) return 1;
    int64_t want = (4096 + qtiles - 1) / qtiles;          // aim for a few thousand workgroups
    const int64_t max_split = (n + 64 * BT - 1) / (64 * BT); // at least 64 tiles per range
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    if (want > 1024) want = 1024;
    return (int)want;
}

}  // namespace knng

using namespace knng;

extern "C" __attribute__((visibility("default"))) uint64_t knng_brute_workspace_bytes(int64_t n, int32_t d, int32_t k, int64_t nq)
{
    if (n < 2 || d < 1 || k < 1 || k > KNNG_MAX_K || (int64_t)k > n - 1 || nq < 0) return 0;
    const uint64_t b = (uint64_t)nq * (uint64_t)brute_nsplit(n, nq) * (uint64_t)k * 8u;
    return b < 256 ? 256 : b;
}

extern "C" __attribute__((visibility("default"))) int knng_brute_knn(const float* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                              const int32_t* query_rows_dev, int64_t nq,
                              int32_t* ids_out_dev, float* dists_out_dev,
                              void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    if (!points_dev || n < 2 || n > 2147483647LL || d < 1 || k < 1 || k > KNNG_MAX_K ||
        (int64_t)k > n - 1 || nq < 0 || (metric != KNNG_METRIC_L2SQ && metric != KNNG_METRIC_IP_UNIT))
        return KNNG_EINVAL;
    if (nq == 0) return KNNG_OK;
    if (!ids_out_dev || !dists_out_dev) return KNNG_EINVAL;
    if (!query_rows_dev && nq > n) return KNNG_EINVAL;
    const uint64_t need = knng_brute_workspace_bytes(n, d, k, nq);
    if (!workspace_dev || workspace_bytes < need) return KNNG_EWORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int nsplit = brute_nsplit(n, nq);
    int64_t chunk = (n + nsplit - 1) / nsplit;
    chunk = (chunk + BT - 1) / BT * BT;
    const unsigned qtiles = (unsigned)((nq + BT - 1) / BT);
    const int lds = 2 * BDC * BLD * 4 + BT * BT * 8 + BT * k * 8 + BT * 8 + BT * 4 + BT * 4;
    u64* part = static_cast<u64*>(workspace_dev);
    hipError_t e;
    if (metric == 0) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_brute<0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute)");
        hipLaunchKernelGGL(k_brute<0>, dim3(qtiles, (unsigned)nsplit), dim3(256), lds, st, points_dev, n, d, k,
                           query_rows_dev, nq, chunk, nsplit, part);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_brute<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute)");
        hipLaunchKernelGGL(k_brute<1>, dim3(qtiles, (unsigned)nsplit), dim3(256), lds, st, points_dev, n, d, k,
                           query_rows_dev, nq, chunk, nsplit, part);
    }
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_brute launch");
    hipLaunchKernelGGL(k_brute_reduce, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, st, nq, k, nsplit, part,
                       ids_out_dev, dists_out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_brute_reduce launch");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return set_hip_error(e, "hipStreamSynchronize");
    return KNNG_OK;
}
