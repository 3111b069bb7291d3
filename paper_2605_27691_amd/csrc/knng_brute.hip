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
//
// k_brute_mfma (rows with d % 4 == 0): the same walk, but a tile is first screened with an fp32
// Gram block on the matrix cores (v_mfma_f32_16x16x4_f32: |q|^2 + |b|^2 - 2<q,b>, or 1 - <q,b>).
// The fp32 value differs from the true distance by at most E = (d + 16) 2^-23 (|q|^2 + |b|^2)
// (more than twice the textbook bound of a length-d fp32 dot product plus the roundings around
// it), so a pair whose screened value minus E lies above a bound on the query's final k-th
// distance cannot be in the result and is skipped; every other pair is evaluated in the exact
// fp64 recipe, and only exact values are ever stored or compared.  The bound is the smaller of the
// k-th distance of the workgroup's own list and the smallest k-th distance any base range of the
// same query has published (one atomic min per query in device memory): with it all ranges
// together evaluate about as many pairs exactly as one pass over all points would.  The result is
// the same bit for bit whatever the timing.
// The walk over (tile, slab of 32 coordinates) is software-pipelined: every thread keeps the
// pieces of the next four slabs in flight in registers (all loads unconditional, from clamped
// addresses), a slab goes to one of two LDS buffers one step before it is multiplied, with one
// barrier per slab, and the stores and the next loads stand between the groups of four matrix
// instructions of the step.
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
        u64* __restrict__ part, const double* __restrict__ nrm64)
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
                    // METRIC 2: nrm64 holds every row's |x|^2 as the sequential fp64 chain gives it
                    const float dist = METRIC == 2 ? cosine_finish(acc[i][j], nrm64[qr], nrm64[b])
                                                   : exact_finish<METRIC == 2 ? 1 : METRIC>(acc[i][j]);
                    const u64 key = pack_key(dist, (int)b, 0);
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

// |x_i|^2 of every point, fp64 sum rounded once (8 lanes per row)
__global__ void __launch_bounds__(256)
k_row_norms(const float* __restrict__ pts, int64_t n, int d, float* __restrict__ nrm)
{
    const int sub = threadIdx.x & 7;
    const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 3;
    double acc = 0.0;
    if (row < n)
        for (int t = sub; t < d; t += 8) { const double x = (double)pts[row * d + t]; acc = fma(x, x, acc); }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    if (row < n && sub == 0) nrm[row] = (float)acc;
}

__global__ void __launch_bounds__(256)
k_fill_u32(uint32_t* __restrict__ p, int64_t count, uint32_t value)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = value;
}

// |x_i|^2 of every point as the distance recipe's own chain gives it: fp64, coordinates in index
// order, fused multiply-add, no rounding to fp32 (general cosine).  One lane per row.
__global__ void __launch_bounds__(256)
k_row_norms_exact(const float* __restrict__ pts, int64_t n, int d, double* __restrict__ nrm64)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= n) return;
    const float* x = pts + row * d;
    double acc = 0.0;
    for (int t = 0; t < d; ++t) acc = exact_step<2>(acc, x[t], x[t]);
    nrm64[row] = acc;
}

// the value of lane - 1 (lane 0: 0), one DPP move per 32-bit half
__device__ __forceinline__ u64 wave_shr1_64(u64 v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, 0x138, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), 0x138, 0xf, 0xf, false);
    return ((u64)hi << 32) | lo;
}

constexpr int MLD = BDC + 4;      // row stride of a row-major slab: conflict-free 16-byte reads

constexpr int SQCAP = BT * BT + 256;   // survivor queue: one whole tile on top of what may wait
constexpr int SQ_BASE_BITS = 26;       // a queue entry: query << 26 | base point - first point of the range
#ifndef KNNG_BRUTE_RING
#define KNNG_BRUTE_RING 4
#endif
constexpr int RING = KNNG_BRUTE_RING;  // slabs in flight from global memory per thread

template <int METRIC, bool RAGGED>
__global__ void __launch_bounds__(256)
k_brute_mfma(const float* __restrict__ pts, const float* __restrict__ nrm, int64_t n, int d, int k,
             const int32_t* __restrict__ query_rows, int64_t nq, int64_t base_chunk, int nsplit,
             u64* __restrict__ part, uint32_t* __restrict__ gthr)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* QS = reinterpret_cast<float*>(smem);            // [2][BT][MLD] query slabs
    float* BS = QS + 2 * BT * MLD;                         // [2][BT][MLD] base slabs
    uint32_t* sq = reinterpret_cast<uint32_t*>(BS + 2 * BT * MLD);   // [SQCAP] survivors of the screen
    u64* list = reinterpret_cast<u64*>(sq + SQCAP);        // [BT][k] ascending
    u64* thr = list + BT * k;                              // [BT] current k-th key
    u64* rk = thr + BT;                                    // [256] exact keys of one round (EMPTY: not better)
    int* rq = reinterpret_cast<int*>(rk + 256);            // [256] their queries
    int* qrow = rq + 256;                                  // [BT] source point of each query
    float* qn = reinterpret_cast<float*>(qrow + BT);       // [BT] |q|^2
    float* bn = qn + BT;                                   // [3][256] |b|^2 of the current tile and of the next, a
                                                           // copy per wavefront; the third: stores nobody reads
    float* thrd = bn + 3 * 256;                            // [BT] k-th distance, +inf while the list is short
    float* gthl = thrd + BT;                               // [2][256] the smallest k-th distance any range has
                                                           // published, a copy per wavefront; the second as above
    int* qcount = reinterpret_cast<int*>(gthl + 2 * 256);  // survivors waiting in sq

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t q0 = (int64_t)blockIdx.x * BT;
    const int64_t b_begin = (int64_t)blockIdx.y * base_chunk;
    const int64_t b_end = (b_begin + base_chunk) < n ? (b_begin + base_chunk) : n;
    const float inf = __uint_as_float(0x7f800000u);
    const float epsd = (float)(d + 16) * 1.1920929e-7f;    // (d + 16) 2^-23

    if (tid < BT) {
        const int64_t q = q0 + tid;
        int r = -1;
        if (q < nq) r = query_rows ? query_rows[q] : (int)q;
        qrow[tid] = r;
        qn[tid] = r >= 0 ? nrm[r] : 0.0f;
        thr[tid] = EMPTY_KEY;
        thrd[tid] = inf;
    }
    gthl[tid] = inf;
    if (tid == 0) *qcount = 0;
    for (int i = tid; i < BT * k; i += 256) list[i] = EMPTY_KEY;
    __syncthreads();

    if (b_begin < b_end) {
        // The walk over (base tile, slab of 32 coordinates) is one sequence of slabs.  Every thread
        // keeps the 16-byte pieces of the next RING slabs in flight in registers: a load takes
        // longer than the matrix cores need for one slab, so one slab of look-ahead leaves them idle.
        // Every load is issued unconditionally from a clamped, valid address (a row past the range
        // reads the range's last row, a piece past d the row's last piece, an unused query row 0):
        // such values are zeroed on the way to LDS or belong to pairs the screen never passes.
        struct Slot { float4 q0, q1, b0, b1; float nb, gt; };   // nb: |b|^2 of the tile's point `lane`; gt: shared bound of query `lane`
        Slot ring[RING];
        const int srow = tid >> 3, spc = tid & 7;          // staging: rows srow and srow + 32, piece spc
        const int sq0 = qrow[srow], sq1 = qrow[srow + 32];
        const float* qp0 = pts + (int64_t)(sq0 > 0 ? sq0 : 0) * d;
        const float* qp1 = pts + (int64_t)(sq1 > 0 ? sq1 : 0) * d;
        // The ranges of one query tile share a bound per query: every range publishes the k-th
        // distance of its full list (an atomic min on the fp32 bits), and every k-th distance of a
        // subset of the points is an upper bound of the final one, so a pair above the smallest
        // published value cannot be in the result.  Without it each of the nsplit ranges would fill
        // and refine a list of its own: nsplit times the exact evaluations of one pass over all points.
        // Which pairs are skipped depends on timing; the result, the exact k smallest, does not.
        const int64_t gq = q0 + lane < nq ? q0 + lane : nq - 1;
        const int nslab = (d + BDC - 1) / BDC;
        constexpr bool ragged = RAGGED;                    // d % BDC != 0: the last slab of a tile is shorter
        const int64_t total = ((b_end - b_begin + BT - 1) / BT) * nslab;
        // rows are below 2^31, and the issue position runs at most RING tiles past the range: 32-bit
        // unsigned row arithmetic, one 32 x 32 -> 64-bit multiply-add per row address
        uint32_t ib0 = (uint32_t)b_begin;                  // the next slab to issue
        int ik0 = 0;
        const uint32_t rlast = (uint32_t)(b_end - 1), du = (uint32_t)d;
        auto issue = [&](Slot& s) {
            int t = ik0 + 4 * spc;
            t = t < d - 4 ? t : d - 4;
            const uint32_t r0 = min(ib0 + (uint32_t)srow, rlast), r1 = min(ib0 + (uint32_t)srow + 32u, rlast);
            s.q0 = *reinterpret_cast<const float4*>(qp0 + t);
            s.q1 = *reinterpret_cast<const float4*>(qp1 + t);
            s.b0 = *reinterpret_cast<const float4*>(pts + ((uint64_t)r0 * du + (uint32_t)t));
            s.b1 = *reinterpret_cast<const float4*>(pts + ((uint64_t)r1 * du + (uint32_t)t));
            s.nb = nrm[min(ib0 + (uint32_t)lane, rlast)];
            s.gt = __uint_as_float(__hip_atomic_load(gthr + gq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            ik0 += BDC;
            if (ik0 >= d) { ik0 = 0; ib0 += BT; }
            // keep the slots' loads in program order: the waits for a slot count the loads issued after it
            __builtin_amdgcn_sched_barrier(0);
        };
#pragma unroll
        for (int i = 0; i < RING; ++i) issue(ring[i]);

        // after the last slab of a tile: lane (r16, kq) holds <q, b> for queries 16w + 4kq + r and
        // base points b0 + 16c + r16.  Screen: pairs the bound cannot rule out are queued; then,
        // once enough of them wait (or the range ends), they get their exact distance, 256 at a
        // time, one per thread, and each wavefront folds the ones of its 16 queries into their lists.
        auto tile_done = [&](const int64_t b0, const floatx4 (&acc)[4], const int tp) {
            // The screen, per pair one add and one compare.  With T the smaller of the query's own
            // k-th distance and the shared bound (+inf while there is none), padded by 2^-20 of itself,
            // and E = epsd (|q|^2 + |b|^2) (squared L2) or epsd (|q|^2 / 2 + |b|^2 / 2 + 1) (1 - <q,b>)
            // the bound on the fp32 value's error, a pair can be ruled out if the fp32 distance
            // minus E lies above T, that is if <q,b> < hq + hb with
            //   squared L2:  hq = (1 - epsd) |q|^2 / 2 - T / 2,   hb = (1 - epsd) |b|^2 / 2
            //   1 - <q,b>:   hq = 1 - T - epsd - epsd |q|^2 / 2,  hb = -epsd |b|^2 / 2
            // (the few roundings of hq + hb are far inside E, which is more than twice the bound of
            // a length-d fp32 dot product).  A pair whose test is not decidedly "below" (a NaN) stays,
            // and so does the pair of a query with itself: the exact step drops that one.
            float hq[4];
            uint32_t vm = 0;                               // the lane's queries that exist
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int qi = 16 * w + 4 * kq + r;
                const float t = fminf(thrd[qi], gthl[64 * w + qi]) * 1.000001f;
                hq[r] = METRIC == 0 ? 0.5f * (1.0f - epsd) * qn[qi] - 0.5f * t : 1.0f - t - epsd - 0.5f * epsd * qn[qi];
                vm |= qrow[qi] >= 0 ? 1u << r : 0u;
            }
            uint32_t pm = 0;                               // one bit per pair of the lane (4c + r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int b = (int)b0 + 16 * c + r16;      // ids fit 31 bits
                const float nb = bn[tp * 256 + 64 * w + 16 * c + r16];
                const float hb = METRIC == 0 ? 0.5f * (1.0f - epsd) * nb : -0.5f * epsd * nb;
                uint32_t pc = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    pc |= !(acc[c][r] < hq[r] + hb) ? 1u << r : 0u;
                pm |= (int64_t)b < b_end ? (pc & vm) << (4 * c) : 0u;
            }
            if (__ballot(pm != 0u) != 0ull) {
                // one reservation in the queue per wavefront: the lanes' counts summed bit by bit,
                // which also gives every lane the number of entries of the lanes before it
                const int cnt = __popc(pm);
                int total = 0, before = 0;
#pragma unroll
                for (int bit = 0; bit < 5; ++bit) {
                    const u64 mb = __ballot(((cnt >> bit) & 1) != 0);
                    total += __popcll(mb) << bit;
                    before += __popcll(mb & lanemask_lt()) << bit;
                }
                int off = 0;
                if (lane == 0) off = atomicAdd(qcount, total);
                off = (int)bcast32((uint32_t)off, 0) + before;
                const uint32_t ent0 = ((uint32_t)(16 * w + 4 * kq) << SQ_BASE_BITS) | ((uint32_t)(b0 - b_begin) + r16);
                while (pm != 0u) {
                    const uint32_t i = (uint32_t)__ffs((int)pm) - 1u;
                    pm &= pm - 1u;
                    sq[off++] = ent0 + ((i & 3u) << SQ_BASE_BITS) + 16u * (i >> 2);
                }
            }
            __syncthreads();
            const int waiting = *qcount;
            if (waiting > 256 || (waiting > 0 && b0 + BT >= b_end)) {
                for (int base = 0; base < waiting; base += 256) {
                    u64 key = EMPTY_KEY;
                    int qi = -1;
                    if (base + tid < waiting) {
                        const uint32_t ent = sq[base + tid];
                        qi = (int)(ent >> SQ_BASE_BITS);
                        const int64_t b = b_begin + (int64_t)(ent & ((1u << SQ_BASE_BITS) - 1u));
                        const float* xq = pts + (int64_t)qrow[qi] * d;
                        const float* xb = pts + b * d;
                        double sacc = 0.0;
                        int t = 0;
                        for (; t + 16 <= d; t += 16) {
                            float4 x[4], y[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                x[u] = *reinterpret_cast<const float4*>(xq + t + 4 * u);
                                y[u] = *reinterpret_cast<const float4*>(xb + t + 4 * u);
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                sacc = exact_step<METRIC>(sacc, x[u].x, y[u].x);
                                sacc = exact_step<METRIC>(sacc, x[u].y, y[u].y);
                                sacc = exact_step<METRIC>(sacc, x[u].z, y[u].z);
                                sacc = exact_step<METRIC>(sacc, x[u].w, y[u].w);
                            }
                        }
                        for (; t < d; t += 4) {
                            const float4 x = *reinterpret_cast<const float4*>(xq + t);
                            const float4 y = *reinterpret_cast<const float4*>(xb + t);
                            sacc = exact_step<METRIC>(sacc, x.x, y.x);
                            sacc = exact_step<METRIC>(sacc, x.y, y.y);
                            sacc = exact_step<METRIC>(sacc, x.z, y.z);
                            sacc = exact_step<METRIC>(sacc, x.w, y.w);
                        }
                        const float dist = exact_finish<METRIC>(sacc);
                        key = pack_key(dist, (int)b, 0);
                        if (!(key < thr[qi]) || dist > gthl[64 * w + qi] || (int)b == qrow[qi]) key = EMPTY_KEY;
                    }
                    rk[tid] = key;
                    rq[tid] = qi;
                    __syncthreads();
                    // Wavefront w owns queries 16w .. 16w+15.  It reads the round's 256 keys once, then
                    // inserts the ones of each of its queries into that query's sorted list, one key at
                    // a time: the list sits in lanes 0 .. k-1, a key's rank is one vote, and the lanes
                    // from that rank on take their left neighbour's entry.
                    u64 rkv[4];
                    int rqv[4];
#pragma unroll
                    for (int ch = 0; ch < 4; ++ch) {
                        rkv[ch] = rk[64 * ch + lane];
                        rqv[ch] = rkv[ch] != EMPTY_KEY ? rq[64 * ch + lane] : -1;
                    }
                    for (int qq = 0; qq < 16; ++qq) {
                        const int mq = 16 * w + qq;
                        u64 cm[4];
#pragma unroll
                        for (int ch = 0; ch < 4; ++ch) cm[ch] = __ballot(rqv[ch] == mq);
                        if ((cm[0] | cm[1] | cm[2] | cm[3]) == 0ull) continue;
                        u64 lk = lane < k ? list[mq * k + lane] : EMPTY_KEY;
#pragma unroll
                        for (int ch = 0; ch < 4; ++ch)
                            for (u64 mm = cm[ch]; mm; mm &= mm - 1) {
                                const u64 c = bcast64(rkv[ch], __ffsll((long long)mm) - 1);
                                const int r = __popcll(__ballot(lk < c));    // lanes >= k hold EMPTY_KEY
                                if (r < k) {
                                    const u64 left = wave_shr1_64(lk);
                                    lk = lane < r ? lk : (lane == r ? c : left);
                                    if (lane >= k) lk = EMPTY_KEY;
                                }
                            }
                        if (lane < k) list[mq * k + lane] = lk;
                        if (lane == k - 1) {
                            thr[mq] = lk;
                            thrd[mq] = lk == EMPTY_KEY ? inf : key_dist(lk);
                            if (lk != EMPTY_KEY && q0 + mq < nq) atomicMin(gthr + (q0 + mq), (uint32_t)(lk >> 32));
                        }
                    }
                    __syncthreads();
                }
                if (tid == 0) *qcount = 0;
                __syncthreads();
            }
        };

        floatx4 acc[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = floatx4{0, 0, 0, 0};
        int64_t b0 = b_begin;                              // the slab being multiplied
        int k0 = 0, buf = 0, tp = 0;                       // tp: parity of its tile (which half of bn)
        int64_t b0n = b_begin;                             // the slab being staged: the one after it
        int k0n = 0, tpn = 0;
        // One slab ahead of the matrix instructions, a slab goes from the ring to the LDS pair the
        // previous step read.  The stores stand after the step's matrix instructions in program
        // order, so they issue in the shadow of those; the barrier that ends the step orders them
        // before the next step's reads, and this step's reads before the stores of the step after.
        auto stage = [&](Slot v, const int to) {
            if (k0n + BDC > d && !(k0n + 4 * spc < d))
                v.q0 = v.q1 = v.b0 = v.b1 = float4{0, 0, 0, 0};
            float* qs = QS + to * (BT * MLD);
            float* bs = BS + to * (BT * MLD);
            bn[(k0n == 0 ? tpn : 2) * 256 + tid] = v.nb;   // a tile's first slab carries its norms and bounds
            gthl[(k0n == 0 ? 0 : 1) * 256 + tid] = v.gt;
            *reinterpret_cast<float4*>(qs + srow * MLD + 4 * spc) = v.q0;
            *reinterpret_cast<float4*>(qs + (srow + 32) * MLD + 4 * spc) = v.q1;
            *reinterpret_cast<float4*>(bs + srow * MLD + 4 * spc) = v.b0;
            *reinterpret_cast<float4*>(bs + (srow + 32) * MLD + 4 * spc) = v.b1;
            k0n += BDC;
            if (k0n >= d) { k0n = 0; tpn ^= 1; b0n += BT; }
        };
        // the slab in LDS pair `buf` times the accumulators: all operands first (ten 16-byte reads),
        // then the 32 matrix instructions as four independent chains taken in turn
        auto multiply = [&]() {
            const float* qs = QS + buf * (BT * MLD);
            const float* bs = BS + buf * (BT * MLD);
            float4 a[2], b[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a[h] = *reinterpret_cast<const float4*>(qs + (16 * w + r16) * MLD + 4 * kq + 16 * h);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    b[h][c] = *reinterpret_cast<const float4*>(bs + (16 * c + r16) * MLD + 4 * kq + 16 * h);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[h].x, b[h][c].x, acc[c], 0, 0, 0);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[h].y, b[h][c].y, acc[c], 0, 0, 0);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[h].z, b[h][c].z, acc[c], 0, 0, 0);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[h].w, b[h][c].w, acc[c], 0, 0, 0);
            }
        };
        // One step of the steady state: the matrix instructions of the slab in LDS pair `buf`, and
        // between them, four at a time, the pieces of what the step also has to do: the next slab
        // from its ring slot to the other LDS pair, then that slot's loads for the slab RING later.
        // A wavefront issues in order, and four of these matrix instructions keep their pipe busy
        // for 128 cycles: what stands between two groups issues in their shadow.  The fences keep
        // the compiler from sorting the groups back together.
        auto step = [&](Slot& nx) {
            const float* qs = QS + buf * (BT * MLD);
            const float* bs = BS + buf * (BT * MLD);
            float* qd = QS + (buf ^ 1) * (BT * MLD) + srow * MLD + 4 * spc;
            float* bd = BS + (buf ^ 1) * (BT * MLD) + srow * MLD + 4 * spc;
            float4 a[2], b[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a[h] = *reinterpret_cast<const float4*>(qs + (16 * w + r16) * MLD + 4 * kq + 16 * h);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    b[h][c] = *reinterpret_cast<const float4*>(bs + (16 * c + r16) * MLD + 4 * kq + 16 * h);
            }
            const bool dead = k0n + BDC > d && !(k0n + 4 * spc < d);   // a piece past d of a last slab
            auto live = [&](float4 x) {
                if (ragged) x = float4{dead ? 0.0f : x.x, dead ? 0.0f : x.y, dead ? 0.0f : x.z, dead ? 0.0f : x.w};
                return x;
            };
            int t = ik0 + 4 * spc;
            t = t < d - 4 ? t : d - 4;
            const uint32_t r0 = min(ib0 + (uint32_t)srow, rlast), r1 = min(ib0 + (uint32_t)srow + 32u, rlast);
            const uint32_t rn = min(ib0 + (uint32_t)lane, rlast);
#define KNNG_MM(h, e) \
            _Pragma("unroll") for (int c = 0; c < 4; ++c) \
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[h].e, b[h][c].e, acc[c], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0)
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(0, x);
            *reinterpret_cast<float4*>(qd) = live(nx.q0);
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(0, y);
            *reinterpret_cast<float4*>(qd + 32 * MLD) = live(nx.q1);
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(0, z);
            *reinterpret_cast<float4*>(bd) = live(nx.b0);
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(0, w);
            *reinterpret_cast<float4*>(bd + 32 * MLD) = live(nx.b1);
            bn[(k0n == 0 ? tpn : 2) * 256 + tid] = nx.nb;
            gthl[(k0n == 0 ? 0 : 1) * 256 + tid] = nx.gt;
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(1, x);
            nx.q0 = *reinterpret_cast<const float4*>(qp0 + t);
            nx.q1 = *reinterpret_cast<const float4*>(qp1 + t);
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(1, y);
            nx.b0 = *reinterpret_cast<const float4*>(pts + ((uint64_t)r0 * du + (uint32_t)t));
            nx.b1 = *reinterpret_cast<const float4*>(pts + ((uint64_t)r1 * du + (uint32_t)t));
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(1, z);
            nx.nb = nrm[rn];
            nx.gt = __uint_as_float(__hip_atomic_load(gthr + gq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            __builtin_amdgcn_sched_barrier(0);
            KNNG_MM(1, w);
#undef KNNG_MM
            k0n += BDC;
            if (k0n >= d) { k0n = 0; tpn ^= 1; b0n += BT; }
            ik0 += BDC;
            if (ik0 >= d) { ik0 = 0; ib0 += BT; }
        };
        auto end_step = [&]() {
            __syncthreads();
            buf ^= 1;
            k0 += BDC;
            if (k0 >= d) {
                tile_done(b0, acc, tp);
                k0 = 0;
                tp ^= 1;
                b0 += BT;
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = floatx4{0, 0, 0, 0};
            }
        };
        stage(ring[0], 0);
        issue(ring[0]);
        __syncthreads();
        // Whole groups of RING slabs run without a condition inside the group: a path on which a
        // step is skipped and the loop goes round again would make the compiler wait, at the first
        // step, for every load in flight.  The last total % RING slabs load what they stage
        // themselves (the ring's loads of those slabs are left to complete unused).
        const int64_t groups = total / RING;
        for (int64_t g = 0; g < groups; ++g) {
#pragma unroll
            for (int i = 0; i < RING; ++i) {
                step(ring[(i + 1) % RING]);            // (past the last slab: a clamped copy nobody reads)
                end_step();
            }
        }
        for (int64_t r = groups * RING; r < total; ++r) {
            multiply();
            Slot v;                                        // the staged slab's successor, loaded here
            {
                int t = k0n + 4 * spc;
                t = t < d - 4 ? t : d - 4;
                int64_t r0 = b0n + srow, r1 = b0n + srow + 32;
                r0 = r0 < b_end ? r0 : b_end - 1;
                r1 = r1 < b_end ? r1 : b_end - 1;
                const int64_t rn = b0n + lane;
                v.q0 = *reinterpret_cast<const float4*>(qp0 + t);
                v.q1 = *reinterpret_cast<const float4*>(qp1 + t);
                v.b0 = *reinterpret_cast<const float4*>(pts + r0 * d + t);
                v.b1 = *reinterpret_cast<const float4*>(pts + r1 * d + t);
                v.nb = nrm[rn < b_end ? rn : b_end - 1];
                v.gt = __uint_as_float(__hip_atomic_load(gthr + gq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            }
            stage(v, buf ^ 1);
            end_step();
        }
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
    // a range's offsets must fit the survivor queue's entries (k_brute_mfma)
    const int64_t min_split = (n + (1ll << SQ_BASE_BITS) - 1) >> SQ_BASE_BITS;
    if (want < min_split) want = min_split;
    return (int)want;
}

}  // namespace knng

using namespace knng;

extern "C" __attribute__((visibility("default"))) uint64_t knng_brute_workspace_bytes(int64_t n, int32_t d, int32_t k, int64_t nq)
{
    if (n < 2 || d < 1 || k < 1 || k > KNNG_MAX_K || (int64_t)k > n - 1 || nq < 0) return 0;
    uint64_t b = (uint64_t)nq * (uint64_t)brute_nsplit(n, nq) * (uint64_t)k * 8u;
    b = (b + 255u) & ~255ull;                     // partial lists, then |x|^2 of every point (fp32, or fp64 for the cosine),
    b += ((uint64_t)n * 8u + 255u) & ~255ull;     // then one shared bound per query (k_brute_mfma)
    return b + (((uint64_t)nq * 4u + 255u) & ~255ull);
}

// candidates: the first n_base of the n_all points; query rows: any of the n_all points
static int brute_impl(const float* points_dev, int64_t n_all, int64_t n, int32_t d, int32_t k, int32_t metric,
                      const int32_t* query_rows_dev, int64_t nq, int32_t* ids_out_dev, float* dists_out_dev,
                      void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    if (!points_dev || n < 2 || n > n_all || n_all > 2147483647LL || d < 1 || k < 1 || k > KNNG_MAX_K ||
        (int64_t)k > n - 1 || nq < 0 ||
        (metric != KNNG_METRIC_L2SQ && metric != KNNG_METRIC_IP_UNIT && metric != KNNG_METRIC_COSINE))
        return KNNG_EINVAL;
    if (nq == 0) return KNNG_OK;
    if (!ids_out_dev || !dists_out_dev) return KNNG_EINVAL;
    if (!query_rows_dev && nq > n_all) return KNNG_EINVAL;
    const uint64_t need = knng_brute_workspace_bytes(n_all, d, k, nq);
    if (!workspace_dev || workspace_bytes < need) return KNNG_EWORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int nsplit = brute_nsplit(n, nq);
    int64_t chunk = (n + nsplit - 1) / nsplit;
    chunk = (chunk + BT - 1) / BT * BT;
    const unsigned qtiles = (unsigned)((nq + BT - 1) / BT);
    const int lds = 2 * BDC * BLD * 4 + BT * BT * 8 + BT * k * 8 + BT * 8 + BT * 4 + BT * 4;
    u64* part = static_cast<u64*>(workspace_dev);
    hipError_t e;
    const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(points_dev) & 15u) == 0);
    if (metric == KNNG_METRIC_COSINE) {
        // every pair in fp64 (the 4x4 register blocks of k_brute), norms from the exact chain
        const uint64_t part_bytes = ((uint64_t)nq * (uint64_t)nsplit * (uint64_t)k * 8u + 255u) & ~255ull;
        double* nrm64 = reinterpret_cast<double*>(static_cast<unsigned char*>(workspace_dev) + part_bytes);
        hipLaunchKernelGGL(k_row_norms_exact, dim3((unsigned)((n_all + 255) / 256)), dim3(256), 0, st, points_dev, n_all, d, nrm64);
        if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_row_norms_exact launch");
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_brute<2>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute)");
        hipLaunchKernelGGL(k_brute<2>, dim3(qtiles, (unsigned)nsplit), dim3(256), lds, st, points_dev, n, d, k,
                           query_rows_dev, nq, chunk, nsplit, part, nrm64);
    } else if (vec) {
        const uint64_t part_bytes = ((uint64_t)nq * (uint64_t)nsplit * (uint64_t)k * 8u + 255u) & ~255ull;
        float* nrm = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace_dev) + part_bytes);
        hipLaunchKernelGGL(k_row_norms, dim3((unsigned)((n_all * 8 + 255) / 256)), dim3(256), 0, st, points_dev, n_all, d, nrm);
        if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_row_norms launch");
        uint32_t* gthr = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace_dev) + part_bytes +
                                                     (((uint64_t)n_all * 8u + 255u) & ~255ull));
        hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, st, gthr, nq, 0x7f800000u);
        if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_fill_u32 launch");
        const int mlds = 4 * BT * MLD * 4 + SQCAP * 4 + BT * k * 8 + BT * 8 + 256 * 8 + 256 * 4 + (3 * BT + 5 * 256) * 4 + 16;
        auto launch = [&](auto kern) -> hipError_t {
            const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, mlds);
            if (ea != hipSuccess) return ea;
            hipLaunchKernelGGL(kern, dim3(qtiles, (unsigned)nsplit), dim3(256), mlds, st, points_dev, nrm,
                               n, d, k, query_rows_dev, nq, chunk, nsplit, part, gthr);
            return hipSuccess;
        };
        const bool ragged = d % BDC != 0;
        if (metric == 0) e = ragged ? launch(k_brute_mfma<0, true>) : launch(k_brute_mfma<0, false>);
        else e = ragged ? launch(k_brute_mfma<1, true>) : launch(k_brute_mfma<1, false>);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute_mfma)");
    } else if (metric == 0) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_brute<0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute)");
        hipLaunchKernelGGL(k_brute<0>, dim3(qtiles, (unsigned)nsplit), dim3(256), lds, st, points_dev, n, d, k,
                           query_rows_dev, nq, chunk, nsplit, part, static_cast<const double*>(nullptr));
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_brute<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return set_hip_error(e, "hipFuncSetAttribute(k_brute)");
        hipLaunchKernelGGL(k_brute<1>, dim3(qtiles, (unsigned)nsplit), dim3(256), lds, st, points_dev, n, d, k,
                           query_rows_dev, nq, chunk, nsplit, part, static_cast<const double*>(nullptr));
    }
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_brute launch");
    hipLaunchKernelGGL(k_brute_reduce, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, st, nq, k, nsplit, part,
                       ids_out_dev, dists_out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_brute_reduce launch");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return set_hip_error(e, "hipStreamSynchronize");
    return KNNG_OK;
}

extern "C" __attribute__((visibility("default"))) int knng_brute_knn(const float* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                              const int32_t* query_rows_dev, int64_t nq,
                              int32_t* ids_out_dev, float* dists_out_dev,
                              void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    return brute_impl(points_dev, n, n, d, k, metric, query_rows_dev, nq, ids_out_dev, dists_out_dev,
                      workspace_dev, workspace_bytes, stream);
}

extern "C" __attribute__((visibility("default"))) int knng_brute_knn_base(const float* points_dev, int64_t n, int64_t n_base, int32_t d, int32_t k,
                                   int32_t metric, const int32_t* query_rows_dev, int64_t nq,
                                   int32_t* ids_out_dev, float* dists_out_dev,
                                   void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    return brute_impl(points_dev, n, n_base, d, k, metric, query_rows_dev, nq, ids_out_dev, dists_out_dev,
                      workspace_dev, workspace_bytes, stream);
}
