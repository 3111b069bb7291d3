// knng_optimize.hip -- search graph G^s from a k-NN graph G (Sec. 3.3: edges that a shorter
// two-hop path bypasses are dropped, reverse edges added; ranks only, no distances).
//
// Input rows list a point's neighbours nearest first, so the column is the rank.  An entry is
// valid if it lies in [0,n), is not the row's own point and does not repeat an earlier entry.
//   1. c(u,j) = number of neighbours w of u, at a rank i < j, whose row holds u's j-th neighbour
//      at a rank r < j (the edge can be bypassed through w); padding entries get c = k.
//   2. P(u) = the d_out entries with the smallest (c, rank), in that order (-1 for padding).
//   3. Every edge u -> v at position p of P(u) hands (p, u) to v; R(v) = those, ascending.
//   4. Row v of G^s = the first d_out - d_out/2 entries of P(v), then R(v) in order, then the
//      rest of P(v), skipping -1 and ids already in the row, until it has d_out entries.
//
// k_opt_prune (1, 2; one wavefront per point; an edge also takes its place in its target's list
// here, with the one atomic that counts the in-degree), a three-kernel prefix sum over the
// in-degrees, k_opt_fill (3: writes every edge's (p, u) word to its place), k_opt_merge (3, 4; one
// wavefront per point picks the smallest words of its list, so the result does not depend on
// the order the places were handed out in).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

__device__ __forceinline__ void wave_lds_sync_opt() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

constexpr int OPT_HT = 128;                       // hash slots per wavefront (>= 2 * 64 entries)

// ------------------------------------------------------------------------------------------
// k_opt_prune: lane j holds entry j of row u.  The row's ids go into a hash table id -> first
// rank (LDS, open addressing).  For every valid neighbour w (rank i) the wavefront reads w's row
// (a lane per entry r; two rows per load at k <= 32), looks each entry up in the table and, where
// it is u's neighbour of a rank j > max(i, r), sets bit i of that neighbour's word: c(u,j) is the
// number of bits.  A repeated id in w's row sets the same bit again, so "some r < j" is counted
// once.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_opt_prune(const int32_t* __restrict__ ids, int64_t n, int k, int d_out, int2* __restrict__ P,
            uint32_t* __restrict__ deg)
{
    __shared__ int hkey[4][OPT_HT];
    __shared__ int hval[4][OPT_HT];
    __shared__ uint32_t bits[4][2][WAVE];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int64_t u = (int64_t)blockIdx.x * 4 + w;
    if (u >= n) return;
    int* hk = hkey[w];
    int* hv = hval[w];
    hk[lane] = -1; hk[lane + 64] = -1;
    hv[lane] = k; hv[lane + 64] = k;
    bits[w][0][lane] = 0u; bits[w][1][lane] = 0u;
    const int my = lane < k ? ids[u * k + lane] : -1;
    const bool inr = lane < k && my >= 0 && (int64_t)my < n && (int64_t)my != u;
    wave_lds_sync_opt();
    if (inr) {
        uint32_t s = hash32((uint32_t)my) & (OPT_HT - 1);
        for (;;) {
            const int prev = atomicCAS(&hk[s], -1, my);
            if (prev == -1 || prev == my) { atomicMin(&hv[s], lane); break; }
            s = (s + 1) & (OPT_HT - 1);
        }
    }
    wave_lds_sync_opt();
    // rank of id x in row u (first occurrence), or k
    auto lookup = [&](int x) -> int {
        uint32_t s = hash32((uint32_t)x) & (OPT_HT - 1);
        for (;;) {
            const int kx = hk[s];
            if (kx == x) return hv[s];
            if (kx == -1) return k;
            s = (s + 1) & (OPT_HT - 1);
        }
    };
    const bool valid = inr && lookup(my) == lane;
    const u64 vmask = __ballot(valid);

    // A wavefront reads 64 / kp neighbour rows per load (kp = the power of two >= k: lane ->
    // row `lane / kp` of the group, entry `lane % kp`), four loads per step, the next step's in
    // flight meanwhile.
    int kp = 1;
    while (kp < k) kp <<= 1;
    const int rpl = WAVE / kp;                                 // rows per load
    const int sub = lane / kp, r = lane & (kp - 1);
    int xn[4];
    auto issue = [&](int i0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i = i0 + t * rpl + sub;
            const int wi = __shfl(my, i < k ? i : 0);          // all lanes take part
            xn[t] = -1;
            if (i < k && r < k && ((vmask >> i) & 1ull)) xn[t] = ids[(int64_t)wi * k + r];
        }
    };
    issue(0);
    for (int i0 = 0; i0 < k; i0 += 4 * rpl) {
        int x[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) x[t] = xn[t];
        if (i0 + 4 * rpl < k) issue(i0 + 4 * rpl);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i = i0 + t * rpl + sub;
            const int j = x[t] >= 0 ? lookup(x[t]) : k;        // x = -1: row absent, padding or past k
            if (j < k && j > i && j > r) atomicOr(&bits[w][i >> 5][j], 1u << (i & 31));
        }
    }
    wave_lds_sync_opt();
    const int c = valid ? __popc(bits[w][0][lane]) + __popc(bits[w][1][lane]) : k;
    const uint32_t key = lane < k ? (uint32_t)(c * 64 + lane) : 0xffffffffu;
    int rank = 0;
    for (int j = 0; j < k; ++j) rank += bcast32(key, j) < key ? 1 : 0;
    if (lane < k && rank < d_out) {
        // {neighbour, place of this edge in the neighbour's reverse list}
        const int place = valid ? (int)atomicAdd(&deg[my], 1u) : 0;
        P[u * d_out + rank] = int2{valid ? my : -1, place};
    }
}

// ------------------------------------------------------------------------------------------
// exclusive prefix sum of deg[n] into start[n + 1]: block sums, their scan, the scan itself
// ------------------------------------------------------------------------------------------
constexpr int SCAN_PER_BLOCK = 2048;              // 256 threads x 8

__device__ __forceinline__ u64 block_sum_256(u64 v, u64* sh)
{
    for (int o = 32; o > 0; o >>= 1) v += (u64)__shfl_xor((unsigned long long)v, o);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const u64 t = sh[0] + sh[1] + sh[2] + sh[3];
    __syncthreads();
    return t;
}

__global__ void __launch_bounds__(256)
k_opt_block_sums(const uint32_t* __restrict__ deg, int64_t n, u64* __restrict__ bsum)
{
    __shared__ u64 sh[4];
    const int64_t base = (int64_t)blockIdx.x * SCAN_PER_BLOCK + (int64_t)threadIdx.x * 8;
    u64 s = 0;
    for (int t = 0; t < 8; ++t) if (base + t < n) s += deg[base + t];
    s = block_sum_256(s, sh);
    if (threadIdx.x == 0) bsum[blockIdx.x] = s;
}

__global__ void __launch_bounds__(256)
k_opt_scan_sums(u64* __restrict__ bsum, int64_t nb)
{
    __shared__ u64 sh[256];
    __shared__ u64 carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t c0 = 0; c0 < nb; c0 += 256) {
        const int64_t i = c0 + threadIdx.x;
        const u64 v = i < nb ? bsum[i] : 0;
        sh[threadIdx.x] = v;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {                    // inclusive scan in LDS
            const u64 add = threadIdx.x >= (unsigned)o ? sh[threadIdx.x - o] : 0;
            __syncthreads();
            sh[threadIdx.x] += add;
            __syncthreads();
        }
        const u64 carry = carry_s;
        if (i < nb) bsum[i] = carry + sh[threadIdx.x] - v;     // exclusive
        __syncthreads();
        if (threadIdx.x == 255) carry_s = carry + sh[255];
        __syncthreads();
    }
}

__global__ void __launch_bounds__(256)
k_opt_scan(const uint32_t* __restrict__ deg, int64_t n, const u64* __restrict__ bsum, u64* __restrict__ start)
{
    __shared__ u64 sh[256];
    const int64_t base = (int64_t)blockIdx.x * SCAN_PER_BLOCK + (int64_t)threadIdx.x * 8;
    uint32_t v[8];
    u64 s = 0;
    for (int t = 0; t < 8; ++t) { v[t] = base + t < n ? deg[base + t] : 0u; s += v[t]; }
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        const u64 add = threadIdx.x >= (unsigned)o ? sh[threadIdx.x - o] : 0;
        __syncthreads();
        sh[threadIdx.x] += add;
        __syncthreads();
    }
    u64 run = bsum[blockIdx.x] + sh[threadIdx.x] - s;
    for (int t = 0; t < 8; ++t) {
        if (base + t < n) start[base + t] = run;
        run += v[t];
        if (base + t == n - 1) start[n] = run;
    }
}

// ------------------------------------------------------------------------------------------
// k_opt_fill: edge (u, p) -> v writes the word (p << 32 | u) to its place in v's list
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_opt_fill(const int2* __restrict__ P, int64_t total, int d_out, const u64* __restrict__ start,
           u64* __restrict__ E)
{
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int2 vp = P[e];
        if (vp.x < 0) continue;
        const int64_t u = e / d_out;
        const int p = (int)(e - u * d_out);
        E[start[vp.x] + (u64)(uint32_t)vp.y] = ((u64)(uint32_t)p << 32) | (u64)(uint32_t)u;
    }
}

// ------------------------------------------------------------------------------------------
// k_opt_merge: one wavefront per point v.  The row is assembled in LDS: the first d_out - h
// entries of P(v); then the reverse candidates, taken from v's list 64 at a time in ascending
// (p, u) order -- the list is streamed through a sorted register array (one word per lane) that
// keeps the 64 smallest words above the last batch's largest; then the rest of P(v).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_opt_merge(const int2* __restrict__ P, const u64* __restrict__ start, const u64* __restrict__ E,
            int64_t n, int d_out, int32_t* __restrict__ out)
{
    __shared__ int rowb[4][WAVE];
    __shared__ u64 sortb[4][WAVE];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int64_t v = (int64_t)blockIdx.x * 4 + w;
    if (v >= n) return;
    int* row = rowb[w];
    const u64 lt = lanemask_lt();
    const int h = d_out / 2, nf = d_out - h;
    const int pv = lane < d_out ? P[v * d_out + lane].x : -1;
    int m;
    {
        const bool f = lane < nf && pv >= 0;
        const u64 fm = __ballot(f);
        if (f) row[__popcll(fm & lt)] = pv;
        m = __popcll(fm);
    }
    wave_lds_sync_opt();
    // append the candidates held by the lanes flagged `has` (in lane order) that the row lacks
    auto append = [&](bool has, int cand) {
        bool ok = has;
        for (int j = 0; j < m; ++j) ok = ok && row[j] != cand;
        const u64 om = __ballot(ok);
        const int pos = m + __popcll(om & lt);
        if (ok && pos < d_out) row[pos] = cand;
        m += __popcll(om);
        if (m > d_out) m = d_out;
        wave_lds_sync_opt();
    };
    const u64 base = start[v];
    const int64_t L = (int64_t)(start[v + 1] - base);
    const u64 INF = ~0ull;
    u64 bound = 0;
    bool have_bound = false;
    int64_t taken = 0;
    if (L <= WAVE && m < d_out && L > 0) {
        // the usual case, a list that fits the lanes: sort it by counting ranks (the words are distinct)
        const u64 key = lane < L ? E[base + lane] : INF;
        int rank = 0;
        for (int j = 0; j < (int)L; ++j) rank += bcast64(key, j) < key ? 1 : 0;
        if (lane < L) sortb[w][rank] = key;
        wave_lds_sync_opt();
        const u64 sorted = lane < L ? sortb[w][lane] : INF;
        append(lane < L, (int)(uint32_t)sorted);
        taken = L;
    }
    while (m < d_out && taken < L) {
        u64 best = INF;                                         // ascending over the lanes
        for (int64_t off = 0; off < L; off += WAVE) {
            u64 key = off + lane < L ? E[base + off + lane] : INF;
            if (have_bound && key <= bound) key = INF;
            for (u64 q = __ballot(key < bcast64(best, WAVE - 1)); q; q &= q - 1) {
                const int src = __ffsll((long long)q) - 1;
                const u64 kj = bcast64(key, src);
                if (kj >= bcast64(best, WAVE - 1)) continue;    // uniform: the array moved on
                const int pos = __popcll(__ballot(best < kj));
                const u64 up = (u64)__shfl_up((unsigned long long)best, 1);
                best = lane == pos ? kj : (lane > pos ? up : best);
            }
        }
        const int got = __popcll(__ballot(best != INF));
        if (got == 0) break;
        append(lane < got, (int)(uint32_t)best);
        taken += got;
        bound = bcast64(best, got - 1);
        have_bound = true;
    }
    if (m < d_out) append(lane >= nf && lane < d_out && pv >= 0, pv);
    if (lane < d_out) out[v * d_out + lane] = lane < m ? row[lane] : -1;
}

}  // namespace knng

using namespace knng;

namespace {
struct OptPlan { uint64_t off_P, off_deg, off_start, off_E, off_bsum, total; int64_t nb; };
bool opt_plan(int64_t n, int32_t k, int32_t d_out, OptPlan* op)
{
    if (n < 1 || n > 2147483647LL || k < 1 || k > KNNG_MAX_K || d_out < 1 || d_out > k) return false;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = (off + bytes + 255) & ~255ull; return o; };
    op->nb = (n + SCAN_PER_BLOCK - 1) / SCAN_PER_BLOCK;
    op->off_P = take((uint64_t)n * d_out * 8);
    op->off_deg = take((uint64_t)n * 4);
    op->off_start = take(((uint64_t)n + 1) * 8);
    op->off_E = take((uint64_t)n * d_out * 8);
    op->off_bsum = take((uint64_t)op->nb * 8);
    op->total = off;
    return true;
}
}  // namespace

extern "C" __attribute__((visibility("default"))) uint64_t knng_optimize_workspace_bytes(int64_t n, int32_t k, int32_t d_out)
{
    OptPlan op;
    return opt_plan(n, k, d_out, &op) ? op.total : 0;
}

extern "C" __attribute__((visibility("default"))) int knng_optimize_graph(const int32_t* ids_dev, int64_t n, int32_t k, int32_t d_out,
                                   int32_t* ids_out_dev, void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    OptPlan op;
    if (!ids_dev || !ids_out_dev || !opt_plan(n, k, d_out, &op)) return KNNG_EINVAL;
    if (!workspace_dev || workspace_bytes < op.total || (reinterpret_cast<uintptr_t>(workspace_dev) & 255u))
        return KNNG_EWORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace_dev);
    int2* P = reinterpret_cast<int2*>(ws + op.off_P);
    uint32_t* deg = reinterpret_cast<uint32_t*>(ws + op.off_deg);
    u64* start = reinterpret_cast<u64*>(ws + op.off_start);
    u64* E = reinterpret_cast<u64*>(ws + op.off_E);
    u64* bsum = reinterpret_cast<u64*>(ws + op.off_bsum);
    hipError_t e;
    if ((e = hipMemsetAsync(deg, 0, (size_t)n * 4, st)) != hipSuccess) return set_hip_error(e, "hipMemsetAsync(in-degrees)");
    const unsigned row_blocks = (unsigned)((n + 3) / 4);
    hipLaunchKernelGGL(k_opt_prune, dim3(row_blocks), dim3(256), 0, st, ids_dev, n, k, d_out, P, deg);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_opt_prune launch");
    hipLaunchKernelGGL(k_opt_block_sums, dim3((unsigned)op.nb), dim3(256), 0, st, deg, n, bsum);
    hipLaunchKernelGGL(k_opt_scan_sums, dim3(1), dim3(256), 0, st, bsum, op.nb);
    hipLaunchKernelGGL(k_opt_scan, dim3((unsigned)op.nb), dim3(256), 0, st, deg, n, bsum, start);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "prefix sum launch");
    const int64_t total = n * d_out;
    int64_t fill_blocks = (total + 255) / 256;
    if (fill_blocks > 1048576) fill_blocks = 1048576;
    hipLaunchKernelGGL(k_opt_fill, dim3((unsigned)fill_blocks), dim3(256), 0, st, P, total, d_out, start, E);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_opt_fill launch");
    hipLaunchKernelGGL(k_opt_merge, dim3(row_blocks), dim3(256), 0, st, P, start, E, n, d_out, ids_out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_opt_merge launch");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return set_hip_error(e, "hipStreamSynchronize");
    return KNNG_OK;
}
