// knng_merge.hip -- update of a k-NN graph's rows with neighbour candidates found elsewhere:
// the local half of the paper's refinement step (Sec. 4.3 step 4: a rank updates its graph with
// the k candidates per point it found on a remote graph; Sec. 4.4: G_{0->0} becomes G_{0->0:1}
// using the search results R_{0->1}, which have the layout of a graph).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

// orders one wavefront's own LDS accesses (wavefront-private regions)
__device__ __forceinline__ void wave_lds_sync_merge() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// One wavefront per row, 4 rows per workgroup.  Lane l holds entry l of row A and entry l of row
// B as one 64-bit word (fp32 distance bits, then the id): unsigned order = (distance, id) order.
//
// Rows as graphs and searches produce them -- each list ascending, padding only at its end, an
// id shared by the two lists carrying the same distance in both -- take the short way: the rank
// of an entry in the union is its own position plus a binary search in the other list, and an
// entry of B equal to one of A is dropped.  That the ids really are distinct otherwise is
// checked exactly with a small hash set in LDS; if that or the ordering fails, the row takes
// the general way below.
//
// General way: pass 1 drops every entry that has the same id as an entry that sorts before it
// (or an equal one at a lower position); pass 2 ranks the rest by counting.  Both walk the other
// entries with v_readlane broadcasts: (ka + kb)^2 compares per row.
constexpr int MSET = 256;                         // hash-set slots per wavefront (>= 2 * 128 entries)

__device__ __forceinline__ void merge_general(u64 key[2], int ka, int kb, int lane, int rank[2])
{
    bool drop[2] = {false, false};
#pragma unroll
    for (int src = 0; src < 2; ++src) {
        const int cnt = src == 0 ? ka : kb;
        for (int j = 0; j < cnt; ++j) {
            const u64 kf = bcast64(key[src], j);
            if (kf == EMPTY_KEY) continue;                      // uniform
#pragma unroll
            for (int me = 0; me < 2; ++me) {
                const bool same_id = (uint32_t)kf == (uint32_t)key[me] && key[me] != EMPTY_KEY;
                const bool earlier = src < me || (src == me && j < lane);   // position of f before mine
                const bool other = src != me || j != lane;
                drop[me] = drop[me] || (other && same_id && (kf < key[me] || (kf == key[me] && earlier)));
            }
        }
    }
    if (drop[0]) key[0] = EMPTY_KEY;
    if (drop[1]) key[1] = EMPTY_KEY;
    rank[0] = rank[1] = 0;
#pragma unroll
    for (int src = 0; src < 2; ++src) {
        const int cnt = src == 0 ? ka : kb;
        for (int j = 0; j < cnt; ++j) {
            const u64 kf = bcast64(key[src], j);
            rank[0] += kf < key[0] ? 1 : 0;
            rank[1] += kf < key[1] ? 1 : 0;
        }
    }
}

__global__ void __launch_bounds__(256)
k_merge_rows(const int32_t* __restrict__ ids_a, const float* __restrict__ dists_a, int ka,
             const int32_t* __restrict__ ids_b, const float* __restrict__ dists_b, int kb,
             int64_t n, int k_out, int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    __shared__ u64 keys_s[4][2][WAVE];            // the two lists of each wavefront's row
    __shared__ int set_s[4][MSET];                // id hash set
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + w;
    if (row >= n) return;
    u64 key[2] = {EMPTY_KEY, EMPTY_KEY};
    if (lane < ka) {
        const int id = ids_a[row * ka + lane];
        if (id >= 0) key[0] = ((u64)__float_as_uint(dists_a[row * ka + lane]) << 32) | (uint32_t)id;
    }
    if (lane < kb) {
        const int id = ids_b[row * kb + lane];
        if (id >= 0) key[1] = ((u64)__float_as_uint(dists_b[row * kb + lane]) << 32) | (uint32_t)id;
    }
    int rank[2];
    // ---- the short way: ordering first
    u64* KA = keys_s[w][0];
    u64* KB = keys_s[w][1];
    KA[lane] = key[0];
    KB[lane] = key[1];
    for (int i = lane; i < MSET; i += WAVE) set_s[w][i] = -1;
    wave_lds_sync_merge();
    bool bad = false;
    if (lane > 0) {
        const u64 pa = KA[lane - 1], pb = KB[lane - 1];
        bad = !(pa < key[0] || key[0] == EMPTY_KEY) || !(pb < key[1] || key[1] == EMPTY_KEY);
    }
    bool fast = __ballot(bad) == 0ull;
    bool dupb = false;
    int less_in_b = 0, less_in_a = 0;
    if (fast) {
        // entries of the other list that sort before mine (both lists ascending, EMPTY last)
        int lo = 0, hi = WAVE;                    // first position of B with KB[pos] >= key[0]
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (KB[mid] < key[0]) lo = mid + 1; else hi = mid; }
        less_in_b = lo;
        lo = 0; hi = WAVE;                        // first position of A with KA[pos] >= key[1]
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (KA[mid] < key[1]) lo = mid + 1; else hi = mid; }
        less_in_a = lo;
        dupb = key[1] != EMPTY_KEY && lo < WAVE && KA[lo] == key[1];   // the same entry sits in A
        // every remaining id once?  insert into the hash set; meeting one's own id means no
        bool clash = false;
#pragma unroll
        for (int me = 0; me < 2; ++me) {
            const bool mine = key[me] != EMPTY_KEY && !(me == 1 && dupb);
            const int id = (int)(uint32_t)key[me];
            uint32_t h = hash32((uint32_t)id) & (MSET - 1);
            bool pending = mine;
            while (__ballot(pending) != 0ull) {
                if (pending) {
                    const int old = atomicCAS(&set_s[w][h], -1, id);
                    if (old == -1) pending = false;
                    else if (old == id) { clash = true; pending = false; }
                    else h = (h + 1) & (MSET - 1);
                }
            }
        }
        fast = __ballot(clash) == 0ull;
    }
    if (fast) {
        const u64 dm = __ballot(dupb);            // dropped entries of B, by position
        const u64 below_b = less_in_b >= 64 ? ~0ull : ((1ull << less_in_b) - 1ull);
        rank[0] = lane + less_in_b - __popcll(dm & below_b);
        rank[1] = lane + less_in_a - __popcll(dm & lanemask_lt());
        if (dupb) key[1] = EMPTY_KEY;
    } else {
        merge_general(key, ka, kb, lane, rank);
    }
    const int total = __popcll(__ballot(key[0] != EMPTY_KEY)) + __popcll(__ballot(key[1] != EMPTY_KEY));
#pragma unroll
    for (int me = 0; me < 2; ++me) {
        if (key[me] != EMPTY_KEY && rank[me] < k_out) {
            ids_out[row * k_out + rank[me]] = (int32_t)(uint32_t)key[me];
            dists_out[row * k_out + rank[me]] = __uint_as_float((uint32_t)(key[me] >> 32));
        }
    }
    for (int p = total + lane; p < k_out; p += WAVE) {         // fewer distinct ids than k_out
        ids_out[row * k_out + p] = -1;
        dists_out[row * k_out + p] = __uint_as_float(0x7f800000u);
    }
}

}  // namespace knng

using namespace knng;

extern "C" __attribute__((visibility("default"))) int knng_merge_graphs(
    const int32_t* ids_a_dev, const float* dists_a_dev, int32_t ka,
    const int32_t* ids_b_dev, const float* dists_b_dev, int32_t kb,
    int64_t n, int32_t k_out, int32_t* ids_out_dev, float* dists_out_dev, void* stream)
{
    if (n < 0 || ka < 0 || kb < 0 || ka > KNNG_MAX_K || kb > KNNG_MAX_K || ka + kb < 1 ||
        k_out < 1 || k_out > 2 * KNNG_MAX_K)
        return KNNG_EINVAL;
    if ((ka && (!ids_a_dev || !dists_a_dev)) || (kb && (!ids_b_dev || !dists_b_dev)) ||
        !ids_out_dev || !dists_out_dev)
        return KNNG_EINVAL;
    if (n == 0) return KNNG_OK;
    if ((n + 3) / 4 > 2147483647LL) return KNNG_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_merge_rows, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, ids_a_dev, dists_a_dev,
                       ka, ids_b_dev, dists_b_dev, kb, n, k_out, ids_out_dev, dists_out_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_hip_error(e, "k_merge_rows launch");
    return KNNG_OK;
}
