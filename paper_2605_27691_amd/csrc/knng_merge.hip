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

// One wavefront per row, 4 rows per workgroup.  Lane l holds entry l of row A and entry l of row
// B as one 64-bit word (fp32 distance bits, then the id): unsigned order = (distance, id) order.
// Pass 1 drops every entry that has the same id as an entry that sorts before it (or an equal one
// at a lower position); pass 2 ranks the rest by counting.  Both walk the other entries with
// v_readlane broadcasts.
__global__ void __launch_bounds__(256)
k_merge_rows(const int32_t* __restrict__ ids_a, const float* __restrict__ dists_a, int ka,
             const int32_t* __restrict__ ids_b, const float* __restrict__ dists_b, int kb,
             int64_t n, int k_out, int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    const int lane = lane_id();
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
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
    // pass 1: repeated ids.  Entry positions: A entries 0..ka-1, then B entries.
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
    // pass 2: ranks among the survivors (their words are distinct: distinct ids)
    int rank[2] = {0, 0};
#pragma unroll
    for (int src = 0; src < 2; ++src) {
        const int cnt = src == 0 ? ka : kb;
        for (int j = 0; j < cnt; ++j) {
            const u64 kf = bcast64(key[src], j);
            rank[0] += kf < key[0] ? 1 : 0;
            rank[1] += kf < key[1] ? 1 : 0;
        }
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
