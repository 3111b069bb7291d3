// knng_recall.hip -- graph recall on the GPU, error text and version of libknng.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <mutex>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

static thread_local char g_hip_msg[256] = "no HIP failure recorded";

int set_hip_error(hipError_t e, const char* what)
{
    snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP failure: %s (%s) in %s", hipGetErrorName(e),
             hipGetErrorString(e), what);
    return KNNG_EHIP;
}

// One thread per (row, test entry) over the nearest at_k entries (paper Sec. 5.3.1).
//   MODE 0: hit if the test id occurs among the reference row's first at_k ids (Sec. 2.1)
//   MODE 1: hit if the test distance is <= the reference row's at_k-th distance (Sec. 5.4.3)
template <int MODE>
__global__ void __launch_bounds__(256)
k_recall(const int32_t* __restrict__ tid_, const float* __restrict__ tdist, int k_test,
         const int32_t* __restrict__ rid, const float* __restrict__ rdist, int k_ref,
         int64_t rows, int at_k, u64* __restrict__ hits)
{
    __shared__ u64 part[4];
    const int64_t total = rows * at_k;
    u64 acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / at_k;
        const int a = (int)(i - row * at_k);
        if (MODE == 0) {
            const int id = tid_[row * k_test + a];
            const int32_t* r = rid + row * k_ref;
            bool hit = false;                                   // padding (id < 0) is no neighbour
            for (int b = 0; b < at_k; ++b) hit = hit || (id >= 0 && r[b] == id);
            acc += hit ? 1u : 0u;
        } else {
            acc += (tdist[row * k_test + a] <= rdist[row * k_ref + (at_k - 1)]) ? 1u : 0u;
        }
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane_id() == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(hits, t);
    }
}

// ---- the variant that allocates nothing ---------------------------------------------------
// Partial hit counts, one per workgroup, live in a file-scope device array: every GPU the library
// runs on holds its own copy at its own address for the life of the process.  In host code the
// array's name is only a stand-in; the address kernels are given comes from
// hipGetSymbolAddress, asked once per device with that device current.
constexpr int RECALL_STATIC_BLOCKS = 8192;
static __device__ __align__(256) u64 scratch[RECALL_STATIC_BLOCKS];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static u64* g_scratch_ptr[MAX_DEVICES];       // per device: address of its copy of `scratch`, null = not asked yet

static int scratch_for_current_device(u64** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_hip_error(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return KNNG_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return set_hip_error(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = static_cast<u64*>(p);
    }
    *out = g_scratch_ptr[dev];
    return KNNG_OK;
}

// the same hit test as k_recall; workgroup b leaves its count in partial[b] (no atomics, so nothing
// has to start at zero: every element that is read was written by this call)
template <int MODE>
__global__ void __launch_bounds__(256)
k_recall_partial(const int32_t* __restrict__ tid_, const float* __restrict__ tdist, int k_test,
                 const int32_t* __restrict__ rid, const float* __restrict__ rdist, int k_ref,
                 int64_t rows, int at_k, u64* __restrict__ partial)
{
    __shared__ u64 part[4];
    const int64_t total = rows * at_k;
    u64 acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / at_k;
        const int a = (int)(i - row * at_k);
        if (MODE == 0) {
            const int id = tid_[row * k_test + a];
            const int32_t* r = rid + row * k_ref;
            bool hit = false;
            for (int b = 0; b < at_k; ++b) hit = hit || (id >= 0 && r[b] == id);
            acc += hit ? 1u : 0u;
        } else {
            acc += (tdist[row * k_test + a] <= rdist[row * k_ref + (at_k - 1)]) ? 1u : 0u;
        }
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane_id() == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// one workgroup: sum of the first nblocks partial counts -> recall (a double, device memory)
__global__ void __launch_bounds__(256)
k_recall_finish(const u64* __restrict__ partial, int nblocks, double denom, double* __restrict__ out)
{
    __shared__ u64 part[4];
    u64 acc = 0;
    for (int i = threadIdx.x; i < nblocks; i += 256) acc += partial[i];
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane_id() == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = (double)(part[0] + part[1] + part[2] + part[3]) / denom;
}

}  // namespace knng

using namespace knng;

extern "C" __attribute__((visibility("default"))) int knng_graph_recall_static(const int32_t* test_ids_dev, const float* test_dists_dev, int32_t k_test,
                                        const int32_t* ref_ids_dev, const float* ref_dists_dev, int32_t k_ref,
                                        int64_t rows, int32_t at_k, int32_t mode,
                                        double* recall_out_dev, void* stream)
{
    if (!recall_out_dev || rows < 1 || at_k < 1 || at_k > k_test || at_k > k_ref || (mode != 0 && mode != 1))
        return KNNG_EINVAL;
    if (mode == 0 && (!test_ids_dev || !ref_ids_dev)) return KNNG_EINVAL;
    if (mode == 1 && (!test_dists_dev || !ref_dists_dev)) return KNNG_EINVAL;
    if (rows > KNNG_RECALL_STATIC_MAX_ENTRIES / at_k) return KNNG_ETOOLARGE;
    u64* partial = nullptr;
    int rc = scratch_for_current_device(&partial);
    if (rc != KNNG_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int64_t total = rows * (int64_t)at_k;
    int64_t blocks = (total + 255) / 256;
    if (blocks > RECALL_STATIC_BLOCKS) blocks = RECALL_STATIC_BLOCKS;
    if (mode == 0)
        hipLaunchKernelGGL(k_recall_partial<0>, dim3((unsigned)blocks), dim3(256), 0, st, test_ids_dev, test_dists_dev,
                           k_test, ref_ids_dev, ref_dists_dev, k_ref, rows, at_k, partial);
    else
        hipLaunchKernelGGL(k_recall_partial<1>, dim3((unsigned)blocks), dim3(256), 0, st, test_ids_dev, test_dists_dev,
                           k_test, ref_ids_dev, ref_dists_dev, k_ref, rows, at_k, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_hip_error(e, "k_recall_partial launch");
    hipLaunchKernelGGL(k_recall_finish, dim3(1), dim3(256), 0, st, partial, (int)blocks,
                       (double)rows * (double)at_k, recall_out_dev);
    if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e, "k_recall_finish launch");
    return KNNG_OK;
}

extern "C" __attribute__((visibility("default"))) int knng_graph_recall(const int32_t* test_ids_dev, const float* test_dists_dev, int32_t k_test,
                                 const int32_t* ref_ids_dev, const float* ref_dists_dev, int32_t k_ref,
                                 int64_t rows, int32_t at_k, int32_t mode,
                                 double* recall_out_host, void* stream)
{
    if (!recall_out_host || rows < 1 || at_k < 1 || at_k > k_test || at_k > k_ref || (mode != 0 && mode != 1))
        return KNNG_EINVAL;
    if (mode == 0 && (!test_ids_dev || !ref_ids_dev)) return KNNG_EINVAL;
    if (mode == 1 && (!test_dists_dev || !ref_dists_dev)) return KNNG_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    u64* hits_dev = nullptr;
    u64 hits = 0;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&hits_dev), sizeof(u64));
    if (e != hipSuccess) return set_hip_error(e, "hipMalloc(recall counter)");
    int rc = KNNG_OK;
    const int64_t total = rows * (int64_t)at_k;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if ((e = hipMemsetAsync(hits_dev, 0, sizeof(u64), st)) != hipSuccess) {
        rc = set_hip_error(e, "hipMemsetAsync");
        goto done;
    }
    if (mode == 0)
        hipLaunchKernelGGL(k_recall<0>, dim3((unsigned)blocks), dim3(256), 0, st, test_ids_dev, test_dists_dev,
                           k_test, ref_ids_dev, ref_dists_dev, k_ref, rows, at_k, hits_dev);
    else
        hipLaunchKernelGGL(k_recall<1>, dim3((unsigned)blocks), dim3(256), 0, st, test_ids_dev, test_dists_dev,
                           k_test, ref_ids_dev, ref_dists_dev, k_ref, rows, at_k, hits_dev);
    if ((e = hipGetLastError()) != hipSuccess) { rc = set_hip_error(e, "k_recall launch"); goto done; }
    if ((e = hipMemcpyAsync(&hits, hits_dev, sizeof(u64), hipMemcpyDeviceToHost, st)) != hipSuccess) {
        rc = set_hip_error(e, "hipMemcpyAsync");
        goto done;
    }
    if ((e = hipStreamSynchronize(st)) != hipSuccess) { rc = set_hip_error(e, "hipStreamSynchronize"); goto done; }
    *recall_out_host = (double)hits / ((double)rows * (double)at_k);
done:
    (void)hipFree(hits_dev);
    return rc;
}

extern "C" __attribute__((visibility("default"))) const char* knng_strerror(int code)
{
    switch (code) {
    case KNNG_OK: return "success";
    case KNNG_EINVAL: return "invalid argument";
    case KNNG_EWORKSPACE: return "workspace missing, misaligned or too small";
    case KNNG_EHIP: return g_hip_msg;
    case KNNG_ETOOLARGE: return "input larger than the fixed scratch of this entry point allows";
    case KNNG_ECHECK: return "debug check: a row broke an invariant";
    default: return "unknown libknng error code";
    }
}

extern "C" __attribute__((visibility("default"))) int knng_version(void) { return KNNG_VERSION; }
