// Device-side helpers shared by the libknng kernels (gfx950, 64-wide wavefronts).
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace knng {

typedef unsigned long long u64;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr int WAVE = 64;
constexpr u64 EMPTY_KEY = ~0ull;

// ---- packed neighbour entries -------------------------------------------------------------
// A neighbour is one 64-bit word: [63:32] fp32 distance bits, [31:1] id, [0] "new" flag.
// Distances are >= +0, so the words order exactly like (distance, id): one integer compare
// (or one 64-bit atomic min) implements the (distance, id) order of the k-NN rows.
__device__ __forceinline__ float nonneg(float x) { return x > 0.0f ? x : 0.0f; }
__device__ __forceinline__ u64 pack_key(float dist, int id, int isnew)
{
    return ((u64)__float_as_uint(dist) << 32) | ((u64)(uint32_t)id << 1) | (u64)(isnew & 1);
}
__device__ __forceinline__ int key_id(u64 key) { return (int)((uint32_t)key >> 1); }
__device__ __forceinline__ float key_dist(u64 key) { return __uint_as_float((uint32_t)(key >> 32)); }
__device__ __forceinline__ u64 key_order(u64 key) { return key & ~1ull; }

// ---- stateless random numbers ---------------------------------------------------------------
// Counter-based: every draw is a hash of (seed, stream tag, row, slot); nothing is stored.
__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}
// hash32 is a bijection of the 32-bit integers; this is its inverse
__device__ __forceinline__ uint32_t unhash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x43021123u;
    x ^= (x >> 15) ^ (x >> 30); x *= 0x1d69e2a5u;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t rnd32(u64 seed, uint32_t tag, uint32_t row, uint32_t slot)
{
    // (seed, tag) and usually row are uniform across a wavefront, so the first two rounds run on
    // the scalar unit; only the last round is per lane
    uint32_t h = hash32(((uint32_t)seed ^ 0x9e3779b9u) + (uint32_t)(seed >> 32) * 0x85ebca6bu + tag * 0x27d4eb2fu);
    h = hash32(h ^ row);
    return hash32(h + slot * 0xc2b2ae35u);
}
// uniform-enough integer in [0, m): high half of a 32x32 product
__device__ __forceinline__ uint32_t below(uint32_t r, uint32_t m) { return __umulhi(r, m); }

// ---- wavefront helpers ------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }
__device__ __forceinline__ u64 lanemask_lt() { return (1ull << lane_id()) - 1ull; }
// value held by lane `src` (src uniform across the wave)
__device__ __forceinline__ uint32_t bcast32(uint32_t v, int src)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src);
}
__device__ __forceinline__ u64 bcast64(u64 v, int src)
{
    uint32_t lo = bcast32((uint32_t)v, src), hi = bcast32((uint32_t)(v >> 32), src);
    return ((u64)hi << 32) | lo;
}

// ---- the exact distance recipe ------------------------------------------------------------------
// Accumulate in fp64 over t ascending with fma, one rounding to fp32 at the end.  The state
// of one (a,b) pair is a single double so the chain can be continued across slabs of d.
template <int METRIC> __device__ __forceinline__ double exact_step(double acc, float a, float b)
{
    if (METRIC == 0) {
        double df = (double)a - (double)b;
        return fma(df, df, acc);
    }
    return fma((double)a, (double)b, acc);
}
template <int METRIC> __device__ __forceinline__ float exact_finish(double acc)
{
    if (METRIC == 0) return (float)acc;
    double r = 1.0 - acc;
    return (float)(r > 0.0 ? r : 0.0);
}
// general cosine (METRIC 2): the chain of <a,b> is exact_step<2>; |a|^2 and |b|^2 are chains of the
// same kind (exact_step<2>(acc, a, a)); a zero vector is at distance 1 from everything
__device__ __forceinline__ float cosine_finish(double dot, double na, double nb)
{
    if (na == 0.0 || nb == 0.0) return 1.0f;
    const double r = 1.0 - dot / sqrt(na * nb);
    return (float)(r > 0.0 ? r : 0.0);
}

// fp16 rows: two halves per 32-bit word
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));   // four bf16 bit patterns (operand of the 16x16x16 bf16 MFMA)
// a - b on the two halves of each word (v_pk_add_f16)
__device__ __forceinline__ uint32_t sub_h2(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, (half2v)(__builtin_bit_cast(half2v, a) - __builtin_bit_cast(half2v, b)));
}
__device__ __forceinline__ float4 sub_h2x4(float4 a, float4 b)
{
    return float4{__uint_as_float(sub_h2(__float_as_uint(a.x), __float_as_uint(b.x))),
                  __uint_as_float(sub_h2(__float_as_uint(a.y), __float_as_uint(b.y))),
                  __uint_as_float(sub_h2(__float_as_uint(a.z), __float_as_uint(b.z))),
                  __uint_as_float(sub_h2(__float_as_uint(a.w), __float_as_uint(b.w)))};
}
__device__ __forceinline__ float h_lo(uint32_t w) { return (float)__builtin_bit_cast(half2v, w)[0]; }
__device__ __forceinline__ float h_hi(uint32_t w) { return (float)__builtin_bit_cast(half2v, w)[1]; }

// an accumulator element as the 32 bits stored in LDS (fp32 Gram tiles / integer Gram tiles)
__device__ __forceinline__ uint32_t acc_bits(float x) { return __float_as_uint(x); }
__device__ __forceinline__ uint32_t acc_bits(int x) { return (uint32_t)x; }

}  // namespace knng
