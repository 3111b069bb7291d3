// knng_build.hip -- lock-free NN-Descent on one MI355X (gfx950).
//
// Implements knng_build_knn_graph: random initial graph, then per iteration
//   k_update   one wavefront per point folds its candidate list into its row   (Sec. 3.1.1)
//              and samples new / old neighbours with reverse edges for the next join (Sec. 3.1)
//   k_plan     fixes the list lengths and compacts the points that have work
//   k_join     local join: gather the sampled neighbours' vectors into LDS, fp32 MFMA Gram
//              block, per-member best candidate, 64-bit atomic-min into the fixed-size
//              candidate lists of the two end points                           (Sec. 3.1.1)
// until an iteration accepts fewer than delta*K*n updates (Sec. 3.1), then
//   k_finalize exact fp64 re-evaluation of every kept distance, sort, cut to k (Sec. 5.3.1).
//
// Memory model: G is only ever written by the wavefront that owns the row (k_init, k_update);
// all cross-row traffic of an iteration goes through the candidate slots with
// order-independent atomic mins, so there are no locks and no retry loops anywhere.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <math.h>

#include "../../include/knng.h"
#include "knng_device.h"
#include "knng_host.h"

namespace knng {

// ------------------------------------------------------------------------------------------
// fp32 distance of (x_v, x_u) by a group of 8 lanes: each lane strides over 16-byte pieces,
// then a 3-step butterfly leaves the sum in all 8 lanes.  Search-time precision only: what
// is written to the caller is recomputed by k_finalize.
// ------------------------------------------------------------------------------------------
template <int METRIC>
__device__ __forceinline__ float dist_group8(const float* __restrict__ a, const float* __restrict__ b,
                                             int d, int sub)
{
    float acc = 0.0f;
    if ((d & 3) == 0) {
        const float4* a4 = reinterpret_cast<const float4*>(a);
        const float4* b4 = reinterpret_cast<const float4*>(b);
        for (int t = sub; t < (d >> 2); t += 8) {
            float4 x = a4[t], y = b4[t];
            if (METRIC == 0) {
                float e0 = x.x - y.x, e1 = x.y - y.y, e2 = x.z - y.z, e3 = x.w - y.w;
                acc = fmaf(e0, e0, acc); acc = fmaf(e1, e1, acc);
                acc = fmaf(e2, e2, acc); acc = fmaf(e3, e3, acc);
            } else {
                acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc);
                acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
            }
        }
    } else {
        for (int t = sub; t < d; t += 8) {
            float x = a[t], y = b[t];
            if (METRIC == 0) { float e = x - y; acc = fmaf(e, e, acc); }
            else acc = fmaf(x, y, acc);
        }
    }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    return METRIC == 0 ? nonneg(acc) : nonneg(1.0f - acc);
}

// ------------------------------------------------------------------------------------------
// uint8 rows (squared L2): sum of (a_i - b_i)^2 over four packed bytes as a.a + b.b - 2 a.b with
// unsigned dot products.  Sums are exact in 32 bits for d <= 65536 (65536 * 255^2 < 2^32).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t sqdiff4_u8(uint32_t a, uint32_t b)
{
    const uint32_t nn = __builtin_amdgcn_udot4(a, a, __builtin_amdgcn_udot4(b, b, 0u, false), false);
    return nn - 2u * __builtin_amdgcn_udot4(a, b, 0u, false);
}
__device__ __forceinline__ uint32_t sqdiff16_u8(uint4 a, uint4 b)
{
    return sqdiff4_u8(a.x, b.x) + sqdiff4_u8(a.y, b.y) + sqdiff4_u8(a.z, b.z) + sqdiff4_u8(a.w, b.w);
}
// distance by a group of 8 lanes, as dist_group8; d % 4 == 0, rows 4-byte aligned
__device__ __forceinline__ float dist_group8_u8(const unsigned char* __restrict__ a,
                                                const unsigned char* __restrict__ b, int d, int sub)
{
    uint32_t acc = 0u;
    if ((d & 15) == 0) {
        const uint4* a4 = reinterpret_cast<const uint4*>(a);
        const uint4* b4 = reinterpret_cast<const uint4*>(b);
        for (int t = sub; t < (d >> 4); t += 8) acc += sqdiff16_u8(a4[t], b4[t]);
    } else {
        const uint32_t* a1 = reinterpret_cast<const uint32_t*>(a);
        const uint32_t* b1 = reinterpret_cast<const uint32_t*>(b);
        for (int t = sub; t < (d >> 2); t += 8) acc += sqdiff4_u8(a1[t], b1[t]);
    }
    acc += (uint32_t)__shfl_xor((int)acc, 1);
    acc += (uint32_t)__shfl_xor((int)acc, 2);
    acc += (uint32_t)__shfl_xor((int)acc, 4);
    return (float)acc;
}

// fp16 rows (squared L2), search-time precision: fp32 accumulation of the squared differences
// of the converted halves; d % 2 == 0, rows 4-byte aligned
__device__ __forceinline__ float dist_group8_f16(const uint32_t* __restrict__ a, const uint32_t* __restrict__ b,
                                                 int d, int sub)
{
    float acc = 0.0f;
    auto word = [&](uint32_t x, uint32_t y) {
        const float e0 = h_lo(x) - h_lo(y), e1 = h_hi(x) - h_hi(y);
        acc = fmaf(e0, e0, acc); acc = fmaf(e1, e1, acc);
    };
    if ((d & 7) == 0) {
        const uint4* a4 = reinterpret_cast<const uint4*>(a);
        const uint4* b4 = reinterpret_cast<const uint4*>(b);
        for (int t = sub; t < (d >> 3); t += 8) {
            const uint4 x = a4[t], y = b4[t];
            word(x.x, y.x); word(x.y, y.y); word(x.z, y.z); word(x.w, y.w);
        }
    } else {
        for (int t = sub; t < (d >> 1); t += 8) word(a[t], b[t]);
    }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    return nonneg(acc);
}

// ------------------------------------------------------------------------------------------
// Row signature: a 256-bit Bloom-style set of the ids in a point's row (bit hash(id) & 255).
// The join uses it to skip partners a member most likely already holds: such offers would be
// rejected by the merge anyway, cost an atomic each, and would shadow real candidates in the
// hashed candidate slots.  A false positive (about 12% at K = 32) only delays a candidate.
// k_update rebuilds every row's signature each iteration, right before the join reads it.
// ------------------------------------------------------------------------------------------
constexpr int SIG_WORDS = 8;
// The bit an id maps to changes with the iteration (salt), so a false positive does not
// shadow the same candidate for good.
__device__ __forceinline__ uint32_t sig_bit(int id, uint32_t salt)
{
    return hash32((uint32_t)id ^ (salt * 0x9e3779b9u + 0x5bd1e995u)) & 255u;
}

// Orders one wavefront's own LDS accesses (they execute in order; this keeps the compiler from
// moving them and makes returned data available): enough for wavefront-private LDS regions.
__device__ __forceinline__ void wave_lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

#ifndef KNNG_REV_MULT
#define KNNG_REV_MULT 2          // reverse buckets per point and kind, in units of s
#endif
constexpr uint32_t EMPTY_REV = 0xffffffffu;            // an empty reverse bucket

// ------------------------------------------------------------------------------------------
// k_init: one wavefront per point.  K distinct ids != v (random, or the caller's warm start
// with bad entries redrawn), their distances, row sorted by (distance, id), all flagged new.
// Also puts the point's candidate slots, counters and threshold into their start state.
// ------------------------------------------------------------------------------------------
// ELEM 1: pts points at uint8 rows of d bytes; ELEM 2: at fp16 rows of d halves.
template <int METRIC, int ELEM>
__global__ void __launch_bounds__(256)
k_init(const float* __restrict__ pts, int64_t n, int d, int K, int C, u64 seed,
       const int32_t* __restrict__ init_ids, u64* __restrict__ G, u64* __restrict__ cand,
       int32_t* __restrict__ cnt, float* __restrict__ worst, uint32_t* __restrict__ rev, int B)
{
    const int lane = lane_id();
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    for (int j = lane; j < C; j += WAVE) cand[v * C + j] = EMPTY_KEY;
    if (lane < 2) cnt[v * 2 + lane] = 0;
    for (int j = lane; j < B; j += WAVE) {           // reverse buckets of the first iteration
        rev[v * B + j] = EMPTY_REV;
        rev[(n + v) * B + j] = EMPTY_REV;
    }

    const bool active = lane < K;
    const uint32_t un = (uint32_t)n;
    int id;
    bool dense = (2 * (int64_t)K > n - 1);
    if (!dense) {
        id = init_ids ? (active ? init_ids[v * K + lane] : -1)
                      : (int)below(rnd32(seed, 0x100u, (uint32_t)v, (uint32_t)lane), un);
        for (int attempt = 1; attempt <= 64; ++attempt) {
            bool bad = active && (id < 0 || (int64_t)id >= n || (int64_t)id == v);
            for (int j = 0; j < K; ++j) {
                int oj = (int)bcast32((uint32_t)id, j);
                if (active && j < lane && oj == id) bad = true;
            }
            if (__ballot(bad) == 0ull) break;
            if (attempt == 64) { dense = true; break; }   // give up on random draws
            if (bad) id = (int)below(rnd32(seed, 0x100u + attempt, (uint32_t)v, (uint32_t)lane), un);
        }
    }
    if (dense) {
        // K consecutive residues from a random start: distinct by construction
        uint32_t start = below(rnd32(seed, 0x1ffu, (uint32_t)v, 0u), un - 1u);
        uint32_t j = (start + (uint32_t)lane) % (un - 1u);
        id = (int)(((uint64_t)v + 1u + j) % (uint64_t)n);
    }
    if (!active) id = (int)v;

    // distances: 8 lanes per entry, 8 entries per pass
    const float* xv = pts + v * (int64_t)d;
    float dist = 0.0f;
    const int sub = lane & 7, grp = lane >> 3;
    for (int pass = 0; pass * 8 < K; ++pass) {
        int e = pass * 8 + grp;
        int uid = __shfl(id, e < K ? e : 0);
        float val;
        if constexpr (ELEM == 1) {
            const unsigned char* p8 = reinterpret_cast<const unsigned char*>(pts);
            val = dist_group8_u8(p8 + v * (int64_t)d, p8 + (int64_t)uid * d, d, sub);
        } else if constexpr (ELEM == 2) {
            const uint32_t* p16 = reinterpret_cast<const uint32_t*>(pts);       // d / 2 words per row
            val = dist_group8_f16(p16 + v * (int64_t)(d >> 1), p16 + (int64_t)uid * (d >> 1), d, sub);
        } else {
            val = dist_group8<METRIC>(xv, pts + (int64_t)uid * d, d, sub);
        }
        float mine = __shfl(val, (lane & 7) * 8);
        if ((lane >> 3) == pass) dist = mine;
    }
    u64 key = active ? pack_key(dist, id, 1) : EMPTY_KEY;
    int rank = 0;
    for (int j = 0; j < K; ++j) rank += (bcast64(key, j) < key) ? 1 : 0;
    if (active) {
        G[v * K + rank] = key;
        if (rank == K - 1) worst[v] = dist;
    }
}

// ------------------------------------------------------------------------------------------
// k_update: the per-point work between two joins, one wavefront per point (persistent
// wavefronts stride over the points and prefetch the next point's row and candidate slots).
//
// Merge (Sec. 3.1.1: a single owner per point folds its candidate list into its row, so no
// races): a candidate is accepted if its id is not already in the row and it sorts before the
// row's K-th entry; the union is re-ranked by counting, the first K kept, accepted entries
// flagged new and counted as updates; used slots are set back to empty.
//
// Sample (Sec. 3.1, rate rho) for the next join, from the merged row while it is still in
// registers: up to s new-flagged entries (a cyclic window of the flagged ones from a random
// start, so every flagged entry is equally likely) become the forward new sample and lose
// their flag; up to s unflagged entries the forward old sample.  Each forward edge v->u also
// enters v into u's reverse sample: u owns B buckets per kind, v falls into bucket
// hash(v) mod B and the bucket keeps the arrival with the smallest random priority (one 32-bit
// atomic min, nothing comes back to the wavefront).  A bucket thus holds a uniformly random one
// of its arrivals, whatever order they came in; k_plan turns the buckets into the reverse list.
// What is stored is hash32(v ^ salt(u)): the priority and, hash32 being a bijection, also v.
// rev[parity][kind][point][bucket]: this launch fills parity iter&1 and resets the point's own
// buckets of the other parity for the next iteration.
// Lists: NEW[v] = [fwd 0..s) [rev s..2s), OLD likewise; cnt[v] = {fwd new, fwd old}.  The
// row's signature for this iteration is rebuilt here as well.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t rev_salt(u64 seed, uint32_t iter)
{
    return hash32((uint32_t)seed ^ (uint32_t)(seed >> 32) * 0x85ebca6bu ^ (iter * 0x9e3779b9u + 0x68e31da4u));
}

__global__ void __launch_bounds__(256)
k_update(int64_t n, int K, int C, int s, u64 seed, uint32_t iter, int do_sample,
         u64* __restrict__ G, u64* __restrict__ cand, int32_t* __restrict__ newl, int32_t* __restrict__ oldl,
         int32_t* __restrict__ cnt, uint32_t* __restrict__ sig, float* __restrict__ worst,
         u64* __restrict__ updates, uint32_t* __restrict__ rev, int B)
{
    __shared__ u64 rowbuf[4][WAVE];
    __shared__ u64 candbuf[4][WAVE];                 // the accepted candidates' order words, compacted
    __shared__ u64 lobuf[4][WAVE];                   // the row's order words
    __shared__ uint32_t sigbuf[4][SIG_WORDS];
    __shared__ u64 part[8];
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // keeps v scalar
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const u64 lt = lanemask_lt();
    const uint32_t tag = 0x200u + 4u * iter;
    u64 accepted = 0;
    uint32_t occupied = 0;                           // candidate slots found occupied (uniform)

    const uint32_t saltp = rev_salt(seed, iter);
    const uint32_t salts = hash32(saltp + 0x3c6ef372u);
    uint32_t* rev_cur = rev + (int64_t)(iter & 1u) * 2 * n * B;          // [kind][point][bucket]
    uint32_t* rev_nxt = rev + (int64_t)((iter & 1u) ^ 1u) * 2 * n * B;

    int64_t v = (int64_t)blockIdx.x * 4 + w;
    u64 lk_n = EMPTY_KEY, ck_n = EMPTY_KEY;
    if (v < n) {
        if (lane < K) lk_n = G[v * K + lane];
        if (lane < C) ck_n = cand[v * C + lane];
    }
    // The first row is waited for here, so that inside the loop the compiler knows the working
    // registers are settled and does not wait for the prefetch it has just issued.
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
    for (; v < n; v += nwaves) {
        u64 row = lk_n;                              // lane < K: entry `lane` of the row
        const u64 ck = ck_n;
        const int64_t vn = v + nwaves;
        lk_n = EMPTY_KEY; ck_n = EMPTY_KEY;
        if (vn < n) {                                // prefetch the next point of this wavefront
            if (lane < K) lk_n = G[vn * K + lane];
            if (lane < C) ck_n = cand[vn * C + lane];
        }
        bool changed = false;
        // ---- merge
        const u64 occm = __ballot(ck != EMPTY_KEY);
        if (occm != 0ull) {
            occupied += (uint32_t)__popcll(occm);
            if (ck != EMPTY_KEY) cand[v * C + lane] = EMPTY_KEY;
            const u64 lo = key_order(row);
            const u64 co = key_order(ck);
            const u64 last = bcast64(lo, K - 1);
            // No test against the row's ids: the join only offers ids that fail the row's
            // signature, which holds every id of the row (no false negatives), and an id always
            // lands in the same slot, so the candidates are distinct from the row and each other.
            const bool valid = ck != EMPTY_KEY && co < last;
            {
                const u64 vm = __ballot(valid);
                if (vm != 0ull) {
                    // ranks in the union of the row and the accepted candidates.  The candidates'
                    // order words are compacted into LDS and every lane walks them (one broadcast
                    // read each): a row entry moves up by the candidates before it, a candidate
                    // lands after the candidates before it and the row entries before it (a
                    // binary search in the row, which is ascending).
                    const int nv = __popcll(vm);
                    if (valid) candbuf[w][__popcll(vm & lt)] = co;
                    if (lane < K) lobuf[w][lane] = lo;
                    wave_lds_sync();
                    int rl = lane;                   // the row is ascending already
                    int rc = 0;
#pragma unroll 4
                    for (int j = 0; j < nv; ++j) {
                        const u64 cj = candbuf[w][j];
                        rl += cj < lo ? 1 : 0;
                        rc += cj < co ? 1 : 0;
                    }
                    {
                        int a = 0, b = K;
                        while (__ballot(a < b) != 0ull) {
                            const int mid = (a + b) >> 1;
                            const u64 lm = lobuf[w][mid < WAVE ? mid : WAVE - 1];
                            if (a < b) { if (lm < co) a = mid + 1; else b = mid; }
                        }
                        rc += a;
                    }
                    const bool in = valid && rc < K;
                    if (lane < K && rl < K) rowbuf[w][rl] = row;
                    if (in) rowbuf[w][rc] = ck | 1ull;
                    wave_lds_sync();
                    row = lane < K ? rowbuf[w][lane] : EMPTY_KEY;
                    wave_lds_sync();
                    changed = true;
                    accepted += (u64)__popcll(__ballot(in));
                    if (lane == K - 1) worst[v] = key_dist(row);
                }
            }
        }
        if (!do_sample) {
            if (changed && lane < K) G[v * K + lane] = row;
            continue;
        }
        // ---- sample for the next join
        const bool active = lane < K;
        const bool isnew = active && (row & 1ull);
        const int id = key_id(row);
        const u64 newmask = __ballot(isnew), oldmask = __ballot(active && !isnew);
        const int cn = __popcll(newmask), co_ = __popcll(oldmask);
        const int64_t base = v * 2 * (int64_t)s;
        bool cleared = false;
        {
            // one code path for both kinds: an entry is either flagged or not
            const int off_n = (int)below(rnd32(seed, tag, (uint32_t)v, 0u), (uint32_t)cn);
            const int off_o = (int)below(rnd32(seed, tag + 1u, (uint32_t)v, 0u), (uint32_t)co_);
            const int cm = isnew ? cn : co_;
            int p = __popcll((isnew ? newmask : oldmask) & lt) - (isnew ? off_n : off_o);
            if (p < 0) p += cm;
            const bool sampled = active && p < s;
            if (sampled) {
                (isnew ? newl : oldl)[base + p] = id;
                if (isnew) { row &= ~1ull; cleared = true; }
                const uint32_t mix = saltp ^ ((uint32_t)id * 0x85ebca6bu);  // per target: independent draws
                const uint32_t bucket = below(hash32((uint32_t)v * 0x9e3779b1u + (mix ^ salts)), (uint32_t)B);
                atomicMin(&rev_cur[((isnew ? 0 : n) + (int64_t)id) * B + bucket], hash32((uint32_t)v ^ mix));
            }
            // the point's own buckets of the other parity: empty for the next iteration
            const int q = lane & 31;
            if (4 * q < B)
                *reinterpret_cast<uint4*>(rev_nxt + ((lane < 32 ? 0 : n) + v) * B + 4 * q) =
                    uint4{EMPTY_REV, EMPTY_REV, EMPTY_REV, EMPTY_REV};
        }
        if (active && (changed || cleared)) G[v * K + lane] = row;
        if (lane == 0) {
            cnt[v * 2 + 0] = cn < s ? cn : s;
            cnt[v * 2 + 1] = co_ < s ? co_ : s;
        }
        // ---- signature of the row for this iteration: OR of one bit per entry, through LDS
        if (lane < SIG_WORDS) sigbuf[w][lane] = 0u;
        wave_lds_sync();
        if (active) {
            const uint32_t h = sig_bit(id, iter);
            atomicOr(&sigbuf[w][h >> 5], 1u << (h & 31u));
        }
        wave_lds_sync();
        if (lane < SIG_WORDS) sig[v * SIG_WORDS + lane] = sigbuf[w][lane];
        wave_lds_sync();
    }
    if (lane == 0) { part[w] = accepted; part[4 + w] = (u64)occupied; }
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(updates, t);
        t = part[4] + part[5] + part[6] + part[7];
        if (t) atomicAdd(updates + 5, t);            // ctr[5]: occupied candidate slots
    }
}

// ------------------------------------------------------------------------------------------
// k_check_rows (debug mode): one wavefront per point, after k_update; counts broken invariants.
// sampled: k_update also sampled (lists, counts and signature are current).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_check_rows(int64_t n, int K, int C, int s, uint32_t iter, int sampled, const u64* __restrict__ G,
             const u64* __restrict__ cand, const int32_t* __restrict__ newl, const int32_t* __restrict__ oldl,
             const int32_t* __restrict__ cnt, const uint32_t* __restrict__ sig, const float* __restrict__ worst,
             u64* __restrict__ violations)
{
    const int lane = lane_id();
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const bool in = lane < K;
    const u64 e = in ? G[v * K + lane] : EMPTY_KEY;
    const int id = key_id(e);
    const uint32_t db = (uint32_t)(e >> 32);
    bool bad = false;
    if (in) {
        bad |= e == EMPTY_KEY;                                   // rows are full from the start
        bad |= id < 0 || (int64_t)id >= n || (int64_t)id == v;
        bad |= (db >> 31) != 0u || db > 0x7f800000u;             // negative, or not a number
    }
    // strictly ascending in (distance, id)
    const u64 nxt = __shfl(key_order(e), lane + 1 < K ? lane + 1 : lane);
    if (lane + 1 < K) bad |= !(key_order(e) < nxt);
    // ids pairwise distinct
    for (int j = 0; j < K; ++j) {
        const int idj = (int)bcast32((uint32_t)id, j);
        if (in && lane != j && idj == id) bad = true;
    }
    if (lane == K - 1) bad |= __float_as_uint(worst[v]) != db;   // the threshold the join compares against
    if (lane < C) bad |= cand[v * C + lane] != EMPTY_KEY;        // the merge empties what it used
    if (sampled) {
        const int cn = cnt[v * 2 + 0], co = cnt[v * 2 + 1];
        if (lane == 0) bad |= cn < 0 || cn > s || co < 0 || co > s;
        if (lane < s) {
            if (lane < cn) { const int u = newl[v * 2 * (int64_t)s + lane]; bad |= u < 0 || (int64_t)u >= n; }
            if (lane < co) { const int u = oldl[v * 2 * (int64_t)s + lane]; bad |= u < 0 || (int64_t)u >= n; }
        }
        if (in && !(id < 0 || (int64_t)id >= n)) {
            const uint32_t h = sig_bit(id, iter);
            bad |= ((sig[v * SIG_WORDS + (h >> 5)] >> (h & 31u)) & 1u) == 0u;
        }
    }
    const u64 m = __ballot(bad);
    if (lane == 0 && m != 0ull) atomicAdd(violations, (u64)__popcll(m));
}

// ------------------------------------------------------------------------------------------
// k_plan: after sampling, turn every point's reverse buckets into its reverse lists (the
// non-empty buckets in bucket order, decoded, at most s: a random subset, since bucket numbers
// are hashes), fix the four list lengths for the join, append the points that have anything new
// around them to the active list, and count the vectors the join will gather.
// A block owns PLAN_CHUNK consecutive points: it takes its share of the active list with one
// atomic.  ctr[1] += vectors, ctr[2] += active points, ctr[3] += pairs to evaluate.
// A wavefront reads whole 16-byte pieces: LPL lanes per list, 64/LPL lists (both kinds of
// 32/LPL points) per step.
// ------------------------------------------------------------------------------------------
constexpr int PLAN_CHUNK = 512;
__global__ void __launch_bounds__(256)
k_plan(int64_t n, int s, int B, u64 seed, uint32_t iter, const uint32_t* __restrict__ rev_cur,
       const int2* __restrict__ cnt, int32_t* __restrict__ newl, int32_t* __restrict__ oldl,
       int4* __restrict__ plan, int32_t* __restrict__ active, u64* __restrict__ ctr)
{
    __shared__ unsigned char actf[PLAN_CHUNK];
    __shared__ u64 wrows[4], wpairs[4];
    __shared__ int wcnt[4];
    __shared__ u64 s_base;
    const uint32_t saltp = rev_salt(seed, iter);
    const int lane = lane_id();
    const int w = (int)(threadIdx.x >> 6);
    const int q4 = B / 4;                            // 16-byte pieces per list (B % 4 == 0, B <= 128)
    int LPL = 1;
    while (LPL < q4) LPL <<= 1;                      // lanes per list, <= 32
    const int pps = 32 / LPL;                        // points per wavefront step
    const int g = lane / LPL, j = lane & (LPL - 1);
    const int kind = g & 1;
    const int64_t p0 = (int64_t)blockIdx.x * PLAN_CHUNK;
    const int npts = (int)((n - p0) < PLAN_CHUNK ? (n - p0) : PLAN_CHUNK);
    const u64 gm = ((1ull << LPL) - 1ull) << (g * LPL);
    const u64 ltg = gm & lanemask_lt();
    u64 rows = 0, pairs = 0;
    auto load_piece = [&](int base) {
        const int pl = base + (g >> 1);
        uint4 key = uint4{EMPTY_REV, EMPTY_REV, EMPTY_REV, EMPTY_REV};
        if (pl < npts && j < q4)
            key = *reinterpret_cast<const uint4*>(rev_cur + ((kind ? n : 0) + p0 + pl) * B + 4 * j);
        return key;
    };
    uint4 key_n = load_piece(w * pps);
    for (int base = w * pps; base < npts; base += 4 * pps) {
        const int pl = base + (g >> 1);
        const bool pin = pl < npts;
        const int64_t p = p0 + pl;
        const uint4 key = key_n;
        key_n = load_piece(base + 4 * pps);          // in flight while this step is written out
        const bool v0 = key.x != EMPTY_REV, v1 = key.y != EMPTY_REV, v2 = key.z != EMPTY_REV, v3 = key.w != EMPTY_REV;
        const u64 b0 = __ballot(v0), b1 = __ballot(v1), b2 = __ballot(v2), b3 = __ballot(v3);
        int r = __popcll(b0 & ltg) + __popcll(b1 & ltg) + __popcll(b2 & ltg) + __popcll(b3 & ltg);
        const int total = __popcll(b0 & gm) + __popcll(b1 & gm) + __popcll(b2 & gm) + __popcll(b3 & gm);
        int32_t* dst = (kind ? oldl : newl) + p * 2 * (int64_t)s + s;
        const uint32_t mix = saltp ^ ((uint32_t)p * 0x85ebca6bu);
        if (v0) { if (r < s) dst[r] = (int32_t)(unhash32(key.x) ^ mix); ++r; }
        if (v1) { if (r < s) dst[r] = (int32_t)(unhash32(key.y) ^ mix); ++r; }
        if (v2) { if (r < s) dst[r] = (int32_t)(unhash32(key.z) ^ mix); ++r; }
        if (v3) { if (r < s) dst[r] = (int32_t)(unhash32(key.w) ^ mix); ++r; }
        const int mine = total < s ? total : s;
        const int other = __shfl(mine, lane ^ LPL);  // the same point's list of the other kind
        if (pin && j == 0 && kind == 0) {
            const int2 c = cnt[p];
            plan[p] = int4{c.x, c.y, mine, other};
            const bool act = (c.x + mine) > 0;
            actf[pl] = act ? 1 : 0;
            if (act) {
                rows += (u64)(c.x + c.y + mine + other);
                const int nn = c.x + mine, no = c.y + other;
                pairs += (u64)(nn * (nn - 1) / 2 + nn * no);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) { rows += __shfl_xor(rows, o); pairs += __shfl_xor(pairs, o); }
    __syncthreads();
    const int t = (int)threadIdx.x;
    const bool a0 = t < npts && actf[t] != 0;
    const bool a1 = t + 256 < npts && actf[t + 256] != 0;
    const u64 m0 = __ballot(a0), m1 = __ballot(a1);
    if (lane == 0) { wcnt[w] = __popcll(m0) + __popcll(m1); wrows[w] = rows; wpairs[w] = pairs; }
    __syncthreads();
    if (t == 0) {
        const int tot = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        s_base = tot ? atomicAdd(ctr + 2, (u64)tot) : 0ull;
        const u64 rt = wrows[0] + wrows[1] + wrows[2] + wrows[3];
        if (rt) atomicAdd(ctr + 1, rt);
        const u64 pt = wpairs[0] + wpairs[1] + wpairs[2] + wpairs[3];
        if (pt) atomicAdd(ctr + 3, pt);
    }
    __syncthreads();
    u64 at = s_base;
    for (int i = 0; i < w; ++i) at += (u64)wcnt[i];
    if (a0) active[at + __popcll(m0 & lanemask_lt())] = (int32_t)(p0 + t);
    if (a1) active[at + __popcll(m0) + __popcll(m1 & lanemask_lt())] = (int32_t)(p0 + t + 256);
}

// ------------------------------------------------------------------------------------------
// k_join: the local join.  Persistent 256-thread workgroups walk the active points; the work
// of a point is split into slabs of DS coordinates, and the loop is software-pipelined over
// (point, slab) units: while the matrix cores and the selection work on the unit in LDS, the
// global loads of the next unit (and the list record of the point after) are already in
// flight into registers.  Barriers wait on LDS traffic only, never on outstanding global loads.
//
// Members of point v: m in [0,nNew) = NEW[v] (forward then reverse sample), m in [nNew,nTot)
// = OLD[v].  Their vectors are gathered with 16-byte loads (a row's pieces in adjacent lanes),
// the pivot x_v is subtracted (keeps |a|^2+|b|^2-2ab away from cancellation: members are near
// v) and the centred slab is stored in LDS.  The four wavefronts compute the NEW x (NEW|OLD)
// Gram block with v_mfma_f32_16x16x4_f32, accumulating over slabs.  The distance block then
// replaces the slab in LDS; every member takes, per residue class of partner index, its
// closest partner that beats the member's farthest neighbour and is not in the member's
// signature, and offers it with one 64-bit atomic min on cand[member][hash(partner) % C].
//
// S16 = number of 16-row tiles of NEW (2s <= 16*S16); DS = slab length in floats.
// ------------------------------------------------------------------------------------------
// Each member's partners are split into residue classes (partner index mod LPM), one per lane.
#ifndef KNNG_OFFERS_PER_MEMBER
#define KNNG_OFFERS_PER_MEMBER 4
#endif
#ifndef KNNG_JOIN_DS
#define KNNG_JOIN_DS 64       // slab length for s <= 16 (the paper's default parameters)
#endif
constexpr int OFFERS_PER_MEMBER = KNNG_OFFERS_PER_MEMBER;

template <int S16, int DS_, int ELEM = 0> struct JoinCfg {
    static constexpr int MROWS = 16 * S16;            // max |NEW|
    static constexpr int NCOLS = 32 * S16;            // max |NEW| + |OLD|
    static constexpr int DS = DS_;
    static constexpr int LD = DS + 4;                 // row stride of the vector slab (floats)
    static constexpr int LDD = NCOLS + 1;             // row stride of the distance block
    static constexpr int NT = (3 * S16 * S16 + 3 * S16 + 7) / 8; // 16x16 tiles per wavefront (upper bound)
    static constexpr int NL = NCOLS * (DS / 4) / 256; // 16-byte pieces a thread gathers per slab
    static constexpr int XBYTES = NCOLS * LD * 4 > MROWS * LDD * 4 ? NCOLS * LD * 4 : MROWS * LDD * 4;
    // ELEM 1 (uint8 rows): + the pivot's row and a row of zeros [2][LD], pivot distances [NCOLS]
    static constexpr int LDS_BYTES = XBYTES + NCOLS * (8 + 8 + 8 + 4 * SIG_WORDS) + 16 + 4 * SIG_WORDS +
                                     (ELEM == 1 ? 2 * LD * 4 + NCOLS * 4 : 0);
};

// 16-byte piece [t, t+4) of a row, zero beyond d.  VEC: d % 4 == 0 and rows 16-byte aligned, so
// a piece is either whole or empty and one vector load serves.
template <bool VEC>
__device__ __forceinline__ float4 load_piece(const float* __restrict__ row, int t, int d)
{
    float4 x = float4{0.0f, 0.0f, 0.0f, 0.0f};
    if (VEC) {
        if (t < d) x = *reinterpret_cast<const float4*>(row + t);
    } else {
        if (t < d) x.x = row[t];
        if (t + 1 < d) x.y = row[t + 1];
        if (t + 2 < d) x.z = row[t + 2];
        if (t + 3 < d) x.w = row[t + 3];
    }
    return x;
}

// 16-byte piece at t; VEC: the caller keeps t inside the row, so the load is unconditional (a
// zero fill before a predicated load would make the compiler wait for every load in flight)
template <bool VEC>
__device__ __forceinline__ float4 load_piece_inside(const float* __restrict__ row, int t, int d)
{
    if (VEC) return *reinterpret_cast<const float4*>(row + t);
    return load_piece<false>(row, t, d);
}

// Workgroup barrier that orders LDS accesses only: outstanding global loads stay in flight.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// thread -> (piece c4 of a row, rows rsub + i*RP) for a slab with q4 pieces per row: pieces are
// rounded up to a power of two QP so a row's pieces sit in QP adjacent lanes
struct SlabMap {
    int len16, q4, qshift, c4, rsub, RP;
    bool col_ok;
};
__device__ __forceinline__ SlabMap slab_map(int d, int k0, int DS, int tid)
{
    SlabMap m;
    const int len = (d - k0) < DS ? (d - k0) : DS;
    m.len16 = (len + 15) & ~15;                        // zero-padded for the MFMA k-loop
    m.q4 = m.len16 >> 2;
    m.qshift = 2;
    while ((1 << m.qshift) < m.q4) ++m.qshift;
    m.RP = 256 >> m.qshift;
    m.c4 = tid & ((1 << m.qshift) - 1);
    m.rsub = tid >> m.qshift;
    m.col_ok = m.c4 < m.q4;
    return m;
}

struct PointPlan { int nfn, nfo, nNew, nTot; };
__device__ __forceinline__ PointPlan make_point(int4 c)
{
    PointPlan p;
    p.nfn = __builtin_amdgcn_readfirstlane(c.x);
    p.nfo = __builtin_amdgcn_readfirstlane(c.y);
    p.nNew = p.nfn + __builtin_amdgcn_readfirstlane(c.z);
    p.nTot = p.nNew + p.nfo + __builtin_amdgcn_readfirstlane(c.w);
    return p;
}
// member index of list slot t (t in [0,2s): NEW list, [2s,4s): OLD list), or -1
__device__ __forceinline__ int member_of_slot(int t, int s, int4 c)
{
    const int nNew = c.x + c.z;
    if (t < s) return t < c.x ? t : -1;
    if (t < 2 * s) return (t - s) < c.z ? c.x + (t - s) : -1;
    if (t < 3 * s) return (t - 2 * s) < c.y ? nNew + (t - 2 * s) : -1;
    if (t < 4 * s) return (t - 3 * s) < c.w ? nNew + c.y + (t - 3 * s) : -1;
    return -1;
}

// Two bf16 halves of four fp32 values, both rounded to nearest (v_cvt_pk_bf16_f32): hi = bf16(x),
// lo = bf16(x - hi) (that difference is exact in fp32).  |x - hi| <= 2^-9 |x|, |x - hi - lo| <= 2^-18 |x|.
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float floatx2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_bf16(float4 x, short4v& hi, short4v& lo)
{
    const bf16x2v h01 = __builtin_convertvector(floatx2v{x.x, x.y}, bf16x2v);
    const bf16x2v h23 = __builtin_convertvector(floatx2v{x.z, x.w}, bf16x2v);
    const floatx2v f01 = __builtin_convertvector(h01, floatx2v), f23 = __builtin_convertvector(h23, floatx2v);
    const bf16x2v l01 = __builtin_convertvector(floatx2v{x.x - f01.x, x.y - f01.y}, bf16x2v);
    const bf16x2v l23 = __builtin_convertvector(floatx2v{x.z - f23.x, x.w - f23.y}, bf16x2v);
    hi = __builtin_bit_cast(short4v, uint2{__builtin_bit_cast(uint32_t, h01), __builtin_bit_cast(uint32_t, h23)});
    lo = __builtin_bit_cast(short4v, uint2{__builtin_bit_cast(uint32_t, l01), __builtin_bit_cast(uint32_t, l23)});
}

// When is a distance from the bf16-split Gram pass good enough?  hi.hi + hi.lo + lo.hi misses <a,b>
// by the dropped lo.lo and by what the two halves do not hold: at most 3 * 2^-18 |a||b| of the
// pivot-centred vectors, and much less on average (the roundings are unbiased, so the terms of
// the sum mostly cancel).  The distance the join compares, |a|^2 + |b|^2 - 2<a,b>, is then off by
// at most 12 * 2^-18 N ~ 2^-14.4 N, N = max(|a - v|^2, |b - v|^2): nothing next to a distance of
// the size of N, but as large as the distance itself for a pair that is tens of thousands of
// times closer to each other than to the pivot (tight clusters far apart, near-duplicate rows).
// Such a value would enter a row as it is and stay there: an id that sits in a row is never
// offered again.  So a chosen partner whose distance is below 2^-9 N is not trusted (above, the
// error is under 2.5 % of the distance in the worst case and a few 1e-4 of it typically); a point
// with such a choice is appended to a list and joined again, whole, by the fp32 kernel in a
// second launch.
// n_a, n_b: |a - v|^2, |b - v|^2; scale: what the compared value is of |a - b|^2 (1, or 1/2 for 1 - <a,b>).
__device__ __forceinline__ bool split_untrusted(uint32_t l_bits, float n_a, float n_b, float scale)
{
    const float nmax = n_a > n_b ? n_a : n_b;
    return __uint_as_float(l_bits) < nmax * (scale * 0.001953125f);
}

// ELEM 1: uint8 rows handled as d 32-bit words, signed bytes x - 128 in LDS, integer Gram tiles
// (v_mfma_i32_16x16x64_i8) -- see knng_join_wave.h; here wavefront w also owns the products of
// the pivot with the member tiles w, w + 4, ... (one accumulator, a column per tile).
// Wavefronts per SIMD the register allocation aims at.  128 member slots: three (left to itself
// the compiler parks the accumulators in 32 AGPRs on top of 152 VGPRs, which allows two; told to
// fit three it needs 149 registers and no spill, and the join runs 28 % faster).  256 member
// slots: one workgroup per CU by LDS (the distance block alone is 132 KB).
#ifndef KNNG_JOIN4_OCC
#define KNNG_JOIN4_OCC 3
#endif
#ifndef KNNG_JOIN3_OCC
#define KNNG_JOIN3_OCC 4
#endif
template <int S16, int ELEM> struct JoinOcc {
    static constexpr int V = S16 == 4 ? KNNG_JOIN4_OCC : S16 == 3 ? (ELEM == 1 ? 3 : KNNG_JOIN3_OCC) : 1;
};
// SPLIT (fp32 rows): the centred values are stored as two bf16 halves and the Gram pass runs on
// v_mfma_f32_16x16x16_bf16 (hi.hi + hi.lo + lo.hi), as in the wavefront kernel: with samples above
// 16 the fp32 matrix instruction is busy for a third of the join, the bf16 one for a fifteenth.
template <int METRIC, int S16, int DS_, bool VEC, int ELEM = 0, bool SPLIT = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(JoinOcc<S16, ELEM>::V, JoinOcc<S16, ELEM>::V)))
k_join(const float* __restrict__ pts, int d, int C, int s, uint32_t iter,
       const int32_t* __restrict__ newl, const int32_t* __restrict__ oldl, const int4* __restrict__ plan,
       const int32_t* __restrict__ active, const u64* __restrict__ nactive_ptr,
       const float* __restrict__ worst, const uint32_t* __restrict__ sig, u64* __restrict__ cand,
       u64* __restrict__ offers_ctr, int32_t* __restrict__ redo, u64* __restrict__ redo_ctr)
{
    static_assert(ELEM == 0 || METRIC == 0, "uint8 and fp16 rows: squared L2 only");
    static_assert(ELEM == 0 || !SPLIT, "the bf16 split is for fp32 rows");
    using Cfg = JoinCfg<S16, DS_, ELEM>;
    using accv = typename std::conditional<ELEM == 1, intx4, floatx4>::type;
    uint32_t n_offers = 0;                                     // this thread's, summed per wavefront at exit
    constexpr int DS = Cfg::DS, LD = Cfg::LD, LDD = Cfg::LDD, NT = Cfg::NT, NL = Cfg::NL, NCOLS = Cfg::NCOLS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* X = reinterpret_cast<float*>(smem);                 // [NCOLS][LD], later D [MROWS][LDD]
    int* midbuf = reinterpret_cast<int*>(smem + Cfg::XBYTES);  // [2][NCOLS] member ids, double-buffered
    int2* mh = reinterpret_cast<int2*>(midbuf + 2 * NCOLS);    // [NCOLS] {member id, its signature bit}
    // [NCOLS] bits of |x_m - x_v|^2 (fp32); ELEM 1: of |x_m - 128|^2 (integer)
    uint32_t* nrm = reinterpret_cast<uint32_t*>(mh + NCOLS);
    float* thr = reinterpret_cast<float*>(nrm + NCOLS);        // [NCOLS] farthest-neighbour distance
    // row signatures, word-major [SIG_WORDS][NCOLS + 1] (column NCOLS: the pivot's): the lanes of a
    // wavefront that read one word of different members' signatures hit different banks
    uint32_t* sg = reinterpret_cast<uint32_t*>(thr + NCOLS);
    constexpr int SGLD = NCOLS + 1;
    float* thr_v = reinterpret_cast<float*>(sg + (NCOLS + 1) * SIG_WORDS);  // [0] the pivot's threshold, [1] ELEM 1: its norm
    // SPLIT: [2] "a chosen distance of this point is not trusted" (see split_untrusted), one flag per
    // parity of the point, since a point's offers are sent while the next point is worked on
    int* untrusted = reinterpret_cast<int*>(thr_v + 2);
    float* PZ = thr_v + 4;                                     // ELEM 1: [2][LD] pivot row, zeros
    float* dpv = PZ + 2 * LD;                                  // ELEM 1: [NCOLS] |x_m - x_v|^2
    if (ELEM == 1 && threadIdx.x < LD) PZ[LD + threadIdx.x] = 0.0f;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront index, kept scalar
    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t nact = (int64_t)*nactive_ptr;
    const int64_t G = gridDim.x;
    int64_t pos = blockIdx.x;
    if (pos >= nact) return;

    // list record of a point: its plan (all threads) and the list slot this thread owns
    auto load_slot = [&](int64_t v) -> int {
        if (tid < 2 * s) return newl[v * 2 * (int64_t)s + tid];
        if (tid < 4 * s) return oldl[v * 2 * (int64_t)s + (tid - 2 * s)];
        return 0;
    };

    // ---- prologue: first point's ids into LDS, its first slab and member data into registers
    int64_t v = active[pos];
    int64_t v_nx = pos + G < nact ? (int64_t)active[pos + G] : -1;       // next point
    int64_t v_nx2 = pos + 2 * G < nact ? (int64_t)active[pos + 2 * G] : -1;
    int4 rc = plan[v];
    int rid = load_slot(v);
    int cur = 0;
    {
        const int m = member_of_slot(tid, s, rc);
        if (m >= 0) midbuf[m] = rid;
    }
    PointPlan P = make_point(rc);
    lds_barrier();

    float4 buf[NL];
    float4 pv;
    float thr_r = 0.0f;
    uint4 sg_r0 = uint4{0, 0, 0, 0}, sg_r1 = uint4{0, 0, 0, 0};
    int my_member = 0;
    // thread tid < nTot holds member tid; thread tid == nTot holds the pivot itself (when all
    // 256 slots are members there is no thread left and the pivot takes no offers of its own)
    auto issue_members = [&](const int* mid, int nTot, int64_t pivot_row) {
        if (tid <= nTot) {
            my_member = tid < nTot ? mid[tid] : (int)pivot_row;
            thr_r = worst[my_member];
            const uint4* sp = reinterpret_cast<const uint4*>(sig + (int64_t)my_member * SIG_WORDS);
            sg_r0 = sp[0];
            sg_r1 = sp[1];
        }
    };
    // All member ids are read from LDS before the first load is issued (one LDS round trip per
    // slab); a group of RP rows is loaded whole (rows past the last member repeat it) or not at
    // all; VEC pieces past the end of the row come from its last piece and are zeroed at the store.
    auto issue_slab = [&](const int* mid, int nTot, int64_t pivot_row, int k0) {
        const SlabMap sm = slab_map(d, k0, DS, tid);
        int t = k0 + 4 * sm.c4;
        if (VEC) t = t < d ? t : d - 4;
        if (nTot > 0) {                                         // uniform
            int rowid[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int row = sm.rsub + i * sm.RP;
                rowid[i] = mid[row < nTot ? row : nTot - 1];
            }
            pv = load_piece_inside<VEC>(pts + pivot_row * d, t, d);
#pragma unroll
            for (int i = 0; i < NL; ++i)
                if (i * sm.RP < nTot)                           // uniform
                    buf[i] = load_piece_inside<VEC>(pts + (int64_t)rowid[i] * d, t, d);
        }
    };

    issue_slab(midbuf, P.nTot, v, 0);
    issue_members(midbuf, P.nTot, v);
    int4 rc_n = int4{0, 0, 0, 0};
    int rid_n = 0;
    if (v_nx >= 0) { rc_n = plan[v_nx]; rid_n = load_slot(v_nx); }

    // Offers of the previous point, sent one point late: right after the last Gram pass, so that
    // their round trip to memory runs under the norm / distance-block / scan work, which never
    // waits for memory.  (Sent right after the scan they would be waited for at the very next use
    // of prefetched data: loads and atomics share one in-order counter.)  One offer per thread and
    // scan pass: member id, partner id (-1: none), distance bits.
    constexpr int NPASS = (NCOLS * OFFERS_PER_MEMBER + 255) / 256;
    int pend_mid[NPASS], pend_pid[NPASS];
    uint32_t pend_l[NPASS];
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) { pend_mid[ps] = 0; pend_pid[ps] = -1; pend_l[ps] = 0u; }
    int v_pend = -1;                                           // the point the pending offers belong to
    // `flag`: the pending point's entry of `untrusted` (its scan lies at least one barrier back)
    auto send_offers = [&](const int* flag) {
        if constexpr (SPLIT) {
            if (v_pend >= 0 && *flag != 0) {
                // left to the fp32 kernel, which runs over the points listed here after this launch
#pragma unroll
                for (int ps = 0; ps < NPASS; ++ps) pend_pid[ps] = -1;
                if (tid == 0) redo[atomicAdd(redo_ctr, 1ull)] = (int32_t)v_pend;
            }
        }
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            if (pend_pid[ps] >= 0) {
                const uint32_t slot = below(hash32((uint32_t)pend_pid[ps]), (uint32_t)C);
                ++n_offers;
                atomicMin(&cand[(int64_t)pend_mid[ps] * C + slot], pack_key(__uint_as_float(pend_l[ps]), pend_pid[ps], 1));
                pend_pid[ps] = -1;
            }
        }
    };

    for (;;) {
        const int* mid = midbuf + cur * NCOLS;
        const int nNew = P.nNew, nTot = P.nTot, nfn = P.nfn, nfo = P.nfo;
        // Output tiles (16x16): rows = NEW members, columns = NEW|OLD members.  Tiles strictly
        // below the diagonal of the NEW x NEW part are skipped (the block is symmetric there).
        // The diagonal tiles of the remaining column tiles are added: the diagonal of the Gram
        // block is |x_m - x_v|^2, so the matrix cores also deliver every member's norm.
        // The tiles are dealt round-robin to the four wavefronts.
        const int nrt = (nNew + 15) >> 4, nct = (nTot + 15) >> 4;
        const int ntm = nrt * nct - nrt * (nrt - 1) / 2;
        const int ntiles = ntm + (nct - nrt);
        accv acc[NT];
        intx4 accp = intx4{0, 0, 0, 0};                     // ELEM 1: <member, pivot> of this wavefront's tiles
        int trow[NT], tcol[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            acc[q] = accv{0, 0, 0, 0};
            int rem = w + 4 * q, rt = 0;
            if (rem < ntm) {
                while (rem >= nct - rt) { rem -= nct - rt; ++rt; }
                trow[q] = rt; tcol[q] = rt + rem;
            } else if (rem < ntiles) {
                trow[q] = tcol[q] = nrt + (rem - ntm);
            } else { trow[q] = -1; tcol[q] = 0; }
        }
        PointPlan Pn = make_point(rc_n);
        // uint8 -> signed bytes x - 128; words past the end of the row stay zero
        auto enc_u8 = [&](float4 f, int t0) -> float4 {
            uint32_t wd[4] = {__float_as_uint(f.x), __float_as_uint(f.y), __float_as_uint(f.z), __float_as_uint(f.w)};
#pragma unroll
            for (int j = 0; j < 4; ++j) wd[j] = (VEC || t0 + j < d) ? (wd[j] ^ 0x80808080u) : 0u;
            return float4{__uint_as_float(wd[0]), __uint_as_float(wd[1]), __uint_as_float(wd[2]), __uint_as_float(wd[3])};
        };

        for (int k0 = 0; k0 < d; k0 += DS) {
            const bool first = k0 == 0, last = k0 + DS >= d;
            const SlabMap sm = slab_map(d, k0, DS, tid);
            // ---- A: registers -> LDS
            if (first) {
                // all 256 threads hold members: no thread is left for the pivot (with 128 member
                // slots thread 128 holds it, and must be the only writer of its threshold)
                if (NCOLS == 256 && tid == NCOLS - 1 && nTot == NCOLS) thr_v[0] = 0.0f;
                if (SPLIT && tid == 0) untrusted[cur] = 0;
                if (tid == nTot) {
                    thr_v[0] = thr_r;
                    sg[0 * SGLD + NCOLS] = sg_r0.x; sg[1 * SGLD + NCOLS] = sg_r0.y;
                    sg[2 * SGLD + NCOLS] = sg_r0.z; sg[3 * SGLD + NCOLS] = sg_r0.w;
                    sg[4 * SGLD + NCOLS] = sg_r1.x; sg[5 * SGLD + NCOLS] = sg_r1.y;
                    sg[6 * SGLD + NCOLS] = sg_r1.z; sg[7 * SGLD + NCOLS] = sg_r1.w;
                }
                if (tid < nTot) {
                    thr[tid] = thr_r;
                    mh[tid] = int2{my_member, (int)sig_bit(my_member, iter)};
                    sg[0 * SGLD + tid] = sg_r0.x; sg[1 * SGLD + tid] = sg_r0.y;
                    sg[2 * SGLD + tid] = sg_r0.z; sg[3 * SGLD + tid] = sg_r0.w;
                    sg[4 * SGLD + tid] = sg_r1.x; sg[5 * SGLD + tid] = sg_r1.y;
                    sg[6 * SGLD + tid] = sg_r1.z; sg[7 * SGLD + tid] = sg_r1.w;
                }
            }
            if (sm.col_ok) {
                float* xdst = X + sm.rsub * LD + 4 * sm.c4;
                // VEC: a piece past the end of the row (loaded from the row's last piece) is zeroed;
                // only the last slab of a row whose length is no multiple of the slab has such pieces
                const bool ragged = VEC && k0 + DS > d;             // uniform
                const bool full = sm.len16 == DS;                   // uniform
                const bool inb = !VEC || k0 + 4 * sm.c4 < d;
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    if (i * sm.RP < nTot) {                     // uniform: the group was loaded
                        float4 x = buf[i];
                        if (ELEM == 1) x = enc_u8(x, k0 + 4 * sm.c4);
                        else if (ELEM == 2) x = sub_h2x4(x, pv);
                        else { x.x -= pv.x; x.y -= pv.y; x.z -= pv.z; x.w -= pv.w; }
                        if (ragged && !inb) x = float4{0.0f, 0.0f, 0.0f, 0.0f};
                        if constexpr (SPLIT) {
                            // the piece keeps its place: two words of hi halves, then two of lo halves
                            short4v hi, lo;
                            split_bf16(x, hi, lo);
                            const uint2 h2 = __builtin_bit_cast(uint2, hi), l2 = __builtin_bit_cast(uint2, lo);
                            x = float4{__uint_as_float(h2.x), __uint_as_float(h2.y), __uint_as_float(l2.x), __uint_as_float(l2.y)};
                        }
                        // A full-width slab has NCOLS / RP groups of RP rows exactly: the rows of a loaded
                        // group past the last member (they repeat it) are stored as they are, nobody
                        // reads them.  A narrower last slab has more rows per group than NCOLS divides
                        // into, so there the store is per row.
                        if (full || sm.rsub + i * sm.RP < nTot) *reinterpret_cast<float4*>(xdst + i * sm.RP * LD) = x;
                    }
                }
                if (ELEM == 1 && sm.rsub == 0) {                // the pivot's own row
                    float4 x = enc_u8(pv, k0 + 4 * sm.c4);
                    if (!inb) x = float4{0.0f, 0.0f, 0.0f, 0.0f};
                    *reinterpret_cast<float4*>(PZ + 4 * sm.c4) = x;
                }
            }
            if (last && v_nx >= 0) {                       // next point's member ids
                const int m = member_of_slot(tid, s, rc_n);
                if (m >= 0) midbuf[(cur ^ 1) * NCOLS + m] = rid_n;
            }
            lds_barrier();
            // ---- B: issue the loads of the next unit
            // (one call site, so the prefetch registers are the same on every path)
            {
                const bool to_next = last;
                const int* nmid = to_next ? midbuf + (cur ^ 1) * NCOLS : mid;
                const int n_tot = to_next ? (v_nx >= 0 ? Pn.nTot : 0) : nTot;
                const int64_t n_piv = to_next ? (v_nx >= 0 ? v_nx : v) : v;
                issue_slab(nmid, n_tot, n_piv, to_next ? 0 : k0 + DS);
            }
            // ---- C: Gram tiles of this slab
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                if (trow[q] >= 0) {
                    const float* xa = X + (trow[q] * 16 + r16) * LD + 4 * kq;
                    const float* xb = X + (tcol[q] * 16 + r16) * LD + 4 * kq;
                    // one k-step (16 words of the slab) of tile q from operands read as 16-byte pieces
                    auto mm = [&](uint4 a, uint4 b) {
                        if constexpr (ELEM == 1) {
                            acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(intx4, a), __builtin_bit_cast(intx4, b), acc[q], 0, 0, 0);
                        } else if constexpr (ELEM == 2) {
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), acc[q], 0, 0, 0);
                        } else if constexpr (SPLIT) {
                            const short4v ah = __builtin_bit_cast(short4v, uint2{a.x, a.y}), al = __builtin_bit_cast(short4v, uint2{a.z, a.w});
                            const short4v bh = __builtin_bit_cast(short4v, uint2{b.x, b.y}), bl = __builtin_bit_cast(short4v, uint2{b.z, b.w});
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bh, acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bl, acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(al, bh, acc[q], 0, 0, 0);
                        } else {
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc[q], 0, 0, 0);
                        }
                    };
                    // two k-steps per round: four operand reads in flight before the first matrix
                    // instruction waits for them (one step per round leaves every LDS round trip bare)
                    // (fp32 rows only: the uint8 and fp16 instantiations have no registers to spare)
                    int kk = 0;
                    for (; ELEM == 0 && kk + 32 <= sm.len16; kk += 32) {
                        const uint4 a0 = *reinterpret_cast<const uint4*>(xa + kk), b0 = *reinterpret_cast<const uint4*>(xb + kk);
                        const uint4 a1 = *reinterpret_cast<const uint4*>(xa + kk + 16), b1 = *reinterpret_cast<const uint4*>(xb + kk + 16);
                        mm(a0, b0);
                        mm(a1, b1);
                    }
                    for (; kk < sm.len16; kk += 16) mm(*reinterpret_cast<const uint4*>(xa + kk), *reinterpret_cast<const uint4*>(xb + kk));
                }
            }
            if constexpr (ELEM == 1) {
                // column c of accp: member tile w + 4c against the pivot; wavefront 0, column 4:
                // the pivot against itself
#pragma unroll
                for (int c = 0; c < 5; ++c) {
                    const int ct = w + 4 * c;
                    if (c < 4 ? ct < nct : w == 0) {            // uniform
                        const float* xa = c < 4 ? X + (ct * 16 + r16) * LD + 4 * kq : PZ + 4 * kq;
                        const float* xb = PZ + (r16 == c ? 0 : LD) + 4 * kq;
                        for (int kk = 0; kk < sm.len16; kk += 16)
                            accp = __builtin_amdgcn_mfma_i32_16x16x64_i8(*reinterpret_cast<const intx4*>(xa + kk),
                                                                         *reinterpret_cast<const intx4*>(xb + kk), accp, 0, 0, 0);
                    }
                }
            }
            if (last) {
                // member norms from the diagonal tiles: lane (r16, kq) holds rows 4kq..4kq+3 of
                // column r16, so the diagonal element sits in lanes with r16 / 4 == kq
                // (one store per accumulator register, the lane that holds the diagonal element in it
                // taking part: a select over a register picked by the lane costs the compiler a
                // chain over every accumulator of the wavefront)
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    if (trow[q] >= 0 && trow[q] == tcol[q]) {   // uniform
                        uint32_t* dst = nrm + trow[q] * 16 + r16;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (r16 == 4 * kq + e) *dst = acc_bits(acc[q][e]);
                    }
                }
                if (ELEM == 1 && w == 0 && lane == 4) thr_v[1] = __uint_as_float((uint32_t)accp[0]);
            }
            lds_barrier();                                 // slab consumed by every wavefront
        }

        // After the last Gram pass: the next point's thresholds and signatures and the list record of
        // the point after next (requested earlier they would hold ten registers through the Gram
        // passes), then the previous point's offers.  All of it completes under the norm /
        // distance-block / scan work below, which never waits for memory.
        if (v_nx >= 0) {
            issue_members(midbuf + (cur ^ 1) * NCOLS, Pn.nTot, v_nx);
            if (v_nx2 >= 0) { rc_n = plan[v_nx2]; rid_n = load_slot(v_nx2); }
        }
        send_offers(untrusted + (cur ^ 1));                // the previous point's
        // The pivot's reverse members hold v in their rows, so |x_m - x_v|^2 is already known:
        // offer them to v itself (closes v<-m edges into v->m without an extra distance).
        auto reverse_offers = [&]() {
          if (tid < nTot) {
            const int m = tid;
            const bool rev = (m >= nfn && m < nNew) || (m >= nNew + nfo);
            if (rev) {
                float l = ELEM == 1 ? dpv[m] : __uint_as_float(nrm[m]);
                if (METRIC == 1) l *= 0.5f;
                l = nonneg(l);
                const int2 me = mh[m];
                const uint32_t h = (uint32_t)me.y;
                const uint32_t vw = sg[(h >> 5) * SGLD + NCOLS];
                if (l < thr_v[0] && !((vw >> (h & 31u)) & 1u)) {
                    const uint32_t slot = below(hash32((uint32_t)me.x), (uint32_t)C);
                    ++n_offers;
                    atomicMin(&cand[v * C + slot], pack_key(l, me.x, 1));
                }
            }
        }
        };
        if (ELEM == 0) reverse_offers();
        // distance block D[row][col] over the slab storage
        float* D = X;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            if (trow[q] >= 0 && trow[q] < nrt) {           // norm-only diagonal tiles have no D rows
                const int col = tcol[q] * 16 + r16;
                const uint32_t nc = nrm[col];
                const uint4 nr = *reinterpret_cast<const uint4*>(nrm + trow[q] * 16 + 4 * kq);
                const uint32_t nra[4] = {nr.x, nr.y, nr.z, nr.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = trow[q] * 16 + 4 * kq + r;
                    float l;
                    if constexpr (ELEM == 1) {
                        l = (float)(nra[r] + nc - 2u * (uint32_t)acc[q][r]);   // exact, >= 0
                    } else {
                        l = __uint_as_float(nra[r]) + __uint_as_float(nc) - 2.0f * acc[q][r];
                        if (METRIC == 1) l *= 0.5f;        // unit rows: 1 - <a,b> = |a-b|^2 / 2
                        l = nonneg(l);
                    }
                    D[row * LDD + col] = l;
                }
            }
        }
        if constexpr (ELEM == 1) {
            // lane (c, kq), c < 4, holds <member 16 (w + 4c) + 4kq + r, pivot> in accp[r]
            const int ct = w + 4 * r16;
            if (r16 < 4 && ct < nct) {
                const uint32_t npiv = __float_as_uint(thr_v[1]);
                const uint4 nm = *reinterpret_cast<const uint4*>(nrm + ct * 16 + 4 * kq);
                float4 o;
                o.x = (float)(nm.x + npiv - 2u * (uint32_t)accp[0]);
                o.y = (float)(nm.y + npiv - 2u * (uint32_t)accp[1]);
                o.z = (float)(nm.z + npiv - 2u * (uint32_t)accp[2]);
                o.w = (float)(nm.w + npiv - 2u * (uint32_t)accp[3]);
                *reinterpret_cast<float4*>(dpv + ct * 16 + 4 * kq) = o;
            }
        }
        lds_barrier();
        if (ELEM == 1) reverse_offers();
        // per-member candidates: LPM lanes per member, each lane scans the partners of one
        // residue class (partner index mod LPM) and offers the closest of its class that beats
        // the member's threshold and is not in the member's signature (branch-free scan)
        constexpr int LPM = OFFERS_PER_MEMBER;
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int m = ps * (256 / LPM) + tid / LPM, sub = tid % LPM;
            if (m >= nTot) continue;
            const int myid = mh[m].x;
            const uint32_t mythr = __float_as_uint(thr[m]);    // non-negative floats order as integers
            uint32_t best_l = mythr, best_j = 0xffffffffu;
            const bool isnew = m < nNew;
            const int jend = isnew ? nTot : nNew;
            // Four partners of the lane's class per step: their distances and records are read
            // together, then their signature words -- two LDS round trips per step instead of
            // three per partner.  D[m][j] sits at [lower tile][higher tile]; with four classes the
            // four partners of a step lie in one 16-wide tile, so a step walks either the member's
            // row (address + 4) or the partners' column (address + 4 LDD).  Index arithmetic in 24
            // bits: one full-rate instruction per address.
            const uint32_t um = (uint32_t)m, mrow = __umul24(um, (uint32_t)LDD);
            for (int j0 = sub; j0 < jend; j0 += 4 * LPM) {
                uint32_t l[4];
                int2 pj[4];
                if constexpr (LPM == 4) {
                    const bool colwalk = !isnew || ((uint32_t)j0 >> 4) < (um >> 4);
                    const uint32_t a0 = colwalk ? __umul24((uint32_t)j0, (uint32_t)LDD) + um : mrow + (uint32_t)j0;
                    const uint32_t st = colwalk ? 4u * LDD : 4u;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + 4 * u;
                        const bool in = j < jend;
                        const uint32_t v = __float_as_uint(D[in ? a0 + (uint32_t)u * st : a0]);
                        l[u] = in ? v : 0xffffffffu;
                        pj[u] = mh[in ? j : j0];
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u * LPM;
                        const bool in = j < jend;
                        const int jj = in ? j : sub;           // any valid partner: its cell is not used
                        const bool tr = isnew && ((jj >> 4) < (m >> 4));
                        const uint32_t v = __float_as_uint(tr ? D[jj * LDD + m] : D[(isnew ? m : jj) * LDD + (isnew ? jj : m)]);
                        l[u] = in ? v : 0xffffffffu;
                        pj[u] = mh[jj];
                    }
                }
                uint32_t wv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wv[u] = sg[__umul24((uint32_t)pj[u].y >> 5, (uint32_t)SGLD) + um];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t known = (wv[u] >> ((uint32_t)pj[u].y & 31u)) & 1u;
                    const bool ok = (l[u] < best_l) & (pj[u].x != myid) & (known == 0u);
                    best_l = ok ? l[u] : best_l;
                    best_j = ok ? (uint32_t)(j0 + u * LPM) : best_j;
                }
            }
            if (best_j != 0xffffffffu) {
                pend_mid[ps] = myid;
                pend_pid[ps] = mh[best_j].x;
                pend_l[ps] = best_l;
                if constexpr (SPLIT) {
                    if (split_untrusted(best_l, __uint_as_float(nrm[m]), __uint_as_float(nrm[best_j]), METRIC == 1 ? 0.5f : 1.0f))
                        untrusted[cur] = 1;
                }
            }
        }
        v_pend = (int)v;
        // ---- advance to the next point of this workgroup
        if (v_nx < 0) break;
        lds_barrier();                                     // D and the member arrays are free again
        pos += G;
        v = v_nx;
        v_nx = v_nx2;
        v_nx2 = pos + 2 * G < nact ? (int64_t)active[pos + 2 * G] : -1;
        P = Pn;
        cur ^= 1;
    }
    lds_barrier();                                         // the last point's flag is complete
    send_offers(untrusted + cur);                          // the last point's
    for (int o = 32; o > 0; o >>= 1) n_offers += __shfl_xor(n_offers, o);
    if ((tid & 63) == 0 && n_offers) atomicAdd(offers_ctr, (u64)n_offers);
}

// ------------------------------------------------------------------------------------------
// k_finalize: lane i of a group of Kp = pow2 >= K lanes owns neighbour i of one point, 64/Kp
// points per wavefront.  The lane evaluates its neighbour's distance in index order with the
// fp64 recipe, so the value written equals a sequential fp64 evaluation bit for bit.  Rows are
// then ranked by (distance, id) and the first k written as ids / distances.
//
// How a neighbour's vector reaches its lane: not by the lane streaming its own row.  Then one
// load instruction touches 64 rows, and on a point set beyond about 2 GB the address
// translations, not the bytes, bound the kernel (1M x 960 fp32: 2 TB/s; a micro-benchmark of
// the pattern falls from 5 to 1.3 TB/s between 2 and 16 GB, while eight lanes per row keep
// 6.2 TB/s).  Instead eight lanes read 128 consecutive bytes of one row (eight rows per
// instruction, like the gathers of k_init and the join), the 64 x 128-byte step goes through
// the wavefront's own LDS region (padded rows: conflict-free 16-byte accesses), and every lane
// picks up its own row's 32 words.  The loads of the next step are in flight while the chain
// runs.  No workgroup barriers: a wavefront only touches its own region, in program order.
// Needs rows of whole, aligned 16-byte pieces; other shapes take k_finalize_scalar.
//
// ELEM 0: fp32 rows.  ELEM 2: fp16 rows, the fp64 recipe on the converted values.  ELEM 1: uint8
// rows, the sum of squared differences is an integer below 2^32, evaluated exactly and rounded
// once to fp32 -- what the fp64 recipe gives on these values.  dw = 32-bit words per row.
// ------------------------------------------------------------------------------------------
constexpr int FIN_CH = 32;                            // words per row and step
constexpr int FIN_LD = FIN_CH + 4;                    // LDS row stride (words)
template <int METRIC, int ELEM>
__global__ void __launch_bounds__(256)
k_finalize(const float* __restrict__ pts, int64_t n, int dw, int K, int Kp, int k,
           const u64* __restrict__ G, int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    static_assert(ELEM == 0 || METRIC == 0, "uint8 and fp16 rows: squared L2 only");
    __shared__ __attribute__((aligned(16))) float stage[4][WAVE * FIN_LD];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int sub = lane / Kp, i = lane & (Kp - 1);
    const int64_t v = ((int64_t)blockIdx.x * 4 + w) * (WAVE / Kp) + sub;
    const bool live = v < n && i < K;
    const int64_t vv = v < n ? v : n - 1;
    const u64 key = live ? G[vv * K + i] : EMPTY_KEY;
    const int id = live ? key_id(key) : (int)vv;
    float* st = stage[w];
    const int g = lane >> 3, c = lane & 7;            // load role: row 8q + g, piece c of the step
    // eight row pointers and eight pieces in flight, as named variables (one per load of a step)
#define KNNG_REP8(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)
#define KNNG_FIN_DECL(q) const float* rp##q = pts + (int64_t)__shfl(id, 8 * q + g) * dw + 4 * c; float4 b##q;
#define KNNG_FIN_LOAD(q) b##q = *reinterpret_cast<const float4*>(rp##q + off);
#define KNNG_FIN_STORE(q) *reinterpret_cast<float4*>(st + (8 * q + g) * FIN_LD + 4 * c) = b##q;
    KNNG_REP8(KNNG_FIN_DECL)
    const float* __restrict__ a = pts + vv * dw;
    // pieces past the end of a row are loaded from its last piece (never used: the chain stops at dw)
    {
        const int off = 4 * c < dw ? 0 : dw - 4 - 4 * c;
        KNNG_REP8(KNNG_FIN_LOAD)
    }
    double acc = 0.0;
    double acc_a = 0.0, acc_b = 0.0;                  // METRIC 2: |a|^2 and |b|^2, chains of the same kind
    uint32_t acc_u = 0u;
    for (int t = 0; t < dw; t += FIN_CH) {
        KNNG_REP8(KNNG_FIN_STORE)
        wave_lds_sync();
        if (t + FIN_CH < dw) {                        // uniform
            const int tn = t + FIN_CH;
            const int off = tn + 4 * c < dw ? tn : dw - 4 - 4 * c;
            KNNG_REP8(KNNG_FIN_LOAD)
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {                 // two halves of 16 words
            if (t + 16 * h < dw) {                    // uniform
                float4 av[4], bv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int tt = t + 16 * h + 4 * j;
                    bv[j] = *reinterpret_cast<const float4*>(st + lane * FIN_LD + 16 * h + 4 * j);
                    av[j] = *reinterpret_cast<const float4*>(a + (tt < dw ? tt : 0));
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (t + 16 * h + 4 * j < dw) {    // uniform
                        if constexpr (ELEM == 1) {
                            acc_u += sqdiff16_u8(uint4{__float_as_uint(av[j].x), __float_as_uint(av[j].y), __float_as_uint(av[j].z), __float_as_uint(av[j].w)},
                                                 uint4{__float_as_uint(bv[j].x), __float_as_uint(bv[j].y), __float_as_uint(bv[j].z), __float_as_uint(bv[j].w)});
                        } else if constexpr (ELEM == 2) {
                            const uint32_t x[4] = {__float_as_uint(av[j].x), __float_as_uint(av[j].y), __float_as_uint(av[j].z), __float_as_uint(av[j].w)};
                            const uint32_t y[4] = {__float_as_uint(bv[j].x), __float_as_uint(bv[j].y), __float_as_uint(bv[j].z), __float_as_uint(bv[j].w)};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                acc = exact_step<0>(acc, h_lo(x[e]), h_lo(y[e]));
                                acc = exact_step<0>(acc, h_hi(x[e]), h_hi(y[e]));
                            }
                        } else {
                            acc = exact_step<METRIC>(acc, av[j].x, bv[j].x);
                            acc = exact_step<METRIC>(acc, av[j].y, bv[j].y);
                            acc = exact_step<METRIC>(acc, av[j].z, bv[j].z);
                            acc = exact_step<METRIC>(acc, av[j].w, bv[j].w);
                            if constexpr (METRIC == 2) {
                                acc_a = exact_step<2>(acc_a, av[j].x, av[j].x); acc_b = exact_step<2>(acc_b, bv[j].x, bv[j].x);
                                acc_a = exact_step<2>(acc_a, av[j].y, av[j].y); acc_b = exact_step<2>(acc_b, bv[j].y, bv[j].y);
                                acc_a = exact_step<2>(acc_a, av[j].z, av[j].z); acc_b = exact_step<2>(acc_b, bv[j].z, bv[j].z);
                                acc_a = exact_step<2>(acc_a, av[j].w, av[j].w); acc_b = exact_step<2>(acc_b, bv[j].w, bv[j].w);
                            }
                        }
                    }
                }
            }
        }
        wave_lds_sync();
    }
#undef KNNG_FIN_STORE
#undef KNNG_FIN_LOAD
#undef KNNG_FIN_DECL
#undef KNNG_REP8
    const float dist = ELEM == 1 ? (float)acc_u : METRIC == 2 ? cosine_finish(acc, acc_a, acc_b) : exact_finish<METRIC>(acc);
    const u64 fk = live ? pack_key(dist, id, 0) : EMPTY_KEY;
    int rank = 0;
    for (int j = 0; j < K; ++j) rank += ((u64)__shfl((unsigned long long)fk, sub * Kp + j) < fk) ? 1 : 0;
    if (live && rank < k) {
        ids_out[v * k + rank] = id;
        dists_out[v * k + rank] = dist;
    }
}

// ------------------------------------------------------------------------------------------
// k_finalize_scalar: the same for rows that are not made of aligned 16-byte pieces (fp32: any d;
// uint8: d % 4 == 0; fp16: d % 2 == 0, rows 4-byte aligned).  Every lane walks its neighbour's
// row and the point's own straight from global memory, one word at a time.  d = coordinates.
// ------------------------------------------------------------------------------------------
template <int METRIC, int ELEM>
__global__ void __launch_bounds__(256)
k_finalize_scalar(const float* __restrict__ pts, int64_t n, int d, int K, int Kp, int k,
                  const u64* __restrict__ G, int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    static_assert(ELEM == 0 || METRIC == 0, "uint8 and fp16 rows: squared L2 only");
    const int lane = lane_id(), w = threadIdx.x >> 6;
    const int sub = lane / Kp, i = lane & (Kp - 1);
    const int64_t v = ((int64_t)blockIdx.x * 4 + w) * (WAVE / Kp) + sub;
    const bool live = v < n && i < K;
    const int64_t vv = v < n ? v : n - 1;
    const u64 key = live ? G[vv * K + i] : EMPTY_KEY;
    const int id = live ? key_id(key) : (int)vv;
    float dist;
    if constexpr (ELEM == 1) {
        const uint32_t* __restrict__ a = reinterpret_cast<const uint32_t*>(pts) + vv * (int64_t)(d >> 2);
        const uint32_t* __restrict__ b = reinterpret_cast<const uint32_t*>(pts) + (int64_t)id * (d >> 2);
        uint32_t acc = 0u;
        for (int t = 0; t < (d >> 2); ++t) acc += sqdiff4_u8(a[t], b[t]);
        dist = (float)acc;
    } else if constexpr (ELEM == 2) {
        const uint32_t* __restrict__ a = reinterpret_cast<const uint32_t*>(pts) + vv * (int64_t)(d >> 1);
        const uint32_t* __restrict__ b = reinterpret_cast<const uint32_t*>(pts) + (int64_t)id * (d >> 1);
        double acc = 0.0;
        for (int t = 0; t < (d >> 1); ++t) {
            acc = exact_step<0>(acc, h_lo(a[t]), h_lo(b[t]));
            acc = exact_step<0>(acc, h_hi(a[t]), h_hi(b[t]));
        }
        dist = exact_finish<0>(acc);
    } else {
        const float* __restrict__ a = pts + vv * d;
        const float* __restrict__ b = pts + (int64_t)id * d;
        double acc = 0.0, acc_a = 0.0, acc_b = 0.0;
        for (int t = 0; t < d; ++t) {
            acc = exact_step<METRIC>(acc, a[t], b[t]);
            if constexpr (METRIC == 2) { acc_a = exact_step<2>(acc_a, a[t], a[t]); acc_b = exact_step<2>(acc_b, b[t], b[t]); }
        }
        dist = METRIC == 2 ? cosine_finish(acc, acc_a, acc_b) : exact_finish<METRIC>(acc);
    }
    const u64 fk = live ? pack_key(dist, id, 0) : EMPTY_KEY;
    int rank = 0;
    for (int j = 0; j < K; ++j) rank += ((u64)__shfl((unsigned long long)fk, sub * Kp + j) < fk) ? 1 : 0;
    if (live && rank < k) {
        ids_out[v * k + rank] = id;
        dists_out[v * k + rank] = dist;
    }
}

// ------------------------------------------------------------------------------------------
// k_unit_rows (general cosine): out = x / |x| row by row, a zero row stays zero.  The joins of a
// cosine build work on these unit-length copies with 1 - <a,b> (search-time precision); what is
// written to the caller is k_finalize's exact cosine of the original rows.  Eight lanes per row.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_unit_rows(const float* __restrict__ pts, int64_t n, int d, float* __restrict__ out)
{
    const int sub = threadIdx.x & 7;
    const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 3;
    if (row >= n) return;                             // whole groups of 8 lanes leave together
    const float* x = pts + row * d;
    float acc = 0.0f;
    for (int t = sub; t < d; t += 8) acc = fmaf(x[t], x[t], acc);
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    const float inv = acc > 0.0f ? 1.0f / sqrtf(acc) : 0.0f;
    for (int t = sub; t < d; t += 8) out[row * d + t] = x[t] * inv;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct BuildPlan {
    int K, C, s, B, S16, max_iters;
    float rho, delta;
    uint64_t off_G, off_cand, off_new, off_old, off_rev, off_cnt, off_plan, off_active, off_redo, off_worst, off_sig, off_ctr, total;
};

static bool make_plan(int64_t n, int32_t d, int32_t k, const knng_params_t* p, BuildPlan* bp)
{
    if (n < 2 || n > 2147483647LL || d < 1 || k < 1) return false;
    int K = (p && p->k_build) ? p->k_build : k;
    float rho = (p && p->rho != 0.0f) ? p->rho : 0.5f;
    float delta = (p && p->delta != 0.0f) ? p->delta : 1e-4f;
    int max_iters = (p && p->max_iters) ? p->max_iters : 100;
    if (max_iters < 0) max_iters = 0;
    if (K < k || K > KNNG_MAX_K || (int64_t)K > n - 1) return false;
    if (!(rho > 0.0f) || rho > 1.0f) return false;
    int C = (p && p->cand_cap) ? p->cand_cap : (2 * K < KNNG_MAX_K ? 2 * K : KNNG_MAX_K);
    if (C < 1 || C > KNNG_MAX_K) return false;
    int s = (int)ceil((double)rho * (double)K);
    if (s < 1) s = 1;
    if (s > K) s = K;
    bp->K = K; bp->C = C; bp->s = s; bp->rho = rho; bp->delta = delta; bp->max_iters = max_iters;
    bp->B = (KNNG_REV_MULT * s + 3) & ~3; if (bp->B > 128) bp->B = 128;              // reverse buckets per point and kind (>= 2s, % 4 == 0)
    bp->S16 = (2 * s <= 16) ? 1 : (2 * s <= 32) ? 2 : (2 * s <= 48) ? 3 : (2 * s <= 64) ? 4 : 8;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = (off + bytes + 255) & ~255ull; return o; };
    bp->off_G = take((uint64_t)n * K * 8);
    bp->off_cand = take((uint64_t)n * C * 8);
    bp->off_new = take((uint64_t)n * 2 * s * 4);
    bp->off_old = take((uint64_t)n * 2 * s * 4);
    bp->off_rev = take((uint64_t)n * 4 * bp->B * 4);   // [parity][kind][point][bucket]
    bp->off_cnt = take((uint64_t)n * 8);
    bp->off_plan = take((uint64_t)n * 16);
    bp->off_active = take((uint64_t)n * 4);
    bp->off_redo = take((uint64_t)n * 4);              // points a split join kernel leaves to the fp32 kernel
    bp->off_worst = take((uint64_t)n * 4);
    bp->off_sig = take((uint64_t)n * SIG_WORDS * 4);
    bp->off_ctr = take(256);
    bp->total = off;
    return true;
}

}  // namespace knng
#include "knng_join_wave.h"
namespace knng {

struct JoinArgs {
    const float* pts; int d; int C; int s; uint32_t iter;
    const int32_t* newl; const int32_t* oldl; const int4* plan; const int32_t* active;
    const u64* nactive; const float* worst; const uint32_t* sig; u64* cand; u64* offers;
    int num_cu; int64_t n;
    int* blocks_per_cu;       // resident workgroups per CU of this build's join kernel; 0 = not yet asked
    int32_t* redo; u64* redo_ctr;   // split kernels: the points left to the fp32 kernel, and their number
};

template <int METRIC, int S16, int DS, bool VEC, int ELEM = 0, bool SPLIT = false>
static hipError_t launch_join_k(hipStream_t st, const JoinArgs& a)
{
    const int lds = JoinCfg<S16, DS, ELEM>::LDS_BYTES;
    auto kern = k_join<METRIC, S16, DS, VEC, ELEM, SPLIT>;
    // asked once per build, on the build's device (a build runs one join kernel): the attribute is
    // per device, and nothing is kept between calls
    if (*a.blocks_per_cu == 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        int occ = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, 256, lds);
        if (e != hipSuccess) return e;
        *a.blocks_per_cu = occ > 0 ? occ : 1;
    }
    int64_t grid = (int64_t)a.num_cu * *a.blocks_per_cu;
    if (grid > a.n) grid = a.n;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, a.pts, a.d, a.C, a.s, a.iter, a.newl,
                       a.oldl, a.plan, a.active, a.nactive, a.worst, a.sig, a.cand, a.offers, a.redo, a.redo_ctr);
    return hipGetLastError();
}

template <int METRIC, int S16, bool VEC, int ELEM = 0, bool SPLIT = false>
static hipError_t launch_join_w(hipStream_t st, const JoinArgs& a)
{
    const int lds = 4 * WaveCfg<S16, ELEM>::WBYTES;
    auto kern = k_join_wave<METRIC, S16, VEC, ELEM, SPLIT>;
    // asked once per build, on the build's device (a build runs one join kernel): the attribute is
    // per device, and nothing is kept between calls
    if (*a.blocks_per_cu == 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        int occ = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, 256, lds);
        if (e != hipSuccess) return e;
        *a.blocks_per_cu = occ > 0 ? occ : 1;
    }
    int64_t grid = (int64_t)a.num_cu * *a.blocks_per_cu;
    if (grid > (a.n + 3) / 4) grid = (a.n + 3) / 4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, a.pts, a.d, a.C, a.s, a.iter, a.newl,
                       a.oldl, a.plan, a.active, a.nactive, a.worst, a.sig, a.cand, a.offers, a.redo, a.redo_ctr);
    return hipGetLastError();
}

#ifndef KNNG_JOINK_SPLIT_MIN_D
#define KNNG_JOINK_SPLIT_MIN_D 64     // fp32 rows from this length on: bf16-split Gram pass in the workgroup join
#endif
#ifndef KNNG_SPLIT_MIN_D
#define KNNG_SPLIT_MIN_D 256      // fp32 rows from this length on: bf16-split Gram pass in the wavefront join
#endif

// uint8 (ELEM 1) or fp16 (ELEM 2) rows, squared L2; a.d counts 32-bit words
template <int ELEM>
static hipError_t launch_join_compact(hipStream_t st, bool vec, int S16, const JoinArgs& a)
{
    if (S16 == 1) return vec ? launch_join_w<0, 1, true, ELEM>(st, a) : launch_join_w<0, 1, false, ELEM>(st, a);
    if (S16 == 2) return vec ? launch_join_w<0, 2, true, ELEM>(st, a) : launch_join_w<0, 2, false, ELEM>(st, a);
    if (S16 == 3) return vec ? launch_join_k<0, 3, 64, true, ELEM>(st, a) : launch_join_k<0, 3, 64, false, ELEM>(st, a);
    if (S16 == 4) return vec ? launch_join_k<0, 4, 64, true, ELEM>(st, a) : launch_join_k<0, 4, 64, false, ELEM>(st, a);
    return vec ? launch_join_k<0, 8, 32, true, ELEM>(st, a) : launch_join_k<0, 8, 32, false, ELEM>(st, a);
}

// the fp32 kernel over the points a split kernel did not trust itself with (the launch reads their
// number on the device; usually none)
static JoinArgs redo_args(const JoinArgs& a)
{
    JoinArgs b = a;
    b.active = a.redo;
    b.nactive = a.redo_ctr;
    b.redo = nullptr;
    b.redo_ctr = nullptr;
    b.blocks_per_cu = a.blocks_per_cu + 1;
    return b;
}

template <int METRIC>
static hipError_t launch_join(hipStream_t st, bool vec, int S16, const JoinArgs& a)
{
    // s <= 16: one wavefront per point; larger samples: one workgroup per point
    // long fp32 rows: the Gram pass on the bf16 matrix instructions (two halves per value), then the
    // fp32 kernel for the points whose choices the narrow pass could not be trusted with
    const bool split = vec && a.d >= KNNG_SPLIT_MIN_D;
    // samples above 16 (the workgroup kernel): from KNNG_JOINK_SPLIT_MIN_D coordinates on
    const bool ksplit = vec && a.d >= KNNG_JOINK_SPLIT_MIN_D;
    hipError_t e;
    if (S16 == 1 && split) {
        if ((e = launch_join_w<METRIC, 1, true, 0, true>(st, a)) != hipSuccess) return e;
        return launch_join_w<METRIC, 1, true>(st, redo_args(a));
    }
    if (S16 == 2 && split) {
        if ((e = launch_join_w<METRIC, 2, true, 0, true>(st, a)) != hipSuccess) return e;
        return launch_join_w<METRIC, 2, true>(st, redo_args(a));
    }
    if (S16 == 1) return vec ? launch_join_w<METRIC, 1, true>(st, a) : launch_join_w<METRIC, 1, false>(st, a);
    if (S16 == 2) return vec ? launch_join_w<METRIC, 2, true>(st, a) : launch_join_w<METRIC, 2, false>(st, a);
#define KNNG_JOIN_CASE(S, DSV)                                                                   \
    do {                                                                                         \
        if (ksplit) {                                                                            \
            if ((e = launch_join_k<METRIC, S, DSV, true, 0, true>(st, a)) != hipSuccess) return e; \
            return launch_join_k<METRIC, S, DSV, true>(st, redo_args(a));                        \
        }                                                                                        \
        return vec ? launch_join_k<METRIC, S, DSV, true>(st, a) : launch_join_k<METRIC, S, DSV, false>(st, a); \
    } while (0)
    switch (S16) {
    case 3: KNNG_JOIN_CASE(3, 64);
    case 4: KNNG_JOIN_CASE(4, 64);
    default: KNNG_JOIN_CASE(8, 32);
    }
#undef KNNG_JOIN_CASE
}

}  // namespace knng

using namespace knng;

extern "C" __attribute__((visibility("default"))) uint64_t knng_build_cosine_extra_bytes(int64_t n, int32_t d)
{
    if (n < 2 || n > 2147483647LL || d < 1) return 0;
    return ((uint64_t)n * (uint64_t)d * 4u + 255u) & ~255ull;
}

extern "C" __attribute__((visibility("default"))) uint64_t knng_build_workspace_bytes(int64_t n, int32_t d, int32_t k, const knng_params_t* params)
{
    if (params && params->struct_size != sizeof(knng_params_t)) return 0;
    BuildPlan bp;
    if (!make_plan(n, d, k, params, &bp)) return 0;
    return bp.total;
}

#define HIPCHK(expr)                                                   \
    do {                                                               \
        hipError_t e_ = (expr);                                        \
        if (e_ != hipSuccess) { rc = set_hip_error(e_, #expr); goto done; } \
    } while (0)

// elem 0: fp32 rows; elem 1: uint8 rows (squared L2, d % 4 == 0, d <= 65536); elem 2: fp16 rows
// (squared L2, d % 2 == 0)
static int build_impl(const void* points_void, int elem, int64_t n, int32_t d, int32_t k, int32_t metric,
                      const knng_params_t* params, int32_t* ids_out_dev, float* dists_out_dev)
{
    const float* points_dev = static_cast<const float*>(points_void);   // kernels cast back for elem 1
    if (!points_dev || !ids_out_dev || !dists_out_dev || !params) return KNNG_EINVAL;
    if (params->struct_size != sizeof(knng_params_t)) return KNNG_EINVAL;
    if (metric != KNNG_METRIC_L2SQ && metric != KNNG_METRIC_IP_UNIT && metric != KNNG_METRIC_COSINE) return KNNG_EINVAL;
    if (metric == KNNG_METRIC_COSINE && elem != 0) return KNNG_EINVAL;
    BuildPlan bp;
    if (!make_plan(n, d, k, params, &bp)) return KNNG_EINVAL;
    // general cosine: the search runs on unit-length copies of the rows (behind the other arrays of
    // the workspace) with 1 - <a,b>; only the last step reads the caller's rows
    const bool cosine = metric == KNNG_METRIC_COSINE;
    const uint64_t ws_need = bp.total + (cosine ? knng_build_cosine_extra_bytes(n, d) : 0);
    const float* points_orig = static_cast<const float*>(points_void);
    if (cosine) metric = KNNG_METRIC_IP_UNIT;
    if (elem == 1) {
        if (metric != KNNG_METRIC_L2SQ || (d & 3) || d > 65536 ||
            (reinterpret_cast<uintptr_t>(points_void) & 3u))
            return KNNG_EINVAL;
    }
    if (elem == 2) {
        if (metric != KNNG_METRIC_L2SQ || (d & 1) || (reinterpret_cast<uintptr_t>(points_void) & 3u))
            return KNNG_EINVAL;
    }
    if (!params->workspace_dev || params->workspace_bytes < ws_need ||
        (reinterpret_cast<uintptr_t>(params->workspace_dev) & 255u))
        return KNNG_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(params->pinned_host) & 7u) return KNNG_EINVAL;

    hipStream_t st = reinterpret_cast<hipStream_t>(params->stream);
    unsigned char* ws = static_cast<unsigned char*>(params->workspace_dev);
    u64* G = reinterpret_cast<u64*>(ws + bp.off_G);
    u64* cand = reinterpret_cast<u64*>(ws + bp.off_cand);
    int32_t* newl = reinterpret_cast<int32_t*>(ws + bp.off_new);
    int32_t* oldl = reinterpret_cast<int32_t*>(ws + bp.off_old);
    int32_t* cnt = reinterpret_cast<int32_t*>(ws + bp.off_cnt);
    uint32_t* rev = reinterpret_cast<uint32_t*>(ws + bp.off_rev);
    int4* plan = reinterpret_cast<int4*>(ws + bp.off_plan);
    int32_t* active = reinterpret_cast<int32_t*>(ws + bp.off_active);
    int32_t* redo = reinterpret_cast<int32_t*>(ws + bp.off_redo);
    float* worst = reinterpret_cast<float*>(ws + bp.off_worst);
    uint32_t* sig = reinterpret_cast<uint32_t*>(ws + bp.off_sig);
    u64* ctr = reinterpret_cast<u64*>(ws + bp.off_ctr);      // [0] updates [1] rows gathered [2] active [3] pairs [4] offers [5] occupied slots [6] points left to the fp32 join [7] check_rows: violations
    knng_stats_t* stats = params->stats_host;
    const bool vec = (d % (elem == 1 ? 16 : elem == 2 ? 8 : 4) == 0) && ((reinterpret_cast<uintptr_t>(points_dev) & 15u) == 0);
    const unsigned row_blocks = (unsigned)((n + 3) / 4);
    unsigned upd_blocks = 0;                          // persistent k_update grid, set once num_cu is known
    const double stop_below = (double)bp.delta * (double)bp.K * (double)n;

    int rc = KNNG_OK;
    int num_cu = 0;
    int join_blocks_per_cu[2] = {0, 0};              // [1]: the fp32 kernel behind a split kernel
    u64* host_ctr = nullptr;
    bool own_ctr = false;
    // events: [0] start, [1] after init, then 4 per iteration (sample, join start, join end, merge), last = end
    const int max_rec = bp.max_iters < KNNG_STATS_MAX_ITERS ? bp.max_iters : KNNG_STATS_MAX_ITERS;
    const int n_ev = stats ? 8 + 4 * max_rec : 0;
    hipEvent_t* ev = nullptr;
    int iters = 0, converged = 0;
    u64 violations = 0;                              // check_rows: broken invariants so far
    if (stats) memset(stats, 0, sizeof(*stats));
    // statistics only: an event per recorded point of the stream, created the first time it is used
    auto record = [&](int i) -> hipError_t {
        if (!ev[i]) {
            hipError_t e = hipEventCreate(&ev[i]);
            if (e != hipSuccess) return e;
        }
        return hipEventRecord(ev[i], st);
    };

    {
        int dev = 0;
        HIPCHK(hipGetDevice(&dev));
        HIPCHK(hipDeviceGetAttribute(&num_cu, hipDeviceAttributeMultiprocessorCount, dev));
        if (num_cu < 1) num_cu = 1;
        upd_blocks = row_blocks < (unsigned)num_cu * 8u ? row_blocks : (unsigned)num_cu * 8u;
    }
    if (params->pinned_host) {
        host_ctr = static_cast<u64*>(params->pinned_host);
    } else {
        HIPCHK(hipHostMalloc(reinterpret_cast<void**>(&host_ctr), 64, hipHostMallocDefault));
        own_ctr = true;
    }
    if (stats) {
        ev = new hipEvent_t[n_ev];
        for (int i = 0; i < n_ev; ++i) ev[i] = nullptr;    // created when first recorded
        HIPCHK(record(0));
    }
    HIPCHK(hipMemsetAsync(ctr, 0, 256, st));
    if (cosine) {
        float* unit = reinterpret_cast<float*>(ws + bp.total);
        hipLaunchKernelGGL(k_unit_rows, dim3((unsigned)((n * 8 + 255) / 256)), dim3(256), 0, st, points_orig, n, d, unit);
        HIPCHK(hipGetLastError());
        points_dev = unit;
    }
    if (elem == 2)
        hipLaunchKernelGGL((k_init<0, 2>), dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst, rev, bp.B);
    else if (elem == 1)
        hipLaunchKernelGGL((k_init<0, 1>), dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst, rev, bp.B);
    else if (metric == 0)
        hipLaunchKernelGGL((k_init<0, 0>), dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst, rev, bp.B);
    else
        hipLaunchKernelGGL((k_init<1, 0>), dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst, rev, bp.B);
    HIPCHK(hipGetLastError());
    if (stats) HIPCHK(record(1));
    if (params->check_rows) {                        // the start state
        hipLaunchKernelGGL(k_check_rows, dim3(row_blocks), dim3(256), 0, st, n, bp.K, bp.C, bp.s, 0u, 0, G, cand,
                           newl, oldl, cnt, sig, worst, ctr + 7);
        HIPCHK(hipGetLastError());
    }

    // Iteration it: k_update merges what join it-1 offered and samples for join it; the host
    // reads the update count of iteration it-1 (the only device->host crossing of the loop)
    // and stops before join it if it fell below delta*K*n.
    for (int it = 0; it <= bp.max_iters; ++it) {
        const bool more = it < bp.max_iters;         // false: final merge-only pass
        if (it == 0 && !more) break;
        const bool rec = stats && it < max_rec;
        hipLaunchKernelGGL(k_update, dim3(upd_blocks), dim3(256), 0, st, n, bp.K, bp.C, bp.s, params->seed,
                           (uint32_t)it, more ? 1 : 0, G, cand, newl, oldl, cnt, sig, worst, ctr, rev, bp.B);
        HIPCHK(hipGetLastError());
        if (rec) HIPCHK(record(2 + 4 * it));
        if (stats && !more) HIPCHK(record(n_ev - 2));
        if (params->check_rows) {
            hipLaunchKernelGGL(k_check_rows, dim3(row_blocks), dim3(256), 0, st, n, bp.K, bp.C, bp.s, (uint32_t)it,
                               more ? 1 : 0, G, cand, newl, oldl, cnt, sig, worst, ctr + 7);
            HIPCHK(hipGetLastError());
        }
        if (it > 0) {
            HIPCHK(hipMemcpyAsync(host_ctr, ctr, 64, hipMemcpyDeviceToHost, st));
            HIPCHK(hipMemsetAsync(ctr, 0, 64, st));
            HIPCHK(hipStreamSynchronize(st));
            violations += host_ctr[7];
            if (stats && it - 1 < max_rec) {
                stats->updates[it - 1] = host_ctr[0];
                stats->join_rows[it - 1] = host_ctr[1];
            }
            if (stats) { stats->pairs += host_ctr[3]; stats->offers += host_ctr[4]; stats->cand_kept += host_ctr[5]; stats->joined += host_ctr[2]; stats->rejoined += host_ctr[6]; }
            if ((double)host_ctr[0] < stop_below) { converged = 1; break; }
        }
        if (!more) break;
        hipLaunchKernelGGL(k_plan, dim3((unsigned)((n + PLAN_CHUNK - 1) / PLAN_CHUNK)), dim3(256), 0, st, n, bp.s, bp.B,
                           params->seed, (uint32_t)it, rev + (int64_t)(it & 1) * 2 * n * bp.B,
                           reinterpret_cast<const int2*>(cnt), newl, oldl, plan, active, ctr);
        HIPCHK(hipGetLastError());
        if (rec) HIPCHK(record(3 + 4 * it));
        {
            JoinArgs ja{points_dev, elem == 1 ? d / 4 : elem == 2 ? d / 2 : d, bp.C, bp.s, (uint32_t)it, newl, oldl, plan, active, ctr + 2,
                        worst, sig, cand, ctr + 4, num_cu, n, join_blocks_per_cu, redo, ctr + 6};
            if (elem == 1) HIPCHK(launch_join_compact<1>(st, vec, bp.S16, ja));
            else if (elem == 2) HIPCHK(launch_join_compact<2>(st, vec, bp.S16, ja));
            else if (metric == 0) HIPCHK(launch_join<0>(st, vec, bp.S16, ja));
            else HIPCHK(launch_join<1>(st, vec, bp.S16, ja));
        }
        if (rec) HIPCHK(record(4 + 4 * it));
        iters = it + 1;
    }
    {
        int Kp = 1;
        while (Kp < bp.K) Kp <<= 1;
        const int64_t per_block = 4 * (WAVE / Kp);
        const dim3 grid((unsigned)((n + per_block - 1) / per_block)), block(256);
        // rows of whole 16-byte pieces: the staged kernel (dw = 32-bit words per row)
        const int dw = elem == 1 ? d / 4 : elem == 2 ? d / 2 : d;
#define KNNG_FIN(M, E)                                                                                            \
    do {                                                                                                          \
        if (vec) hipLaunchKernelGGL((k_finalize<M, E>), grid, block, 0, st, points_dev, n, dw, bp.K, Kp, k, G,   \
                                    ids_out_dev, dists_out_dev);                                                  \
        else hipLaunchKernelGGL((k_finalize_scalar<M, E>), grid, block, 0, st, points_dev, n, d, bp.K, Kp, k, G, \
                                ids_out_dev, dists_out_dev);                                                      \
    } while (0)
        if (cosine) points_dev = points_orig;          // the exact cosine of the caller's rows
        if (elem == 1) KNNG_FIN(0, 1);
        else if (elem == 2) KNNG_FIN(0, 2);
        else if (cosine) KNNG_FIN(2, 0);
        else if (metric == 0) KNNG_FIN(0, 0);
        else KNNG_FIN(1, 0);
#undef KNNG_FIN
        HIPCHK(hipGetLastError());
    }
    if (stats) HIPCHK(record(n_ev - 1));
    if (params->check_rows && bp.max_iters == 0) {   // no iteration read the counter: the start state's check
        HIPCHK(hipMemcpyAsync(host_ctr, ctr, 64, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        violations += host_ctr[7];
    }
    HIPCHK(hipStreamSynchronize(st));
    if (violations) rc = KNNG_ECHECK;
    if (stats) {
        stats->row_violations = violations;
        stats->iterations = iters;
        stats->converged = converged;
        float ms = 0.0f;
        HIPCHK(hipEventElapsedTime(&ms, ev[0], ev[1])); stats->ms_init = ms;
        const int recd = iters < max_rec ? iters : max_rec;
        for (int it = 0; it < recd; ++it) {
            hipEvent_t prev = it == 0 ? ev[1] : ev[4 + 4 * (it - 1)];
            HIPCHK(hipEventElapsedTime(&ms, prev, ev[2 + 4 * it])); stats->ms_sample += ms;
            HIPCHK(hipEventElapsedTime(&ms, ev[3 + 4 * it], ev[4 + 4 * it]));
            stats->join_ms[it] = ms; stats->ms_join += ms;
        }
        // the k_update after the last join (merge; when stopped by convergence also a sample)
        hipEvent_t lastj = recd > 0 ? ev[4 + 4 * (recd - 1)] : ev[1];
        if (recd > 0) {
            hipEvent_t lastu = (iters == bp.max_iters) ? ev[n_ev - 2] : ev[2 + 4 * (recd < max_rec ? recd : max_rec - 1)];
            if (iters == bp.max_iters || recd < max_rec) {
                HIPCHK(hipEventElapsedTime(&ms, lastj, lastu)); stats->ms_merge = ms;
                lastj = lastu;
            }
        }
        HIPCHK(hipEventElapsedTime(&ms, lastj, ev[n_ev - 1])); stats->ms_finalize = ms;
        HIPCHK(hipEventElapsedTime(&ms, ev[0], ev[n_ev - 1])); stats->ms_total = ms;
    }
done:
    if (rc != KNNG_OK) (void)hipStreamSynchronize(st);
    if (ev) {
        for (int i = 0; i < n_ev; ++i) if (ev[i]) (void)hipEventDestroy(ev[i]);
        delete[] ev;
    }
    if (own_ctr) (void)hipHostFree(host_ctr);
    return rc;
}

extern "C" __attribute__((visibility("default"))) int knng_build_knn_graph(const float* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                                    const knng_params_t* params, int32_t* ids_out_dev, float* dists_out_dev)
{
    return build_impl(points_dev, 0, n, d, k, metric, params, ids_out_dev, dists_out_dev);
}

extern "C" __attribute__((visibility("default"))) int knng_build_knn_graph_f16(const uint16_t* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                                        const knng_params_t* params, int32_t* ids_out_dev, float* dists_out_dev)
{
    return build_impl(points_dev, 2, n, d, k, metric, params, ids_out_dev, dists_out_dev);
}

extern "C" __attribute__((visibility("default"))) int knng_build_knn_graph_u8(const uint8_t* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                                       const knng_params_t* params, int32_t* ids_out_dev, float* dists_out_dev)
{
    return build_impl(points_dev, 1, n, d, k, metric, params, ids_out_dev, dists_out_dev);
}
