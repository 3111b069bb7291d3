// knng_build.hip -- lock-free NN-Descent on one MI355X (gfx950).
//
// Implements knng_build_knn_graph: random initial graph, then per iteration
//   k_sample   per-point sampling of new / old neighbours with reverse edges  (paper Sec. 3.1)
//   k_join     local join: gather the sampled neighbours' vectors into LDS, fp32 MFMA Gram
//              block, per-member best candidate, 64-bit atomic-min into the fixed-size
//              candidate lists of the two end points                           (Sec. 3.1.1)
//   k_merge    one wavefront per point folds its candidate list into its row   (Sec. 3.1.1)
// until an iteration accepts fewer than delta*K*n updates (Sec. 3.1), then
//   k_finalize exact fp64 re-evaluation of every kept distance, sort, cut to k (Sec. 5.3.1).
//
// Memory model: G is only ever written by the wavefront that owns the row (k_init, k_sample,
// k_merge); all cross-row traffic of an iteration goes through the candidate slots with
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
// Row signature: a 256-bit Bloom-style set of the ids in a point's row (bit hash(id) & 255).
// The join uses it to skip partners a member most likely already holds: such offers would be
// rejected by the merge anyway, cost an atomic each, and would shadow real candidates in the
// hashed candidate slots.  A false positive (about 12% at K = 32) only delays a candidate.
// k_sample rebuilds every row's signature each iteration, right before the join reads it.
// ------------------------------------------------------------------------------------------
constexpr int SIG_WORDS = 8;
// The bit an id maps to changes with the iteration (salt), so a false positive does not
// shadow the same candidate for good.
__device__ __forceinline__ uint32_t sig_bit(int id, uint32_t salt)
{
    return hash32((uint32_t)id ^ (salt * 0x9e3779b9u + 0x5bd1e995u)) & 255u;
}
// every lane contributes id (if has); lane w < 8 writes word w of the OR
__device__ __forceinline__ void store_signature(uint32_t* __restrict__ dst, int id, bool has, uint32_t salt)
{
    const uint32_t h = sig_bit(id, salt);
    uint32_t mine = 0;
#pragma unroll
    for (int w = 0; w < SIG_WORDS; ++w) {
        uint32_t x = (has && (h >> 5) == (uint32_t)w) ? (1u << (h & 31u)) : 0u;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) x |= __shfl_xor(x, o);
        if (lane_id() == w) mine = x;
    }
    if (lane_id() < SIG_WORDS) dst[lane_id()] = mine;
}

// ------------------------------------------------------------------------------------------
// k_init: one wavefront per point.  K distinct ids != v (random, or the caller's warm start
// with bad entries redrawn), their distances, row sorted by (distance, id), all flagged new.
// Also puts the point's candidate slots, counters and threshold into their start state.
// ------------------------------------------------------------------------------------------
template <int METRIC>
__global__ void __launch_bounds__(256)
k_init(const float* __restrict__ pts, int64_t n, int d, int K, int C, u64 seed,
       const int32_t* __restrict__ init_ids, u64* __restrict__ G, u64* __restrict__ cand,
       int32_t* __restrict__ cnt, float* __restrict__ worst)
{
    const int lane = lane_id();
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    for (int j = lane; j < C; j += WAVE) cand[v * C + j] = EMPTY_KEY;
    if (lane < 4) cnt[v * 4 + lane] = 0;

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
        float val = dist_group8<METRIC>(xv, pts + (int64_t)uid * d, d, sub);
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
// k_sample: one wavefront per point.  Up to s new-flagged entries (a cyclic window of the
// flagged ones from a random start, so every flagged entry is equally likely) become the
// forward new sample and lose their flag; up to s unflagged entries the forward old sample.
// Each forward edge v->u also puts v into u's reverse sample: an atomic counter hands out the
// first s slots, later arrivals replace a random slot with probability s/(arrivals so far).
// Lists: NEW[v] = [fwd 0..s) [rev s..2s), OLD likewise; cnt[v] = {fwd new, fwd old, rev new, rev old}.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_sample(int64_t n, int K, int s, u64 seed, uint32_t iter, u64* __restrict__ G,
         int32_t* __restrict__ newl, int32_t* __restrict__ oldl, int32_t* __restrict__ cnt,
         uint32_t* __restrict__ sig)
{
    const int lane = lane_id();
    const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const bool active = lane < K;
    u64 e = active ? G[v * K + lane] : 0ull;
    const bool isnew = active && (e & 1ull);
    const bool isold = active && !(e & 1ull);
    const int id = key_id(e);
    store_signature(sig + v * SIG_WORDS, id, active, iter);
    const u64 newmask = __ballot(isnew), oldmask = __ballot(isold);
    const int cn = __popcll(newmask), co = __popcll(oldmask);
    const u64 lt = lanemask_lt();
    const int64_t base = v * 2 * (int64_t)s;
    const uint32_t tag = 0x200u + 4u * iter;
    if (isnew) {
        int off = (int)below(rnd32(seed, tag, (uint32_t)v, 0u), (uint32_t)cn);
        int p = __popcll(newmask & lt) - off;
        if (p < 0) p += cn;
        if (p < s) {
            newl[base + p] = id;
            G[v * K + lane] = e & ~1ull;
            int pos = atomicAdd(&cnt[(int64_t)id * 4 + 2], 1);
            if (pos < s) newl[(int64_t)id * 2 * s + s + pos] = (int32_t)v;
            else {
                int r = (int)below(rnd32(seed, tag + 2u, (uint32_t)v, (uint32_t)lane), (uint32_t)pos + 1u);
                if (r < s) newl[(int64_t)id * 2 * s + s + r] = (int32_t)v;
            }
        }
    }
    if (isold) {
        int off = (int)below(rnd32(seed, tag + 1u, (uint32_t)v, 0u), (uint32_t)co);
        int p = __popcll(oldmask & lt) - off;
        if (p < 0) p += co;
        if (p < s) {
            oldl[base + p] = id;
            int pos = atomicAdd(&cnt[(int64_t)id * 4 + 3], 1);
            if (pos < s) oldl[(int64_t)id * 2 * s + s + pos] = (int32_t)v;
            else {
                int r = (int)below(rnd32(seed, tag + 3u, (uint32_t)v, (uint32_t)lane), (uint32_t)pos + 1u);
                if (r < s) oldl[(int64_t)id * 2 * s + s + r] = (int32_t)v;
            }
        }
    }
    if (lane == 0) {
        cnt[v * 4 + 0] = cn < s ? cn : s;
        cnt[v * 4 + 1] = co < s ? co : s;
    }
}

// Number of vectors the next join launch gathers (statistics only).
__global__ void __launch_bounds__(256)
k_count_rows(int64_t n, int s, const int32_t* __restrict__ cnt, u64* __restrict__ out)
{
    __shared__ u64 part[4];
    u64 acc = 0;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        int4 c = reinterpret_cast<const int4*>(cnt)[v];
        int nn = c.x + (c.z < s ? c.z : s);
        if (nn > 0) acc += (u64)(nn + c.y + (c.w < s ? c.w : s));
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane_id() == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(out, part[0] + part[1] + part[2] + part[3]);
}

// ------------------------------------------------------------------------------------------
// k_join: the local join, one 256-thread workgroup per point v.
//
// Members: m in [0,nNew) = NEW[v], m in [nNew,nTot) = OLD[v].  Their vectors are gathered
// from HBM with 16-byte coalesced loads, the pivot x_v is subtracted (keeps the Gram form
// |a|^2+|b|^2-2ab away from cancellation: all members are near v), and the centred slab is
// staged in LDS.  Four wavefronts then compute the NEW x (NEW|OLD) Gram block with
// v_mfma_f32_16x16x4_f32, 16x32 outputs per work item, accumulating over slabs of d.
// The distance block goes to LDS (over the vector slab), each member takes its closest
// partner, and if that beats the member's current farthest neighbour the pair is offered to
// the member's candidate list: one 64-bit atomic min on slot hash(partner) % C.
//
// S16 = number of 16-row tiles of NEW (2s <= 16*S16); DS = slab length in floats.
// ------------------------------------------------------------------------------------------
// Each member's partners are split into 4 residue classes (partner index mod 4), one per
// lane; the closest partner of each class is offered (1, 2 or 4 offers per member and join).
#ifndef KNNG_OFFERS_PER_MEMBER
#define KNNG_OFFERS_PER_MEMBER 4
#endif
constexpr int OFFERS_PER_MEMBER = KNNG_OFFERS_PER_MEMBER;

template <int S16> struct JoinCfg {
    static constexpr int MROWS = 16 * S16;            // max |NEW|
    static constexpr int NCOLS = 32 * S16;            // max |NEW| + |OLD|
    // short slabs keep the LDS footprint near 20 KB so seven workgroups fit a CU: the join is
    // latency-bound and measured 1.6x faster at 64 than at 128 floats per slab (d = 128)
    static constexpr int DS = S16 <= 2 ? 64 : (S16 == 4 ? 64 : 32);
    static constexpr int LD = DS + 4;                 // row stride of the vector slab (floats)
    static constexpr int LDD = NCOLS + 1;             // row stride of the distance block
    static constexpr int NT = (2 * S16 * S16 + 3) / 4; // 16x16 output tiles per wavefront (upper bound)
    static constexpr int NL = NCOLS * (DS / 4) / 256; // 16-byte pieces a thread gathers per slab
    static constexpr int XBYTES = NCOLS * LD * 4 > MROWS * LDD * 4 ? NCOLS * LD * 4 : MROWS * LDD * 4;
    static constexpr int LDS_BYTES = XBYTES + NCOLS * (16 + 4 * SIG_WORDS);
};

template <bool VEC>
__device__ __forceinline__ float4 load_piece(const float* __restrict__ row, int t, int d)
{
    if (VEC && t + 3 < d) return *reinterpret_cast<const float4*>(row + t);
    float4 x;
    x.x = t < d ? row[t] : 0.0f;         x.y = t + 1 < d ? row[t + 1] : 0.0f;
    x.z = t + 2 < d ? row[t + 2] : 0.0f; x.w = t + 3 < d ? row[t + 3] : 0.0f;
    return x;
}

template <int METRIC, int S16, bool VEC>
__global__ void __launch_bounds__(256)
k_join(const float* __restrict__ pts, int64_t n, int d, int K, int C, int s, uint32_t iter,
       const int32_t* __restrict__ newl, const int32_t* __restrict__ oldl, int32_t* __restrict__ cnt,
       const float* __restrict__ worst, const uint32_t* __restrict__ sig, u64* __restrict__ cand)
{
    using Cfg = JoinCfg<S16>;
    constexpr int DS = Cfg::DS, LD = Cfg::LD, LDD = Cfg::LDD, NT = Cfg::NT, NL = Cfg::NL;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* X = reinterpret_cast<float*>(smem);                 // [NCOLS][LD], later D [MROWS][LDD]
    int* mid = reinterpret_cast<int*>(smem + Cfg::XBYTES);     // [NCOLS] member ids
    float* nrm = reinterpret_cast<float*>(mid + Cfg::NCOLS);   // [NCOLS] |x_m - x_v|^2
    float* thr = nrm + Cfg::NCOLS;                             // [NCOLS] farthest-neighbour distance
    uint32_t* hb = reinterpret_cast<uint32_t*>(thr + Cfg::NCOLS);  // [NCOLS] signature bit of the id
    uint32_t* sg = hb + Cfg::NCOLS;                            // [NCOLS][SIG_WORDS] row signatures

    const int64_t v = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;

    const int4 c = reinterpret_cast<const int4*>(cnt)[v];
    const int nfn = c.x, nfo = c.y;
    const int nrn = c.z < s ? c.z : s, nro = c.w < s ? c.w : s;
    const int nNew = nfn + nrn, nOld = nfo + nro, nTot = nNew + nOld;
    if (tid == 0 && (c.z | c.w)) {            // hand the reverse counters back at zero
        cnt[v * 4 + 2] = 0;
        cnt[v * 4 + 3] = 0;
    }
    if (nNew == 0) return;                    // nothing new around v: no pair to evaluate

    // member ids (one member per thread: NCOLS <= 256)
    const int64_t lbase = v * 2 * (int64_t)s;
    int my_member = -1;
    if (tid < nTot) {
        const int m = tid;
        if (m < nNew) my_member = newl[lbase + (m < nfn ? m : s + (m - nfn))];
        else { int o = m - nNew; my_member = oldl[lbase + (o < nfo ? o : s + (o - nfo))]; }
        mid[m] = my_member;
        nrm[m] = 0.0f;
    }
    __syncthreads();
    // thresholds and signatures of the members: issued now, parked in registers while the
    // vector gather below is in flight
    float thr_r = 0.0f;
    uint4 sg_r0 = uint4{0, 0, 0, 0}, sg_r1 = uint4{0, 0, 0, 0};
    if (tid < nTot) {
        thr_r = worst[my_member];
        const uint4* sp = reinterpret_cast<const uint4*>(sig + (int64_t)my_member * SIG_WORDS);
        sg_r0 = sp[0];
        sg_r1 = sp[1];
    }

    // Output tiles (16x16): rows = NEW members, columns = NEW|OLD members.  Tiles strictly below
    // the diagonal of the NEW x NEW part are skipped (the block is symmetric there); the kept
    // tiles are dealt round-robin to the four wavefronts so every SIMD gets matrix work.
    const int nrt = (nNew + 15) >> 4, nct = (nTot + 15) >> 4;
    const int ntiles = nrt * nct - nrt * (nrt - 1) / 2;
    floatx4 acc[NT];
    int trow[NT], tcol[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        acc[q] = floatx4{0, 0, 0, 0};
        int rem = w + 4 * q, rt = 0;
        if (rem < ntiles) {
            while (rem >= nct - rt) { rem -= nct - rt; ++rt; }
            trow[q] = rt; tcol[q] = rt + rem;
        } else { trow[q] = -1; tcol[q] = 0; }
    }

    const int r16 = lane & 15, kq = lane >> 4;
    const float* xv = pts + v * (int64_t)d;

    for (int k0 = 0; k0 < d; k0 += DS) {
        const int len = (d - k0) < DS ? (d - k0) : DS;     // valid floats in this slab
        const int len16 = (len + 15) & ~15;                // padded with zeros for the MFMA k-loop
        const int q4 = len16 >> 2;                         // 16-byte pieces per row
        // thread -> (piece c4 of the row, row rsub + i*RP): QP = pieces rounded up to a power of
        // two, so a row's pieces sit in QP adjacent lanes and c4 is the same in every pass
        int qshift = 2;
        while ((1 << qshift) < q4) ++qshift;
        const int QP = 1 << qshift, RP = 256 >> qshift;
        const int c4 = tid & (QP - 1), rsub = tid >> qshift;
        const int t = k0 + 4 * c4;
        const bool col_ok = c4 < q4;
        float4 buf[NL];
        float4 pv = float4{0, 0, 0, 0};
        if (col_ok) pv = load_piece<VEC>(xv, t, d);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int row = rsub + i * RP;
            buf[i] = float4{0, 0, 0, 0};
            if (col_ok && row < nTot) buf[i] = load_piece<VEC>(pts + (int64_t)mid[row] * d, t, d);
        }
        if (k0 == 0 && tid < nTot) {
            thr[tid] = thr_r;
            hb[tid] = sig_bit(my_member, iter);
            reinterpret_cast<uint4*>(sg)[2 * tid] = sg_r0;
            reinterpret_cast<uint4*>(sg)[2 * tid + 1] = sg_r1;
        }
        if (k0 > 0) __syncthreads();                       // previous slab fully consumed
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int row = rsub + i * RP;
            float4 x = buf[i];
            x.x -= pv.x; x.y -= pv.y; x.z -= pv.z; x.w -= pv.w;
            float ss = x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
            for (int o = QP >> 1; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
            if (row < nTot) {
                if (col_ok) *reinterpret_cast<float4*>(X + row * LD + 4 * c4) = x;
                if (c4 == 0) nrm[row] += ss;
            }
        }
        __syncthreads();
        // Gram tiles of this slab
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            if (trow[q] >= 0) {
                const float* xa = X + (trow[q] * 16 + r16) * LD + 4 * kq;
                const float* xb = X + (tcol[q] * 16 + r16) * LD + 4 * kq;
                for (int kk = 0; kk < len16; kk += 16) {
                    const float4 a = *reinterpret_cast<const float4*>(xa + kk);
                    const float4 b = *reinterpret_cast<const float4*>(xb + kk);
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc[q], 0, 0, 0);
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc[q], 0, 0, 0);
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc[q], 0, 0, 0);
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc[q], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();                                       // all wavefronts done with the slab
    // The pivot's reverse members hold v in their rows, so |x_m - x_v|^2 is already known here:
    // offer them to v itself (closes v<-m edges into v->m without an extra distance).
    for (int m = tid; m < nTot; m += 256) {
        const bool rev = (m >= nfn && m < nNew) || (m >= nNew + nfo);
        if (!rev) continue;
        float l = nrm[m];
        if (METRIC == 1) l *= 0.5f;
        l = nonneg(l);
        const int pid = mid[m];
        const uint32_t h = hb[m];
        const uint32_t vw = sig[v * SIG_WORDS + (h >> 5)];
        if (l < worst[v] && !((vw >> (h & 31u)) & 1u)) {
            const uint32_t slot = below(hash32((uint32_t)pid), (uint32_t)C);
            atomicMin(&cand[v * C + slot], pack_key(l, pid, 1));
        }
    }
    // distance block D[row][col] over the slab storage
    float* D = X;
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        if (trow[q] >= 0) {
            const int col = tcol[q] * 16 + r16;
            const float nc = nrm[col < nTot ? col : 0];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = trow[q] * 16 + 4 * kq + r;
                float l = nrm[row < nTot ? row : 0] + nc - 2.0f * acc[q][r];
                if (METRIC == 1) l *= 0.5f;                // unit rows: 1 - <a,b> = |a-b|^2 / 2
                D[row * LDD + col] = nonneg(l);
            }
        }
    }
    __syncthreads();
    // per-member candidates: LPM lanes per member, each lane scans the partners of one residue
    // class (partner index mod LPM) and offers the closest of its class
    constexpr int LPM = OFFERS_PER_MEMBER;
    for (int m0 = 0; m0 < nTot; m0 += 256 / LPM) {
        const int m = m0 + tid / LPM, sub = tid % LPM;
        if (m >= nTot) continue;
        const int myid = mid[m];
        const uint32_t* msig = sg + m * SIG_WORDS;
        const float mythr = thr[m];
        u64 best = EMPTY_KEY;
        if (m < nNew) {
            for (int j = sub; j < nTot; j += LPM) {
                const float l = ((j >> 4) < (m >> 4)) ? D[j * LDD + m] : D[m * LDD + j];
                if (!(l < mythr)) continue;
                const uint32_t h = hb[j];
                if (mid[j] == myid || ((msig[h >> 5] >> (h & 31u)) & 1u)) continue;
                u64 cnd = ((u64)__float_as_uint(l) << 32) | (uint32_t)j;
                best = cnd < best ? cnd : best;
            }
        } else {
            for (int i = sub; i < nNew; i += LPM) {
                const float l = D[i * LDD + m];
                if (!(l < mythr)) continue;
                const uint32_t h = hb[i];
                if (mid[i] == myid || ((msig[h >> 5] >> (h & 31u)) & 1u)) continue;
                u64 cnd = ((u64)__float_as_uint(l) << 32) | (uint32_t)i;
                best = cnd < best ? cnd : best;
            }
        }
        if (best != EMPTY_KEY) {
            const float l = __uint_as_float((uint32_t)(best >> 32));
            {
                const int pid = mid[(int)(uint32_t)best];
                const uint32_t slot = below(hash32((uint32_t)pid), (uint32_t)C);
                atomicMin(&cand[(int64_t)myid * C + slot], pack_key(l, pid, 1));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// k_merge: one wavefront per point folds the candidate slots into the row (Sec. 3.1.1: a
// single owner per point, so no races).  A candidate is accepted if its id is not already in
// the row and it sorts before the row's K-th entry; the union is re-ranked by counting, the
// first K kept, accepted entries flagged new and counted; used slots are set back to empty.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_merge(int64_t n, int K, int C, u64* __restrict__ G, u64* __restrict__ cand,
        float* __restrict__ worst, u64* __restrict__ updates)
{
    __shared__ u64 part[4];
    const int lane = lane_id();
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    u64 accepted = 0;
    for (int64_t v = wave0; v < n; v += nwaves) {
        u64 ck = lane < C ? cand[v * C + lane] : EMPTY_KEY;
        if (__ballot(ck != EMPTY_KEY) == 0ull) continue;
        if (ck != EMPTY_KEY) cand[v * C + lane] = EMPTY_KEY;
        const u64 lk = lane < K ? G[v * K + lane] : EMPTY_KEY;
        const u64 lo = key_order(lk);
        const u64 co = key_order(ck);
        const u64 last = bcast64(lo, K - 1);
        bool valid = ck != EMPTY_KEY && co < last;
        const int cid = key_id(ck), lid = key_id(lk);
        if (__ballot(valid) == 0ull) continue;
        for (int i = 0; i < K; ++i) {
            int li = (int)bcast32((uint32_t)lid, i);
            if (li == cid) valid = false;
        }
        u64 vm = __ballot(valid);
        if (vm == 0ull) continue;
        // ranks in the union of the row and the accepted candidates
        int rl = lane;                           // the row is ascending already
        int rc = 0;
        for (u64 m = vm; m; m &= m - 1) {
            int j = __ffsll((long long)m) - 1;
            u64 cj = bcast64(co, j);
            rl += (cj < lo) ? 1 : 0;
            rc += (cj < co) ? 1 : 0;
        }
        for (int i = 0; i < K; ++i) rc += (bcast64(lo, i) < co) ? 1 : 0;
        if (lane < K && rl < K) {
            G[v * K + rl] = lk;
            if (rl == K - 1) worst[v] = key_dist(lk);
        }
        const bool in = valid && rc < K;
        if (in) {
            G[v * K + rc] = ck | 1ull;
            if (rc == K - 1) worst[v] = key_dist(ck);
        }
        accepted += (u64)__popcll(__ballot(in));
    }
    if (lane == 0) part[threadIdx.x >> 6] = accepted;
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(updates, t);
    }
}

// ------------------------------------------------------------------------------------------
// k_finalize: one wavefront per point, 4 points per workgroup.  The K neighbour vectors are
// staged slab by slab in LDS (coalesced), then lane i walks neighbour i's slab in index order
// with the fp64 recipe, so the value written equals a sequential fp64 evaluation bit for bit.
// Rows are then ranked by (distance, id) and the first k written as ids / distances.
// ------------------------------------------------------------------------------------------
constexpr int FIN_SL = 32;                        // slab length (floats)
constexpr int FIN_LD = FIN_SL + 1;                // odd stride: lanes on distinct banks

template <int METRIC>
__global__ void __launch_bounds__(256)
k_finalize(const float* __restrict__ pts, int64_t n, int d, int K, int k,
           const u64* __restrict__ G, int32_t* __restrict__ ids_out, float* __restrict__ dists_out)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    float* X = reinterpret_cast<float*>(smem) + w * (K + 1) * FIN_LD;   // [K+1][FIN_LD], row K = x_v
    int64_t v = (int64_t)blockIdx.x * 4 + w;
    const bool live = v < n;
    if (!live) v = n - 1;                         // keep every wavefront in the barriers
    const u64 key = lane < K ? G[v * K + lane] : EMPTY_KEY;
    const int id = lane < K ? key_id(key) : (int)v;
    double acc = 0.0;
    for (int k0 = 0; k0 < d; k0 += FIN_SL) {
        const int len = (d - k0) < FIN_SL ? (d - k0) : FIN_SL;
        __syncthreads();
        // 32 consecutive lanes read one row's 128-byte slab
        for (int base = 0; base < (K + 1) * FIN_SL; base += WAVE) {   // uniform trip count
            const int idx = base + lane;
            const bool ok = idx < (K + 1) * FIN_SL;
            const int row = ok ? idx / FIN_SL : 0, t = idx - row * FIN_SL;
            const int src = __shfl(id, row < K ? row : 0);
            const int rid = row < K ? src : (int)v;
            if (ok && t < len) X[row * FIN_LD + t] = pts[(int64_t)rid * d + k0 + t];
        }
        __syncthreads();
        if (lane < K) {
            const float* xr = X + lane * FIN_LD;
            const float* xp = X + K * FIN_LD;
            for (int t = 0; t < len; ++t) acc = exact_step<METRIC>(acc, xp[t], xr[t]);
        }
    }
    const float dist = exact_finish<METRIC>(acc);
    const u64 fk = lane < K ? pack_key(dist, id, 0) : EMPTY_KEY;
    int rank = 0;
    for (int j = 0; j < K; ++j) rank += (bcast64(fk, j) < fk) ? 1 : 0;
    if (live && lane < K && rank < k) {
        ids_out[v * k + rank] = id;
        dists_out[v * k + rank] = dist;
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct BuildPlan {
    int K, C, s, S16, max_iters;
    float rho, delta;
    uint64_t off_G, off_cand, off_new, off_old, off_cnt, off_worst, off_sig, off_ctr, total;
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
    int C = (p && p->cand_cap) ? p->cand_cap : K;
    if (C < 1 || C > KNNG_MAX_K) return false;
    int s = (int)ceil((double)rho * (double)K);
    if (s < 1) s = 1;
    if (s > K) s = K;
    bp->K = K; bp->C = C; bp->s = s; bp->rho = rho; bp->delta = delta; bp->max_iters = max_iters;
    bp->S16 = (2 * s <= 16) ? 1 : (2 * s <= 32) ? 2 : (2 * s <= 64) ? 4 : 8;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = (off + bytes + 255) & ~255ull; return o; };
    bp->off_G = take((uint64_t)n * K * 8);
    bp->off_cand = take((uint64_t)n * C * 8);
    bp->off_new = take((uint64_t)n * 2 * s * 4);
    bp->off_old = take((uint64_t)n * 2 * s * 4);
    bp->off_cnt = take((uint64_t)n * 16);
    bp->off_worst = take((uint64_t)n * 4);
    bp->off_sig = take((uint64_t)n * SIG_WORDS * 4);
    bp->off_ctr = take(256);
    bp->total = off;
    return true;
}

template <int METRIC, int S16>
static hipError_t launch_join(hipStream_t st, bool vec, uint32_t iter, const float* pts, int64_t n, int d,
                              const BuildPlan& bp, const int32_t* newl, const int32_t* oldl,
                              int32_t* cnt, const float* worst, const uint32_t* sig, u64* cand)
{
    const int lds = JoinCfg<S16>::LDS_BYTES;
    auto kv = k_join<METRIC, S16, true>;
    auto ks = k_join<METRIC, S16, false>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(vec ? kv : ks),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    if (vec) hipLaunchKernelGGL(kv, dim3((unsigned)n), dim3(256), lds, st, pts, n, d, bp.K, bp.C, bp.s, iter,
                                newl, oldl, cnt, worst, sig, cand);
    else hipLaunchKernelGGL(ks, dim3((unsigned)n), dim3(256), lds, st, pts, n, d, bp.K, bp.C, bp.s, iter,
                            newl, oldl, cnt, worst, sig, cand);
    return hipGetLastError();
}

template <int METRIC>
static hipError_t launch_join_m(hipStream_t st, bool vec, uint32_t iter, const float* pts, int64_t n, int d,
                                const BuildPlan& bp, const int32_t* newl, const int32_t* oldl,
                                int32_t* cnt, const float* worst, const uint32_t* sig, u64* cand)
{
    switch (bp.S16) {
    case 1: return launch_join<METRIC, 1>(st, vec, iter, pts, n, d, bp, newl, oldl, cnt, worst, sig, cand);
    case 2: return launch_join<METRIC, 2>(st, vec, iter, pts, n, d, bp, newl, oldl, cnt, worst, sig, cand);
    case 4: return launch_join<METRIC, 4>(st, vec, iter, pts, n, d, bp, newl, oldl, cnt, worst, sig, cand);
    default: return launch_join<METRIC, 8>(st, vec, iter, pts, n, d, bp, newl, oldl, cnt, worst, sig, cand);
    }
}

}  // namespace knng

using namespace knng;

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

extern "C" __attribute__((visibility("default"))) int knng_build_knn_graph(const float* points_dev, int64_t n, int32_t d, int32_t k, int32_t metric,
                                    const knng_params_t* params, int32_t* ids_out_dev, float* dists_out_dev)
{
    if (!points_dev || !ids_out_dev || !dists_out_dev || !params) return KNNG_EINVAL;
    if (params->struct_size != sizeof(knng_params_t)) return KNNG_EINVAL;
    if (metric != KNNG_METRIC_L2SQ && metric != KNNG_METRIC_IP_UNIT) return KNNG_EINVAL;
    BuildPlan bp;
    if (!make_plan(n, d, k, params, &bp)) return KNNG_EINVAL;
    if (!params->workspace_dev || params->workspace_bytes < bp.total ||
        (reinterpret_cast<uintptr_t>(params->workspace_dev) & 255u))
        return KNNG_EWORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(params->stream);
    unsigned char* ws = static_cast<unsigned char*>(params->workspace_dev);
    u64* G = reinterpret_cast<u64*>(ws + bp.off_G);
    u64* cand = reinterpret_cast<u64*>(ws + bp.off_cand);
    int32_t* newl = reinterpret_cast<int32_t*>(ws + bp.off_new);
    int32_t* oldl = reinterpret_cast<int32_t*>(ws + bp.off_old);
    int32_t* cnt = reinterpret_cast<int32_t*>(ws + bp.off_cnt);
    float* worst = reinterpret_cast<float*>(ws + bp.off_worst);
    uint32_t* sig = reinterpret_cast<uint32_t*>(ws + bp.off_sig);
    u64* ctr = reinterpret_cast<u64*>(ws + bp.off_ctr);      // [0] updates, [1] rows gathered
    knng_stats_t* stats = params->stats_host;
    const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(points_dev) & 15u) == 0);
    const unsigned row_blocks = (unsigned)((n + 3) / 4);
    const unsigned merge_blocks = row_blocks < 256u * 16u ? row_blocks : 256u * 16u;
    const double stop_below = (double)bp.delta * (double)bp.K * (double)n;

    int rc = KNNG_OK;
    u64* host_ctr = nullptr;
    // events: [0] start, [1] after init, then 4 per iteration (sample, join start, join end, merge), last = end
    const int max_rec = bp.max_iters < KNNG_STATS_MAX_ITERS ? bp.max_iters : KNNG_STATS_MAX_ITERS;
    const int n_ev = stats ? 4 + 4 * max_rec : 0;
    hipEvent_t* ev = nullptr;
    int iters = 0, converged = 0;
    if (stats) memset(stats, 0, sizeof(*stats));

    HIPCHK(hipHostMalloc(reinterpret_cast<void**>(&host_ctr), 64, hipHostMallocDefault));
    if (stats) {
        ev = new hipEvent_t[n_ev];
        for (int i = 0; i < n_ev; ++i) ev[i] = nullptr;
        for (int i = 0; i < n_ev; ++i) HIPCHK(hipEventCreate(&ev[i]));
        HIPCHK(hipEventRecord(ev[0], st));
    }
    HIPCHK(hipMemsetAsync(ctr, 0, 256, st));
    if (metric == 0)
        hipLaunchKernelGGL(k_init<0>, dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst);
    else
        hipLaunchKernelGGL(k_init<1>, dim3(row_blocks), dim3(256), 0, st, points_dev, n, d, bp.K, bp.C,
                           params->seed, params->init_ids_dev, G, cand, cnt, worst);
    HIPCHK(hipGetLastError());
    if (stats) HIPCHK(hipEventRecord(ev[1], st));

    for (int it = 0; it < bp.max_iters; ++it) {
        const bool rec = stats && it < max_rec;
        hipLaunchKernelGGL(k_sample, dim3(row_blocks), dim3(256), 0, st, n, bp.K, bp.s, params->seed,
                           (uint32_t)it, G, newl, oldl, cnt, sig);
        HIPCHK(hipGetLastError());
        if (rec) {
            HIPCHK(hipEventRecord(ev[2 + 4 * it], st));
            hipLaunchKernelGGL(k_count_rows, dim3(1024), dim3(256), 0, st, n, bp.s, cnt, ctr + 1);
            HIPCHK(hipGetLastError());
            HIPCHK(hipEventRecord(ev[3 + 4 * it], st));
        }
        if (metric == 0) HIPCHK(launch_join_m<0>(st, vec, (uint32_t)it, points_dev, n, d, bp, newl, oldl, cnt, worst, sig, cand));
        else HIPCHK(launch_join_m<1>(st, vec, (uint32_t)it, points_dev, n, d, bp, newl, oldl, cnt, worst, sig, cand));
        if (rec) HIPCHK(hipEventRecord(ev[4 + 4 * it], st));
        hipLaunchKernelGGL(k_merge, dim3(merge_blocks), dim3(256), 0, st, n, bp.K, bp.C, G, cand, worst, ctr);
        HIPCHK(hipGetLastError());
        if (rec) HIPCHK(hipEventRecord(ev[5 + 4 * it], st));
        HIPCHK(hipMemcpyAsync(host_ctr, ctr, 16, hipMemcpyDeviceToHost, st));
        HIPCHK(hipMemsetAsync(ctr, 0, 16, st));
        HIPCHK(hipStreamSynchronize(st));
        iters = it + 1;
        if (rec) { stats->updates[it] = host_ctr[0]; stats->join_rows[it] = host_ctr[1]; }
        if ((double)host_ctr[0] < stop_below) { converged = 1; break; }
    }
    {
        const int lds = 4 * (bp.K + 1) * FIN_LD * 4;
        if (metric == 0)
            hipLaunchKernelGGL(k_finalize<0>, dim3(row_blocks), dim3(256), lds, st, points_dev, n, d, bp.K, k,
                               G, ids_out_dev, dists_out_dev);
        else
            hipLaunchKernelGGL(k_finalize<1>, dim3(row_blocks), dim3(256), lds, st, points_dev, n, d, bp.K, k,
                               G, ids_out_dev, dists_out_dev);
        HIPCHK(hipGetLastError());
    }
    if (stats) HIPCHK(hipEventRecord(ev[n_ev - 1], st));
    HIPCHK(hipStreamSynchronize(st));
    if (stats) {
        stats->iterations = iters;
        stats->converged = converged;
        float ms = 0.0f;
        HIPCHK(hipEventElapsedTime(&ms, ev[0], ev[1])); stats->ms_init = ms;
        const int recd = iters < max_rec ? iters : max_rec;
        for (int it = 0; it < recd; ++it) {
            hipEvent_t prev = it == 0 ? ev[1] : ev[5 + 4 * (it - 1)];
            HIPCHK(hipEventElapsedTime(&ms, prev, ev[2 + 4 * it])); stats->ms_sample += ms;
            HIPCHK(hipEventElapsedTime(&ms, ev[3 + 4 * it], ev[4 + 4 * it]));
            stats->join_ms[it] = ms; stats->ms_join += ms;
            HIPCHK(hipEventElapsedTime(&ms, ev[4 + 4 * it], ev[5 + 4 * it])); stats->ms_merge += ms;
        }
        hipEvent_t lastit = recd > 0 ? ev[5 + 4 * (recd - 1)] : ev[1];
        HIPCHK(hipEventElapsedTime(&ms, lastit, ev[n_ev - 1])); stats->ms_finalize = ms;
        HIPCHK(hipEventElapsedTime(&ms, ev[0], ev[n_ev - 1])); stats->ms_total = ms;
    }
done:
    if (rc != KNNG_OK) (void)hipStreamSynchronize(st);
    if (ev) {
        for (int i = 0; i < n_ev; ++i) if (ev[i]) (void)hipEventDestroy(ev[i]);
        delete[] ev;
    }
    if (host_ctr) (void)hipHostFree(host_ctr);
    return rc;
}
