// knng_join_wave.h -- the local join for s <= 16 (the paper's default parameters): one
// wavefront per point, no workgroup barriers.  Included by knng_build.hip.
//
// With at most 64 members per point a point maps onto one 64-lane wavefront: lane m owns
// member m (its id, threshold and signature bit live in that lane's registers; other lanes
// read them with v_readlane), the wavefront owns every Gram tile of the point, and all
// cross-lane traffic goes through the wavefront's private LDS region in program order, so no
// s_barrier is needed.  Four wavefronts of a workgroup work on four different points and only
// share the LDS allocation.  Each wavefront is persistent and software-pipelined over
// (point, slab) units of 32 coordinates: while the matrix cores and the selection work on the
// unit in LDS, the global loads of the next unit and the list record of the point after next
// are in flight into registers.
//
// Per unit:  A  prefetched 16-byte pieces - pivot -> LDS slab X[64][36]
//            B  issue the loads of the next unit
//            C  one pass of v_mfma_f32_16x16x4_f32 over all tiles of the point: the operand
//               tiles (16 members x 16 coordinates) are read once per k-step and shared by all
//               output tiles, so up to 36 MFMAs follow 4 LDS reads
// After the last slab: member norms from the diagonal tiles, distance block D to LDS (over X),
// then lane m scans member m's partners: per residue class (partner index mod 4) the closest
// partner that beats the member's threshold and is not in the member's signature is offered
// with one 64-bit atomic min on cand[member][hash(partner) % C].
//
// The kernel is bound by instruction issue inside the CU, not by HBM (it runs at the same
// speed on a cache-resident point set), so the code below trades generality for straight-line
// instruction streams and a small register footprint (three wavefronts per SIMD without
// spills): the gather has one uniform guard per group of rows, the Gram pass reads each
// operand tile once per k-step, and the partner scan advances one LDS address per partner.
// (Specialising the Gram pass on the tile counts was tried: the extra code paths cost 40
// registers, spills, and 25% of the speed.)
//
// ELEM = 1: uint8 rows (squared L2 only).  A row is handled as d/4 32-bit words, so a slab of 32
// words is 128 coordinates and the gather and the LDS slab are the same bytes as for floats.
// The bytes are stored as signed values x - 128 (one xor) and not centred; the Gram pass is
// v_mfma_i32_16x16x64_i8, one instruction where the fp32 pass needs sixteen, exact in 32-bit
// integers, and |a-b|^2 = |a|^2 + |b|^2 - 2<a,b> is evaluated in integers before the one
// conversion to fp32.  The products with the pivot (for its reverse members) come from one more
// accumulator tile: column c of that tile takes the pivot as B operand for member tile c and a
// row of zeros for the others, column 4 the pivot against itself.
//
// ELEM = 2: fp16 rows (squared L2 only), d/2 words per row: a slab is 64 coordinates in the same
// bytes.  The rows are centred on the pivot in fp16 (one v_pk_add_f16 per word) and stay fp16 in
// LDS; the Gram pass is v_mfma_f32_16x16x32_f16 with fp32 accumulators, one instruction per
// operand read, and everything after it is the fp32 kernel's.  The centring rounds to fp16, so
// the distances the join compares carry a relative error of about 1e-3: search-time precision
// only, what is written to the caller is recomputed exactly from the fp16 values.
//
// SPLIT (fp32 rows of 256 coordinates or more, where the fp32 matrix instruction is the busiest
// unit of the kernel): the centred values are split into two bf16 halves when the slab is stored
// (a 16-byte piece = two words of hi halves, then two of lo halves: the same bytes, the same LDS
// addresses and bank pattern as the fp32 slab), and the Gram pass
// takes <a,b> as hi.hi + hi.lo + lo.hi on v_mfma_f32_16x16x16_bf16 -- three instructions of 8
// cycles where fp32 needs four of 32.  The products miss <a,b> by at most 3 * 2^-18 |a||b| of the
// centred vectors; a choice that this could have decided is not made here: the point goes to a
// list the fp32 kernel works off afterwards (split_untrusted in knng_build.hip).
#pragma once

namespace knng {

template <int S16, int ELEM = 0> struct WaveCfg {
    static constexpr int NCOLS = 32 * S16;            // max members (<= 64 lanes)
    static constexpr int MROWS = 16 * S16;            // max |NEW|
    static constexpr int CT = 2 * S16;                // 16-member operand tiles
#ifndef KNNG_WAVE_DS
#define KNNG_WAVE_DS 32
#endif
    static constexpr int DS = KNNG_WAVE_DS;           // slab length (floats)
    static constexpr int LD = DS + 4;                 // slab row stride: conflict-free ds_read_b128
    static constexpr int LDD = NCOLS + 1;             // distance-block row stride (last column: +inf cell)
    static constexpr int NL = NCOLS * (DS / 4) / 64;  // 16-byte pieces per lane and slab
    static constexpr int NTILES = (3 * S16 * S16 + 3 * S16) / 2;  // upper triangle rows<S16 + extra diagonals
    static_assert(NCOLS * LD >= MROWS * LDD, "the distance block lies over the slab rows");
    // ELEM 1: two more slab rows (the pivot, zeros) and the pivot distances dpv[NCOLS]
    static constexpr int XBYTES = (NCOLS + (ELEM == 1 ? 2 : 0)) * LD * 4;
    // X/D | mid[2][NCOLS] | nrm[NCOLS] | sg[8][NCOLS+1] | dpv[NCOLS]
    static constexpr int WBYTES = ((XBYTES + NCOLS * (8 + 4) + (NCOLS + 1) * 4 * SIG_WORDS +
                                    (ELEM == 1 ? NCOLS * 4 : 0)) + 255) & ~255;
};

#ifndef KNNG_WAVE_OCC
#define KNNG_WAVE_OCC 3
#endif
// Wavefronts per SIMD the register allocation aims at: three; two for uint8 and fp16 rows with
// up to 64 members (the extra accumulator tile of the uint8 kernel does not fit beside the rest
// in 168 registers, and the fp16 kernel spills 39 there).
template <int S16, int ELEM> struct WaveOcc { static constexpr int V = (ELEM != 0 && S16 == 2) ? 2 : KNNG_WAVE_OCC; };

template <int METRIC, int S16, bool VEC, int ELEM = 0, bool SPLIT = false>
__global__ void __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu(WaveOcc<S16, ELEM>::V, WaveOcc<S16, ELEM>::V)))
k_join_wave(const float* __restrict__ pts, int d, int C, int s, uint32_t iter,
            const int32_t* __restrict__ newl, const int32_t* __restrict__ oldl, const int4* __restrict__ plan,
            const int32_t* __restrict__ active, const u64* __restrict__ nactive_ptr,
            const float* __restrict__ worst, const uint32_t* __restrict__ sig, u64* __restrict__ cand,
            u64* __restrict__ offers_ctr, int32_t* __restrict__ redo, u64* __restrict__ redo_ctr)
{
    // ELEM 1 / 2: pts points at uint8 / fp16 rows of 4 d bytes, d counts 32-bit words
    static_assert(ELEM == 0 || METRIC == 0, "uint8 and fp16 rows: squared L2 only");
    static_assert(ELEM == 0 || !SPLIT, "the bf16 split is for fp32 rows");
    using Cfg = WaveCfg<S16, ELEM>;
    using accv = typename std::conditional<ELEM == 1, intx4, floatx4>::type;
    constexpr int NCOLS = Cfg::NCOLS, CT = Cfg::CT, DS = Cfg::DS, LD = Cfg::LD, LDD = Cfg::LDD,
                  NL = Cfg::NL, NTILES = Cfg::NTILES;
    constexpr int INF_CELL = NCOLS;                             // D[0][NCOLS]: holds +inf
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = lane_id();
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    unsigned char* wbase = smem + wib * Cfg::WBYTES;
    float* X = reinterpret_cast<float*>(wbase);                 // [NCOLS][LD], later D [MROWS][LDD]
    int* midbuf = reinterpret_cast<int*>(wbase + Cfg::XBYTES);  // [2][NCOLS] member ids, double-buffered
    // [NCOLS] bits of |x_m - x_v|^2 (fp32); ELEM 1: of |x_m - 128|^2 (integer)
    uint32_t* nrm = reinterpret_cast<uint32_t*>(midbuf + 2 * NCOLS);
    uint32_t* sg = nrm + NCOLS;                                 // [SIG_WORDS][NCOLS + 1], column nTot = pivot
    constexpr int SGLD = NCOLS + 1;
    float* dpv = reinterpret_cast<float*>(sg + SIG_WORDS * SGLD);   // ELEM 1: [NCOLS] |x_m - x_v|^2
    constexpr int PIV_ROW = NCOLS * LD, ZERO_ROW = (NCOLS + 1) * LD;   // ELEM 1: two more slab rows
    if (ELEM == 1 && lane < LD) X[ZERO_ROW + lane] = 0.0f;

    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t nact = (int64_t)*nactive_ptr;
    const int64_t GW = (int64_t)gridDim.x * 4;                  // wavefronts in the grid
    int64_t pos = (int64_t)blockIdx.x * 4 + wib;
    if (pos >= nact) return;

    auto load_slot = [&](int64_t v) -> int {
        if (lane < 2 * s) return newl[v * 2 * (int64_t)s + lane];
        if (lane < 4 * s) return oldl[v * 2 * (int64_t)s + (lane - 2 * s)];
        return 0;
    };

    // ---- prologue
    int64_t v = active[pos];
    int64_t v_nx = pos + GW < nact ? (int64_t)active[pos + GW] : -1;
    int64_t v_nx2 = pos + 2 * GW < nact ? (int64_t)active[pos + 2 * GW] : -1;
    int4 rc = plan[v];
    int rid = load_slot(v);
    int cur = 0;
    PointPlan P = make_point(rc);
    {
        const int m = member_of_slot(lane, s, rc);
        if (m >= 0) midbuf[m] = rid;
        if (lane >= P.nTot && lane < NCOLS) midbuf[lane] = (int)v;
    }
    wave_lds_sync();

    float4 buf[NL];
    float4 pv;
    // lane m < nTot: member m; lane nTot (if any): the pivot itself
    int id_r = 0;
    float thr_r = 0.0f;
    uint4 sg_r0 = uint4{0, 0, 0, 0}, sg_r1 = uint4{0, 0, 0, 0};
    auto issue_members = [&](const int* mid, int nTot, int64_t pivot_row) {
        if (lane <= nTot) {
            id_r = lane < nTot ? mid[lane] : (int)pivot_row;
            thr_r = worst[id_r];
            const uint4* sp = reinterpret_cast<const uint4*>(sig + (int64_t)id_r * SIG_WORDS);
            sg_r0 = sp[0];
            sg_r1 = sp[1];
        }
    };
    // slab pieces: lane -> (piece c4 = lane & 7, rows (lane >> 3) + 8 i).  A group of 8 rows is
    // loaded whole or not at all: the id slots past the last member hold the pivot's id (its
    // centred row is zero and its cells are masked out of the distance block).  All ids are read
    // from LDS before the first load is issued: one LDS round trip per slab, not one per group.
    constexpr int QP = DS / 4, RPW = 64 / QP;              // pieces per row, rows per load
    const int c4 = lane & (QP - 1), rsub = lane / QP;
    auto issue_slab = [&](const int* mid, int nTot, int64_t pivot_row, int k0) {
        int t = k0 + 4 * c4;
        // VEC: pieces past the end of the row are loaded from its last piece and zeroed when
        // they are stored to LDS (a zero fill before a predicated load would make the compiler
        // wait for every load in flight)
        if (VEC) t = t < d ? t : d - 4;
        int rowid[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) rowid[i] = mid[rsub + RPW * i];
        pv = load_piece_inside<VEC>(pts + pivot_row * d, t, d);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (RPW * i < nTot)                                 // uniform
                buf[i] = load_piece_inside<VEC>(pts + (int64_t)rowid[i] * d, t, d);
        }
    };

    issue_slab(midbuf, P.nTot, v, 0);
    issue_members(midbuf, P.nTot, v);
    int4 rc_n = int4{0, 0, 0, 0};
    int rid_n = 0;
    if (v_nx >= 0) { rc_n = plan[v_nx]; rid_n = load_slot(v_nx); }

    // Offers of the previous point, sent one point late: right after the last Gram pass, so
    // that their round trip to memory runs under the norm / distance-block / scan work, which
    // never waits for memory.  (Sent right after the scan they would be waited for at the very
    // next use of prefetched data: loads and atomics share one in-order counter.)
    // pend_id: the previous point's member id per lane; pend_j: partner lane per class, 0xff none.
    int pend_id = 0;
    uint32_t pend_j = 0xffffffffu;
    uint32_t pend_l[OFFERS_PER_MEMBER];
#pragma unroll
    for (int u = 0; u < OFFERS_PER_MEMBER; ++u) pend_l[u] = 0u;
    uint32_t n_offers = 0;                                     // wavefront total (uniform)
    auto send_offers = [&]() {
#pragma unroll
        for (int u = 0; u < OFFERS_PER_MEMBER; ++u) {
            const uint32_t j = (pend_j >> (8 * u)) & 0xffu;
            const int pid = __shfl(pend_id, (int)(j & 63u));   // all lanes take part in the shuffle
            n_offers += (uint32_t)__popcll(__ballot(j != 0xffu));
            if (j != 0xffu) {
                const uint32_t slot = below(hash32((uint32_t)pid), (uint32_t)C);
                atomicMin(&cand[(int64_t)pend_id * C + slot], pack_key(__uint_as_float(pend_l[u]), pid, 1));
            }
        }
        pend_j = 0xffffffffu;
    };
    static_assert(OFFERS_PER_MEMBER <= 4, "pend_j packs one byte per class");

    for (;;) {
        const int* mid = midbuf + cur * NCOLS;
        const int nNew = P.nNew, nTot = P.nTot, nfn = P.nfn, nfo = P.nfo;
        const int nrt = (nNew + 15) >> 4, nct = (nTot + 15) >> 4;
        const PointPlan Pn = make_point(rc_n);

        // this point's member registers (loaded during the previous unit)
        const int my_id = id_r;
        const uint32_t my_thr = __float_as_uint(thr_r);
        const uint32_t my_hb = sig_bit(my_id, iter);
        if (lane <= nTot) {                                     // slot nTot <= NCOLS exists
            // word-major: lanes that read one word of their own signatures hit different banks
            sg[0 * SGLD + lane] = sg_r0.x; sg[1 * SGLD + lane] = sg_r0.y;
            sg[2 * SGLD + lane] = sg_r0.z; sg[3 * SGLD + lane] = sg_r0.w;
            sg[4 * SGLD + lane] = sg_r1.x; sg[5 * SGLD + lane] = sg_r1.y;
            sg[6 * SGLD + lane] = sg_r1.z; sg[7 * SGLD + lane] = sg_r1.w;
        }

        accv acc[NTILES];
#pragma unroll
        for (int q = 0; q < NTILES; ++q) acc[q] = accv{0, 0, 0, 0};
        intx4 accp = intx4{0, 0, 0, 0};                         // ELEM 1: <member, pivot>, <pivot, pivot>

        // uint8 -> signed bytes x - 128; words past the end of the row (zero-filled by the
        // predicated loads of the unaligned path) stay zero
        auto enc_u8 = [&](float4 f, int k0) -> float4 {
            uint32_t w[4] = {__float_as_uint(f.x), __float_as_uint(f.y), __float_as_uint(f.z), __float_as_uint(f.w)};
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = (VEC || k0 + 4 * c4 + j < d) ? (w[j] ^ 0x80808080u) : 0u;
            return float4{__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3])};
        };
        // ---- A: registers -> LDS (rows up to the end of the last loaded group of 8)
        auto store_slab = [&](int k0) {
            float* xdst = X + rsub * LD + 4 * c4;
            const bool inb = !VEC || k0 + 4 * c4 < d;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                if (RPW * i < nTot) {                           // uniform
                    float4 x = buf[i];
                    if (ELEM == 1) x = enc_u8(x, k0);
                    else if (ELEM == 2) x = sub_h2x4(x, pv);
                    else { x.x -= pv.x; x.y -= pv.y; x.z -= pv.z; x.w -= pv.w; }
                    if (!inb) x = float4{0.0f, 0.0f, 0.0f, 0.0f};
                    if constexpr (SPLIT) {
                        // the piece keeps its place: two words of hi halves, then two of lo halves
                        short4v hi, lo;
                        split_bf16(x, hi, lo);
                        const uint2 h2 = __builtin_bit_cast(uint2, hi), l2 = __builtin_bit_cast(uint2, lo);
                        *reinterpret_cast<uint4*>(xdst + RPW * i * LD) = uint4{h2.x, h2.y, l2.x, l2.y};
                    } else {
                        *reinterpret_cast<float4*>(xdst + RPW * i * LD) = x;
                    }
                }
            }
            if (ELEM == 1 && rsub == 0) {                       // the pivot's own row
                float4 x = enc_u8(pv, k0);
                if (!inb) x = float4{0.0f, 0.0f, 0.0f, 0.0f};
                *reinterpret_cast<float4*>(X + PIV_ROW + 4 * c4) = x;
            }
        };
        store_slab(0);
        for (int k0 = 0; k0 < d; k0 += DS) {
            const bool last = k0 + DS >= d;
            const int len = (d - k0) < DS ? (d - k0) : DS;
            const int len16 = (len + 15) & ~15;
            if (last && v_nx >= 0) {                            // next point's member ids
                const int m = member_of_slot(lane, s, rc_n);
                if (m >= 0) midbuf[(cur ^ 1) * NCOLS + m] = rid_n;
                if (lane >= Pn.nTot && lane < NCOLS) midbuf[(cur ^ 1) * NCOLS + lane] = (int)v_nx;
            }
            wave_lds_sync();
            // ---- B: issue the loads of the next unit (one call site)
            if (!last || v_nx >= 0) {
                const int* nmid = last ? midbuf + (cur ^ 1) * NCOLS : mid;
                const int n_tot = last ? Pn.nTot : nTot;
                const int64_t n_piv = last ? v_nx : v;
                // the slab first: whatever the compiler makes the wavefront wait for before it
                // reuses a prefetch register must not include the member gathers below
                issue_slab(nmid, n_tot, n_piv, last ? 0 : k0 + DS);
            }
            // ---- C: all Gram tiles of the point for this slab
            if constexpr (ELEM == 1) {
                for (int kk = 0; kk < len16; kk += 16) {
                    intx4 x[CT];
#pragma unroll
                    for (int t = 0; t < CT; ++t)
                        if (t < nct) x[t] = *reinterpret_cast<const intx4*>(X + (t * 16 + r16) * LD + 4 * kq + kk);
                    const intx4 xp = *reinterpret_cast<const intx4*>(X + PIV_ROW + 4 * kq + kk);
                    int q = 0;
#pragma unroll
                    for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                        for (int ct = rt; ct < CT; ++ct, ++q) {
                            if (ct < nct && (rt < nrt || rt == ct))
                                acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x[rt], x[ct], acc[q], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int ct = S16; ct < CT; ++ct, ++q) {
                        if (ct < nct) acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(x[ct], x[ct], acc[q], 0, 0, 0);
                    }
                    // column c of accp: members of tile c against the pivot; column CT: the pivot's norm
#pragma unroll
                    for (int ct = 0; ct <= CT; ++ct) {
                        if (ct < nct || ct == CT) {
                            const intx4 b = *reinterpret_cast<const intx4*>(X + (r16 == ct ? PIV_ROW : ZERO_ROW) + 4 * kq + kk);
                            accp = __builtin_amdgcn_mfma_i32_16x16x64_i8(ct < CT ? x[ct < CT ? ct : 0] : xp, b, accp, 0, 0, 0);
                        }
                    }
                }
            } else if constexpr (ELEM == 2) {
                for (int kk = 0; kk < len16; kk += 16) {
                    half8v x[CT];
#pragma unroll
                    for (int t = 0; t < CT; ++t)
                        if (t < nct) x[t] = *reinterpret_cast<const half8v*>(X + (t * 16 + r16) * LD + 4 * kq + kk);
                    int q = 0;
#pragma unroll
                    for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                        for (int ct = rt; ct < CT; ++ct, ++q) {
                            if (ct < nct && (rt < nrt || rt == ct))
                                acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x[rt], x[ct], acc[q], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int ct = S16; ct < CT; ++ct, ++q) {
                        if (ct < nct) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x[ct], x[ct], acc[q], 0, 0, 0);
                    }
                }
            } else if constexpr (SPLIT) {
                // fp32 rows, long: the centred values sit in LDS as two bf16 halves (split when the
                // slab is stored) and <a,b> is taken as hi.hi + hi.lo + lo.hi on
                // v_mfma_f32_16x16x16_bf16 -- three instructions of 8 cycles where fp32 needs four
                // of 32, for a relative error below 2^-13 of |a||b| in what the join compares
                for (int kk = 0; kk < len16; kk += 16) {
                    short4v xh[CT], xl[CT];
#pragma unroll
                    for (int t = 0; t < CT; ++t) {
                        if (t < nct) {
                            const uint4 p = *reinterpret_cast<const uint4*>(X + (t * 16 + r16) * LD + 4 * kq + kk);
                            xh[t] = __builtin_bit_cast(short4v, uint2{p.x, p.y});
                            xl[t] = __builtin_bit_cast(short4v, uint2{p.z, p.w});
                        }
                    }
                    int q = 0;
#pragma unroll
                    for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                        for (int ct = rt; ct < CT; ++ct, ++q) {
                            if (ct < nct && (rt < nrt || rt == ct)) {
                                acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xh[rt], xh[ct], acc[q], 0, 0, 0);
                                acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xh[rt], xl[ct], acc[q], 0, 0, 0);
                                acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xl[rt], xh[ct], acc[q], 0, 0, 0);
                            }
                        }
                    }
#pragma unroll
                    for (int ct = S16; ct < CT; ++ct, ++q) {
                        if (ct < nct) {
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xh[ct], xh[ct], acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xh[ct], xl[ct], acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(xl[ct], xh[ct], acc[q], 0, 0, 0);
                        }
                    }
                }
            } else {
            for (int kk = 0; kk < len16; kk += 16) {
                float4 x[CT];
#pragma unroll
                for (int t = 0; t < CT; ++t)
                    if (t < nct) x[t] = *reinterpret_cast<const float4*>(X + (t * 16 + r16) * LD + 4 * kq + kk);
                int q = 0;
#pragma unroll
                for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                    for (int ct = rt; ct < CT; ++ct, ++q) {
                        if (ct < nct && (rt < nrt || rt == ct)) {
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[rt].x, x[ct].x, acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[rt].y, x[ct].y, acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[rt].z, x[ct].z, acc[q], 0, 0, 0);
                            acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[rt].w, x[ct].w, acc[q], 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int ct = S16; ct < CT; ++ct, ++q) {
                    if (ct < nct) {
                        acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ct].x, x[ct].x, acc[q], 0, 0, 0);
                        acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ct].y, x[ct].y, acc[q], 0, 0, 0);
                        acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ct].z, x[ct].z, acc[q], 0, 0, 0);
                        acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ct].w, x[ct].w, acc[q], 0, 0, 0);
                    }
                }
            }
            }
            wave_lds_sync();
            if (!last) store_slab(k0 + DS);
        }
        // After the last Gram pass, when the accumulators are the only big thing left in
        // registers: the next point's thresholds and signatures, the list record of the point after
        // next, and the previous point's offers.  All of it completes under the norm /
        // distance-block / scan work below, which never waits for memory.
        if (v_nx >= 0) {
            issue_members(midbuf + (cur ^ 1) * NCOLS, Pn.nTot, v_nx);
            if (v_nx2 >= 0) { rc_n = plan[v_nx2]; rid_n = load_slot(v_nx2); }
        }
        send_offers();                                          // the previous point's

        // ---- member norms from the diagonal tiles: lane (r16, kq) holds rows 4kq..4kq+3 of
        // column r16, so the diagonal element sits in the lanes with r16 / 4 == kq
        {
            const int e = r16 & 3;
            int q = 0;
#pragma unroll
            for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                for (int ct = rt; ct < CT; ++ct, ++q) {
                    if (ct == rt && ct < nct && (r16 >> 2) == kq)
                        nrm[ct * 16 + r16] = acc_bits(e == 0 ? acc[q][0] : e == 1 ? acc[q][1] : e == 2 ? acc[q][2] : acc[q][3]);
                }
            }
#pragma unroll
            for (int ct = S16; ct < CT; ++ct, ++q) {
                if (ct < nct && (r16 >> 2) == kq)
                    nrm[ct * 16 + r16] = acc_bits(e == 0 ? acc[q][0] : e == 1 ? acc[q][1] : e == 2 ? acc[q][2] : acc[q][3]);
            }
        }
        wave_lds_sync();
        if constexpr (ELEM == 1) {
            // lane (c, kq), c < CT, holds <member 16c + 4kq + r, pivot> in accp[r]; column CT is <pivot, pivot>
            const uint32_t npiv = (uint32_t)__builtin_amdgcn_readlane(accp[0], CT);
            if (r16 < CT) {
                const uint4 nm = *reinterpret_cast<const uint4*>(nrm + r16 * 16 + 4 * kq);
                float4 o;
                o.x = (float)(nm.x + npiv - 2u * (uint32_t)accp[0]);
                o.y = (float)(nm.y + npiv - 2u * (uint32_t)accp[1]);
                o.z = (float)(nm.z + npiv - 2u * (uint32_t)accp[2]);
                o.w = (float)(nm.w + npiv - 2u * (uint32_t)accp[3]);
                *reinterpret_cast<float4*>(dpv + r16 * 16 + 4 * kq) = o;
            }
        }
        // ---- distance block D[row][col] over the slab storage; cells outside NEW x members are
        // +inf so the partner scan needs no bounds tests
        float* D = X;
        {
            const float inf = __uint_as_float(0x7f800000u);
            int q = 0;
#pragma unroll
            for (int rt = 0; rt < S16; ++rt) {
#pragma unroll
                for (int ct = rt; ct < CT; ++ct, ++q) {
                    if (ct < nct && rt < nrt) {
                        const int col = ct * 16 + r16;
                        const uint32_t nc = nrm[col];
                        const uint4 nr = *reinterpret_cast<const uint4*>(nrm + rt * 16 + 4 * kq);
                        const uint32_t nra[4] = {nr.x, nr.y, nr.z, nr.w};
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int row = rt * 16 + 4 * kq + r;
                            float l;
                            if constexpr (ELEM == 1) {
                                l = (float)(nra[r] + nc - 2u * (uint32_t)acc[q][r]);   // exact, >= 0
                            } else {
                                l = __uint_as_float(nra[r]) + __uint_as_float(nc) - 2.0f * acc[q][r];
                                if (METRIC == 1) l *= 0.5f;    // unit rows: 1 - <a,b> = |a-b|^2 / 2
                                l = nonneg(l);
                            }
                            D[row * LDD + col] = (row < nNew && col < nTot) ? l : inf;
                        }
                    }
                }
            }
            if (lane == 0) D[INF_CELL] = inf;
        }
        // ---- the pivot's reverse members hold v in their rows, so |x_m - x_v|^2 is already
        // known: offer them to v itself (closes v<-m edges into v->m without an extra distance)
        {
            const int m = lane;
            const bool rev = m < nTot && ((m >= nfn && m < nNew) || (m >= nNew + nfo));
            const uint32_t pthr = nTot < 64 ? (uint32_t)__builtin_amdgcn_readlane((int)my_thr, nTot & 63) : 0u;
            float l = 0.0f;
            uint32_t vw = 0xffffffffu;
            if (rev) {
                l = ELEM == 1 ? dpv[m] : __uint_as_float(nrm[m]);
                if (METRIC == 1) l *= 0.5f;
                l = nonneg(l);
                vw = sg[(my_hb >> 5) * SGLD + nTot];
            }
            const bool go = rev && __float_as_uint(l) < pthr && !((vw >> (my_hb & 31u)) & 1u);
            n_offers += (uint32_t)__popcll(__ballot(go));
            if (go) {
                const uint32_t slot = below(hash32((uint32_t)my_id), (uint32_t)C);
                atomicMin(&cand[v * C + slot], pack_key(l, my_id, 1));
            }
        }
        wave_lds_sync();
        // ---- selection: lane m scans member m's partners j (j uniform, 4 residue classes).
        // D[m][j] is stored at [lower tile][higher tile]: a lane walks its row (address + 1 per
        // partner) or, where the partner's tile is the lower one, the partner's column
        // (address + LDD).  OLD members pair with NEW partners only (column walk); lanes with
        // nothing to look at sit on the +inf cell.
        {
            const int m = lane;
            const bool ismem = m < nTot, isnew = m < nNew;
            const int mt = m >> 4;
            constexpr int NCLS = OFFERS_PER_MEMBER;            // residue classes = offers per member
            uint32_t bl[NCLS], bj[NCLS];
#pragma unroll
            for (int u = 0; u < NCLS; ++u) { bl[u] = ismem ? my_thr : 0u; bj[u] = 0xffffffffu; }
            const uint32_t* msig = sg + m;
            const int nNew4 = (nNew + 3) & ~3, nTot4 = (nTot + 3) & ~3;
            // four partners per step: their distances are read together, a wavefront-wide vote
            // skips groups in which nobody improves, then the four signature words are read
            // together -- two LDS round trips per four partners
            auto scan = [&](int jb, int je, int addr, int step) {
                for (int j0 = jb; j0 < je; j0 += 4) {
                    uint32_t l[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) l[u] = __float_as_uint(D[addr + u * step]);
                    addr += 4 * step;
                    bool any = false;
#pragma unroll
                    for (int u = 0; u < 4; ++u) any = any || (l[u] < bl[u % NCLS]);
                    if (__ballot(any) == 0ull) continue;
                    uint32_t hj[4], wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        hj[u] = (uint32_t)__builtin_amdgcn_readlane((int)my_hb, j0 + u);
                        wv[u] = msig[(hj[u] >> 5) * SGLD];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        // bitwise, not short-circuit: no branches around the signature words
                        const int idj = __builtin_amdgcn_readlane(my_id, j0 + u);
                        const uint32_t known = __builtin_amdgcn_ubfe(wv[u], hj[u] & 31u, 1u);
                        const bool ok = (l[u] < bl[u % NCLS]) & (idj != my_id) & (known == 0u);
                        bl[u % NCLS] = ok ? l[u] : bl[u % NCLS];
                        bj[u % NCLS] = ok ? (uint32_t)(j0 + u) : bj[u % NCLS];
                    }
                }
            };
            // NEW partners below 16: NEW members of tile 0 walk their row, everyone else the column
            {
                const int je = nNew4 < 16 ? nNew4 : 16;
                const bool row = isnew && mt == 0;
                scan(0, je, !ismem ? INF_CELL : row ? m * LDD : m, !ismem ? 0 : row ? 1 : LDD);
            }
            // NEW partners from 16: NEW members walk their row, OLD members the column
            if (nNew4 > 16)
                scan(16, nNew4, !ismem ? INF_CELL : isnew ? m * LDD + 16 : 16 * LDD + m, !ismem ? 0 : isnew ? 1 : LDD);
            // OLD partners: NEW members only
            if (nTot4 > nNew4)
                scan(nNew4, nTot4, isnew ? m * LDD + nNew4 : INF_CELL, isnew ? 1 : 0);
            pend_id = my_id;
            pend_j = 0u;
#pragma unroll
            for (int u = 0; u < NCLS; ++u) {
                pend_l[u] = bl[u];
                pend_j |= (bj[u] & 0xffu) << (8 * u);
            }
#pragma unroll
            for (int u = NCLS; u < 4; ++u) pend_j |= 0xffu << (8 * u);
            if constexpr (SPLIT) {
                // Is every chosen distance good enough?  (See split_untrusted.)  If not the point is
                // left to the fp32 kernel, which runs over the points listed here after this launch,
                // and none of its offers is sent from here.
                bool bad = false;
                const float n_m = __uint_as_float(nrm[m & (NCOLS - 1)]);
#pragma unroll
                for (int u = 0; u < NCLS; ++u) {
                    const float n_j = __uint_as_float(nrm[bj[u] & (NCOLS - 1)]);
                    bad = bad | ((bj[u] != 0xffffffffu) & split_untrusted(bl[u], n_m, n_j, METRIC == 1 ? 0.5f : 1.0f));
                }
                if (__ballot(bad) != 0ull) {
                    pend_j = 0xffffffffu;
                    if (lane == 0) redo[atomicAdd(redo_ctr, 1ull)] = (int32_t)v;
                }
            }
        }
        // ---- advance
        if (v_nx < 0) break;
        wave_lds_sync();
        pos += GW;
        v = v_nx;
        v_nx = v_nx2;
        v_nx2 = pos + 2 * GW < nact ? (int64_t)active[pos + 2 * GW] : -1;
        P = Pn;
        cur ^= 1;
    }
    send_offers();
    if (lane == 0 && n_offers) atomicAdd(offers_ctr, (u64)n_offers);
}

}  // namespace knng
