// Batched exact-mode scan on the matrix cores, for one word count W (-DRBE_W=1|2).
//
// For several queries per call the scoring is a dense contraction: with the
// query reconstructed as qhat = sum_i c_i b_q^i in R^d (Eq. 11 unrolled), Eq. 14 is
//     s(q, z) = sum_j a_j[z] * ( qhat . b_z^j ),
// i.e. per plane j a [queries x d] by [d x items] product whose right factor is
// +-1.  One wave handles a row of 256 items: it stages the row's plane words and
// scales in LDS and feeds v_mfma_f32_16x16x32_f16 with 16 queries x 16 items x 32
// dims per instruction.
//
// Item operand.  Turning bits into +-1.0 halves costs either a table read of 16 bytes
// per eight bits (random 16-byte reads: the LDS bank conflicts then bound the kernel) or
// two vector operations per pair of bits.  Instead the bits are used where they are: a
// half whose only set bit is bit 10 + t (t = 0..3) is the number 2^-14, 2^-13, 2^-11 or
// 2^-7, so ONE AND of the (rotated) plane word with 0x04000400 << t yields a dword of
// two operand halves, each 0 or val_t.  The query operand absorbs the rest: with
// rho = 2b - 1,
//     qhat . rho = sum_d (2 qhat_d / val_t(d)) * (b_d val_t(d))  -  sum_d qhat_d ,
// so the host stores 2 qhat_d / val_t in the order the kernel picks the bits and the
// accumulators start at -sum_d qhat_d.  The contraction is free to visit the dimensions
// in any order, which is what lets lane group g take bits (10 + 16h + t - 4g) mod 32 of
// every 32-bit part with one rotate and four ANDs.
//
// Schedule.  Vector instructions overlap with the MFMAs of the same SIMD only if they
// are independent of them, so the row is processed two item groups at a time in one
// straight-line block (the survivor test comes once per block): the expansion of the
// next group and the fp32 combination of the previous one issue while a group's MFMAs
// are in the pipeline.
//
// Precision.  qhat is scaled by a power of two into (-1, 1); products are exact and
// accumulate in fp32.  Dyadic modes: every operand is exact in one half, so the
// contraction is the score.  General scales: the operand is each component rounded to
// one half, the contraction is a filter with a margin the host computes, and whatever
// passes it is scored again in the arithmetic of the one-query scan, so the results
// carry no trace of the half precision.  The per-pair VALU work drops from ~58
// lane-ops to P fused multiply-adds and one compare; bit expansion is paid once per
// item, whatever the number of queries.
//
// Integer operands (OP = 1; general scales, binary and fp32 queries).  The filter needs no more than a few bits of the
// query: with qhat rounded to eight-bit integers T_d (times a power of two), v_mfma_i32_16x16x64_i8 contracts a
// whole 64-dimension plane per instruction -- half the matrix instructions -- and a dword of four operand BYTES
// comes out of one AND: lane group g shifts the plane's two 32-bit parts left by 6 - 2g, and the masks
// 0x40404040 / 0x80808080 then leave bits 2g / 2g + 1 of every byte as the byte values 64 / -128.  The query
// operand holds T_d against the 64s and -T_d / 2 against the -128s, the accumulators start at the bit pattern
// of the float 1.5 * 2^23 minus 32 sum_d T_d, and so they END as the bit pattern of the float
// 1.5 * 2^23 + 32 sum_d T_d rho_d: no conversion instruction; the constant leaves through the multiply-adds
// that apply the item's scales.  The rounding of the query and of those multiply-adds is part of the margin.
#include <type_traits>

#include "rbe_internal.hpp"

#ifndef RBE_W
#error "compile with -DRBE_W=1|2"
#endif

namespace rbe {

constexpr int kBatchStage = 256;   // staged survivors per wave (all sub-queues together)
constexpr int kMaxPlanes = 4;      // query planes (RBE_MAX_PLANES of the C interface)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

// Where the integer accumulators start, as a float: adding an integer n (|n| < 2^22) to its bit pattern gives the
// bit pattern of kAccBase + n.
constexpr float kAccBase = 12582912.0f;   // 1.5 * 2^23

// A wave works through its row of 256 items in SEG segments.  One segment (d = 64) keeps the loads widest; at
// d = 128 a whole row in flight costs 160 registers and 80 KB of LDS per workgroup with 4 planes -- one wave per
// SIMD -- so the row is taken in quarters of 64 items (one 16-byte plane load per lane and plane).
template <int W>
constexpr int row_segments() { return W == 2 ? 4 : 1; }

// Raw (still packed) segment as it comes from memory: 16-byte plane loads, matching scale loads.
template <int W, int P, int S>
struct RawRow {
    static constexpr int SEG = row_segments<W>();
    u32x4 pl[P][2 * W / SEG];              // W=1: items (2l,2l+1) and (128+2l,129+2l); W=2: item seg*64 + l
    float sc[S > 0 ? S : 1][kItemsPerLane / SEG];
};

// JP, JS: planes 0 .. JP-1 and scale arrays 0 .. JS-1 only (the lean stream leaves the last plane and the fp32 scales out).
template <int W, int P, int S, int JP = P, int JS = S>
__device__ __forceinline__ void load_raw(RawRow<W, P, S>& r, const char* __restrict__ tile, int wave, int seg, int lane)
{
    constexpr int SEG = row_segments<W>();
    const TileGeom g{(uint32_t)W, (uint32_t)P, (uint32_t)S};
#pragma unroll
    for (int j = 0; j < JP; ++j) {
        const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes()) + (size_t)wave * kRow * W;
#pragma unroll
        for (int s = 0; s < 2 * W / SEG; ++s) {
            const uint64_t* src = (W == 1) ? pj + s * 128 + 2 * lane
                                           : pj + (size_t)((seg * (4 / SEG) + s) * 64 + lane) * 2;
            r.pl[j][s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
        }
    }
#pragma unroll
    for (int j = 0; j < JS; ++j) {
        const float* sj = reinterpret_cast<const float*>(tile + g.scales_offset()) + j * kTileItems + wave * kRow;
        if (W == 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const f32x2 a = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sj + s * 128 + 2 * lane));
                r.sc[j][2 * s] = a.x; r.sc[j][2 * s + 1] = a.y;
            }
        } else {
#pragma unroll
            for (int m = 0; m < kItemsPerLane / SEG; ++m)
                r.sc[j][m] = __builtin_nontemporal_load(sj + (seg * (kItemsPerLane / SEG) + m) * 64 + lane);
        }
    }
}

// RS != 0 (general scales): the contraction runs with the hi half of the query only and is used as a filter -- its
// distance from the true score is at most a.margin * sum_j a_j[item] (the host adds up the part of every query
// component that the half does not hold) -- and what passes the filter is scored again exactly as the one-query
// scan scores it: RS = 1, binary queries, in the arithmetic of the XOR/popcount scan; RS = 2, fp32 queries, from
// the byte tables of the hybrid scan.  Half the MFMAs, and results that do not depend on how many queries share
// a call.
// CALIB: the measurement variant (BatchArgs::calib_repeat), a separate instantiation so that the scan proper carries
// none of it.
// OP: 0 = half operands (v_mfma_f32_16x16x32_f16), 1 = eight-bit integer operands (v_mfma_i32_16x16x64_i8).
// LEAN (integer operands, binary queries, two or more planes, an index that holds one-byte copies of its scales):
// the stream carries planes 0 .. P-2 and the one-byte copies of their scale arrays only -- 8W(P-1) + P-1 instead
// of (8W + 4)P bytes per item.  The first look is formed with the copies in place of the scales (its threshold
// lowered by the most the copies can be off, per row), over the whole segment; the blocks of 32 items in which
// some pair passes it then have their last plane and their fp32 scales read, all at once, and are looked at again
// with every plane and the true scales -- the look a wave takes that has given the first look up.  What passes
// that is scored exactly as before, so the results do not change.  A wave that looks again at more than half of
// its blocks goes back to whole rows.  Dyadic modes: there are no scale arrays to copy (the stored inverse norm,
// if any, stays in the stream); the stream leaves the last plane out -- 8W(P-1) [+ 4] instead of 8WP [+ 4] bytes
// per item -- and the first look is the one these modes take anyway (the most the last plane could add in its place).
template <int W, int P, int MODE, int NQT, int RS, int OP = 0, bool CALIB = false, bool LEAN = false>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu((NQT == 1 && W == 1 && P <= 3) ? 3 : 1)))
void scan_batch_mfma(const BatchArgs a)
{
    constexpr int S = scale_arrays(MODE, P);
    constexpr int KP = 2 * W;                          // 32-dimension parts of a plane
    constexpr bool kI8 = OP == 1;
    static_assert(!kI8 || (MODE == kModeScaled ? (RS == 1 || RS == 2) : RS == 0), "integer operands: the filter on general scales, the exact score in the dyadic modes");
    using acc_t = std::conditional_t<kI8, intx4, floatx4>;
    // General scales: one accumulator per plane (the item's a_j is applied afterwards); the query's hi half
    // filters.  Dyadic modes: the plane weight 2^-j is folded into a per-plane copy of the query operand, all
    // planes add into one accumulator, and the query (a short dyadic fraction) is exact in one half.
    constexpr bool kDy = MODE != kModeScaled;
    constexpr bool kRescore = !kDy;
    constexpr bool kBinary = kRescore && RS == 1;
    static_assert(kDy ? RS == 0 : (RS == 1 || RS == 2), "general scales filter and rescore; dyadic modes are exact");
    // Binary queries, two or more planes: the last plane (the smallest weights) stays out of the contraction; the
    // first look adds the most it could contribute instead (general scales: a_{P-1}[item] * sum_d |v_d|; dyadic
    // modes: a.q_mass), and only a block of items in which that leaves some pair above its threshold contracts the
    // last plane as well (dyadic modes: that is then the exact score) before anything is queued or scored exactly.
    // (With fp32 queries the saving did not pay for the extra table reads.)
    // (fp32 queries on the lean stream: its second phase is the all-planes look they take anyway, so the saving comes
    // without more survivors for the byte tables)
    constexpr bool kCanSkip = (kBinary || kDy || LEAN) && P >= 2;
    static_assert(!LEAN || (kI8 && P >= 2 && !CALIB), "the lean stream: integer operands, two or more planes");
    constexpr int PA = kDy ? P : 1;
    constexpr int PD_MAX = kDy ? 1 : P;
    constexpr int SEG = row_segments<W>();
    constexpr int kSegItems = kRow / SEG;
    __shared__ uint64_t s_pl[kWavesPerBlock][P][kSegItems * W];
    __shared__ float s_sc[kWavesPerBlock][S > 0 ? S : 1][kSegItems];
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kBatchStage];
    __shared__ uint32_t s_cnt_all[kWavesPerBlock][16 * NQT + 1];
    // what the survivor path needs of this launch's queries, close at hand: at one wave per SIMD (d = 128 with
    // 3 or 4 planes) a global read there would stall the whole SIMD
    __shared__ uint64_t s_tau[16 * NQT];
    __shared__ float s_unscale[16 * NQT];
    __shared__ uint32_t s_qw[kBinary ? 16 * NQT : 1][kMaxPlanes][2 * W];
    __shared__ float s_qc[kBinary ? 16 * NQT : 1][kMaxPlanes + 1];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 4;       // lane group: which 8 dims of a 32-dim part / which 4 queries of a tile
    const int col = lane & 15;     // item column inside a 16-item group, query row when loading A
    const MultiStage ms{s_keys_all[wave], s_cnt_all[wave], (uint32_t)kBatchStage / (16u * NQT), a.q_begin, 16u * NQT};
    if (lane < 16 * NQT) s_cnt_all[wave][lane] = 0;
    if (lane == 0) s_cnt_all[wave][16 * NQT] = 0;

    for (uint32_t ql = threadIdx.x; ql < 16u * NQT; ql += kBlock) {
        const uint32_t q = a.q_begin + ql;
        const bool live = q < a.n_queries;
        s_tau[ql] = live ? a.tau[q] : ~0ull;
        s_unscale[ql] = live ? a.q_unscale[q] : 1.0f;
        if (kBinary) {
            for (uint32_t i = 0; i <= a.PQ; ++i) s_qc[ql][i] = live ? a.qcoef[(size_t)q * (a.PQ + 1) + i] : 0.0f;
            for (uint32_t i = 0; i < a.PQ; ++i)
                for (int h = 0; h < 2 * W; ++h) s_qw[ql][i][h] = live ? a.qwords[((size_t)q * a.PQ + i) * 2 * W + h] : 0u;
        }
    }
    __syncthreads();

    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;

    // query operands (16 queries per tile, one half per component, KP parts), already in lane order
    // (integer operands: one 16-byte operand per 64-dimension part, [tile][part][lane])
    half8 A[kI8 ? 1 : NQT][PA][KP];
    intx4 A8[kI8 ? NQT : 1][PA][W];
    if constexpr (kI8) {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
            for (int pa = 0; pa < PA; ++pa)
#pragma unroll
                for (int kp = 0; kp < W; ++kp)
                    A8[qt][pa][kp] = __builtin_bit_cast(
                        intx4, reinterpret_cast<const u32x4*>(a.a_ops)[(((a.q_begin / 16 + qt) * PA + pa) * W + kp) * 64 + lane]);
    } else {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
            for (int pa = 0; pa < PA; ++pa)
#pragma unroll
                for (int kp = 0; kp < KP; ++kp) {
                    const u32x4 v =
                        reinterpret_cast<const u32x4*>(a.a_ops)[(((a.q_begin / 16 + qt) * PA + pa) * KP + kp) * 64 + lane];
                    A[qt][pa][kp] = __builtin_bit_cast(half8, v);
                }
    }
    // this lane's queries: tile qt, rows 4g .. 4g+3 (query a.q_begin + 16 qt + 4g + r).  Scores are formed in the
    // query's scaled domain (qhat * 2^k); thresholds are moved there, survivors are moved back (both exact).
    // Only what the common path needs stays in registers; the rare survivor path re-reads the rest.
    float taus[NQT][4], bias[NQT][4], qmass[NQT][4];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t q = a.q_begin + qt * 16 + 4 * g + r;
            taus[qt][r] = q < a.n_queries ? threshold_score(a.tau[q]) / a.q_unscale[q] : __builtin_inff();
            bias[qt][r] = q < a.n_queries ? a.q_bias[q] : 0.0f;
            qmass[qt][r] = (kCanSkip && q < a.n_queries) ? a.q_mass[q] : 0.0f;
        }

    const uint32_t i8_shift = 6u - 2u * (uint32_t)g;
    // the accumulators' start value, and what a finished accumulator reads as (integer operands: the same bits)
    auto acc_start = [&](int qt) {
        if constexpr (kI8)
            return intx4{__float_as_int(bias[qt][0]), __float_as_int(bias[qt][1]), __float_as_int(bias[qt][2]), __float_as_int(bias[qt][3])};
        else
            return floatx4{bias[qt][0], bias[qt][1], bias[qt][2], bias[qt][3]};
    };
    auto acc_value = [](const acc_t& d, int r) {
        if constexpr (kI8) return __int_as_float(d[r]);
        else return d[r];
    };
    // contracts one plane of one item group into the accumulators D[qt]
    auto contract_plane = [&](acc_t (&D)[NQT], const uint32_t (&part)[KP], int pa) {
        if constexpr (kI8) {
#pragma unroll
            for (int kp = 0; kp < W; ++kp) {
                // item bits as bytes: 0 or 64 (bit 2g of every byte), 0 or -128 (bit 2g + 1)
                const uint32_t lo = part[2 * kp] << i8_shift, hi = part[2 * kp + 1] << i8_shift;
                const intx4 B = {(int)(lo & 0x40404040u), (int)(lo & 0x80808080u), (int)(hi & 0x40404040u), (int)(hi & 0x80808080u)};
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt)
                    D[qt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A8[qt][pa][kp], B, D[qt], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
                // item bits as halves: 0, or the power of two whose only set bit is bit 10 + t
                const uint32_t xr = __builtin_rotateleft32(part[kp], 4u * (uint32_t)g);
                u32x4 bw;
#pragma unroll
                for (int t = 0; t < 4; ++t) bw[t] = xr & (0x04000400u << t);
                const half8 B = __builtin_bit_cast(half8, bw);
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt)
                    D[qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[qt][pa][kp], B, D[qt], 0, 0, 0);
            }
        }
    };

    bool skip_last = kCanSkip;              // wave-uniform
    uint32_t blocks_seen = 0, second_looks = 0;
    uint32_t lean_units = 0;
    RawRow<W, P, S> cur;
    int seg = 0;
    // LEAN: the lane's one-byte scale copies of the row in `cur` (word j = array j, byte m = the lane's item m), what
    // a copy decodes to, and the most the copies of arrays 0 .. P-2 can be off for scales below their smallest code
    constexpr int NW = P - 1 == 3 ? 4 : (P >= 2 ? P - 1 : 1);
    uint32_t hw[NW] = {};
    uint32_t hint_lo[3] = {0u, 0u, 0u};
    float hint_floor = 0.0f;
    if constexpr (LEAN && !kDy) {
#pragma unroll
        for (int j = 0; j < P - 1; ++j) {
            hint_lo[j] = (uint32_t)a.hint_base[j] << 5;
            hint_floor += __uint_as_float((uint32_t)a.hint_base[j] << 23);
        }
        hint_floor *= 1.0001f;
    }
    // loads a segment into `cur`: everything, or (LEAN, while the wave leaves the last plane out) the lean stream
    auto load_segment = [&](uint32_t tile_p, int sg, bool full) __attribute__((always_inline)) {
        if constexpr (LEAN) {
            if (!full) {
                if constexpr (kDy) {
                    load_raw<W, P, S, P - 1, S>(cur, a.tiles + (size_t)tile_p * tile_bytes, wave, sg, lane);
                    return;
                }
                load_raw<W, P, S, P - 1, 0>(cur, a.tiles + (size_t)tile_p * tile_bytes, wave, sg, lane);
                const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
                if constexpr (NW == 1) {
                    hw[0] = __builtin_nontemporal_load(src);
                } else if constexpr (NW == 2) {
                    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
                    hw[0] = v.x; hw[1] = v.y;
                } else {
                    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
                    hw[0] = v.x; hw[1] = v.y; hw[2] = v.z; hw[3] = v.w;
                }
                return;
            }
        }
        load_raw<W, P, S>(cur, a.tiles + (size_t)tile_p * tile_bytes, wave, sg, lane);
    };
    bool cur_full = !(LEAN && skip_last);     // wave-uniform: what `cur` holds
    load_segment(p, seg, cur_full);
    uint32_t calib_left = CALIB ? a.calib_repeat : 0u;   // measurement variant: segments to go through again without loading them
    for (;;) {
        const bool again = CALIB && calib_left != 0;     // wave-uniform
        const int segn = again ? seg : (seg + 1 == SEG ? 0 : seg + 1);
        const uint32_t pn = again ? p : (segn == 0 ? p + G : p);
        const bool has_next = again || pn < a.p_end;
        // stage the segment in this wave's LDS area, in item order
        const bool lean_now = LEAN && !cur_full;        // wave-uniform: this segment came by the lean stream
#pragma unroll
        for (int j = 0; j < P; ++j)
            if (j < P - 1 || !lean_now) {
#pragma unroll
                for (int s = 0; s < 2 * W / SEG; ++s) {
                    uint64_t* dst = (W == 1) ? &s_pl[wave][j][s * 128 + 2 * lane] : &s_pl[wave][j][(s * 64 + lane) * 2];
                    *reinterpret_cast<u32x4*>(dst) = cur.pl[j][s];
                }
            }
        if (lean_now && !kDy) {
            // (the one-byte copies stand where the first look expects the scales)
#pragma unroll
            for (int j = 0; j < P - 1; ++j)
#pragma unroll
                for (int m = 0; m < kItemsPerLane / SEG; ++m) {
                    const uint32_t c = (hw[j] >> (8 * (SEG == 1 ? m : seg))) & 255u;
                    s_sc[wave][j][SEG == 1 ? lane_item<W>(lane, m) : m * 64 + lane] = __uint_as_float((c + hint_lo[j]) << 18);
                }
        } else {
#pragma unroll
            for (int j = 0; j < S; ++j)
#pragma unroll
                for (int m = 0; m < kItemsPerLane / SEG; ++m)
                    s_sc[wave][j][SEG == 1 ? lane_item<W>(lane, m) : m * 64 + lane] = cur.sc[j][m];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // the staged copy is what the segment is worked from: its registers are free for the next segment, whose
        // loads stay in flight while this one is contracted (one register set instead of two)
        __builtin_amdgcn_sched_barrier(0);
        if (again) --calib_left;                // (the registers still hold the segment)
        else if (has_next) {
            cur_full = !(LEAN && skip_last);
            load_segment(pn, segn, cur_full);
        }

        const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow +
                                (uint64_t)seg * kSegItems;
        constexpr int U = 2;   // item groups per straight-line block
        // the segment's blocks, with the last plane left out of the first look (SKIP) or not: two copies of the
        // code, one of which runs per segment
        // PHASE 0: first look, second look where it is needed, survivors.  PHASE 1 (lean stream, SKIP): the first look
        // alone, with the one-byte copies for scales; returns the set of blocks to look at again.  PHASE 2 (lean
        // stream, not SKIP): the blocks of `only`, with everything read for them by now; they were counted in phase 1.
        auto blocks = [&](auto skip_tag, auto phase_tag, uint32_t only) -> uint32_t {
        // skip_tag: planes the first look leaves out -- 0, 1 (the last), or 2 (general scales, four planes, whole rows
        // streamed: the last plane by the row's largest last scale as before, the one before it by the item's own
        // scale, a_{P-2} mass_q added per pair in place of its multiply-add)
        constexpr int SKIPN = (int)decltype(skip_tag)::value;
        constexpr bool SKIP = SKIPN != 0;
        constexpr int PHASE = decltype(phase_tag)::value;
        static_assert(PHASE == 0 || (LEAN && SKIPN == (PHASE == 1 ? 1 : 0)), "phases of the lean stream");
        static_assert(SKIPN <= 1 || (MODE == kModeScaled && P >= 4), "two planes are left out on general scales with four planes only");
        constexpr int F = P - SKIPN;
        constexpr int PD = kDy ? 1 : F;
        static_assert(PD <= PD_MAX, "accumulators");
        uint32_t look_again = 0;
        // General scales, last plane left out: a pair can only reach its threshold if
        //     sum_{j<P-1} a_j D_j  >=  tau - a_{P-1} mass_q - margin sum_j a_j,
        // and with the row's largest last scale and largest scale sum the right-hand side is the same for every item
        // of the row: one subtraction per query and row instead of a multiply-add per pair.
        float row_taus[NQT][4];
        if constexpr (MODE == kModeScaled && F < P) {
            const float amax = a.row_amax[(size_t)p * kWavesPerBlock + wave], smax = a.row_asum[(size_t)p * kWavesPerBlock + wave];
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if constexpr (PHASE == 1) {
                        // the copies of arrays 0 .. P-2 add up to hs at most; each is within 2^-6 * 1.016 of its
                        // scale, or (a scale below the smallest code) above it by less than that code; a plane's
                        // contraction of the rounded query stays within mass_q + margin
                        const float hs = __fmaf_rn(1.016f, smax, hint_floor);
                        const float off = __fmaf_rn(0.015875f, hs, hint_floor);
                        row_taus[qt][r] = taus[qt][r] - 1.000001f * (__fmaf_rn(amax, qmass[qt][r], a.margin * hs) + off * (qmass[qt][r] + a.margin));
                    } else {
                        row_taus[qt][r] = taus[qt][r] - 1.000001f * __fmaf_rn(amax, qmass[qt][r], a.margin * smax);
                    }
                }
        }
        for (int cb = 0; cb < kSegItems / (16 * U); ++cb) {
            if (PHASE == 2 && !((only >> cb) & 1u)) continue;       // wave-uniform
            float s[U][NQT][4];
            bool any = false;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int item = 16 * (cb * U + u) + col;
                acc_t D[PD][NQT];
#pragma unroll
                for (int j = 0; j < PD; ++j)
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) D[j][qt] = acc_start(qt);
#pragma unroll
                for (int j = 0; j < F; ++j) {
                    uint32_t part[KP];
                    if constexpr (W == 1) {
                        const uint64_t w = s_pl[wave][j][item];
                        part[0] = (uint32_t)w; part[1] = (uint32_t)(w >> 32);
                    } else {
                        const u32x4 w = *reinterpret_cast<const u32x4*>(&s_pl[wave][j][item * 2]);
                        part[0] = w.x; part[1] = w.y; part[2] = w.z; part[3] = w.w;
                    }
                    contract_plane(D[kDy ? 0 : j], part, kDy ? j : 0);
                }
                float aj[P];
                float adj = 0.0f;      // filter slack of this item (general scales)
                if (MODE == kModeScaled) {
                    // first look without the last plane: its largest possible contribution and the filter slack
                    // are taken with the row's largest last scale and scale sum and sit in row_taus already
#pragma unroll
                    for (int j = 0; j < F; ++j) aj[j] = s_sc[wave][j][item];
                    if ((kRescore && F == P) || kI8) {
                        float asum = aj[0];
#pragma unroll
                        for (int j = 1; j < F; ++j) asum += aj[j];
                        if (kRescore && F == P) adj = a.margin * asum;
                        // integer operands: every accumulator reads kAccBase too high
                        if (kI8) adj = __fmaf_rn(-kAccBase, asum, adj);
                    }
                } else if (MODE == kModeDyadicNorm) {
                    aj[0] = s_sc[wave][0][item];
                }
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float v;
                        if (MODE == kModeScaled) {
                            v = adj;
#pragma unroll
                            for (int j = 0; j < F; ++j) v = __fmaf_rn(aj[j], acc_value(D[j][qt], r), v);
                            if constexpr (SKIPN == 2) {
                                // (kept apart from what the second look continues: s holds the chain, the test adds the bound)
                                s[u][qt][r] = v;
                                any |= (__fmaf_rn(s_sc[wave][P - 2][item], qmass[qt][r], v) >= row_taus[qt][r]);
                                continue;
                            }
                        } else {
                            // (integer operands: the accumulator reads kAccBase too high; all terms are integers
                            // below 2^24 in magnitude, so the sum in brackets and the addition are exact)
                            const float dv = acc_value(D[0][qt], r) + ((F < P ? qmass[qt][r] : 0.0f) - (kI8 ? kAccBase : 0.0f));
                            v = MODE == kModeDyadicNorm ? aj[0] * dv : dv;
                        }
                        s[u][qt][r] = v;
                        any |= (v >= ((MODE == kModeScaled && F < P) ? row_taus[qt][r] : taus[qt][r]));
                    }
            }
            bool go = __ballot(any) != 0;
            if (PHASE != 2) ++blocks_seen;
            if constexpr (PHASE == 1) {
                look_again |= go ? (1u << cb) : 0u;
                continue;
            }
            if (F < P && go) {
                ++second_looks;
                // second look, with the planes that the first look left out contracted too
                bool any2 = false;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int item = 16 * (cb * U + u) + col;
                    auto plane_words = [&](int j, uint32_t (&part)[KP]) {
                        if constexpr (W == 1) {
                            const uint64_t w = s_pl[wave][j][item];
                            part[0] = (uint32_t)w; part[1] = (uint32_t)(w >> 32);
                        } else {
                            const u32x4 w = *reinterpret_cast<const u32x4*>(&s_pl[wave][j][item * 2]);
                            part[0] = w.x; part[1] = w.y; part[2] = w.z; part[3] = w.w;
                        }
                    };
                    float a_item = 1.0f, adj2 = 0.0f;
                    if constexpr (MODE == kModeScaled) {
                        // general scales: the planes the first look left out, one after the other, each with the
                        // item's own scale (integer operands: each accumulator's start constant leaves with it)
#pragma unroll
                        for (int j = F; j < P; ++j) {
                            acc_t DL[NQT];
#pragma unroll
                            for (int qt = 0; qt < NQT; ++qt) DL[qt] = acc_start(qt);
                            uint32_t part[KP];
                            plane_words(j, part);
                            contract_plane(DL, part, 0);
                            const float a_j = s_sc[wave][j][item];
#pragma unroll
                            for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                                for (int r = 0; r < 4; ++r) {
                                    const float sofar = kI8 ? __fmaf_rn(-kAccBase, a_j, s[u][qt][r]) : s[u][qt][r];
                                    s[u][qt][r] = __fmaf_rn(a_j, acc_value(DL[qt], r), sofar);
                                }
                        }
                        float asum = s_sc[wave][P - 1][item];
#pragma unroll
                        for (int j = 0; j < P - 1; ++j) asum += s_sc[wave][j][item];
                        adj2 = a.margin * asum;          // the item's own filter slack
                    } else if constexpr (MODE == kModeDyadicNorm) {
                        a_item = s_sc[wave][0][item];
                    }
                    // dyadic modes: every plane again (the exact score)
                    acc_t DL[NQT];
                    if constexpr (kDy) {
#pragma unroll
                        for (int qt = 0; qt < NQT; ++qt) DL[qt] = acc_start(qt);
#pragma unroll
                        for (int j = 0; j < P; ++j) {
                            uint32_t part[KP];
                            plane_words(j, part);
                            contract_plane(DL, part, j);
                        }
                    }
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if constexpr (MODE == kModeScaled) {
                                s[u][qt][r] += adj2;
                            } else {
                                const float dv = acc_value(DL[qt], r) - (kI8 ? kAccBase : 0.0f);      // (exact)
                                s[u][qt][r] = MODE == kModeDyadicNorm ? a_item * dv : dv;
                            }
                            any2 |= (s[u][qt][r] >= taus[qt][r]);
                        }
                }
                go = __ballot(any2) != 0;
            }
            if (go) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint64_t id = row_id + (uint64_t)(16 * (cb * U + u) + col);
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            bool ok = (s[u][qt][r] >= taus[qt][r]) && (id < a.n_items);   // false for padding queries
                            const uint32_t ql = (uint32_t)(qt * 16 + 4 * g + r);
                            uint64_t key = 0;
                            if (ok) {
                                float score;
                                const uint32_t it = (uint32_t)(16 * (cb * U + u) + col);
                                if (kRescore && !kBinary) {
                                    // exact score of the hybrid scan: byte-table entries added in byte order
                                    const float(*lut)[256] =
                                        reinterpret_cast<const float(*)[256]>(a.lut + (size_t)(a.q_begin + ql) * (8 * W * 256));
                                    score = 0.0f;
                                    for (int j = 0; j < P; ++j) {
                                        const uint32_t* kw = reinterpret_cast<const uint32_t*>(&s_pl[wave][j][it * W]);
                                        float t = 0.0f;
                                        for (int h = 0; h < 2 * W; ++h) {
                                            const uint32_t w = kw[h];
                                            t += lut[4 * h + 0][w & 255u];
                                            t += lut[4 * h + 1][(w >> 8) & 255u];
                                            t += lut[4 * h + 2][(w >> 16) & 255u];
                                            t += lut[4 * h + 3][w >> 24];
                                        }
                                        score = __fmaf_rn(s_sc[wave][j][it], t, score);
                                    }
                                } else if (kBinary) {
                                    // exact score, in the arithmetic of the XOR/popcount scan (i inner, j outer)
                                    const float* qc = s_qc[ql];
                                    score = 0.0f;
                                    for (int j = 0; j < P; ++j) {
                                        const uint32_t* kw = reinterpret_cast<const uint32_t*>(&s_pl[wave][j][it * W]);
                                        float t = qc[a.PQ];
                                        for (uint32_t i = 0; i < a.PQ; ++i) {
                                            uint32_t pc = 0;
                                            for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(kw[h] ^ s_qw[ql][i][h]);
                                            t = __fmaf_rn(qc[i], (float)pc, t);
                                        }
                                        score = __fmaf_rn(s_sc[wave][j][it], t, score);
                                    }
                                    score += 0.0f;
                                } else {
                                    score = s[u][qt][r] * s_unscale[ql];
                                }
                                key = make_key(score, (uint32_t)id);
                                ok = key >= s_tau[ql];
                            }
                            mstage_append(ok, key, ql, ms, a.out, lane);
                        }
                }
            }
        }
        return look_again;
        };
        using phase0 = std::integral_constant<int, 0>;
        if constexpr (LEAN) {
            if (lean_now) {
                const uint32_t again_mask = blocks(std::true_type{}, std::integral_constant<int, 1>{}, 0u);
                if (again_mask) {
                    second_looks += (uint32_t)__builtin_popcount(again_mask);
                    lean_units += (uint32_t)__builtin_popcount(again_mask) * (32u * W + (kDy ? 0u : 16u * S));       // 8-byte units asked for beyond the stream
                    // the last plane and the fp32 scales of the blocks to look at again: every lane asks for what it
                    // would have staged of them, all loads in flight together, then they take their places in LDS
                    const char* tile = a.tiles + (size_t)p * tile_bytes;
                    const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + (P - 1) * geom.plane_bytes()) + (size_t)wave * kRow * W;
                    const float* sj0 = reinterpret_cast<const float*>(tile + geom.scales_offset()) + wave * kRow;
                    constexpr int SLOTS = 2 * W / SEG, PER = kItemsPerLane / SEG / SLOTS;     // item slots of a lane, items per slot
                    constexpr int GS = kDy ? 0 : S;       // scale arrays to read (dyadic modes: the norm came with the stream)
                    u32x4 gpl[SLOTS];
                    float gsc[GS > 0 ? GS : 1][SLOTS][PER];
                    bool mine[SLOTS];
#pragma unroll
                    for (int sl = 0; sl < SLOTS; ++sl) {
                        const int item0 = (W == 1) ? sl * 128 + 2 * lane : sl * 64 + lane;        // (first) item of the slot, in the segment
                        mine[sl] = ((again_mask >> (item0 >> 5)) & 1u) != 0u;
                        gpl[sl] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                        for (int j = 0; j < GS; ++j)
#pragma unroll
                            for (int e = 0; e < PER; ++e) gsc[j][sl][e] = 0.0f;
                        if (mine[sl]) {
                            const uint64_t* src = (W == 1) ? pj + sl * 128 + 2 * lane : pj + (size_t)((seg * (4 / SEG) + sl) * 64 + lane) * 2;
                            gpl[sl] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
#pragma unroll
                            for (int j = 0; j < GS; ++j) {
                                const float* sj = sj0 + j * kTileItems;
                                if constexpr (W == 1) {
                                    const f32x2 v = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sj + sl * 128 + 2 * lane));
                                    gsc[j][sl][0] = v.x; gsc[j][sl][1] = v.y;
                                } else {
                                    gsc[j][sl][0] = __builtin_nontemporal_load(sj + (seg * (kItemsPerLane / SEG) + sl) * 64 + lane);
                                }
                            }
                        }
                    }
#pragma unroll
                    for (int sl = 0; sl < SLOTS; ++sl)
                        if (mine[sl]) {
                            const int item0 = (W == 1) ? sl * 128 + 2 * lane : sl * 64 + lane;
                            *reinterpret_cast<u32x4*>(&s_pl[wave][P - 1][item0 * W]) = gpl[sl];
#pragma unroll
                            for (int j = 0; j < GS; ++j)
#pragma unroll
                                for (int e = 0; e < PER; ++e) s_sc[wave][j][item0 + e] = gsc[j][sl][e];
                        }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    blocks(std::false_type{}, std::integral_constant<int, 2>{}, again_mask);
                }
                if (second_looks * 2 > blocks_seen + 16) skip_last = false;
            } else {
                blocks(std::false_type{}, phase0{}, 0u);
            }
        } else if constexpr (kCanSkip) {
            constexpr int kLeaveOut = (MODE == kModeScaled && P >= 4) ? 2 : 1;       // planes the first look leaves out
            if (skip_last) blocks(std::integral_constant<int, kLeaveOut>{}, phase0{}, 0u);
            else blocks(std::false_type{}, phase0{}, 0u);
            // a wave that takes the second look for more than half of its blocks (a loose threshold, or weights
            // that do not decay) contracts every plane in the first look from then on
            if (skip_last && second_looks * 2 > blocks_seen + 16) skip_last = false;
        } else {
            blocks(std::false_type{}, phase0{}, 0u);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (!has_next) break;
        p = pn;
        seg = segn;
    }
    mstage_drain(ms, a.out, lane);
    if (LEAN && a.deep_units && lane == 0 && lean_units) atomicAdd(a.deep_units, lean_units);
    if (kCanSkip && a.look_stats && lane == 0 && blocks_seen) {
        atomicAdd(&a.look_stats[0], 1u);
        if (!skip_last) atomicAdd(&a.look_stats[1], 1u);
    }
}

namespace {
using BatchFn = void (*)(const BatchArgs);

template <int W, int P, int MODE>
BatchFn batch_fn_q(uint32_t nqt, uint32_t rescore, uint32_t operand, bool calib, bool lean)
{
    if (nqt != 1 && nqt != 2) return nullptr;
    if constexpr (MODE == kModeScaled) {
        if (operand == 1) {     // eight-bit integer operands
            if (rescore == 2) {
                if (calib) return nullptr;
                if constexpr (P >= 2)
                    if (lean && nqt == 1) return scan_batch_mfma<W, P, MODE, 1, 2, 1, false, true>;
                return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 2, 1> : scan_batch_mfma<W, P, MODE, 2, 2, 1>;
            }
            if (rescore != 1) return nullptr;
            if (calib) return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 1, 1, true> : scan_batch_mfma<W, P, MODE, 2, 1, 1, true>;
            // (one query tile per launch only: with two, 32 queries share every byte read, and the second set of
            // loads and the two-phase segment cost more than the bytes they save -- 1e9 items, 32 queries: 10.9 ms
            // with whole rows, 12.0 ms with the lean stream)
            if constexpr (P >= 2)
                if (lean && nqt == 1) return scan_batch_mfma<W, P, MODE, 1, 1, 1, false, true>;
            return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 1, 1> : scan_batch_mfma<W, P, MODE, 2, 1, 1>;
        }
        if (calib) return nullptr;      // the measurement variant is built for the default operands only
        if (rescore == 1) return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 1> : scan_batch_mfma<W, P, MODE, 2, 1>;
        if (rescore == 2) return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 2> : scan_batch_mfma<W, P, MODE, 2, 2>;
        return nullptr;
    } else {
        if (rescore != 0 || operand > 1 || calib) return nullptr;
        if (operand == 1) {
            if constexpr (P >= 2)
                if (lean && nqt == 1) return scan_batch_mfma<W, P, MODE, 1, 0, 1, false, true>;
            return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 0, 1> : scan_batch_mfma<W, P, MODE, 2, 0, 1>;
        }
        return nqt == 1 ? scan_batch_mfma<W, P, MODE, 1, 0> : scan_batch_mfma<W, P, MODE, 2, 0>;
    }
}

template <int W, int P>
BatchFn batch_fn_m(int mode, uint32_t nqt, uint32_t rescore, uint32_t operand, bool calib, bool lean)
{
    switch (mode) {
        case kModeScaled: return batch_fn_q<W, P, kModeScaled>(nqt, rescore, operand, calib, lean);
        case kModeDyadicNorm: return batch_fn_q<W, P, kModeDyadicNorm>(nqt, 0, operand, calib, lean);
        case kModeDyadic: return batch_fn_q<W, P, kModeDyadic>(nqt, 0, operand, calib, lean);
        default: return nullptr;
    }
}
}  // namespace

template <>
hipError_t launch_scan_batch_w<RBE_W>(const KernelSel& k, const BatchArgs& a, uint32_t n_query_tiles, uint32_t n_cu,
                                      uint32_t per_cu, hipStream_t st, uint32_t* grid_out)
{
    BatchFn fn = nullptr;
    // the lean stream: where the index holds one-byte copies of its scales (and so the rows' largest values too)
    const bool lean = a.lean != 0 && a.operand == 1 && a.calib_repeat == 0 &&
                      (k.mode == kModeScaled ? (a.hints != nullptr && a.row_amax != nullptr && a.row_asum != nullptr &&
                                                // (fp32 queries: 1e9 items, whole rows / lean stream, 3 queries 7.7 / 6.9 ms, 8 queries
                                                // 8.4 / 8.3, 16 queries 9.3 / 10.1: their second phase pays for the byte tables)
                                                (a.rescore == 1 || (a.rescore == 2 && a.n_queries <= 8)))
                                             : a.rescore == 0);
    switch (k.P) {
        case 1: fn = batch_fn_m<RBE_W, 1>(k.mode, n_query_tiles, a.rescore, a.operand, a.calib_repeat != 0, lean); break;
        case 2: fn = batch_fn_m<RBE_W, 2>(k.mode, n_query_tiles, a.rescore, a.operand, a.calib_repeat != 0, lean); break;
        case 3: fn = batch_fn_m<RBE_W, 3>(k.mode, n_query_tiles, a.rescore, a.operand, a.calib_repeat != 0, lean); break;
        case 4: fn = batch_fn_m<RBE_W, 4>(k.mode, n_query_tiles, a.rescore, a.operand, a.calib_repeat != 0, lean); break;
        default: break;
    }
    if (!fn) return hipErrorInvalidValue;
    if (a.p_end <= a.p_begin) return hipSuccess;
    if (per_cu == 0) {
        int nb = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kBlock, 0);
        if (e != hipSuccess) return e;
        per_cu = (uint32_t)(nb > 0 ? nb : 1);
    }
    const uint32_t units = a.p_end - a.p_begin;
    const uint32_t grid = units < n_cu * per_cu ? units : n_cu * per_cu;
    if (grid_out) *grid_out = grid;
    fn<<<dim3(grid), dim3(kBlock), 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace rbe
