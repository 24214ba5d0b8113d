// Device code shared by the scan kernels of the RBE retrieval library (gfx950).
//
//   keys                 64-bit (ordered fp32 score, ~id) candidates
//   QueryRegs/load_query per-query words and coefficients
//   RowRegs/load_row     one lane's share of a 256-item row of a tile
//   score_item           Eq. 14 by XOR/popcount (Sec. 5.1), three scoring modes
//   stage_*1 / mstage_*  per-wave LDS queues of survivors -> global candidate lists
//
// Wavefronts are 64 wide.  One wave reads a "row" of 256 consecutive items per
// step: every plane with 16-byte loads per lane (1 KiB contiguous per wave
// instruction), every scale array with the matching 8- or 4-byte loads.  The
// four waves of a workgroup read the four rows of one 1024-item tile, which is
// one contiguous block of memory (rbe_layout.hpp).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rbe_layout.hpp"

namespace rbe {

constexpr int kBlock = 256;             // threads per workgroup of the scans
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kRow = 256;               // items one wave handles per step
constexpr int kItemsPerLane = 4;
static_assert(kRow * kWavesPerBlock == kTileItems, "a workgroup step covers one tile");

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------- keys
// A candidate is one 64-bit key: high word = the fp32 score mapped to an
// unsigned integer with the same order, low word = ~id.  Larger key = better
// under (score descending, id ascending); keys of distinct items never tie.
__device__ __forceinline__ uint32_t score_to_ordered(float s)
{
    s += 0.0f;  // -0.0 -> +0.0 so that equal scores give equal words
    const uint32_t b = __float_as_uint(s);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float ordered_to_score(uint32_t k)
{
    const uint32_t b = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(b);
}
__device__ __forceinline__ uint64_t make_key(float s, uint32_t id)
{
    return ((uint64_t)score_to_ordered(s) << 32) | (uint32_t)(~id);
}
// Threshold key 0 means "no lower bound yet".
__device__ __forceinline__ float threshold_score(uint64_t tau)
{
    return tau == 0 ? -__builtin_inff() : ordered_to_score((uint32_t)(tau >> 32));
}

// ---------------------------------------------------------------- per-query constants
// Query words are read as 32-bit halves; coef = (-2 c_0, ..., -2 c_{PQ-1}, dim * sum_i c_i)
// (unused in the dyadic modes).
template <int W, int PQ>
struct QueryRegs {
    uint32_t w[PQ][2 * W];
    float m2c[PQ];
    float bias;
};

template <int W, int PQ>
__device__ __forceinline__ QueryRegs<W, PQ> load_query(const uint32_t* __restrict__ qwords,
                                                       const float* __restrict__ qcoef, uint32_t q)
{
    QueryRegs<W, PQ> r;
    const uint32_t* pw = qwords + (size_t)q * PQ * 2 * W;
    const float* pc = qcoef + (size_t)q * (PQ + 1);
#pragma unroll
    for (int i = 0; i < PQ; ++i) {
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[i][h] = pw[i * 2 * W + h];
        r.m2c[i] = pc[i];
    }
    r.bias = pc[PQ];
    return r;
}

// A query's registers and its two masses, kept in LDS by the scans that take a few queries per row.  A load from
// global memory inside a loop that also stores cannot go through the scalar cache, so it becomes a vector load, and
// waiting for it waits for every vector load asked for before it -- the next row's prefetch included.  LDS reads are
// counted apart from those.
template <int W, int PQ>
struct alignas(16) QuerySlot {
    uint32_t w[PQ][2 * W];
    float m2c[PQ];
    float bias;
    float mass_x, mass_y;
};

// Fills slots[0 .. nq) from the query arrays (thread q fills slot q; nq <= blockDim.x) and synchronises the workgroup.
// All threads of the workgroup.
template <int W, int PQ>
__device__ __forceinline__ void stage_queries(QuerySlot<W, PQ>* slots, const uint32_t* __restrict__ qwords,
                                              const float* __restrict__ qcoef, const float* __restrict__ masses,
                                              uint32_t nq)
{
    const uint32_t q = threadIdx.x;
    if (q < nq) {
        const QueryRegs<W, PQ> r = load_query<W, PQ>(qwords, qcoef, q);
        QuerySlot<W, PQ>& d = slots[q];
#pragma unroll
        for (int i = 0; i < PQ; ++i) {
#pragma unroll
            for (int h = 0; h < 2 * W; ++h) d.w[i][h] = r.w[i][h];
            d.m2c[i] = r.m2c[i];
        }
        d.bias = r.bias;
        d.mass_x = masses[2 * q];
        d.mass_y = masses[2 * q + 1];
    }
    __syncthreads();
}

template <int W, int PQ>
__device__ __forceinline__ QueryRegs<W, PQ> slot_query(const QuerySlot<W, PQ>& s)
{
    QueryRegs<W, PQ> r;
#pragma unroll
    for (int i = 0; i < PQ; ++i) {
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[i][h] = s.w[i][h];
        r.m2c[i] = s.m2c[i];
    }
    r.bias = s.bias;
    return r;
}

// ---------------------------------------------------------------- one lane's share of a row
template <int W, int P, int S>
struct RowRegs {
    uint32_t w[P][kItemsPerLane][2 * W];     // plane words of the lane's 4 items
    float a[S > 0 ? S : 1][kItemsPerLane];   // their scales (S arrays)
};

// Item handled by (lane, m) relative to the row base.
template <int W>
__device__ __forceinline__ uint32_t lane_item(int lane, int m)
{
    if (W == 1) return (uint32_t)((m >> 1) * 128 + 2 * lane + (m & 1));
    return (uint32_t)(m * 64 + lane);
}

// Loads planes [J0, J1) of the wave's row (`wave` = 0..3) of the tile that starts at `tile`.
template <int W, int P, int S, int J0, int J1>
__device__ __forceinline__ void load_row_planes(RowRegs<W, P, S>& r, const char* __restrict__ tile, int wave, int lane)
{
    const TileGeom g{(uint32_t)W, (uint32_t)P, (uint32_t)S};
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes()) + (size_t)wave * kRow * W;
        if (W == 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + s * 128 + 2 * lane));
                r.w[j][2 * s][0] = v.x; r.w[j][2 * s][1] = v.y;
                r.w[j][2 * s + 1][0] = v.z; r.w[j][2 * s + 1][1] = v.w;
            }
        } else {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
#pragma unroll
                for (int h = 0; h < W / 2; ++h) {
                    const u32x4 v = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4*>(pj + (size_t)(m * 64 + lane) * W) + h);
                    r.w[j][m][4 * h + 0] = v.x; r.w[j][m][4 * h + 1] = v.y;
                    r.w[j][m][4 * h + 2] = v.z; r.w[j][m][4 * h + 3] = v.w;
                }
            }
        }
    }
}

// ... and its scale arrays [J0, J1).
template <int W, int P, int S, int J0 = 0, int J1 = S>
__device__ __forceinline__ void load_row_scales(RowRegs<W, P, S>& r, const char* __restrict__ tile, int wave, int lane)
{
    const TileGeom g{(uint32_t)W, (uint32_t)P, (uint32_t)S};
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        const float* sj = reinterpret_cast<const float*>(tile + g.scales_offset()) + j * kTileItems + wave * kRow;
        if (W == 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const f32x2 a = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sj + s * 128 + 2 * lane));
                r.a[j][2 * s] = a.x; r.a[j][2 * s + 1] = a.y;
            }
        } else {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) r.a[j][m] = __builtin_nontemporal_load(sj + m * 64 + lane);
        }
    }
}

// The whole row.
template <int W, int P, int S>
__device__ __forceinline__ void load_row(RowRegs<W, P, S>& r, const char* __restrict__ tile, int wave, int lane)
{
    load_row_planes<W, P, S, 0, P>(r, tile, wave, lane);
    load_row_scales<W, P, S>(r, tile, wave, lane);
}

// Score of the lane's item m against one query.  The popcounts are exact in every mode.
//
// kModeScaled:  s = sum_j a_j * ( bias + sum_i (-2 c_i) * popcount(Q_i ^ K_j) ), fp32 fused
//               multiply-adds, i inner, j outer.
// Dyadic modes: weights 2^-i (query) and 2^-j (item), the paper's residual weights
//               (Sec. 4.3), applied with shift-adds in Horner order as Sec. 5.1's footnote
//               suggests:  H = sum_j 2^(P-1-j) sum_i 2^(PQ-1-i) popcount(Q_i ^ K_j),
//               sum_ij 2^-(i+j) (d - 2 popcount) = 2^-(P+PQ-2) * ( d (2^P - 1)(2^PQ - 1) - 2 H ),
//               an exact integer times a power of two; kModeDyadicNorm multiplies it by the
//               item's single scale (one rounding).
template <int W, int P, int PQ, int MODE>
__device__ __forceinline__ float score_item(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m,
                                            const QueryRegs<W, PQ>& q)
{
    if (MODE == kModeScaled) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            float t = q.bias;
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                uint32_t pc = 0;
#pragma unroll
                for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(r.w[j][m][h] ^ q.w[i][h]);
                t = __fmaf_rn(q.m2c[i], (float)pc, t);
            }
            s = __fmaf_rn(r.a[j][m], t, s);
        }
        return s;
    } else {
        uint32_t H = 0;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            uint32_t h_j = 0;
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                uint32_t pc = 0;
#pragma unroll
                for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(r.w[j][m][h] ^ q.w[i][h]);
                h_j = (h_j << 1) + pc;
            }
            H = (H << 1) + h_j;
        }
        constexpr int kAll = 64 * W * ((1 << P) - 1) * ((1 << PQ) - 1);
        constexpr float kScale = 1.0f / (float)(1 << (P + PQ - 2));
        const float f = (float)(kAll - 2 * (int)H) * kScale;   // exact
        return MODE == kModeDyadicNorm ? f * r.a[0][m] : f;
    }
}

// Upper bound on score_item from planes 0 .. F-1 alone (1 <= F < P): whatever the other planes hold, the inner
// sum of plane j lies in [-M, M] with M = sum_d |sum_i c_i rho_i[d]|, the query's mass (the sum is qhat . rho_j
// and rho_j is a sign vector), and the scales are not negative.
//
// kModeScaled:  the first F steps exactly as score_item takes them, then  + (a_F + .. + a_{P-1}) * mass.x,  plus
//               (a_0 + .. + a_{P-1}) * mass.y for the roundings on either side.  The host supplies mass.x >= M
//               plus the rounding of the inner sums (which happen at magnitude d sum_i |c_i|, possibly far above
//               M), and mass.y = 2^-19 mass.x.
// Dyadic modes: integers.  Plane j contributes 2^(P-1-j) h_j to H and h_j >= h_min (the mismatch count of the
//               best possible plane), so H >= sum_{j<F} 2^(P-1-j) h_j + (2^(P-F) - 1) h_min; mass.x carries
//               h_min as an integer.  The conversion and the item's scale are monotone, so the bound is exact.
struct QueryMass { float x, y; };

// score_item taken in two steps: planes [0, F) first, the rest later, through exactly the same operations in
// the same order, so that finish_item(partial_item(..)) == score_item(..) bit for bit.
struct PartialScore { float s; uint32_t H; };

template <int W, int P, int PQ, int MODE, int J0, int J1>
__device__ __forceinline__ PartialScore score_planes(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m,
                                                     const QueryRegs<W, PQ>& q, PartialScore acc)
{
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        if constexpr (MODE == kModeScaled) {
            float t = q.bias;
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                uint32_t pc = 0;
#pragma unroll
                for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(r.w[j][m][h] ^ q.w[i][h]);
                t = __fmaf_rn(q.m2c[i], (float)pc, t);
            }
            acc.s = __fmaf_rn(r.a[j][m], t, acc.s);
        } else {
            uint32_t h_j = 0;
#pragma unroll
            for (int i = 0; i < PQ; ++i) {
                uint32_t pc = 0;
#pragma unroll
                for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(r.w[j][m][h] ^ q.w[i][h]);
                h_j = (h_j << 1) + pc;
            }
            acc.H = (acc.H << 1) + h_j;
        }
    }
    return acc;
}

template <int W, int P, int PQ, int MODE, int F>
__device__ __forceinline__ PartialScore partial_item(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m,
                                                     const QueryRegs<W, PQ>& q)
{
    return score_planes<W, P, PQ, MODE, 0, F>(r, m, q, PartialScore{0.0f, 0u});
}

template <int W, int P, int MODE>
__device__ __forceinline__ float score_value(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m, uint32_t H, float s,
                                             int PQ)
{
    if (MODE == kModeScaled) return s;
    const int all = 64 * W * ((1 << P) - 1) * ((1 << PQ) - 1);
    const float f = (float)(all - 2 * (int)H) * (1.0f / (float)(1 << (P + PQ - 2)));   // exact
    return MODE == kModeDyadicNorm ? f * r.a[0][m] : f;
}

template <int W, int P, int PQ, int MODE, int F>
__device__ __forceinline__ float finish_item(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m,
                                             const QueryRegs<W, PQ>& q, PartialScore part)
{
    const PartialScore full = score_planes<W, P, PQ, MODE, F, P>(r, m, q, part);
    return score_value<W, P, MODE>(r, m, full.H, full.s, PQ);
}

// The bound from a partial score (1 <= F < P).
template <int W, int P, int PQ, int MODE, int F>
__device__ __forceinline__ float bound_item(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m, PartialScore part,
                                            const QueryMass& mass)
{
    static_assert(F >= 1 && F < P, "a bound needs planes to compute and planes to skip");
    if constexpr (MODE == kModeScaled) {
        float tail = r.a[F][m];
#pragma unroll
        for (int j = F + 1; j < P; ++j) tail += r.a[j][m];
        float all = tail;
#pragma unroll
        for (int j = 0; j < F; ++j) all += r.a[j][m];
        return __fmaf_rn(all, mass.y, __fmaf_rn(tail, mass.x, part.s));
    } else {
        const uint32_t H = (part.H << (P - F)) + ((1u << (P - F)) - 1u) * __float_as_uint(mass.x);
        return score_value<W, P, MODE>(r, m, H, 0.0f, PQ);
    }
}

// The same bound with F = P - 1 and the last scale array (a_{P-1}; the single inverse-norm array of
// kModeDyadicNorm) replaced by its largest value over the wave's row, so that the stream need not carry that
// array either.  A product of an upper bound and a larger non-negative factor is an upper bound only while the
// first is positive; a score whose bound is negative is bounded by 0.
template <int W, int P, int PQ, int MODE>
__device__ __forceinline__ float bound_item_rowmax(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m, PartialScore part,
                                                   const QueryMass& mass, float amax)
{
    static_assert(P >= 2, "a bound needs planes to compute and a plane to skip");
    if constexpr (MODE == kModeScaled) {
        float all = amax;
#pragma unroll
        for (int j = 0; j < P - 1; ++j) all += r.a[j][m];
        return __fmaf_rn(all, mass.y, __fmaf_rn(amax, mass.x, part.s));
    } else {
        const uint32_t H = (part.H << 1) + __float_as_uint(mass.x);
        const int all = 64 * W * ((1 << P) - 1) * ((1 << PQ) - 1);
        const float f = (float)(all - 2 * (int)H) * (1.0f / (float)(1 << (P + PQ - 2)));   // exact
        if (MODE == kModeDyadic) return f;
        return f > 0.0f ? f * amax : 0.0f;
    }
}

// ---------------------------------------------------------------- per-wave candidate staging
// Survivors are first written to a queue in LDS that belongs to one wave (no
// atomics, no workgroup barrier), and moved to the query's global candidate list
// in bulk: one global atomic per flushed group instead of one per survivor.
constexpr int kStage = 512;  // entries per wave; an append adds at most 64

struct CandList {
    uint64_t* cand;   // [Q][cap]
    uint32_t* count;  // [Q], kCountStride words apart
    uint64_t* kmax;   // [Q], kKmaxStride words apart: largest key ever appended (the selection starts its radix descent below
                      //     the bits that the threshold and this maximum have in common)
    uint32_t cap;
};

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const uint64_t o = __shfl_xor(v, d);
        v = o > v ? o : v;
    }
    return v;
}

// One query per launch: a single queue per wave.
__device__ __forceinline__ void stage_flush1(uint64_t* s_keys, uint32_t fill, const CandList& a, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(a.count, fill);
    base = __shfl(base, 0);
    uint64_t mx = 0;
    for (uint32_t i0 = 0; i0 < fill; i0 += 64) {   // wave-uniform trip count
        const uint32_t i = i0 + (uint32_t)lane;
        if (i < fill) {
            const uint32_t pos = base + i;
            const uint64_t key = s_keys[i];
            mx = key > mx ? key : mx;
            if (pos < a.cap) a.cand[pos] = key;  // the count keeps running so that overflow is seen
        }
    }
    mx = wave_max_u64(mx);
    if (lane == 0 && mx > *reinterpret_cast<const volatile uint64_t*>(a.kmax)) atomicMax((unsigned long long*)a.kmax, (unsigned long long)mx);
    __builtin_amdgcn_wave_barrier();
}

// Must be reached by all lanes of the wave.  Returns the new fill level.
__device__ __forceinline__ uint32_t stage_append1(bool ok, uint64_t key, uint64_t* s_keys, uint32_t fill,
                                                  const CandList& a, int lane)
{
    const uint64_t mask = __ballot(ok);
    if (mask == 0) return fill;
    const uint32_t n = (uint32_t)__popcll(mask);
    if (fill + n > (uint32_t)kStage) {
        stage_flush1(s_keys, fill, a, lane);
        fill = 0;
    }
    if (ok) s_keys[fill + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull))] = key;
    return fill + n;
}

// Several queries per launch: the wave's queue is split into one sub-queue per query
// (`qcap` entries each, counters in LDS), so that a flush reserves a whole sub-queue in
// the query's global list with ONE atomic.  With a queue shared by all queries every group
// of 64 staged entries held up to 16 different queries and needed as many atomics; thousands
// of waves then serialised on the few per-query counters.
// Per-query counters (appended candidates, largest key) sit one to a 128-byte line: every wave of a scan adds to
// them, and atomics on one line are served one after the other (16 queries' counters in one line made the coarse
// levels of a 16-query search wait for 10^5 atomics in single file).
constexpr uint32_t kCountStride = 32;   // in uint32_t
constexpr uint32_t kKmaxStride = 16;    // in uint64_t

struct MultiStage {
    uint64_t* keys;    // [n_sub][qcap] this wave's LDS
    uint32_t* cnt;     // [n_sub + 1]: fill of each sub-queue, then a spare word (see mstage_append)
    uint32_t qcap;     // entries per sub-queue (power of two)
    uint32_t q_base;   // global query index of sub-queue 0
    uint32_t n_sub;    // sub-queues
};

// Moves the first n entries of sub-queue q to the global list.  All lanes of the wave.
__device__ __forceinline__ void mstage_flush_query(const MultiStage& ms, uint32_t q, uint32_t n, const CandList& a,
                                                   int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const uint32_t gq = ms.q_base + q;
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(a.count + gq * kCountStride, n);
    base = __shfl(base, 0);
    uint64_t mx = 0;
    if ((uint32_t)lane < n) {   // n <= qcap <= 64
        const uint32_t pos = base + (uint32_t)lane;
        mx = ms.keys[q * ms.qcap + (uint32_t)lane];
        if (pos < a.cap) a.cand[(size_t)gq * a.cap + pos] = mx;
    }
    mx = wave_max_u64(mx);
    // (most flushes do not raise the maximum: a plain look first saves the atomic)
    if (lane == 0 && mx > *reinterpret_cast<const volatile uint64_t*>(a.kmax + gq * kKmaxStride))
        atomicMax((unsigned long long*)(a.kmax + gq * kKmaxStride), (unsigned long long)mx);
    __builtin_amdgcn_wave_barrier();
}

// Queues `key` for sub-queue q of every lane with ok == true.  All lanes of the wave.
//
// Written without a branch on per-lane state around the wave-wide steps: the loop state is the wave-uniform mask
// `pend` of lanes still holding an entry, and lanes with nothing to draw increment a spare counter (index n_sub)
// instead of skipping the atomic.  With `if (ok) pos = atomicAdd(...)` in front of the loop the compiler split the
// loop by that condition and the two halves of the wave ran the ballots and flushes separately.
__device__ __forceinline__ void mstage_append(bool ok, uint64_t key, uint32_t q, const MultiStage& ms, const CandList& a,
                                              int lane)
{
    uint64_t pend = __ballot(ok);
    if (pend == 0) return;
    uint32_t pos = atomicAdd(&ms.cnt[ok ? q : ms.n_sub], 1u);
    for (;;) {
        const bool fits = ((pend >> lane) & 1ull) != 0 && pos < ms.qcap;
        if (fits) ms.keys[q * ms.qcap + pos] = key;
        pend &= ~__ballot(fits);
        if (pend == 0) break;
        // a sub-queue is full (its counter overshot): flush it, reset it, let its lanes draw again
        const int lead = __ffsll((long long)pend) - 1;
        const uint32_t q0 = __shfl(q, lead);
        mstage_flush_query(ms, q0, ms.qcap, a, lane);
        if (lane == lead) ms.cnt[q0] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const bool again = ((pend >> lane) & 1ull) != 0 && q == q0;
        const uint32_t drawn = atomicAdd(&ms.cnt[again ? q0 : ms.n_sub], 1u);
        pos = again ? drawn : pos;
    }
}

// End of kernel: flush whatever is left.  All lanes of the wave.
// Every sub-queue reserves its place in its query's list at once (lane q for sub-queue q: one round trip for all
// of them; taken one after the other, 64 returning atomics were 0.1 ms at the end of every wave), then the entries
// are copied queue by queue, and the largest keys are raised together at the end.
__device__ __forceinline__ void mstage_drain(const MultiStage& ms, const CandList& a, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint32_t n = 0;
    if ((uint32_t)lane < ms.n_sub) {
        n = ms.cnt[lane];
        n = n < ms.qcap ? n : ms.qcap;
    }
    const uint32_t gq_lane = ms.q_base + (uint32_t)lane;
    uint32_t base = 0;
    if (n) base = atomicAdd(a.count + gq_lane * kCountStride, n);
    uint64_t mx_lane = 0;
    uint64_t live = __ballot(n != 0);      // wave-uniform loop state
    while (live) {
        const int q = __ffsll((long long)live) - 1;
        live &= live - 1;
        const uint32_t n_q = __shfl(n, q), base_q = __shfl(base, q);
        uint64_t key = 0;
        if ((uint32_t)lane < n_q) {   // n_q <= qcap <= 64
            key = ms.keys[(uint32_t)q * ms.qcap + (uint32_t)lane];
            const uint32_t pos = base_q + (uint32_t)lane;
            if (pos < a.cap) a.cand[(size_t)(ms.q_base + (uint32_t)q) * a.cap + pos] = key;
        }
        const uint64_t mx = wave_max_u64(key);
        if (lane == q) mx_lane = mx;
    }
    if (n && mx_lane > *reinterpret_cast<const volatile uint64_t*>(a.kmax + gq_lane * kKmaxStride))
        atomicMax((unsigned long long*)(a.kmax + gq_lane * kKmaxStride), (unsigned long long)mx_lane);
}

// Sub-queue count for n queries: 16, 32 or 64 (power of two so that qcap is one too).
__device__ __forceinline__ uint32_t sub_queues_for(uint32_t n) { return n <= 16 ? 16u : (n <= 32 ? 32u : 64u); }

// ---------------------------------------------------------------- kernel arguments
struct ScanArgs {
    const char* tiles;        // physical tile 0
    Layout layout;
    uint64_t n_items;
    const uint32_t* qwords;   // [Q][PQ][2W]
    const float* qcoef;       // [Q][PQ+1], then the queries' masses [Q][2] (see bound_item)
    uint32_t n_queries;
    const uint64_t* tau;      // [Q] threshold keys
    CandList out;
    uint32_t p_begin, p_end;  // physical tile range this launch covers
    uint32_t* deep_rows;      // progressive scan: += rows whose planes 1.. had to be read
    uint32_t* deep_units;     // one-query progressive scans: += what the lanes asked for beyond the stream, in units of 8 bytes
    uint32_t* deep_pairs;     // scan_exact_batch_prog: += (query, row) pairs that were scored in full (may be null)
    const float* row_amax;    // [physical tile][4 rows] largest value of the last scale array over the row (one-query
                              // progressive scans; unused where there is no scale array)
    const uint32_t* hints;    // general scales: one-byte copies of the scale arrays 0 .. P-2 in lane order (scale_hints)
    int hint_base[3];         // ... and the exponent base of each array's hints
    const uint32_t* hints_last;  // three or more planes: one-byte copies of the LAST scale array, [tile][wave][lane] (a byte
                                 // per item of the lane), for the first stage of scan_exact_prog2_hint
    int hint_base_last;          // ... and their exponent base
    uint32_t stage_entries;   // several queries: LDS queue entries per wave (512..4096), split into sub-queues
    uint32_t q_slice;         // batch form of scan_exact: queries per workgroup row (blockIdx.y takes queries
                              // [y * q_slice, (y + 1) * q_slice)); 0 = every workgroup applies all queries.  Set by the launcher
    uint32_t calib_repeat;    // measurement only (batch form of scan_exact): every tile is scored this many more times
                              // without being loaded again, so the launch runs the scan's arithmetic free of memory traffic
};

// Hybrid scoring (fp32 query against RBE items, the paper's model m_5, Sec. 8.1): one query per
// launch; `lut` holds, for every byte position p of a plane and every byte value v,
// sum_{b<8} q[8p+b] * (bit b of v ? +1 : -1).
struct FqArgs {
    const char* tiles;
    Layout layout;
    uint64_t n_items;
    const float* lut;         // [8W][256]
    const uint64_t* tau_ptr;  // [1] threshold key of this query
    CandList out;             // this query's list (pointers already offset)
    uint32_t p_begin, p_end;
    QueryMass mass;           // progressive scan: x >= sum_d |q_d| plus the rounding of the table sums, y = 2^-19 x
    uint32_t* deep_rows;      // progressive scan: += rows whose last plane had to be read
    const float* row_amax;    // as in ScanArgs
    const uint32_t* hints;    // as in ScanArgs
    int hint_base[3];         // as in ScanArgs
    uint32_t* deep_units;     // as in ScanArgs (counted by scan_exact_fq_prog_hint)
    // scan_exact_fq_prog_hint<.., BIN = true>: the bound is formed from a 4-plane binary approximation qhat of the
    // query with XOR/popcounts instead of table sums
    const uint32_t* qwords;   // [4][2W] this query's approximation (pointers already offset)
    const float* qcoef;       // [5]
    QueryMass bmass;          // mass of qhat (query_mass)
    float resid;              // >= sum_d |q_d - qhat_d|
    const uint32_t* hints_last;  // as in ScanArgs (scan_exact_fq_prog2_hint)
    int hint_base_last;
};

// Batched scan on the matrix cores (rbe_batch.hip).
struct BatchArgs {
    const char* tiles;
    Layout layout;
    uint64_t n_items;
    const uint32_t* a_ops;    // operand 0: [query tile][plane copy][32-dim part][lane][4 dwords = 8 halves]: the scaled
                              // reconstructed queries in the A-operand order of v_mfma_f32_16x16x32_f16,
                              // dimensions permuted and weighted to match the kernel's B operand.
                              // operand 1: [query tile][64-dim part][lane][4 dwords = 16 bytes], eight-bit integers in
                              // the A-operand order of v_mfma_i32_16x16x64_i8; q_bias then holds the float whose bit
                              // pattern the accumulators start from
    uint32_t operand;         // 0: halves; 1: eight-bit integers (rescore = 1 only)
    const float* q_unscale;   // [Q] 2^-k: what a score formed from the scaled query is multiplied by
    const float* q_bias;      // [Q] minus the (plane-weighted) sum of the scaled query's components: where
                              // every accumulator starts
    const float* q_mass;      // [Q] what lets the first look leave the last plane out.  General scales: sum_d |v_d| of
                              // the scaled query, rounded up (no plane's qhat . rho exceeds it).  Dyadic modes: the most
                              // the last plane's term can add to the accumulator, 2^-(P-1) (sum_d |v_d| + sum_d v_d)
    const float* row_amax;    // [physical tile][4 rows] largest last scale of the row, and ...
    const float* row_asum;    // ... largest sum of an item's scales in the row (general scales)
    const uint32_t* hints;    // one-byte copies of the scale arrays 0 .. P-2 (see scale_hints), or null: integer operands
                              // and binary queries then take the lean stream (planes 0 .. P-2 and these copies)
    uint8_t hint_base[3];     // exponent base of each array's copies
    uint32_t lean;            // nonzero: the lean stream where the launch allows it (a level with a threshold worth pruning by)
    uint32_t* deep_units;     // += bytes / 8 that the lean stream's second looks asked for (may be null)
    uint32_t* look_stats;     // [2] += waves that ran, waves that gave up leaving the last plane out (may be null)
    const uint64_t* tau;      // [Q] threshold keys
    uint32_t n_queries;       // Q
    uint32_t q_begin;         // first query of this launch (a multiple of 16); it handles 16 or 32 from there
    // hi-half filter + exact rescoring (general scales): what the one-query scan scores with -- the staged binary
    // queries of the XOR/popcount scan (rescore = 1) or the byte tables of fp32 queries (rescore = 2) -- and the
    // bound on |true - filter score| per unit of sum_j a_j[item], in the scaled domain
    uint32_t rescore;         // 0: a_ops is exact (dyadic modes) and the contraction is the score
    uint32_t PQ;              // query planes (rescore = 1)
    const uint32_t* qwords;   // [Q][PQ][2W] (rescore = 1)
    const float* qcoef;       // [Q][PQ+1] (rescore = 1)
    const float* lut;         // [Q][8W][256] (rescore = 2)
    float margin;
    CandList out;
    uint32_t p_begin, p_end;
    uint32_t calib_repeat;    // measurement only: every row is staged and contracted this many more times without being
                              // loaded again (the kernel's instruction mix free of memory traffic)
};

struct GroupArgs {
    const char* tiles;
    Layout layout;
    uint64_t n_items;
    uint32_t rows_total;      // ceil(n_items / 256)
    uint32_t I;               // rows per super-block
    const uint32_t* qwords;   // [Q][PQ][2W]
    const float* qcoef;       // [Q][PQ+1]
    uint32_t q_begin, nq;     // queries handled by this launch (nq <= QB)
    const uint64_t* tau;
    CandList out;
    uint32_t v_begin, v_end;  // range of super-block ranks this launch covers
    uint32_t stride, skip;    // super-block = unit * stride; unit = rank, or the rank-th non-multiple of skip
};

}  // namespace rbe
