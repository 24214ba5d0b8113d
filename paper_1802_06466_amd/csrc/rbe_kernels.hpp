// Device code of the RBE retrieval library for gfx950 (MI355X).
//
// Kernels:
//   scan_exact<W,P,PQ,SINGLE>  streaming exhaustive match (Eq. 14 by XOR/popcount,
//                              Sec. 5.1) fused with local selection: an item whose
//                              (score, id) key reaches the query's proven lower bound
//                              is staged in the wave's LDS queue and later appended
//                              to the query's global candidate list.
//   select_topk                per query: k-th largest candidate key by radix
//                              descent, compaction of the k best to the front of the
//                              list, new threshold, sorted output on the last round
//                              (the per-GPU global selection of Sec. 5 / Sec. 6).
//   scatter_chunk              load path: caller's [P][n][W] / [P][n] arrays -> tiles.
//   dense_popcounts / dense_scores / gather_scales / fold_cosine / init_state /
//   calib_copy                 small helpers.
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

constexpr int kBlock = 256;             // threads per workgroup of the scan
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kRow = 256;               // items one wave handles per step
constexpr int kItemsPerLane = 4;
static_assert(kRow * kWavesPerBlock == kTileItems, "a workgroup step covers one tile");

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
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
// Query words are read as 32-bit halves; coef = (-2 c_0, ..., -2 c_{PQ-1}, dim * sum_i c_i).
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

// ---------------------------------------------------------------- one lane's share of a row
template <int W, int P>
struct RowRegs {
    uint32_t w[P][kItemsPerLane][2 * W];  // plane words of the lane's 4 items
    float a[P][kItemsPerLane];            // their scales
};

// Item handled by (lane, m) relative to the row base.
template <int W>
__device__ __forceinline__ uint32_t lane_item(int lane, int m)
{
    if (W == 1) return (uint32_t)((m >> 1) * 128 + 2 * lane + (m & 1));
    return (uint32_t)(m * 64 + lane);
}

// Loads the wave's row (`wave` = 0..3) of the tile that starts at `tile`.
template <int W, int P>
__device__ __forceinline__ void load_row(RowRegs<W, P>& r, const char* __restrict__ tile, int wave, int lane)
{
    const TileGeom g{(uint32_t)W, (uint32_t)P};
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes()) + (size_t)wave * kRow * W;
        const float* sj = reinterpret_cast<const float*>(tile + g.scales_offset()) + j * kTileItems + wave * kRow;
        if (W == 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int it = s * 128 + 2 * lane;
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + it));
                r.w[j][2 * s][0] = v.x; r.w[j][2 * s][1] = v.y;
                r.w[j][2 * s + 1][0] = v.z; r.w[j][2 * s + 1][1] = v.w;
                const f32x2 a = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sj + it));
                r.a[j][2 * s] = a.x; r.a[j][2 * s + 1] = a.y;
            }
        } else {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                const int it = m * 64 + lane;
#pragma unroll
                for (int h = 0; h < W / 2; ++h) {
                    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + (size_t)it * W) + h);
                    r.w[j][m][4 * h + 0] = v.x; r.w[j][m][4 * h + 1] = v.y;
                    r.w[j][m][4 * h + 2] = v.z; r.w[j][m][4 * h + 3] = v.w;
                }
                r.a[j][m] = __builtin_nontemporal_load(sj + it);
            }
        }
    }
}

// s = sum_j a_j * ( bias + sum_i (-2 c_i) * popcount(Q_i ^ K_j) ), fp32, fused multiply-adds,
// i inner, j outer.  The popcounts are exact.
template <int W, int P, int PQ>
__device__ __forceinline__ float score_item(const RowRegs<W, P>& r, int m, const QueryRegs<W, PQ>& q)
{
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
}

// ---------------------------------------------------------------- per-wave candidate staging
// Survivors are first written to a queue in LDS that belongs to one wave (no
// atomics, no workgroup barrier), and moved to the query's global candidate list
// in bulk: one global atomic per flushed group instead of one per survivor.
constexpr int kStage = 512;  // entries per wave; an append adds at most 64

struct ScanArgs {
    const char* tiles;        // physical tile 0
    Layout layout;
    uint64_t n_items;
    const uint32_t* qwords;   // [Q][PQ][2W]
    const float* qcoef;       // [Q][PQ+1]
    uint32_t n_queries;
    const uint64_t* tau;      // [Q] threshold keys
    uint64_t* cand;           // [Q][cap]
    uint32_t* count;          // [Q]
    uint32_t cap;
    uint32_t p_begin, p_end;  // physical tile range this launch covers
};

template <bool SINGLE>
__device__ __forceinline__ void stage_flush(uint64_t* s_keys, uint8_t* s_q, uint32_t fill, const ScanArgs& a, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (SINGLE) {
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(a.count, fill);
        base = __shfl(base, 0);
        for (uint32_t i = lane; i < fill; i += 64) {
            const uint32_t pos = base + i;
            if (pos < a.cap) a.cand[pos] = s_keys[i];  // the count keeps running so that overflow is seen
        }
    } else {
        for (uint32_t i0 = 0; i0 < fill; i0 += 64) {
            const uint32_t i = i0 + lane;
            const bool valid = i < fill;
            const uint64_t key = valid ? s_keys[i] : 0;
            const uint32_t myq = valid ? s_q[i] : 0xFFFFFFFFu;
            uint64_t todo = __ballot(valid);
            while (todo) {  // one round per distinct query present in this group of 64
                const int lead = __ffsll((long long)todo) - 1;
                const uint32_t q0 = __shfl(myq, lead);
                const uint64_t sel = __ballot(valid && myq == q0);
                uint32_t base = 0;
                if (lane == lead) base = atomicAdd(a.count + q0, (uint32_t)__popcll(sel));
                base = __shfl(base, lead);
                if (valid && myq == q0) {
                    const uint32_t pos = base + (uint32_t)__popcll(sel & ((1ull << lane) - 1ull));
                    if (pos < a.cap) a.cand[(size_t)q0 * a.cap + pos] = key;
                }
                todo &= ~sel;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Must be reached by all lanes of the wave.  Returns the new fill level.
template <bool SINGLE>
__device__ __forceinline__ uint32_t stage_append(bool ok, uint64_t key, uint32_t q, uint64_t* s_keys, uint8_t* s_q,
                                                 uint32_t fill, const ScanArgs& a, int lane)
{
    const uint64_t mask = __ballot(ok);
    if (mask == 0) return fill;
    const uint32_t n = (uint32_t)__popcll(mask);
    if (fill + n > (uint32_t)kStage) {
        stage_flush<SINGLE>(s_keys, s_q, fill, a, lane);
        fill = 0;
    }
    if (ok) {
        const uint32_t pos = fill + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        s_keys[pos] = key;
        if (!SINGLE) s_q[pos] = (uint8_t)q;
    }
    return fill + n;
}

// Scores the lane's 4 items of `cur` against one query and queues the survivors.
template <int W, int P, int PQ, bool SINGLE>
__device__ __forceinline__ uint32_t score_and_stage(const RowRegs<W, P>& cur, const QueryRegs<W, PQ>& qr, uint64_t tau,
                                                    float taus, uint32_t q, uint32_t p, int wave, int lane,
                                                    uint64_t* s_keys, uint8_t* s_q, uint32_t fill, const ScanArgs& a)
{
    float s[kItemsPerLane];
    bool any = false;
#pragma unroll
    for (int m = 0; m < kItemsPerLane; ++m) {
        s[m] = score_item<W, P, PQ>(cur, m, qr);
        any |= (s[m] >= taus);
    }
    if (__ballot(any)) {   // rare: at least one lane of the wave has a survivor
        const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow;
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            const uint64_t id = row_id + lane_item<W>(lane, m);
            bool ok = (s[m] >= taus) && (id < a.n_items);
            uint64_t key = 0;
            if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
            fill = stage_append<SINGLE>(ok, key, q, s_keys, s_q, fill, a, lane);
        }
    }
    return fill;
}

// Streaming exhaustive match + local selection over physical tiles
// [p_begin, p_end).  Persistent workgroups: workgroup b takes tiles p_begin + b,
// + grid, ....
// SINGLE (one query, HBM-bound): the query lives in SGPRs and the next tile's loads
// are issued before the current one is scored (register double buffering).
// Batch (VALU-bound): one tile in registers, all queries applied to it; the next
// query's words and coefficients are fetched by scalar loads while the current
// one is being applied, and memory latency is covered by the other resident waves.
template <int W, int P, int PQ, bool SINGLE>
__global__ __launch_bounds__(kBlock) void scan_exact(const ScanArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ uint8_t s_q_all[SINGLE ? 1 : kWavesPerBlock][SINGLE ? 1 : kStage];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    uint8_t* s_q = SINGLE ? s_q_all[0] : s_q_all[wave];
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    uint32_t fill = 0;

    if (SINGLE) {
        const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
        const uint64_t tau0 = a.tau[0];
        const float taus0 = threshold_score(tau0);
        RowRegs<W, P> cur, nxt;
        load_row<W, P>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
        for (;;) {
            const uint32_t pn = p + G;
            const bool has_next = pn < a.p_end;
            if (has_next) load_row<W, P>(nxt, a.tiles + (size_t)pn * tile_bytes, wave, lane);
            fill = score_and_stage<W, P, PQ, SINGLE>(cur, q0, tau0, taus0, 0, p, wave, lane, s_keys, s_q, fill, a);
            if (!has_next) break;
            cur = nxt;
            p = pn;
        }
    } else {
        const uint32_t nq = a.n_queries;
        for (; p < a.p_end; p += G) {
            RowRegs<W, P> cur;
            load_row<W, P>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
            QueryRegs<W, PQ> qn = load_query<W, PQ>(a.qwords, a.qcoef, 0);
            uint64_t tau_n = a.tau[0];
            for (uint32_t q = 0; q < nq; ++q) {
                const QueryRegs<W, PQ> qr = qn;
                const uint64_t tau = tau_n;
                if (q + 1 < nq) {
                    qn = load_query<W, PQ>(a.qwords, a.qcoef, q + 1);
                    tau_n = a.tau[q + 1];
                }
                fill = score_and_stage<W, P, PQ, SINGLE>(cur, qr, tau, threshold_score(tau), q, p, wave, lane,
                                                         s_keys, s_q, fill, a);
            }
        }
    }
    if (fill) stage_flush<SINGLE>(s_keys, s_q, fill, a, lane);
}

// ---------------------------------------------------------------- near-lossless local selection
// Algorithm 1 with a priority queue of length 1: thread y of block x visits
// items x*256*I + y, + 256, ... (I of them) and forwards only its best one.  In
// rows of 256 items: "super-block" x is rows [x*I, (x+1)*I), and the group of an
// item is (super-block, column = id mod 256).  One workgroup takes one
// super-block per step; wave w scans rows w, w+4, ... keeping, per lane and
// column, the best (score, row) seen; the four waves' partial winners are merged
// through LDS and the group winners that reach the threshold are queued like the
// survivors of the exact scan.
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
    uint64_t* cand;
    uint32_t* count;
    uint32_t cap;
    uint32_t v_begin, v_end;  // range of super-block ranks this launch covers
    uint32_t stride, skip;    // super-block = nth_non_multiple-style unit * stride (skip == 0: unit = rank)
};

// Physical address of logical row `row` (wave-uniform).
__device__ __forceinline__ const char* row_tile(const GroupArgs& a, const TileGeom& g, uint32_t row)
{
    return a.tiles + (size_t)tile_to_phys(a.layout, row >> 2) * g.tile_bytes();
}

template <int W, int P, int PQ, int QB>
__global__ __launch_bounds__(kBlock) void scan_groupmax(const GroupArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ uint8_t s_q_all[kWavesPerBlock][kStage];
    __shared__ float s_best[QB][kWavesPerBlock][kItemsPerLane][64];
    __shared__ uint32_t s_brow[QB][kWavesPerBlock][kItemsPerLane][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint64_t* s_keys = s_keys_all[wave];
    uint8_t* s_q = s_q_all[wave];
    const TileGeom geom{(uint32_t)W, (uint32_t)P};
    const float ninf = -__builtin_inff();

    // the staging/flush helpers take ScanArgs: only the candidate-list fields are used
    ScanArgs sa{};
    sa.cand = a.cand; sa.count = a.count; sa.cap = a.cap;

    QueryRegs<W, PQ> qr[QB];
    uint64_t tau[QB];
    float taus[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const uint32_t q = a.q_begin + (b < (int)a.nq ? b : 0);
        qr[b] = load_query<W, PQ>(a.qwords, a.qcoef, q);
        tau[b] = a.tau[q];
        taus[b] = threshold_score(tau[b]);
    }

    uint32_t fill = 0;
    for (uint32_t v = a.v_begin + blockIdx.x; v < a.v_end; v += gridDim.x) {
        const uint32_t x = (a.skip ? nth_non_multiple(v, a.skip) : v) * a.stride;
        const uint32_t row0 = x * a.I;
        const uint32_t n_rows = a.rows_total - row0 < a.I ? a.rows_total - row0 : a.I;

        float best[QB][kItemsPerLane];
        uint32_t brow[QB][kItemsPerLane];
#pragma unroll
        for (int b = 0; b < QB; ++b)
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) { best[b][m] = ninf; brow[b][m] = 0xFFFFFFFFu; }

        uint32_t r = (uint32_t)wave;
        RowRegs<W, P> cur, nxt;
        if (r < n_rows) load_row<W, P>(cur, row_tile(a, geom, row0 + r), (int)((row0 + r) & 3), lane);
        while (r < n_rows) {
            const uint32_t rn = r + kWavesPerBlock;
            if (rn < n_rows) load_row<W, P>(nxt, row_tile(a, geom, row0 + rn), (int)((row0 + rn) & 3), lane);
            const uint64_t row_id = (uint64_t)(row0 + r) * kRow;
            const bool tail = row_id + kRow > a.n_items;   // only the corpus' last row can hold missing slots
#pragma unroll
            for (int b = 0; b < QB; ++b) {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    float s = score_item<W, P, PQ>(cur, m, qr[b]) + 0.0f;
                    if (tail && row_id + lane_item<W>(lane, m) >= a.n_items) s = ninf;
                    // rows are visited in ascending order: ">" keeps the lowest id among equal scores
                    if (s > best[b][m]) { best[b][m] = s; brow[b][m] = r; }
                }
            }
            if (rn < n_rows) cur = nxt;
            r = rn;
        }

        // merge the four waves' partial winners: wave w finalises item slot m = w of every lane
#pragma unroll
        for (int b = 0; b < QB; ++b)
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) { s_best[b][wave][m][lane] = best[b][m]; s_brow[b][wave][m][lane] = brow[b][m]; }
        __syncthreads();
        for (int b = 0; b < QB; ++b) {
            if (b >= (int)a.nq) break;
            float ws = ninf;
            uint32_t wr = 0xFFFFFFFFu;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                const float s = s_best[b][w][wave][lane];
                const uint32_t rr = s_brow[b][w][wave][lane];
                if (rr != 0xFFFFFFFFu && (wr == 0xFFFFFFFFu || s > ws || (s == ws && rr < wr))) { ws = s; wr = rr; }
            }
            bool ok = (wr != 0xFFFFFFFFu) && (ws >= taus[b]);
            uint64_t key = 0;
            if (ok) {
                const uint64_t id = (uint64_t)(row0 + wr) * kRow + lane_item<W>(lane, wave);
                key = make_key(ws, (uint32_t)id);
                ok = key >= tau[b];
            }
            fill = stage_append<false>(ok, key, a.q_begin + b, s_keys, s_q, fill, sa, lane);
        }
        __syncthreads();
    }
    if (fill) stage_flush<false>(s_keys, s_q, fill, sa, lane);
}

// ---------------------------------------------------------------- selection
constexpr int kSelBlock = 1024;
constexpr int kSelMaxK = 4096;
constexpr int kSelBins = 2048;      // 11-bit digits
constexpr int kSelBound = 1024;     // boundary keys finished by an LDS sort
constexpr int kSelUnroll = 8;

enum : uint32_t { kStatusOverflow = 1u };

struct SelectArgs {
    uint64_t* cand;      // [Q][cap], in/out: on return the best min(n,k) keys at the front
    uint32_t* count;     // [Q] in: appended so far; out: number kept
    uint64_t* tau;       // [Q] out: k-th best key once at least k candidates exist
    uint32_t cap;
    uint32_t k;
    uint32_t* status;    // bit 0 set if any query's count exceeded cap
    uint32_t* count_seen;  // [Q] out: candidate count before selection (for statistics)
    int final_pass;
    int64_t* ids_out;    // [Q][k]   (final pass; sorted)
    float* scores_out;   // [Q][k]
};

// Inclusive prefix sum over the 1024 threads of the select workgroup.
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t* s_wave /*[16]*/)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint32_t add = 0;
    for (int w = 0; w < wave; ++w) add += s_wave[w];
    __syncthreads();
    return incl + add;
}

// Bitonic sort of `pow2` keys in LDS, descending.  All threads of the workgroup call it.
__device__ __forceinline__ void bitonic_desc(uint64_t* keys, uint32_t pow2)
{
    for (uint32_t size = 2; size <= pow2; size <<= 1) {
        for (uint32_t st = size >> 1; st > 0; st >>= 1) {
            for (uint32_t i = threadIdx.x; i < pow2 / 2; i += kSelBlock) {
                const uint32_t lo = 2 * i - (i & (st - 1));
                const uint32_t hi = lo + st;
                const bool desc = ((lo & size) == 0);
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
            __syncthreads();
        }
    }
}

// One workgroup per query.
__global__ __launch_bounds__(kSelBlock) void select_topk(const SelectArgs a)
{
    __shared__ uint64_t skeys[kSelMaxK];    // keys known to be kept
    __shared__ uint64_t sbound[kSelBound];  // keys of the boundary bin
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t s_wave[16];
    __shared__ uint64_t s_and, s_or;
    __shared__ uint32_t s_digit, s_remaining, s_binpop, s_fill_keep, s_fill_bound;

    const uint32_t q = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    uint64_t* keys = a.cand + (size_t)q * a.cap;
    const uint32_t appended = a.count[q];
    const uint32_t n = appended < a.cap ? appended : a.cap;
    const uint32_t k = a.k;
    if (tid == 0) {
        a.count_seen[q] = appended;
        if (appended > a.cap) atomicOr(a.status, kStatusOverflow);
    }

    uint32_t m;  // number of keys kept
    if (n <= k) {
        // everything is kept; nothing to prune.  Only the final round needs them sorted.
        m = n;
        if (!a.final_pass) return;
        for (uint32_t i = tid; i < n; i += kSelBlock) skeys[i] = keys[i];
    } else {
        m = k;
        // ---- bits that differ between any two keys
        uint64_t vand = ~0ull, vor = 0;
        for (uint32_t base = 0; base < n; base += kSelBlock * kSelUnroll) {
            uint64_t kk[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const uint32_t i = base + u * kSelBlock + tid;
                kk[u] = i < n ? keys[i] : 0;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const uint32_t i = base + u * kSelBlock + tid;
                if (i < n) { vand &= kk[u]; vor |= kk[u]; }
            }
        }
        if (tid == 0) { s_and = ~0ull; s_or = 0; }
        __syncthreads();
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            vand &= __shfl_xor(vand, d);
            vor |= __shfl_xor(vor, d);
        }
        if ((tid & 63) == 0) { atomicAnd((unsigned long long*)&s_and, (unsigned long long)vand); atomicOr((unsigned long long*)&s_or, (unsigned long long)vor); }
        __syncthreads();
        const uint64_t diff = s_and ^ s_or;       // non-zero: the n > k >= 1 keys are distinct
        int pos = 64 - __clzll((long long)diff);   // low `pos` bits are undetermined
        uint64_t mask = pos >= 64 ? 0ull : ~((1ull << pos) - 1ull);
        uint64_t prefix = s_or & mask;
        uint32_t remaining = k;                    // rank of the wanted key among keys matching the prefix

        // ---- radix descent, 11 bits per round, until the boundary bin fits an LDS sort
        for (;;) {
            const int bits = pos < 11 ? pos : 11;
            const int shift = pos - bits;
            const uint32_t dmask = (1u << bits) - 1u;
            for (uint32_t i = tid; i < kSelBins; i += kSelBlock) hist[i] = 0;
            __syncthreads();
            for (uint32_t base = 0; base < n; base += kSelBlock * kSelUnroll) {
                uint64_t kk[kSelUnroll];
#pragma unroll
                for (int u = 0; u < kSelUnroll; ++u) {
                    const uint32_t i = base + u * kSelBlock + tid;
                    kk[u] = i < n ? keys[i] : 0;
                }
#pragma unroll
                for (int u = 0; u < kSelUnroll; ++u) {
                    const uint32_t i = base + u * kSelBlock + tid;
                    if (i < n && (kk[u] & mask) == prefix) atomicAdd(&hist[(uint32_t)(kk[u] >> shift) & dmask], 1u);
                }
            }
            __syncthreads();
            // thread t owns digits 2047-2t and 2046-2t (descending order)
            const uint32_t d1 = kSelBins - 1 - 2 * tid, d0 = d1 - 1;
            const uint32_t c1 = hist[d1], c0 = hist[d0];
            const uint32_t incl = block_scan_incl(c1 + c0, s_wave);
            const uint32_t before = incl - (c1 + c0);
            if (before < remaining && incl >= remaining) {
                if (before + c1 >= remaining) { s_digit = d1; s_remaining = remaining - before; s_binpop = c1; }
                else { s_digit = d0; s_remaining = remaining - before - c1; s_binpop = c0; }
            }
            __syncthreads();
            prefix |= (uint64_t)s_digit << shift;
            mask |= (uint64_t)dmask << shift;
            remaining = s_remaining;
            pos = shift;
            const uint32_t binpop = s_binpop;
            __syncthreads();
            if (binpop <= (uint32_t)kSelBound || pos == 0) break;
        }

        // ---- gather: keys above the boundary bin are kept; the bin itself is sorted in LDS
        if (tid == 0) { s_fill_keep = 0; s_fill_bound = 0; }
        __syncthreads();
        for (uint32_t base = 0; base < n; base += kSelBlock * kSelUnroll) {
            uint64_t kk[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const uint32_t i = base + u * kSelBlock + tid;
                kk[u] = i < n ? keys[i] : 0;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const uint32_t i = base + u * kSelBlock + tid;
                if (i < n) {
                    const uint64_t hi = kk[u] & mask;
                    if (hi > prefix) {
                        const uint32_t o = atomicAdd(&s_fill_keep, 1u);
                        if (o < (uint32_t)kSelMaxK) skeys[o] = kk[u];
                    } else if (hi == prefix) {
                        const uint32_t o = atomicAdd(&s_fill_bound, 1u);
                        if (o < (uint32_t)kSelBound) sbound[o] = kk[u];
                    }
                }
            }
        }
        __syncthreads();
        const uint32_t n_keep = k - remaining;      // == s_fill_keep
        const uint32_t n_bound = s_fill_bound < (uint32_t)kSelBound ? s_fill_bound : (uint32_t)kSelBound;
        uint32_t bp2 = 1;
        while (bp2 < n_bound) bp2 <<= 1;
        for (uint32_t i = n_bound + tid; i < bp2; i += kSelBlock) sbound[i] = 0;
        __syncthreads();
        bitonic_desc(sbound, bp2);
        const uint32_t take = remaining < n_bound ? remaining : n_bound;   // == remaining (keys are distinct)
        for (uint32_t i = tid; i < take; i += kSelBlock) skeys[n_keep + i] = sbound[i];
        __syncthreads();
        if (tid == 0 && take > 0) a.tau[q] = sbound[take - 1];   // k-th best of everything seen so far
    }
    __syncthreads();

    if (!a.final_pass) {
        for (uint32_t i = tid; i < m; i += kSelBlock) keys[i] = skeys[i];
        if (tid == 0) a.count[q] = m;
        return;
    }

    // ---- final round: sort the kept keys and emit ids and scores
    uint32_t pow2 = 1;
    while (pow2 < m) pow2 <<= 1;
    for (uint32_t i = m + tid; i < pow2; i += kSelBlock) skeys[i] = 0;
    __syncthreads();
    bitonic_desc(skeys, pow2);
    if (tid == 0) a.count[q] = m;
    for (uint32_t i = tid; i < k; i += kSelBlock) {
        int64_t id = -1;
        float sc = -__builtin_inff();
        if (i < m) {
            const uint64_t key = skeys[i];
            keys[i] = key;
            id = (int64_t)(uint32_t)(~(uint32_t)key);
            sc = ordered_to_score((uint32_t)(key >> 32));
        }
        a.ids_out[(size_t)q * k + i] = id;
        a.scores_out[(size_t)q * k + i] = sc;
    }
}

__global__ void init_state(uint32_t* count, uint64_t* tau, uint32_t* status, uint32_t n_queries)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_queries) { count[i] = 0; tau[i] = 0; }
    if (i == 0) *status = 0;
}

// ---------------------------------------------------------------- load path
// Address of item z's plane-j words / scale inside the tiled layout.
__device__ __forceinline__ char* item_tile(char* tiles, const Layout& l, const TileGeom& g, uint64_t z)
{
    return tiles + (size_t)tile_to_phys(l, (uint32_t)(z / kTileItems)) * g.tile_bytes();
}

// Caller's chunk ([P][count][W] words, [P][count] scales, items first..first+count) -> tiles.
// One thread per item.
__global__ void scatter_chunk(char* __restrict__ tiles, const Layout l, const TileGeom g,
                              const uint64_t* __restrict__ planes, const float* __restrict__ scales,
                              uint64_t first, uint64_t count)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    char* tile = item_tile(tiles, l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    for (uint32_t j = 0; j < g.P; ++j) {
        uint64_t* dst = reinterpret_cast<uint64_t*>(tile + j * g.plane_bytes()) + (size_t)o * g.W;
        for (uint32_t w = 0; w < g.W; ++w) dst[w] = planes[((size_t)j * count + t) * g.W + w];
        reinterpret_cast<float*>(tile + g.scales_offset())[j * kTileItems + o] = scales[(size_t)j * count + t];
    }
}

// ---------------------------------------------------------------- calibration
// Plain 16-byte-per-lane copy of a known size: the yardstick that hardware
// counter readings of the scan are scaled by.
__global__ __launch_bounds__(256) void calib_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------- dense helpers (tests, cosine fold)
__global__ void dense_popcounts(const char* __restrict__ tiles, const Layout l, const TileGeom g,
                                const uint64_t* __restrict__ qplanes, uint32_t PQ,
                                uint64_t first, uint64_t count, int32_t* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const char* tile = item_tile(const_cast<char*>(tiles), l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    for (uint32_t j = 0; j < g.P; ++j) {
        const uint64_t* kw = reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes()) + (size_t)o * g.W;
        for (uint32_t i = 0; i < PQ; ++i) {
            int32_t pc = 0;
            for (uint32_t w = 0; w < g.W; ++w) pc += __popcll(kw[w] ^ qplanes[i * g.W + w]);
            out[(t * g.P + j) * PQ + i] = pc;
        }
    }
}

template <int W, int P, int PQ>
__global__ void dense_scores(const char* __restrict__ tiles, const Layout l,
                             const uint32_t* __restrict__ qwords, const float* __restrict__ qcoef,
                             uint64_t first, uint64_t count, float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const TileGeom g{(uint32_t)W, (uint32_t)P};
    const char* tile = item_tile(const_cast<char*>(tiles), l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    const QueryRegs<W, PQ> q = load_query<W, PQ>(qwords, qcoef, 0);
    RowRegs<W, P> r;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint32_t* pw = reinterpret_cast<const uint32_t*>(tile + j * g.plane_bytes()) + (size_t)o * 2 * W;
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[j][0][h] = pw[h];
        r.a[j][0] = reinterpret_cast<const float*>(tile + g.scales_offset())[j * kTileItems + o];
    }
    out[t] = score_item<W, P, PQ>(r, 0, q);
}

// out[j][t] = scale j of item first + t
__global__ void gather_scales(const char* __restrict__ tiles, const Layout l, const TileGeom g,
                              uint64_t first, uint64_t count, float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const char* tile = item_tile(const_cast<char*>(tiles), l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    for (uint32_t j = 0; j < g.P; ++j)
        out[(size_t)j * count + t] = reinterpret_cast<const float*>(tile + g.scales_offset())[j * kTileItems + o];
}

// Divide each item's scales by the norm of its reconstructed vector:
// ||sum_j a_j b_j||^2 = dim * sum_j a_j^2 + 2 sum_{j<j'} a_j a_j' (dim - 2 popcount(K_j ^ K_j')).
// One thread per physical slot; slots never loaded have scale 0 and are left alone.
__global__ void fold_cosine(char* __restrict__ tiles, const TileGeom g, uint64_t n_slots)
{
    const uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_slots) return;
    char* tile = tiles + (size_t)(s / kTileItems) * g.tile_bytes();
    const uint32_t o = (uint32_t)(s % kTileItems);
    float* sc = reinterpret_cast<float*>(tile + g.scales_offset());
    const double dim = 64.0 * g.W;
    double a[4];
    for (uint32_t j = 0; j < g.P; ++j) a[j] = (double)sc[j * kTileItems + o];
    double n2 = 0.0;
    for (uint32_t j = 0; j < g.P; ++j) {
        n2 += dim * a[j] * a[j];
        const uint64_t* kj = reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes()) + (size_t)o * g.W;
        for (uint32_t jj = j + 1; jj < g.P; ++jj) {
            const uint64_t* kk = reinterpret_cast<const uint64_t*>(tile + jj * g.plane_bytes()) + (size_t)o * g.W;
            int pc = 0;
            for (uint32_t w = 0; w < g.W; ++w) pc += __popcll(kj[w] ^ kk[w]);
            n2 += 2.0 * a[j] * a[jj] * (dim - 2.0 * pc);
        }
    }
    if (n2 > 0.0) {
        const double nrm = sqrt(n2);
        for (uint32_t j = 0; j < g.P; ++j) sc[j * kTileItems + o] = (float)(a[j] / nrm);
    }
}

}  // namespace rbe
