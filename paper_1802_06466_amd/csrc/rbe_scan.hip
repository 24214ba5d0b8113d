// Exact-mode scan kernels and the dense score dump, for one word count W
// (compile with -DRBE_W=1, 2 or 4).
#include "rbe_internal.hpp"

#ifndef RBE_W
#error "compile with -DRBE_W=1|2|4"
#endif

namespace rbe {

// Queues the survivors among the lane's 4 scores.
template <int W, bool SINGLE>
__device__ __forceinline__ uint32_t stage_scores(const float (&s)[kItemsPerLane], uint64_t tau, float taus, uint32_t q,
                                                 uint32_t p, int wave, int lane, uint64_t* s_keys, const MultiStage& ms,
                                                 uint32_t fill, const ScanArgs& a)
{
    const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow;
#pragma unroll
    for (int m = 0; m < kItemsPerLane; ++m) {
        const uint64_t id = row_id + lane_item<W>(lane, m);
        bool ok = (s[m] >= taus) && (id < a.n_items);
        uint64_t key = 0;
        if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
        if (SINGLE) fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
        else mstage_append(ok, key, q, ms, a.out, lane);
    }
    return fill;
}

// Scores the lane's 4 items of `cur` against one query and queues the survivors.
template <int W, int P, int PQ, bool SINGLE, int MODE>
__device__ __forceinline__ uint32_t score_and_stage(RowRegs<W, P, scale_arrays(MODE, P)>& cur, const QueryRegs<W, PQ>& qr, uint64_t tau,
                                                    float taus, uint32_t q, uint32_t p, int wave, int lane,
                                                    uint64_t* s_keys, const MultiStage& ms, uint32_t fill, const ScanArgs& a)
{
    float s[kItemsPerLane];
    bool any = false;
#pragma unroll
    for (int m = 0; m < kItemsPerLane; ++m) {
        s[m] = score_item<W, P, PQ, MODE>(cur, m, qr);
        any |= (s[m] >= taus);
        // Batch kernel only: the empty asm makes the next item's plane words "depend" on this
        // item's score, at no cost.  Without it the scheduler interleaves the popcount chains of
        // all four items; wide configurations then spill to the accumulation registers, and the
        // VALU-bound kernel loses 10 % (d=64, 3x3 planes) to 30 % (d=128, 4x4).  The one-query
        // kernel is HBM-bound and measurably prefers the interleaved schedule.
        if (!SINGLE && m + 1 < kItemsPerLane) {
#pragma unroll
            for (int j = 0; j < P; ++j)
#pragma unroll
                for (int h = 0; h < 2 * W; ++h) asm volatile("" : "+v"(s[m]), "+v"(cur.w[j][m + 1][h]));
        }
    }
    if (__ballot(any))     // rare: at least one lane of the wave has a survivor
        fill = stage_scores<W, SINGLE>(s, tau, taus, q, p, wave, lane, s_keys, ms, fill, a);
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
template <int W, int P, int PQ, bool SINGLE, int MODE>
__global__ __launch_bounds__(kBlock) void scan_exact(const ScanArgs a)
{
    // one query: a fixed queue per wave.  Several: a.stage_entries per wave from the launch's dynamic LDS --
    // a batch forwards Q times as many survivors, and with 64 sub-queues in 512 entries a flush (one returning
    // global atomic, a microsecond of waiting) came every 8 survivors
    __shared__ uint64_t s_keys_fixed[SINGLE ? kWavesPerBlock : 1][SINGLE ? kStage : 1];
    extern __shared__ __align__(16) unsigned char s_dynamic[];
    __shared__ uint32_t s_cnt_all[SINGLE ? 1 : kWavesPerBlock][SINGLE ? 1 : 65];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = SINGLE ? s_keys_fixed[SINGLE ? wave : 0] : reinterpret_cast<uint64_t*>(s_dynamic) + (size_t)wave * a.stage_entries;
    MultiStage ms{};
    if (!SINGLE) {
        const uint32_t n_sub = sub_queues_for(a.n_queries);
        const uint32_t per_sub = a.stage_entries / n_sub;
        ms = MultiStage{s_keys, s_cnt_all[wave], per_sub > 64u ? 64u : per_sub, 0u, n_sub};   // a flush moves <= 64 entries
        s_cnt_all[wave][lane] = 0;
        if (lane == 0) s_cnt_all[wave][64] = 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    const uint32_t G = gridDim.x;
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    uint32_t fill = 0;

    if (SINGLE) {
        const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
        const uint64_t tau0 = a.tau[0];
        const float taus0 = threshold_score(tau0);
        RowRegs<W, P, S> cur, nxt;
        load_row<W, P, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
        for (;;) {
            const uint32_t pn = p + G;
            const bool has_next = pn < a.p_end;
            load_row<W, P, S>(nxt, a.tiles + (size_t)(has_next ? pn : p) * tile_bytes, wave, lane);   // unconditional: see scan_exact_prog_hint
            fill = score_and_stage<W, P, PQ, SINGLE, MODE>(cur, q0, tau0, taus0, 0, p, wave, lane, s_keys, ms, fill, a);
            if (!has_next) break;
            cur = nxt;
            p = pn;
        }
    } else {
        // (a short range is given to several rows of workgroups, each with a slice of the queries: see the launcher)
        const uint32_t q_lo = a.q_slice ? blockIdx.y * a.q_slice : 0u;
        const uint32_t nq = a.q_slice && q_lo + a.q_slice < a.n_queries ? q_lo + a.q_slice : a.n_queries;
        if (q_lo >= nq) return;
        for (; p < a.p_end; p += G) {
            RowRegs<W, P, S> cur;
            load_row<W, P, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
            // do not start scoring piecemeal as individual loads land: that keeps every partial
            // popcount of the tile alive at once and overflows the register file
            __builtin_amdgcn_sched_barrier(0);
            for (uint32_t rep = 0; rep <= a.calib_repeat; ++rep) {      // (once, except in the measurement mode)
                QueryRegs<W, PQ> qn = load_query<W, PQ>(a.qwords, a.qcoef, q_lo);
                uint64_t tau_n = a.tau[q_lo];
                for (uint32_t q = q_lo; q < nq; ++q) {
                    const QueryRegs<W, PQ> qr = qn;
                    const uint64_t tau = tau_n;
                    if (q + 1 < nq) {
                        qn = load_query<W, PQ>(a.qwords, a.qcoef, q + 1);
                        tau_n = a.tau[q + 1];
                    }
                    fill = score_and_stage<W, P, PQ, SINGLE, MODE>(cur, qr, tau, threshold_score(tau), q, p, wave, lane,
                                                             s_keys, ms, fill, a);
                }
            }
        }
    }
    if (SINGLE) { if (fill) stage_flush1(s_keys, fill, a.out, lane); }
    else mstage_drain(ms, a.out, lane);
}

// Several queries (a few in practice: larger batches go to the matrix cores), P >= 2, progressive: one row in registers, planes 0 .. P-2 and the scales
// first; every query forms its partial scores and bounds from them, and the first query for which some item of
// the row can still reach the threshold has the row's last plane read (once per row), after which it and any
// later such query continue their partial chains to the full scores.  Most (query, row) pairs stop at the bound:
// a third fewer XOR/popcounts at P = 3, and most rows never read their last plane.  Appends what the batch form
// of scan_exact appends.
template <int W, int P, int PQ, int MODE>
__global__ __launch_bounds__(kBlock) void scan_exact_batch_prog(const ScanArgs a)
{
    extern __shared__ __align__(16) unsigned char s_dynamic[];
    __shared__ uint32_t s_cnt_all[kWavesPerBlock][65];
    constexpr int F = P - 1;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = reinterpret_cast<uint64_t*>(s_dynamic) + (size_t)wave * a.stage_entries;
    const uint32_t n_sub = sub_queues_for(a.n_queries);
    const uint32_t per_sub = a.stage_entries / n_sub;
    const MultiStage ms{s_keys, s_cnt_all[wave], per_sub > 64u ? 64u : per_sub, 0u, n_sub};
    s_cnt_all[wave][lane] = 0;
    if (lane == 0) s_cnt_all[wave][64] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const uint32_t G = gridDim.x;
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    const uint32_t nq = a.n_queries;
    const float* masses = a.qcoef + (size_t)nq * (PQ + 1);
    uint32_t full_rows = 0, rows = 0, full_pairs = 0;
    uint32_t probed = 0, probe_full = 0;   // (query, row) pairs taken the progressive way, and those of them scored in full
    for (uint32_t p = a.p_begin + blockIdx.x; p < a.p_end; p += G) {
        const char* tile = a.tiles + (size_t)p * tile_bytes;
        RowRegs<W, P, S> cur;
        load_row_planes<W, P, S, 0, F>(cur, tile, wave, lane);
        load_row_scales<W, P, S>(cur, tile, wave, lane);
        // a wave for which more than half of the (query, row) pairs go on to the full score (a loose threshold) asks
        // for the last plane together with the others and, bounds being of no use to it, scores like scan_exact; one
        // row in sixteen still goes the progressive way, to notice when that changes.  (Pairs, not rows: with many
        // queries most rows are needed by some query while most pairs still stop at the bound.)
        const bool plain = probe_full * 2 > probed + 16 * nq && (rows & 15u) != 0u;     // wave-uniform
        bool have_last = plain;
        if (plain) { load_row_planes<W, P, S, F, P>(cur, tile, wave, lane); ++full_rows; full_pairs += nq; }
        ++rows;
        __builtin_amdgcn_sched_barrier(0);
        if (plain) {
            QueryRegs<W, PQ> qn = load_query<W, PQ>(a.qwords, a.qcoef, 0);
            uint64_t tau_n = a.tau[0];
            for (uint32_t q = 0; q < nq; ++q) {
                const QueryRegs<W, PQ> qr = qn;
                const uint64_t tau = tau_n;
                if (q + 1 < nq) {
                    qn = load_query<W, PQ>(a.qwords, a.qcoef, q + 1);
                    tau_n = a.tau[q + 1];
                }
                score_and_stage<W, P, PQ, false, MODE>(cur, qr, tau, threshold_score(tau), q, p, wave, lane, s_keys, ms, 0, a);
            }
            continue;
        }
        probed += nq;
        QueryRegs<W, PQ> qn = load_query<W, PQ>(a.qwords, a.qcoef, 0);
        uint64_t tau_n = a.tau[0];
        QueryMass mass_n{masses[0], masses[1]};
        for (uint32_t q = 0; q < nq; ++q) {
            const QueryRegs<W, PQ> qr = qn;
            const uint64_t tau = tau_n;
            const QueryMass mass = mass_n;
            if (q + 1 < nq) {
                qn = load_query<W, PQ>(a.qwords, a.qcoef, q + 1);
                tau_n = a.tau[q + 1];
                mass_n = QueryMass{masses[2 * (q + 1)], masses[2 * (q + 1) + 1]};
            }
            const float taus = threshold_score(tau);
            PartialScore part[kItemsPerLane];
            bool reach = false;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                part[m] = partial_item<W, P, PQ, MODE, F>(cur, m, qr);
                reach |= !(bound_item<W, P, PQ, MODE, F>(cur, m, part[m], mass) < taus);
                if (m + 1 < kItemsPerLane) {     // one item's popcount chains at a time (see score_and_stage)
#pragma unroll
                    for (int j = 0; j < F; ++j)
#pragma unroll
                        for (int h = 0; h < 2 * W; ++h) {
                            if (MODE == kModeScaled) asm volatile("" : "+v"(part[m].s), "+v"(cur.w[j][m + 1][h]));
                            else asm volatile("" : "+v"(part[m].H), "+v"(cur.w[j][m + 1][h]));
                        }
                }
            }
            if (__ballot(reach)) {
                if (!have_last) {
                    load_row_planes<W, P, S, F, P>(cur, tile, wave, lane);
                    have_last = true;
                    ++full_rows;
                }
                ++probe_full;
                ++full_pairs;
                float s[kItemsPerLane];
                bool any = false;
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    s[m] = finish_item<W, P, PQ, MODE, F>(cur, m, qr, part[m]);
                    any |= (s[m] >= taus);
                }
                if (__ballot(any)) stage_scores<W, false>(s, tau, taus, q, p, wave, lane, s_keys, ms, 0, a);
            }
        }
    }
    mstage_drain(ms, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_pairs && lane == 0 && full_pairs) atomicAdd(a.deep_pairs, full_pairs);
}

// One query, P >= 2, progressive: the stream carries planes 0 .. F-1 (F = P - 1) and the scale arrays 0 .. S-2
// only; the row's largest last scale (row_amax) stands in for the last scale array.  From them every item gets an
// upper bound on its score (bound_item_rowmax); only where some item of the wave's row can still reach the
// threshold are the row's last plane and last scales read (a dependent load, exposed, but rare once the threshold
// is tight: the rows that hold items of the query's own neighbourhood) and the partial scores continued to the
// full ones, exactly as scan_exact forms them.  What is appended is therefore identical to scan_exact's; what is
// read is (8W + 4)(P-1) of the (8W + 4) P bytes of most items (general scales; see scan_exact_prog_hint for the
// variant that streams one-byte scale copies).  (The residual scales decay from plane to plane, so the last plane is the one
// whose absence costs the bound least; with fewer planes in the stream the bound let most rows through on
// clustered data.)
// A wave that finds itself fetching the last plane for more than a quarter of its rows (a loose threshold, or
// scales that do not decay) streams whole rows like scan_exact until the rate falls again.
template <int W, int P, int PQ, int MODE>
__global__ __launch_bounds__(kBlock) void scan_exact_prog(const ScanArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    const MultiStage ms{};
    const uint32_t G = gridDim.x;
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    constexpr int F = P - 1;
    uint32_t fill = 0, rows = 0, deep = 0, full_rows = 0;   // rows seen, rows the bound let through, rows read in full
    uint32_t extra8 = 0;                                    // bytes / 8 asked for beyond the stream
    const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
    const float* pm = a.qcoef + (size_t)a.n_queries * (PQ + 1);
    const QueryMass mass{pm[0], pm[1]};
    const uint64_t tau0 = a.tau[0];
    const float taus0 = threshold_score(tau0);

    // the last scale array stays out of the stream as well: its largest value over the row stands in for it
    constexpr int SS = S > 0 ? S - 1 : 0;
    RowRegs<W, P, S> cur, nxt;
    load_row_planes<W, P, S, 0, F>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_row_scales<W, P, S, 0, SS>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    float amax = S > 0 ? a.row_amax[(size_t)p * kWavesPerBlock + wave] : 0.0f, amax_n = 0.0f;
    bool whole = false;    // wave-uniform: cur holds every plane and scale already
    for (;;) {
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const bool whole_next = deep * 4 > rows + 32;     // wave-uniform
        const uint32_t pl = has_next ? pn : p;      // prefetch not under a branch: see scan_exact_prog_hint
        const char* tn = a.tiles + (size_t)pl * tile_bytes;
        load_row_planes<W, P, S, 0, F>(nxt, tn, wave, lane);
        load_row_scales<W, P, S, 0, SS>(nxt, tn, wave, lane);
        if (S > 0) amax_n = a.row_amax[(size_t)pl * kWavesPerBlock + wave];
        if (whole_next) {
            load_row_planes<W, P, S, F, P>(nxt, tn, wave, lane);
            load_row_scales<W, P, S, SS, S>(nxt, tn, wave, lane);
            extra8 += has_next ? kRow * W + (S > 0 ? kRow / 2 : 0) : 0;
        }
        PartialScore part[kItemsPerLane];
        uint32_t mine = 0;     // which of this lane's items can still reach the threshold (a NaN bound does not prune)
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            part[m] = partial_item<W, P, PQ, MODE, F>(cur, m, q0);
            mine |= !(bound_item_rowmax<W, P, PQ, MODE>(cur, m, part[m], mass, amax) < taus0) ? (1u << m) : 0u;
        }
        const bool reach = __ballot(mine != 0u) != 0;
        ++rows;
        full_rows += (whole || reach) ? 1u : 0u;
        if (reach) {
            if (!whole) {
                // only the lanes that hold such an item read the rest of their items' data: the memory system then
                // fetches the cache lines they touch, not the row
                const char* tile = a.tiles + (size_t)p * tile_bytes;
                const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + (P - 1) * geom.plane_bytes()) + (size_t)wave * kRow * W;
                const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset()) + (size_t)SS * kTileItems + wave * kRow;
                if constexpr (W == 1) {
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
                        extra8 += (uint32_t)__builtin_popcountll(__ballot((mine & (3u << (2 * h2))) != 0u)) * (2 + (S > 0 ? 1 : 0));
                } else {
#pragma unroll
                    for (int m = 0; m < kItemsPerLane; ++m)
                        extra8 += ((uint32_t)__builtin_popcountll(__ballot((mine & (1u << m)) != 0u)) * (2 * W + (S > 0 ? 1 : 0))) / 2;
                }
                if constexpr (W == 1) {
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
                        if (mine & (3u << (2 * h2))) {
                            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + h2 * 128 + 2 * lane));
                            cur.w[P - 1][2 * h2][0] = v.x; cur.w[P - 1][2 * h2][1] = v.y;
                            cur.w[P - 1][2 * h2 + 1][0] = v.z; cur.w[P - 1][2 * h2 + 1][1] = v.w;
                            if constexpr (S > 0) {
                                const f32x2 av = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sc + h2 * 128 + 2 * lane));
                                cur.a[SS][2 * h2] = av.x; cur.a[SS][2 * h2 + 1] = av.y;
                            }
                        }
                } else {
#pragma unroll
                    for (int m = 0; m < kItemsPerLane; ++m)
                        if (mine & (1u << m)) {
#pragma unroll
                            for (int h = 0; h < W / 2; ++h) {
                                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + (size_t)(m * 64 + lane) * W) + h);
                                cur.w[P - 1][m][4 * h + 0] = v.x; cur.w[P - 1][m][4 * h + 1] = v.y;
                                cur.w[P - 1][m][4 * h + 2] = v.z; cur.w[P - 1][m][4 * h + 3] = v.w;
                            }
                            if constexpr (S > 0) cur.a[SS][m] = __builtin_nontemporal_load(sc + m * 64 + lane);
                        }
                }
            }
            ++deep;
            float s[kItemsPerLane];
            bool any = false;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                // an item whose bound is below the threshold cannot be a survivor (and in the lane-wise path its data
                // was not read)
                s[m] = -__builtin_inff();
                if (mine & (1u << m)) s[m] = finish_item<W, P, PQ, MODE, F>(cur, m, q0, part[m]);
                any |= (s[m] >= taus0);
            }
            if (__ballot(any)) fill = stage_scores<W, true>(s, tau0, taus0, 0, p, wave, lane, s_keys, ms, fill, a);
        }
        if (!has_next) break;
        cur = nxt;
        amax = amax_n;
        whole = whole_next;
        p = pn;
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}


// scan_exact_prog for general scales: the stream carries no fp32 scale array at all.  The scale arrays 0 .. P-2
// come as one-byte copies h_j (scale_hints: a_j = h_j (1 +- 2^-6), so a_j t_j <= h_j t_j + 2^-6 h_j |t_j|
// <= h_j t_j + 2^-6 h_j M, slightly more in the kernel), the last one as its largest value over the row.  A row that the bound lets through reads its last plane
// and its P fp32 scale arrays and is scored from scratch by score_item, so what is appended is still exactly
// what scan_exact appends.  16 + 2 instead of 16 + 8 streamed bytes per item at d = 64, P = 3.
// A wave whose bound lets more than a quarter of its rows through gives it up and takes the rest of its rows as
// scan_exact does (whole rows, prefetched).  The two register sets (this row, the next one in flight) hold the
// streamed planes only and swap roles from row to row.
// The rows of a wave from tile p on (p, p + grid, ...), with what the wave has queued and counted so far: the whole
// of scan_exact_prog_hint, and what scan_exact_prog2_hint falls back to.  STREAM_EXTRA (a number of planes): count the planes A .. P-2
// that this stream carries as bytes beyond the (plane 0 only) stream of the caller.
template <int W, int P, int PQ, int STREAM_EXTRA>
__device__ __forceinline__ void prog_hint_rows(const ScanArgs& a, uint32_t p, uint32_t fill, uint32_t full_rows, uint32_t extra8,
                                               uint64_t* s_keys, int wave, int lane)
{
    constexpr int MODE = kModeScaled;
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;   // hint words per lane and row (one byte per item and array)
    const MultiStage ms{};
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    uint32_t probed = 0, passed = 0;
    const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
    const float* pm = a.qcoef + (size_t)a.n_queries * (PQ + 1);
    const QueryMass mass{pm[0], pm[1]};
    const float slack_all = 2.0f * mass.y + 0.015875f * mass.x;
    const uint64_t tau0 = a.tau[0];
    const float taus0 = threshold_score(tau0);

    struct Hints { uint32_t w[NW]; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 1) {
            h.w[0] = __builtin_nontemporal_load(src);
        } else if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };
    // hint byte (3-bit exponent above base_j, 5-bit mantissa) -> fp32
    const uint32_t hb0 = (uint32_t)a.hint_base[0] << 5, hb1 = (uint32_t)a.hint_base[1] << 5, hb2 = (uint32_t)a.hint_base[2] << 5;
    auto hint = [&](const Hints& h, int j, int m) {
        const uint32_t c = (h.w[j] >> (8 * m)) & 255u;
        return __uint_as_float((c + (j == 0 ? hb0 : (j == 1 ? hb1 : hb2))) << 18);
    };
    // a scale below the smallest hint of its array, 2^(base_j - 127), is off by up to that much instead
    float floor_c = 0.0f;
    for (int j = 0; j < F; ++j) floor_c += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_c *= 1.0001f * mass.x;
    const float mass_last = mass.x + 2.0f * mass.y;

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, F>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    float amax = a.row_amax[(size_t)p * kWavesPerBlock + wave], amax_n = 0.0f;
    bool plain = false;    // wave-uniform: the bound lets most rows through; the rest of the wave's rows go the plain way
    // One row: start the loads of the next one into the other register set, judge and score this one.  The two
    // register sets swap roles from row to row (two copies of the code) instead of being copied.
    auto step = [&](RowRegs<W, P, S>& cur, Hints& hc, float& amax, RowRegs<W, P, S>& nxt, Hints& hn, float& amax_n)
                    __attribute__((always_inline)) -> bool {
        if (passed * 4 > probed + 32) { plain = true; return false; }     // wave-uniform; this row is not done yet
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        // The prefetch is not under a branch (a workgroup's last step fetches its own row once more): with
        // `if (has_next)` around it the compiler, merging the path that loaded with the one that did not, makes
        // the first use of THIS row's registers wait for half of the loads just issued -- every step then stalls
        // for a memory round trip and nothing is prefetched.
        const uint32_t pl = has_next ? pn : p;
        load_row_planes<W, P, S, 0, F>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
        amax_n = a.row_amax[(size_t)pl * kWavesPerBlock + wave];
        bool reach = true;
        uint32_t mine = 0;     // which of this lane's items can still reach the threshold
        {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                float s = floor_c, all = 0.0f;
#pragma unroll
                for (int j = 0; j < F; ++j) {
                    float t = q0.bias;
#pragma unroll
                    for (int i = 0; i < PQ; ++i) {
                        uint32_t pc = 0;
#pragma unroll
                        for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ q0.w[i][h]);
                        t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                    }
                    const float hj = hint(hc, j, m);
                    s = __fmaf_rn(hj, t, s);
                    all += hj;
                }
                // |a_j t_j - h_j t_j| <= 2^-6 (1 + 2^-6) h_j |t_j| <= 0.015875 h_j mass.x, and the roundings of
                // either chain: both per unit of the scale sum (slack_all)
                const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(amax, mass_last, s));
                mine |= !(ub < taus0) ? (1u << m) : 0u;      // (a NaN bound does not prune)
            }
            reach = __ballot(mine != 0u) != 0;
            ++probed;
            passed += reach ? 1u : 0u;
        }
        full_rows += reach ? 1u : 0u;
        if (STREAM_EXTRA) extra8 += kRow * (uint32_t)W * (uint32_t)STREAM_EXTRA;
        if (reach) {
            // only the lanes that hold such an item read the rest of their items' data (the memory system fetches
            // the cache lines they touch, not the row) and score; an item whose bound is below the threshold cannot
            // be a survivor
            const char* tile = a.tiles + (size_t)p * tile_bytes;
            const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + (P - 1) * geom.plane_bytes()) + (size_t)wave * kRow * W;
            const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset()) + wave * kRow;
            // what the lanes ask for: per pair of items (W = 1) or per item, the last plane and S scales
            if constexpr (W == 1) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) extra8 += (uint32_t)__builtin_popcountll(__ballot((mine & (3u << (2 * h2))) != 0u)) * (2 + S);
            } else {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m)
                    extra8 += ((uint32_t)__builtin_popcountll(__ballot((mine & (1u << m)) != 0u)) * (2 * W + S)) / 2;
            }
            if constexpr (W == 1) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
                    if (mine & (3u << (2 * h2))) {
                        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + h2 * 128 + 2 * lane));
                        cur.w[P - 1][2 * h2][0] = v.x; cur.w[P - 1][2 * h2][1] = v.y;
                        cur.w[P - 1][2 * h2 + 1][0] = v.z; cur.w[P - 1][2 * h2 + 1][1] = v.w;
#pragma unroll
                        for (int j = 0; j < S; ++j) {
                            const f32x2 av = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sc + j * kTileItems + h2 * 128 + 2 * lane));
                            cur.a[j][2 * h2] = av.x; cur.a[j][2 * h2 + 1] = av.y;
                        }
                    }
            } else {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m)
                    if (mine & (1u << m)) {
#pragma unroll
                        for (int h = 0; h < W / 2; ++h) {
                            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + (size_t)(m * 64 + lane) * W) + h);
                            cur.w[P - 1][m][4 * h + 0] = v.x; cur.w[P - 1][m][4 * h + 1] = v.y;
                            cur.w[P - 1][m][4 * h + 2] = v.z; cur.w[P - 1][m][4 * h + 3] = v.w;
                        }
#pragma unroll
                        for (int j = 0; j < S; ++j) cur.a[j][m] = __builtin_nontemporal_load(sc + j * kTileItems + m * 64 + lane);
                    }
            }
            float sv[kItemsPerLane];
            bool any = false;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                sv[m] = -__builtin_inff();
                if (mine & (1u << m)) sv[m] = score_item<W, P, PQ, MODE>(cur, m, q0);
                any |= (sv[m] >= taus0);
            }
            if (__ballot(any)) fill = stage_scores<W, true>(sv, tau0, taus0, 0, p, wave, lane, s_keys, ms, fill, a);
        }
        p = pn;
        return has_next;
    };
    for (;;) {
        if (!step(cur, hc, amax, nxt, hn, amax_n)) break;
        if (!step(nxt, hn, amax_n, cur, hc, amax)) break;
    }
    if (plain) {
        // from row p on as scan_exact does it: whole rows, the next one in flight while this one is scored
        load_row<W, P, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
        for (;;) {
            const uint32_t pn = p + G;
            const bool has_next = pn < a.p_end;
            load_row<W, P, S>(nxt, a.tiles + (size_t)(has_next ? pn : p) * tile_bytes, wave, lane);   // unconditional: see scan_exact_prog_hint
            fill = score_and_stage<W, P, PQ, true, MODE>(cur, q0, tau0, taus0, 0, p, wave, lane, s_keys, ms, fill, a);
            ++full_rows;
            extra8 += kRow * (W + S / 2) + (kRow * (S & 1)) / 2;     // 8W + 4S bytes per item beyond the stream's
            if (STREAM_EXTRA) extra8 += kRow * (uint32_t)W * (uint32_t)STREAM_EXTRA;
            if (!has_next) break;
            cur = nxt;
            p = pn;
        }
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}

template <int W, int P, int PQ>
__global__ __launch_bounds__(kBlock) void scan_exact_prog_hint(const ScanArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    prog_hint_rows<W, P, PQ, 0>(a, p, 0u, 0u, 0u, s_keys_all[wave], wave, lane);
}

// scan_exact_prog_hint in two stages (P >= 3): the stream carries plane 0 and the one-byte scale copies only
// -- here of ALL P scale arrays, the last one from a side array of its own -- (8W + P bytes per item: 11 instead of
// 18 at d = 64, P = 3).  Stage A bounds an item's score from plane 0 alone: h_0 t_0 plus the most the other planes
// (their scale copies times the query's mass) could add.  A plane of 64 signs already tells most items of a corpus
// apart from a query: about one item in 100 to 200 passes on clustered data, but nearly every ROW of 256 holds one,
// so what passes is not followed up row by row: it goes to a queue in the wave's LDS area (item, partial score,
// scale copies, row maximum), and whenever 64 entries have gathered, stage B takes one per lane: the lane reads the
// item's words of planes 1 .. P-2 (8W bytes each: 64 loads in flight for one round trip) and forms the bound of
// scan_exact_prog_hint -- the same operations in the same order.  What passes that too (stage C: a few items in
// 10^4) has all its planes and fp32 scales read by the same lane and is scored from scratch by score_item, so what
// is appended is still exactly what scan_exact appends.  A wave of whose items more than one in 16 pass stage A
// gives the first stage up and takes the rest of its rows as scan_exact_prog_hint does (which has its own
// fallback to whole rows).
// A: planes in the stream (written above for A = 1).  With three planes the sign plane and the two other scale
// copies rule out 98 of 100 items; with four, what three residual planes could still add lets one item in ten
// through, and the first stage is formed from planes 0 and 1 (A = 2: 16W + 4 bytes per item instead of 24W + 3,
// next to no item passes), stage B reads plane 2.
template <int W, int P, int PQ, int A = 1>
__global__ __launch_bounds__(kBlock) void scan_exact_prog2_hint(const ScanArgs a)
{
    static_assert(P >= 3, "with two planes scan_exact_prog_hint streams plane 0 alone already");
    static_assert(A >= 1 && A <= P - 2, "stage B reads planes A .. P-2");
    constexpr int MODE = kModeScaled;
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;   // hint words per lane and row (one byte per item and array)
    constexpr int kQueue = 128;                  // entries per wave: a batch of 64 leaves when 64 have gathered
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ uint32_t s_qid[kWavesPerBlock][kQueue];    // physical tile * 1024 + item of the tile
    __shared__ float s_qs0[kWavesPerBlock][kQueue];       // floor + h_0 t_0: where the bound's chain stands after plane 0
    __shared__ uint32_t s_qhb[kWavesPerBlock][kQueue];    // the item's scale copies, array j in byte j
    __shared__ float s_qam[kWavesPerBlock][kQueue];       // the copy of the item's last scale
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    uint32_t fill = 0, full_rows = 0, extra8 = 0;
    uint32_t qfill = 0;                       // entries waiting for stage B (wave-uniform)
    uint32_t last_row = 0xFFFFFFFFu;          // row of the last item that reached stage C (wave-uniform)
    uint32_t probed = 0, passed = 0;          // items judged by stage A, items it let through (wave-uniform)
    const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
    const float* pm = a.qcoef + (size_t)a.n_queries * (PQ + 1);
    const QueryMass mass{pm[0], pm[1]};
    const float slack_all = 2.0f * mass.y + 0.015875f * mass.x;      // as in scan_exact_prog_hint
    const uint64_t tau0 = a.tau[0];
    const float taus0 = threshold_score(tau0);
    const uint32_t hb[3] = {(uint32_t)a.hint_base[0] << 5, (uint32_t)a.hint_base[1] << 5, (uint32_t)a.hint_base[2] << 5};
    auto decode = [&](uint32_t byte, int j) { return __uint_as_float((byte + hb[j]) << 18); };
    // a scale below the smallest copy of its array, 2^(base - 127), is off by up to that much instead (all P arrays here)
    float floor_c = __uint_as_float((uint32_t)a.hint_base_last << 23);
    for (int j = 0; j < F; ++j) floor_c += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_c *= 1.0001f * mass.x;
    const float mass_last = mass.x + 2.0f * mass.y;
    const float mass_hint = mass_last + slack_all;      // what a plane whose scale is known by its copy can add, per unit of the copy
    float floor_j[A];      // (the smallest copy of each streamed plane's array)
#pragma unroll
    for (int j = 0; j < A; ++j) floor_j[j] = 1.0001f * __uint_as_float((uint32_t)a.hint_base[j] << 23);
    const uint32_t hb_last = (uint32_t)a.hint_base_last << 5;

    struct Hints { uint32_t w[NW]; uint32_t last; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        h.last = __builtin_nontemporal_load(a.hints_last + ((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane);
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };

    // Stage B (and C) for the entries [base, base + n) of the wave's queue, one per lane.  All lanes of the wave.
    auto follow_up = [&](uint32_t base, uint32_t n) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const bool act = (uint32_t)lane < n;
        const uint32_t e = base + (act ? (uint32_t)lane : 0u);
        const uint32_t id = s_qid[wave][e], hbytes = s_qhb[wave][e];
        const float h_last = s_qam[wave][e];
        float s = s_qs0[wave][e];
        const uint32_t tp = id >> 10, idx = id & 1023u;
        const char* tile = a.tiles + (size_t)tp * tile_bytes;
        RowRegs<W, P, S> it;          // this lane's item, in slot 0
        bool pass2 = false;
        if (act) {
            float all = 0.0f;
#pragma unroll
            for (int j = 0; j < A; ++j) all += decode((hbytes >> (8 * j)) & 255u, j);
#pragma unroll
            for (int j = A; j < F; ++j) {
                const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
                if constexpr (W == 1) {
                    const u32x2 v = *reinterpret_cast<const u32x2*>(kw);
                    it.w[j][0][0] = v.x; it.w[j][0][1] = v.y;
                } else {
#pragma unroll
                    for (int h = 0; h < W / 2; ++h) {
                        const u32x4 v = reinterpret_cast<const u32x4*>(kw)[h];
                        it.w[j][0][4 * h + 0] = v.x; it.w[j][0][4 * h + 1] = v.y; it.w[j][0][4 * h + 2] = v.z; it.w[j][0][4 * h + 3] = v.w;
                    }
                }
                float t = q0.bias;
#pragma unroll
                for (int i = 0; i < PQ; ++i) {
                    uint32_t pc = 0;
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(it.w[j][0][h] ^ q0.w[i][h]);
                    t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                }
                const float hj = decode((hbytes >> (8 * j)) & 255u, j);
                s = __fmaf_rn(hj, t, s);
                all += hj;
            }
            // the bound of scan_exact_prog_hint, with the item's own last scale (by its copy) for the row's largest
            const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(h_last, mass_hint, s));
            pass2 = !(ub < taus0);
        }
        extra8 += n * (uint32_t)W * (uint32_t)(F - A);
        const uint64_t m2 = __ballot(pass2);
        if (m2) {
            float score = -__builtin_inff();
            uint64_t logical = 0;
            if (pass2) {
                // the rest of the item: the streamed planes again (another lane had them), the last plane, the fp32 scales
#pragma unroll
                for (int jj = 0; jj <= A; ++jj) {
                    const int j = jj < A ? jj : P - 1;
                    const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) it.w[j][0][h] = kw[h];
                }
                const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset());
#pragma unroll
                for (int j = 0; j < S; ++j) it.a[j][0] = sc[j * kTileItems + idx];
                score = score_item<W, P, PQ, MODE>(it, 0, q0);
                logical = (uint64_t)phys_to_tile_per_lane(a.layout, tp) * kTileItems + idx;
            }
            bool ok = pass2 && (score >= taus0) && (logical < a.n_items);
            uint64_t key = 0;
            if (ok) { key = make_key(score, (uint32_t)logical); ok = key >= tau0; }
            fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
            const uint32_t n2 = (uint32_t)__builtin_popcountll(m2);
            extra8 += n2 * ((uint32_t)(A + 1) * W + (uint32_t)S / 2u) + (n2 * ((uint32_t)S & 1u)) / 2u;
            // rows that hold such an item: entries leave the queue in the order of their rows, so an item opens a
            // new row if the nearest lower lane with such an item (or, for the lowest, the last batch) holds another one
            const uint64_t below = m2 & ((1ull << lane) - 1ull);
            const int prev = below ? 63 - __builtin_clzll(below) : lane;
            const uint32_t row = id >> 8, row_prev = __shfl(row, prev);
            full_rows += (uint32_t)__builtin_popcountll(__ballot(pass2 && row != (below ? row_prev : last_row)));
            last_row = __shfl(row, 63 - __builtin_clzll(m2));
        }
        __builtin_amdgcn_wave_barrier();
    };

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, A>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    bool give_up = false;
    for (;;) {
        if (passed * 10 > probed + 4096) { give_up = true; break; }         // wave-uniform; row p is not done yet
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const uint32_t pl = has_next ? pn : p;          // (unconditional prefetch: see scan_exact_prog_hint)
        load_row_planes<W, P, S, 0, A>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            uint32_t hbytes = 0;
            float rest = 0.0f;
#pragma unroll
            for (int j = 0; j < F; ++j) {
                const uint32_t c = (hc.w[j] >> (8 * m)) & 255u;
                hbytes |= c << (8 * j);
                if (j >= A) rest += decode(c, j);
            }
            const float h_last = __uint_as_float((((hc.last >> (8 * m)) & 255u) + hb_last) << 18);
            float s0 = floor_c;          // the chain of scan_exact_prog_hint's bound after the streamed planes (stage B takes it up)
            float seen = 0.0f;           // what the streamed planes add to this stage's bound
            float h_seen = 0.0f;         // their scale copies, added up
#pragma unroll
            for (int j = 0; j < A; ++j) {
                float t = q0.bias;
#pragma unroll
                for (int i = 0; i < PQ; ++i) {
                    uint32_t pc = 0;
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ q0.w[i][h]);
                    t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                }
                const float hj = decode((hbytes >> (8 * j)) & 255u, j);
                s0 = __fmaf_rn(hj, t, s0);
                seen = __fmaf_rn(__builtin_fabsf(t), __fmaf_rn(0.015875f, hj, floor_j[j]), __fmaf_rn(hj, t, seen));
                h_seen += hj;
            }
            // For a streamed plane, a_j t_j <= h_j t_j + (0.015875 h_j + floor_j) |t_j|: the copy is within 2^-6 of the
            // scale, or, for a scale below the smallest copy, above it by less than that copy (floor_j); t_j is known
            // here, so its own size stands where scan_exact_prog_hint has the query's mass.  Every other plane adds at
            // most (its copy) x (mass + slack): |t_j| <= mass_last, and a copy that is not within 2^-6 of its scale is
            // above it.  The roundings of this line and of the chains it stands for are inside 2 mass.y per unit
            // of the scale sum, as there.
            const float ub = __fmaf_rn(rest + h_last, mass_hint, __fmaf_rn(2.0f * mass.y, h_seen, seen));
            const bool pass = !(ub < taus0);            // (a NaN bound does not prune)
            const uint64_t mk = __ballot(pass);
            if (mk) {
                if (pass) {
                    const uint32_t at = qfill + (uint32_t)__builtin_popcountll(mk & ((1ull << lane) - 1ull));
                    s_qid[wave][at] = p * (uint32_t)kTileItems + (uint32_t)wave * kRow + lane_item<W>(lane, m);
                    s_qs0[wave][at] = s0;
                    s_qhb[wave][at] = hbytes;
                    s_qam[wave][at] = h_last;
                }
                const uint32_t n = (uint32_t)__builtin_popcountll(mk);
                qfill += n;
                passed += n;
                if (qfill >= 64) {
                    // the 64 oldest entries leave; the rest (fewer than 64) move to the front
                    follow_up(0, 64);
                    qfill -= 64;
                    const bool mv = (uint32_t)lane < qfill;
                    const uint32_t from = 64u + (mv ? (uint32_t)lane : 0u);
                    const uint32_t e_id = s_qid[wave][from], e_hb = s_qhb[wave][from];
                    const float e_s0 = s_qs0[wave][from], e_am = s_qam[wave][from];
                    __builtin_amdgcn_wave_barrier();
                    if (mv) { s_qid[wave][lane] = e_id; s_qhb[wave][lane] = e_hb; s_qs0[wave][lane] = e_s0; s_qam[wave][lane] = e_am; }
                }
            }
        }
        probed += kRow;
        if (!has_next) { p = pn; break; }
        cur = nxt; hc = hn;
        p = pn;
    }
    if (qfill) follow_up(0, qfill);
    if (give_up) {
        prog_hint_rows<W, P, PQ, P - 1 - A>(a, p, fill, full_rows, extra8, s_keys, wave, lane);
        return;
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}

// scan_exact_prog_hint for several queries per call (2 .. 4 in practice): the same stream (planes 0 .. P-2, their
// one-byte scale copies, the row's largest last scale), every query's bound per item, and for the items that some
// query's bound lets through the lanes that hold them read the last plane and the fp32 scales once; every query
// then scores those items from scratch.  Appends what the batch form of scan_exact appends.  Against
// scan_exact_batch_prog, which streams the fp32 scales (28 instead of 18 bytes per item at d = 64, P = 3), the gain
// is in the small batches that are still bound by memory.
// The rows of a wave from tile p on, with what the wave has counted so far (see prog_hint_rows): the whole of
// scan_exact_batch_prog_hint, and what scan_exact_batch_prog2_hint falls back to.
template <int W, int P, int PQ, int STREAM_EXTRA>
__device__ __forceinline__ void batch_prog_hint_rows(const ScanArgs& a, uint32_t p, uint32_t full_rows, uint32_t full_pairs, uint32_t extra8,
                                                     uint64_t* s_keys, const MultiStage& ms, const QuerySlot<W, PQ>* slots,
                                                     int wave, int lane)
{
    constexpr int MODE = kModeScaled;
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;   // hint words per lane and row (one byte per item and array)
    const uint32_t nq = __builtin_amdgcn_readfirstlane(a.n_queries);     // (kept in a scalar register: the loops over the queries are the wave's, not the lanes')
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    uint32_t rows = 0;
    uint32_t probed = 0, passed = 0;   // (query, row) pairs whose bound was evaluated, and those of them it let through

    struct Hints { uint32_t w[NW]; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 1) {
            h.w[0] = __builtin_nontemporal_load(src);
        } else if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };
    // hint byte (3-bit exponent above base_j, 5-bit mantissa) -> fp32
    const uint32_t hb0 = (uint32_t)a.hint_base[0] << 5, hb1 = (uint32_t)a.hint_base[1] << 5, hb2 = (uint32_t)a.hint_base[2] << 5;
    auto hint = [&](const Hints& h, int j, int m) {
        const uint32_t c = (h.w[j] >> (8 * m)) & 255u;
        return __uint_as_float((c + (j == 0 ? hb0 : (j == 1 ? hb1 : hb2))) << 18);
    };
    // a scale below the smallest hint of its array, 2^(base_j - 127), is off by up to that much instead
    float floor_h = 0.0f;
    for (int j = 0; j < F; ++j) floor_h += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_h *= 1.0001f;

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, F>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    float amax = a.row_amax[(size_t)p * kWavesPerBlock + wave], amax_n = 0.0f;
    // The thresholds a row is judged by are asked for while the row BEFORE it is judged, along with that row's
    // prefetch (the host sends at most four queries to this scan): loads return in order, so waiting for a threshold
    // asked for after the prefetch would wait for all of it, and nothing would be in flight while the row is judged.
    uint64_t tau_a[4], tau_b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) tau_a[q] = a.tau[(uint32_t)q < nq ? q : 0];
    bool whole = false;    // wave-uniform: whole-row fallback, the bound is not evaluated for this row
    // One row: start the loads of the next one into the other register set, judge and score this one.  The two
    // register sets swap roles from row to row (two copies of the code) instead of being copied.
    auto step = [&](RowRegs<W, P, S>& cur, Hints& hc, float& amax, const uint64_t (&tau_c)[4],
                    RowRegs<W, P, S>& nxt, Hints& hn, float& amax_n, uint64_t (&tau_n)[4]) __attribute__((always_inline)) -> bool {
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const bool whole_next = passed * 4 > probed + 32 * nq;     // wave-uniform
        const uint32_t pl = has_next ? pn : p;      // prefetch not under a branch: see scan_exact_prog_hint
        auto tau_of = [&](uint32_t q) { return q == 0 ? tau_c[0] : (q == 1 ? tau_c[1] : (q == 2 ? tau_c[2] : tau_c[3])); };
        load_row_planes<W, P, S, 0, F>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
        amax_n = a.row_amax[(size_t)pl * kWavesPerBlock + wave];
#pragma unroll
        for (int q = 0; q < 4; ++q) tau_n[q] = a.tau[(uint32_t)q < nq ? q : 0];
        bool reach = true;
        uint32_t mine = (1u << kItemsPerLane) - 1u;     // which of this lane's items can still reach some query's threshold
        uint32_t row_pairs = nq;                         // queries for which some item of the row can
        if (!whole || (rows & 7u) == 0u) {
            mine = 0;
            row_pairs = 0;
            for (uint32_t q = 0; q < nq; ++q) {
                const QueryRegs<W, PQ> q0 = slot_query(slots[q]);
                const float taus0 = threshold_score(tau_of(q));
                const QueryMass mass{slots[q].mass_x, slots[q].mass_y};
                const float slack_all = 2.0f * mass.y + 0.015875f * mass.x;
                const float floor_c = floor_h * mass.x;
                const float mass_last = mass.x + 2.0f * mass.y;
                uint32_t mine_q = 0;
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    float s = floor_c, all = 0.0f;
#pragma unroll
                    for (int j = 0; j < F; ++j) {
                        float t = q0.bias;
#pragma unroll
                        for (int i = 0; i < PQ; ++i) {
                            uint32_t pc = 0;
#pragma unroll
                            for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ q0.w[i][h]);
                            t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                        }
                        const float hj = hint(hc, j, m);
                        s = __fmaf_rn(hj, t, s);
                        all += hj;
                    }
                    // (the bound of scan_exact_prog_hint)
                    const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(amax, mass_last, s));
                    mine_q |= !(ub < taus0) ? (1u << m) : 0u;      // (a NaN bound does not prune)
                }
                mine |= mine_q;
                row_pairs += __ballot(mine_q != 0u) != 0 ? 1u : 0u;
            }
            reach = __ballot(mine != 0u) != 0;
            probed += nq;
            passed += row_pairs;
        }
        ++rows;
        full_rows += reach ? 1u : 0u;
        if (STREAM_EXTRA) extra8 += kRow * (uint32_t)W * (uint32_t)STREAM_EXTRA;       // (planes that the caller's stream left out)
        if (reach) {
            full_pairs += row_pairs;
            // only the lanes that hold such an item read the rest of their items' data (the memory system fetches
            // the cache lines they touch, not the row) and score; an item whose bound is below the threshold cannot
            // be a survivor.  (Whole-row fallback, rows that are not probed: every lane, every item.)
            const char* tile = a.tiles + (size_t)p * tile_bytes;
            const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + (P - 1) * geom.plane_bytes()) + (size_t)wave * kRow * W;
            const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset()) + wave * kRow;
            // what the lanes ask for: per pair of items (W = 1) or per item, the last plane and S scales
            if constexpr (W == 1) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) extra8 += (uint32_t)__builtin_popcountll(__ballot((mine & (3u << (2 * h2))) != 0u)) * (2 + S);
            } else {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m)
                    extra8 += ((uint32_t)__builtin_popcountll(__ballot((mine & (1u << m)) != 0u)) * (2 * W + S)) / 2;
            }
            if constexpr (W == 1) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
                    if (mine & (3u << (2 * h2))) {
                        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + h2 * 128 + 2 * lane));
                        cur.w[P - 1][2 * h2][0] = v.x; cur.w[P - 1][2 * h2][1] = v.y;
                        cur.w[P - 1][2 * h2 + 1][0] = v.z; cur.w[P - 1][2 * h2 + 1][1] = v.w;
#pragma unroll
                        for (int j = 0; j < S; ++j) {
                            const f32x2 av = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sc + j * kTileItems + h2 * 128 + 2 * lane));
                            cur.a[j][2 * h2] = av.x; cur.a[j][2 * h2 + 1] = av.y;
                        }
                    }
            } else {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m)
                    if (mine & (1u << m)) {
#pragma unroll
                        for (int h = 0; h < W / 2; ++h) {
                            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + (size_t)(m * 64 + lane) * W) + h);
                            cur.w[P - 1][m][4 * h + 0] = v.x; cur.w[P - 1][m][4 * h + 1] = v.y;
                            cur.w[P - 1][m][4 * h + 2] = v.z; cur.w[P - 1][m][4 * h + 3] = v.w;
                        }
#pragma unroll
                        for (int j = 0; j < S; ++j) cur.a[j][m] = __builtin_nontemporal_load(sc + j * kTileItems + m * 64 + lane);
                    }
            }
            // every query scores the items that some query's bound let through (an item whose own bound is below
            // the threshold scores below it too, and is not appended)
            for (uint32_t q = 0; q < nq; ++q) {
                const QueryRegs<W, PQ> qr = slot_query(slots[q]);
                const uint64_t tau = a.tau[q];
                const float taus = threshold_score(tau);
                float sv[kItemsPerLane];
                bool any = false;
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    sv[m] = -__builtin_inff();
                    if (mine & (1u << m)) sv[m] = score_item<W, P, PQ, MODE>(cur, m, qr);
                    any |= (sv[m] >= taus);
                }
                if (__ballot(any)) stage_scores<W, false>(sv, tau, taus, q, p, wave, lane, s_keys, ms, 0, a);
            }
        }
        whole = whole_next;
        p = pn;
        return has_next;
    };
    for (;;) {
        if (!step(cur, hc, amax, tau_a, nxt, hn, amax_n, tau_b)) break;
        if (!step(nxt, hn, amax_n, tau_b, cur, hc, amax, tau_a)) break;
    }
    mstage_drain(ms, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_pairs && lane == 0 && full_pairs) atomicAdd(a.deep_pairs, full_pairs);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}


template <int W, int P, int PQ>
__global__ __launch_bounds__(kBlock) void scan_exact_batch_prog_hint(const ScanArgs a)
{
    extern __shared__ __align__(16) unsigned char s_dynamic[];
    __shared__ uint32_t s_cnt_all[kWavesPerBlock][65];
    __shared__ QuerySlot<W, PQ> s_query[4];           // (the host sends at most four queries to this scan)
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if (a.n_queries > 4u) return;                     // (every thread alike)
    stage_queries<W, PQ>(s_query, a.qwords, a.qcoef, a.qcoef + (size_t)a.n_queries * (PQ + 1), a.n_queries);
    uint64_t* s_keys = reinterpret_cast<uint64_t*>(s_dynamic) + (size_t)wave * a.stage_entries;
    const uint32_t n_sub = sub_queues_for(a.n_queries);
    const uint32_t per_sub = a.stage_entries / n_sub;
    const MultiStage ms{s_keys, s_cnt_all[wave], per_sub > 64u ? 64u : per_sub, 0u, n_sub};
    s_cnt_all[wave][lane] = 0;
    if (lane == 0) s_cnt_all[wave][64] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    batch_prog_hint_rows<W, P, PQ, 0>(a, p, 0u, 0u, 0u, s_keys, ms, s_query, wave, lane);
}


// scan_exact_prog2_hint for 2 .. 4 queries per call: the stream is the same (plane 0, the one-byte copies of all P
// scale arrays), stage A forms every query's bound from the one popcount pass per query over plane 0, and an item
// that some query's bound lets through is queued once, with each query's partial score and the set of queries that
// still want it.  Stage B reads the item's planes 1 .. P-2 once and continues the chains of those queries; stage C
// reads the rest once and scores the item from scratch for each query whose second bound it passed.  What is
// appended is what the batch form of scan_exact appends.  A wave of whose items more than one in 10 pass stage A
// takes the rest of its rows as scan_exact_batch_prog_hint does.  A: planes in the stream, as there (1 with three
// planes, 2 with four).
template <int W, int P, int PQ, int A = 1>
__global__ __launch_bounds__(kBlock) void scan_exact_batch_prog2_hint(const ScanArgs a)
{
    static_assert(P >= 3, "with two planes scan_exact_batch_prog_hint streams plane 0 alone already");
    static_assert(A >= 1 && A <= P - 2, "stage B reads planes A .. P-2");
    constexpr int MODE = kModeScaled;
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;   // hint words per lane and row (one byte per item and array)
    constexpr int kQueue = 128;                  // entries per wave: a batch of 64 leaves when 64 have gathered
    constexpr int QB = 4;                        // most queries per call
    extern __shared__ __align__(16) unsigned char s_dynamic[];
    __shared__ uint32_t s_cnt_all[kWavesPerBlock][65];
    __shared__ uint32_t s_qid[kWavesPerBlock][kQueue];      // physical tile * 1024 + item of the tile
    __shared__ float s_qs0[kWavesPerBlock][QB][kQueue];     // per query: where the bound's chain stands after the streamed planes
    __shared__ uint32_t s_qhb[kWavesPerBlock][kQueue];      // scale copies of arrays 0 .. P-2 in bytes 0 .. P-2, the queries that want the item in byte 3
    __shared__ float s_qam[kWavesPerBlock][kQueue];         // the copy of the item's last scale
    __shared__ QuerySlot<W, PQ> s_query[QB];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if (a.n_queries > (uint32_t)QB) return;                 // (the host sends at most QB; every thread alike)
    stage_queries<W, PQ>(s_query, a.qwords, a.qcoef, a.qcoef + (size_t)a.n_queries * (PQ + 1), a.n_queries);
    uint64_t* s_keys = reinterpret_cast<uint64_t*>(s_dynamic) + (size_t)wave * a.stage_entries;
    const uint32_t n_sub = sub_queues_for(a.n_queries);
    const uint32_t per_sub = a.stage_entries / n_sub;
    const MultiStage ms{s_keys, s_cnt_all[wave], per_sub > 64u ? 64u : per_sub, 0u, n_sub};
    s_cnt_all[wave][lane] = 0;
    if (lane == 0) s_cnt_all[wave][64] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const uint32_t nq = __builtin_amdgcn_readfirstlane(a.n_queries);     // (kept in a scalar register: the loops over the queries are the wave's, not the lanes')
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    uint32_t full_rows = 0, full_pairs = 0, extra8 = 0;
    uint32_t qfill = 0;                       // entries waiting for stage B (wave-uniform)
    uint32_t last_row = 0xFFFFFFFFu;          // row of the last item that reached stage C (wave-uniform)
    uint32_t probed = 0, passed = 0;          // items judged by stage A, items it let through for some query (wave-uniform)
    const uint32_t hb[3] = {(uint32_t)a.hint_base[0] << 5, (uint32_t)a.hint_base[1] << 5, (uint32_t)a.hint_base[2] << 5};
    auto decode = [&](uint32_t byte, int j) { return __uint_as_float((byte + hb[j]) << 18); };
    // (the constants of scan_exact_prog2_hint, per unit of a query's mass where they depend on it)
    float floor_all = __uint_as_float((uint32_t)a.hint_base_last << 23);
    for (int j = 0; j < F; ++j) floor_all += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_all *= 1.0001f;
    float floor_j[A];      // (the smallest copy of each streamed plane's array)
#pragma unroll
    for (int j = 0; j < A; ++j) floor_j[j] = 1.0001f * __uint_as_float((uint32_t)a.hint_base[j] << 23);
    const uint32_t hb_last = (uint32_t)a.hint_base_last << 5;

    struct Hints { uint32_t w[NW]; uint32_t last; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        h.last = __builtin_nontemporal_load(a.hints_last + ((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane);
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };

    // Stages B and C for the entries [base, base + n) of the wave's queue, one per lane.  All lanes of the wave.
    auto follow_up = [&](uint32_t base, uint32_t n) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const bool act = (uint32_t)lane < n;
        const uint32_t e = base + (act ? (uint32_t)lane : 0u);
        const uint32_t id = s_qid[wave][e], hbytes = s_qhb[wave][e];
        const float h_last = s_qam[wave][e];
        const uint32_t want = act ? hbytes >> 24 : 0u;        // queries whose first bound the item passed
        const uint32_t tp = id >> 10, idx = id & 1023u;
        const char* tile = a.tiles + (size_t)tp * tile_bytes;
        RowRegs<W, P, S> it;          // this lane's item, in slot 0
        float all = 0.0f;
#pragma unroll
        for (int j = 0; j < A; ++j) all += decode((hbytes >> (8 * j)) & 255u, j);
        float hj[F];
        if (act) {
#pragma unroll
            for (int j = A; j < F; ++j) {
                const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
                if constexpr (W == 1) {
                    const u32x2 v = *reinterpret_cast<const u32x2*>(kw);
                    it.w[j][0][0] = v.x; it.w[j][0][1] = v.y;
                } else {
#pragma unroll
                    for (int h = 0; h < W / 2; ++h) {
                        const u32x4 v = reinterpret_cast<const u32x4*>(kw)[h];
                        it.w[j][0][4 * h + 0] = v.x; it.w[j][0][4 * h + 1] = v.y; it.w[j][0][4 * h + 2] = v.z; it.w[j][0][4 * h + 3] = v.w;
                    }
                }
                hj[j] = decode((hbytes >> (8 * j)) & 255u, j);
                all += hj[j];
            }
        }
        extra8 += n * (uint32_t)W * (uint32_t)(F - A);
        uint32_t want2 = 0;           // queries whose second bound it passed too
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            if ((uint32_t)q >= nq) break;                     // wave-uniform
            const QueryRegs<W, PQ> q0 = slot_query(s_query[q]);
            const QueryMass mass{s_query[q].mass_x, s_query[q].mass_y};
            const float taus = threshold_score(a.tau[q]);
            const float slack_all = 2.0f * mass.y + 0.015875f * mass.x;
            const float mass_hint = mass.x + 2.0f * mass.y + slack_all;
            if ((want >> q) & 1u) {
                float s = s_qs0[wave][q][e];
#pragma unroll
                for (int j = A; j < F; ++j) {
                    float t = q0.bias;
#pragma unroll
                    for (int i = 0; i < PQ; ++i) {
                        uint32_t pc = 0;
#pragma unroll
                        for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(it.w[j][0][h] ^ q0.w[i][h]);
                        t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                    }
                    s = __fmaf_rn(hj[j], t, s);
                }
                // (the second bound of scan_exact_prog2_hint)
                const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(h_last, mass_hint, s));
                want2 |= !(ub < taus) ? (1u << q) : 0u;
            }
        }
        const uint64_t m2 = __ballot(want2 != 0u);
        if (m2) {
            uint64_t logical = 0;
            if (want2) {
                // the rest of the item: the streamed planes again (another lane had them), the last plane, the fp32 scales
#pragma unroll
                for (int jj = 0; jj <= A; ++jj) {
                    const int j = jj < A ? jj : P - 1;
                    const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) it.w[j][0][h] = kw[h];
                }
                const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset());
#pragma unroll
                for (int j = 0; j < S; ++j) it.a[j][0] = sc[j * kTileItems + idx];
                logical = (uint64_t)phys_to_tile_per_lane(a.layout, tp) * kTileItems + idx;
            }
#pragma unroll
            for (int q = 0; q < QB; ++q) {
                if ((uint32_t)q >= nq) break;                 // wave-uniform
                const QueryRegs<W, PQ> qr = slot_query(s_query[q]);
                const uint64_t tau = a.tau[q];
                const float taus = threshold_score(tau);
                const bool mine = ((want2 >> q) & 1u) != 0u;
                float score = -__builtin_inff();
                if (mine) score = score_item<W, P, PQ, MODE>(it, 0, qr);
                bool ok = mine && (score >= taus) && (logical < a.n_items);
                uint64_t key = 0;
                if (ok) { key = make_key(score, (uint32_t)logical); ok = key >= tau; }
                mstage_append(ok, key, (uint32_t)q, ms, a.out, lane);
                full_pairs += (uint32_t)__builtin_popcountll(__ballot(mine));
            }
            const uint32_t n2 = (uint32_t)__builtin_popcountll(m2);
            extra8 += n2 * ((uint32_t)(A + 1) * W + (uint32_t)S / 2u) + (n2 * ((uint32_t)S & 1u)) / 2u;
            // rows that hold such an item (see scan_exact_prog2_hint)
            const uint64_t below = m2 & ((1ull << lane) - 1ull);
            const int prev = below ? 63 - __builtin_clzll(below) : lane;
            const uint32_t row = id >> 8, row_prev = __shfl(row, prev);
            full_rows += (uint32_t)__builtin_popcountll(__ballot(want2 != 0u && row != (below ? row_prev : last_row)));
            last_row = __shfl(row, 63 - __builtin_clzll(m2));
        }
        __builtin_amdgcn_wave_barrier();
    };

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, A>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    // The thresholds a row is judged by are asked for while the row BEFORE it is judged, along with that row's
    // prefetch: loads return in order, so waiting for a threshold asked for after the prefetch would wait for all of
    // it, and nothing would be in flight while the row is judged.
    uint64_t tau_c[QB], tau_n[QB];
#pragma unroll
    for (int q = 0; q < QB; ++q) tau_c[q] = a.tau[(uint32_t)q < nq ? q : 0];
    bool give_up = false;
    for (;;) {
        if (passed * 10 > probed + 4096) { give_up = true; break; }         // wave-uniform; row p is not done yet
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const uint32_t pl = has_next ? pn : p;          // (unconditional prefetch: see scan_exact_prog_hint)
        load_row_planes<W, P, S, 0, A>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
#pragma unroll
        for (int q = 0; q < QB; ++q) tau_n[q] = a.tau[(uint32_t)q < nq ? q : 0];
        // what does not depend on the query
        uint32_t hbytes[kItemsPerLane];
        float hs[kItemsPerLane][A], h_seen[kItemsPerLane], h_last[kItemsPerLane], others[kItemsPerLane];
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            hbytes[m] = 0;
            float rest = 0.0f;
            h_seen[m] = 0.0f;
#pragma unroll
            for (int j = 0; j < F; ++j) {
                const uint32_t c = (hc.w[j] >> (8 * m)) & 255u;
                hbytes[m] |= c << (8 * j);
                if (j >= A) rest += decode(c, j);
                else { hs[m][j] = decode(c, j); h_seen[m] += hs[m][j]; }
            }
            h_last[m] = __uint_as_float((((hc.last >> (8 * m)) & 255u) + hb_last) << 18);
            others[m] = rest + h_last[m];
        }
        float s0[kItemsPerLane][QB];
        uint32_t want[kItemsPerLane];
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            want[m] = 0;
#pragma unroll
            for (int q = 0; q < QB; ++q) s0[m][q] = 0.0f;
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            if ((uint32_t)q >= nq) break;                     // wave-uniform
            const QueryRegs<W, PQ> q0 = slot_query(s_query[q]);
            const QueryMass mass{s_query[q].mass_x, s_query[q].mass_y};
            const float taus = threshold_score(tau_c[q]);
            const float slack_all = 2.0f * mass.y + 0.015875f * mass.x;
            const float mass_hint = mass.x + 2.0f * mass.y + slack_all;
            const float floor_c = floor_all * mass.x;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                float chain = floor_c;       // (where stage B takes the chain up)
                float seen = 0.0f;
#pragma unroll
                for (int j = 0; j < A; ++j) {
                    float t = q0.bias;
#pragma unroll
                    for (int i = 0; i < PQ; ++i) {
                        uint32_t pc = 0;
#pragma unroll
                        for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ q0.w[i][h]);
                        t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                    }
                    chain = __fmaf_rn(hs[m][j], t, chain);
                    seen = __fmaf_rn(__builtin_fabsf(t), __fmaf_rn(0.015875f, hs[m][j], floor_j[j]), __fmaf_rn(hs[m][j], t, seen));
                }
                s0[m][q] = chain;
                // (the first bound of scan_exact_prog2_hint)
                const float ub = __fmaf_rn(others[m], mass_hint, __fmaf_rn(2.0f * mass.y, h_seen[m], seen));
                want[m] |= !(ub < taus) ? (1u << q) : 0u;     // (a NaN bound does not prune)
            }
        }
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            const bool pass = want[m] != 0u;
            const uint64_t mk = __ballot(pass);
            if (mk) {
                if (pass) {
                    const uint32_t at = qfill + (uint32_t)__builtin_popcountll(mk & ((1ull << lane) - 1ull));
                    s_qid[wave][at] = p * (uint32_t)kTileItems + (uint32_t)wave * kRow + lane_item<W>(lane, m);
#pragma unroll
                    for (int q = 0; q < QB; ++q) s_qs0[wave][q][at] = s0[m][q];
                    s_qhb[wave][at] = hbytes[m] | (want[m] << 24);
                    s_qam[wave][at] = h_last[m];
                }
                const uint32_t n = (uint32_t)__builtin_popcountll(mk);
                qfill += n;
                passed += n;
                if (qfill >= 64) {
                    // the 64 oldest entries leave; the rest (fewer than 64) move to the front
                    follow_up(0, 64);
                    qfill -= 64;
                    const bool mv = (uint32_t)lane < qfill;
                    const uint32_t from = 64u + (mv ? (uint32_t)lane : 0u);
                    const uint32_t e_id = s_qid[wave][from], e_hb = s_qhb[wave][from];
                    const float e_am = s_qam[wave][from];
                    float e_s0[QB];
#pragma unroll
                    for (int q = 0; q < QB; ++q) e_s0[q] = s_qs0[wave][q][from];
                    __builtin_amdgcn_wave_barrier();
                    if (mv) {
                        s_qid[wave][lane] = e_id; s_qhb[wave][lane] = e_hb; s_qam[wave][lane] = e_am;
#pragma unroll
                        for (int q = 0; q < QB; ++q) s_qs0[wave][q][lane] = e_s0[q];
                    }
                }
            }
        }
        probed += kRow;
        if (!has_next) { p = pn; break; }
        cur = nxt; hc = hn;
#pragma unroll
        for (int q = 0; q < QB; ++q) tau_c[q] = tau_n[q];
        p = pn;
    }
    if (qfill) follow_up(0, qfill);
    if (give_up) {
        batch_prog_hint_rows<W, P, PQ, P - 1 - A>(a, p, full_rows, full_pairs, extra8, s_keys, ms, s_query, wave, lane);
        return;
    }
    mstage_drain(ms, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_pairs && lane == 0 && full_pairs) atomicAdd(a.deep_pairs, full_pairs);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}


// ---------------------------------------------------------------- hybrid scoring (fp32 query)
// t_j = sum over the 8W bytes of plane j of lut[p][byte], accumulated in fp32 in byte order;
// kModeScaled: s = sum_j fma(a_j, t_j, s).  Dyadic modes: s = (sum_j 2^-j t_j) [* the item's scale].
template <int W, int P, int MODE, int J0, int J1>
__device__ __forceinline__ float fq_planes(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m, const float (*lut)[256],
                                           float s)
{
#pragma unroll
    for (int j = J0; j < J1; ++j) {
        float t = 0.0f;
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) {
            const uint32_t w = r.w[j][m][h];
            t += lut[4 * h + 0][w & 255u];
            t += lut[4 * h + 1][(w >> 8) & 255u];
            t += lut[4 * h + 2][(w >> 16) & 255u];
            t += lut[4 * h + 3][w >> 24];
        }
        if (MODE == kModeScaled) s = __fmaf_rn(r.a[j][m], t, s);
        else s = __fmaf_rn(1.0f / (float)(1 << j), t, s);
    }
    return s;
}

template <int W, int P, int MODE>
__device__ __forceinline__ float score_item_fq(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m,
                                               const float (*lut)[256])
{
    const float s = fq_planes<W, P, MODE, 0, P>(r, m, lut, 0.0f);
    return MODE == kModeDyadicNorm ? s * r.a[0][m] : s;
}

// Upper bound on score_item_fq from planes 0 .. P-2 (see bound_item_rowmax): no plane's table sum exceeds the
// query's mass sum_d |q_d| (mass.x, rounding of the table entries and of their sum included), the last plane's
// weight is at most amax (the row's largest a_{P-1}) or is 2^-(P-1), and mass.y per unit of weight covers the
// roundings of the chain.  kModeDyadicNorm: the row's largest inverse norm multiplies a positive bound.
template <int W, int P, int MODE>
__device__ __forceinline__ float bound_item_fq(const RowRegs<W, P, scale_arrays(MODE, P)>& r, int m, float part,
                                               const QueryMass& mass, float amax)
{
    float tail, all;
    if (MODE == kModeScaled) {
        tail = amax;
        all = amax;
#pragma unroll
        for (int j = 0; j < P - 1; ++j) all += r.a[j][m];
    } else {
        tail = 1.0f / (float)(1 << (P - 1));
        all = 2.0f;
    }
    const float ub = __fmaf_rn(all, mass.y, __fmaf_rn(tail, mass.x, part));
    if (MODE == kModeDyadicNorm) return ub > 0.0f ? ub * amax : 0.0f;
    return ub;
}

template <int W, int P, int MODE>
__global__ __launch_bounds__(kBlock) void scan_exact_fq(const FqArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ float s_lut[8 * W][256];
    constexpr int S = scale_arrays(MODE, P);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    for (int i = threadIdx.x; i < 8 * W * 256; i += kBlock) (&s_lut[0][0])[i] = a.lut[i];
    __syncthreads();

    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    const uint64_t tau = a.tau_ptr[0];
    const float taus = threshold_score(tau);
    uint32_t fill = 0;
    RowRegs<W, P, S> cur, nxt;
    load_row<W, P, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    for (;;) {
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        load_row<W, P, S>(nxt, a.tiles + (size_t)(has_next ? pn : p) * tile_bytes, wave, lane);   // unconditional: see scan_exact_prog_hint
        float s[kItemsPerLane];
        bool any = false;
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            s[m] = score_item_fq<W, P, MODE>(cur, m, s_lut);
            any |= (s[m] >= taus);
        }
        if (__ballot(any)) {
            const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                const uint64_t id = row_id + lane_item<W>(lane, m);
                bool ok = (s[m] >= taus) && (id < a.n_items);
                uint64_t key = 0;
                if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
                fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
            }
        }
        if (!has_next) break;
        cur = nxt;
        p = pn;
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
}

// scan_exact_fq, progressive (P >= 2): as scan_exact_prog, with the table sums in place of the popcounts.
template <int W, int P, int MODE>
__global__ __launch_bounds__(kBlock) void scan_exact_fq_prog(const FqArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ float s_lut[8 * W][256];
    constexpr int S = scale_arrays(MODE, P);
    constexpr int F = P - 1;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    for (int i = threadIdx.x; i < 8 * W * 256; i += kBlock) (&s_lut[0][0])[i] = a.lut[i];
    __syncthreads();

    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    const uint64_t tau = a.tau_ptr[0];
    const float taus = threshold_score(tau);
    const QueryMass mass = a.mass;
    uint32_t fill = 0, rows = 0, deep = 0, full_rows = 0;
    constexpr int SS = S > 0 ? S - 1 : 0;
    RowRegs<W, P, S> cur, nxt;
    load_row_planes<W, P, S, 0, F>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_row_scales<W, P, S, 0, SS>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    float amax = S > 0 ? a.row_amax[(size_t)p * kWavesPerBlock + wave] : 0.0f, amax_n = 0.0f;
    bool whole = false;
    for (;;) {
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const bool whole_next = deep * 4 > rows + 32;
        const uint32_t pl = has_next ? pn : p;      // prefetch not under a branch: see scan_exact_prog_hint
        const char* tn = a.tiles + (size_t)pl * tile_bytes;
        load_row_planes<W, P, S, 0, F>(nxt, tn, wave, lane);
        load_row_scales<W, P, S, 0, SS>(nxt, tn, wave, lane);
        if (S > 0) amax_n = a.row_amax[(size_t)pl * kWavesPerBlock + wave];
        if (whole_next) {
            load_row_planes<W, P, S, F, P>(nxt, tn, wave, lane);
            load_row_scales<W, P, S, SS, S>(nxt, tn, wave, lane);
        }
        float part[kItemsPerLane];
        bool reach = false;
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            part[m] = fq_planes<W, P, MODE, 0, F>(cur, m, s_lut, 0.0f);
            reach |= !(bound_item_fq<W, P, MODE>(cur, m, part[m], mass, amax) < taus);
        }
        reach = __ballot(reach) != 0;
        ++rows;
        full_rows += (whole || reach) ? 1u : 0u;
        if (reach) {
            if (!whole) {
                load_row_planes<W, P, S, F, P>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
                load_row_scales<W, P, S, SS, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
            }
            ++deep;
            float s[kItemsPerLane];
            bool any = false;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                const float v = fq_planes<W, P, MODE, F, P>(cur, m, s_lut, part[m]);
                s[m] = MODE == kModeDyadicNorm ? v * cur.a[0][m] : v;
                any |= (s[m] >= taus);
            }
            if (__ballot(any)) {
                const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow;
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    const uint64_t id = row_id + lane_item<W>(lane, m);
                    bool ok = (s[m] >= taus) && (id < a.n_items);
                    uint64_t key = 0;
                    if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
                    fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
                }
            }
        }
        if (!has_next) break;
        cur = nxt;
        amax = amax_n;
        whole = whole_next;
        p = pn;
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
}

// scan_exact_fq_prog for general scales with the one-byte scale copies in the stream (see
// scan_exact_prog_hint): rows that pass the bound are scored from scratch by score_item_fq.
// BIN: the bound is formed from a 4-plane binary approximation qhat of the query by XOR/popcounts, as in the
// binary-query scan, instead of from table sums (8W LDS reads per plane and item).  A plane's table sum q . b is
// qhat . b + (q - qhat) . b, and the second term is at most R = sum_d |q_d - qhat_d| (a.resid): the bound gains
// R per unit of the scale sum, about 6 % of the query's mass against the 25 % that the left-out plane costs anyway.
// The rows of a wave from tile p on, with what the wave has queued and counted so far (see prog_hint_rows): the whole
// of scan_exact_fq_prog_hint, and what scan_exact_fq_prog2_hint falls back to.
template <int W, int P, bool BIN, int STREAM_EXTRA>
__device__ __forceinline__ void fq_prog_hint_rows(const FqArgs& a, uint32_t p, uint32_t fill, uint32_t full_rows, uint32_t extra8,
                                                  uint64_t* s_keys, const float (&s_lut)[8 * W][256], int wave, int lane)
{
    constexpr int PQB = 4;
    constexpr int MODE = kModeScaled;
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();
    const uint64_t tau = a.tau_ptr[0];
    const float taus = threshold_score(tau);
    const QueryMass mass = a.mass;
    // |a_j t_j - h_j t_j| <= 0.015875 h_j |t_j| with |t_j| at most the mass of what t_j is formed from; BIN: the
    // roundings of both chains, and a_j R <= 1.04 h_j R
    const float slack_all = BIN ? 2.0f * (mass.y + a.bmass.y) + 0.015875f * a.bmass.x + 1.04f * a.resid
                                : 2.0f * mass.y + 0.015875f * mass.x;
    QueryRegs<W, PQB> qb{};
    if constexpr (BIN) qb = load_query<W, PQB>(a.qwords, a.qcoef, 0);
    uint32_t probed = 0, passed = 0;

    struct Hints { uint32_t w[NW]; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 1) {
            h.w[0] = __builtin_nontemporal_load(src);
        } else if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };
    // hint byte (3-bit exponent above base_j, 5-bit mantissa) -> fp32
    const uint32_t hb0 = (uint32_t)a.hint_base[0] << 5, hb1 = (uint32_t)a.hint_base[1] << 5, hb2 = (uint32_t)a.hint_base[2] << 5;
    auto hint = [&](const Hints& h, int j, int m) {
        const uint32_t c = (h.w[j] >> (8 * m)) & 255u;
        return __uint_as_float((c + (j == 0 ? hb0 : (j == 1 ? hb1 : hb2))) << 18);
    };
    // a scale below the smallest hint of its array, 2^(base_j - 127), is off by up to that much instead
    float floor_c = 0.0f;
    for (int j = 0; j < F; ++j) floor_c += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_c *= 1.0001f * (BIN ? a.bmass.x + a.resid : mass.x);
    const float mass_last = mass.x + 2.0f * mass.y;      // (the last plane's term is bounded by the query's own mass)

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, F>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    float amax = a.row_amax[(size_t)p * kWavesPerBlock + wave], amax_n = 0.0f;
    bool plain = false;    // wave-uniform: the bound lets most rows through; the rest of the wave's rows go the plain way
    // scores the items `mine` of this lane in the row held by r (every plane and scale of them loaded) and queues
    // what reaches the threshold
    auto score_row = [&](const RowRegs<W, P, S>& r, uint32_t mine, uint32_t p) __attribute__((always_inline)) {
        float s[kItemsPerLane];
        bool any = false;
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            s[m] = -__builtin_inff();
            if (mine & (1u << m)) s[m] = score_item_fq<W, P, MODE>(r, m, s_lut);
            any |= (s[m] >= taus);
        }
        if (__ballot(any)) {
            const uint64_t row_id = (uint64_t)phys_to_tile(a.layout, p) * kTileItems + (uint64_t)wave * kRow;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                const uint64_t id = row_id + lane_item<W>(lane, m);
                bool ok = (s[m] >= taus) && (id < a.n_items);
                uint64_t key = 0;
                if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
                fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
            }
        }
    };
    // one row, as in scan_exact_prog_hint: the two register sets swap roles from row to row
    auto step = [&](RowRegs<W, P, S>& cur, Hints& hc, float& amax, RowRegs<W, P, S>& nxt, Hints& hn, float& amax_n)
                    __attribute__((always_inline)) -> bool {
        if (passed * 4 > probed + 32) { plain = true; return false; }     // wave-uniform; this row is not done yet
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        // The prefetch is not under a branch (a workgroup's last step fetches its own row once more): with
        // `if (has_next)` around it the compiler, merging the path that loaded with the one that did not, makes
        // the first use of THIS row's registers wait for half of the loads just issued -- every step then stalls
        // for a memory round trip and nothing is prefetched.
        const uint32_t pl = has_next ? pn : p;
        load_row_planes<W, P, S, 0, F>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
        amax_n = a.row_amax[(size_t)pl * kWavesPerBlock + wave];
        bool reach = true;
        uint32_t mine = 0;     // which of this lane's items can still reach the threshold
        {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                float s = floor_c, all = 0.0f;
#pragma unroll
                for (int j = 0; j < F; ++j) {
                    float t = 0.0f;
                    if constexpr (BIN) {
                        t = qb.bias;
#pragma unroll
                        for (int i = 0; i < PQB; ++i) {
                            uint32_t pc = 0;
#pragma unroll
                            for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ qb.w[i][h]);
                            t = __fmaf_rn(qb.m2c[i], (float)pc, t);
                        }
                    } else {
#pragma unroll
                        for (int h = 0; h < 2 * W; ++h) {
                            const uint32_t w = cur.w[j][m][h];
                            t += s_lut[4 * h + 0][w & 255u];
                            t += s_lut[4 * h + 1][(w >> 8) & 255u];
                            t += s_lut[4 * h + 2][(w >> 16) & 255u];
                            t += s_lut[4 * h + 3][w >> 24];
                        }
                    }
                    const float hj = hint(hc, j, m);
                    s = __fmaf_rn(hj, t, s);
                    all += hj;
                }
                const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(amax, mass_last, s));
                mine |= !(ub < taus) ? (1u << m) : 0u;      // (a NaN bound does not prune)
            }
            reach = __ballot(mine != 0u) != 0;
            ++probed;
            passed += reach ? 1u : 0u;
        }
        full_rows += reach ? 1u : 0u;
        if (STREAM_EXTRA) extra8 += kRow * (uint32_t)W * (uint32_t)STREAM_EXTRA;
        if (reach) {
            {
                // lane-wise, as in scan_exact_prog_hint
                const char* tile = a.tiles + (size_t)p * tile_bytes;
                const uint64_t* pj = reinterpret_cast<const uint64_t*>(tile + (P - 1) * geom.plane_bytes()) + (size_t)wave * kRow * W;
                const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset()) + wave * kRow;
                if constexpr (W == 1) {
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) extra8 += (uint32_t)__builtin_popcountll(__ballot((mine & (3u << (2 * h2))) != 0u)) * (2 + S);
                } else {
#pragma unroll
                    for (int m = 0; m < kItemsPerLane; ++m)
                        extra8 += ((uint32_t)__builtin_popcountll(__ballot((mine & (1u << m)) != 0u)) * (2 * W + S)) / 2;
                }
                if constexpr (W == 1) {
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
                        if (mine & (3u << (2 * h2))) {
                            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + h2 * 128 + 2 * lane));
                            cur.w[P - 1][2 * h2][0] = v.x; cur.w[P - 1][2 * h2][1] = v.y;
                            cur.w[P - 1][2 * h2 + 1][0] = v.z; cur.w[P - 1][2 * h2 + 1][1] = v.w;
#pragma unroll
                            for (int j = 0; j < S; ++j) {
                                const f32x2 av = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sc + j * kTileItems + h2 * 128 + 2 * lane));
                                cur.a[j][2 * h2] = av.x; cur.a[j][2 * h2 + 1] = av.y;
                            }
                        }
                } else {
#pragma unroll
                    for (int m = 0; m < kItemsPerLane; ++m)
                        if (mine & (1u << m)) {
#pragma unroll
                            for (int h = 0; h < W / 2; ++h) {
                                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + (size_t)(m * 64 + lane) * W) + h);
                                cur.w[P - 1][m][4 * h + 0] = v.x; cur.w[P - 1][m][4 * h + 1] = v.y;
                                cur.w[P - 1][m][4 * h + 2] = v.z; cur.w[P - 1][m][4 * h + 3] = v.w;
                            }
#pragma unroll
                            for (int j = 0; j < S; ++j) cur.a[j][m] = __builtin_nontemporal_load(sc + j * kTileItems + m * 64 + lane);
                        }
                }
            }
            score_row(cur, mine, p);
        }
        p = pn;
        return has_next;
    };
    for (;;) {
        if (!step(cur, hc, amax, nxt, hn, amax_n)) break;
        if (!step(nxt, hn, amax_n, cur, hc, amax)) break;
    }
    if (plain) {
        // from row p on as scan_exact_fq does it: whole rows, the next one in flight while this one is scored
        load_row<W, P, S>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
        for (;;) {
            const uint32_t pn = p + G;
            const bool has_next = pn < a.p_end;
            load_row<W, P, S>(nxt, a.tiles + (size_t)(has_next ? pn : p) * tile_bytes, wave, lane);   // unconditional: see scan_exact_prog_hint
            score_row(cur, (1u << kItemsPerLane) - 1u, p);
            ++full_rows;
            extra8 += kRow * (W + S / 2) + (kRow * (S & 1)) / 2;     // 8W + 4S bytes per item beyond the stream's
            if (STREAM_EXTRA) extra8 += kRow * (uint32_t)W * (uint32_t)STREAM_EXTRA;
            if (!has_next) break;
            cur = nxt;
            p = pn;
        }
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}

template <int W, int P, bool BIN>
__global__ __launch_bounds__(kBlock) void scan_exact_fq_prog_hint(const FqArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ float s_lut[8 * W][256];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 8 * W * 256; i += kBlock) (&s_lut[0][0])[i] = a.lut[i];
    __syncthreads();
    const uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    fq_prog_hint_rows<W, P, BIN, 0>(a, p, 0u, 0u, 0u, s_keys_all[wave], s_lut, wave, lane);
}

// scan_exact_prog2_hint for an fp32 query (hybrid scoring): the bounds of both stages are formed from the 4-plane
// binary approximation qhat of the query by XOR/popcounts, as in scan_exact_fq_prog_hint<.., true> (the query's own
// sums differ from qhat's by at most a.resid per plane); what passes both is scored from the byte tables.
// A: planes in the stream (1 with three planes, 2 with four: see scan_exact_prog2_hint).
template <int W, int P, int A = 1>
__global__ __launch_bounds__(kBlock) void scan_exact_fq_prog2_hint(const FqArgs a)
{
    static_assert(P >= 3, "with two planes scan_exact_fq_prog_hint streams plane 0 alone already");
    static_assert(A >= 1 && A <= P - 2, "stage B reads planes A .. P-2");
    constexpr int MODE = kModeScaled;
    constexpr int PQ = 4;                        // planes of the query's binary approximation
    constexpr int S = P, F = P - 1;
    constexpr int NW = S - 1 == 3 ? 4 : S - 1;   // hint words per lane and row (one byte per item and array)
    constexpr int kQueue = 128;                  // entries per wave: a batch of 64 leaves when 64 have gathered
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ uint32_t s_qid[kWavesPerBlock][kQueue];    // physical tile * 1024 + item of the tile
    __shared__ float s_qs0[kWavesPerBlock][kQueue];       // floor + h_0 t_0: where the bound's chain stands after plane 0
    __shared__ uint32_t s_qhb[kWavesPerBlock][kQueue];    // the item's scale copies, array j in byte j
    __shared__ float s_qam[kWavesPerBlock][kQueue];       // the copy of the item's last scale
    __shared__ float s_lut[8 * W][256];
    for (int i = threadIdx.x; i < 8 * W * 256; i += kBlock) (&s_lut[0][0])[i] = a.lut[i];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint64_t* s_keys = s_keys_all[wave];
    const uint32_t G = gridDim.x;
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const size_t tile_bytes = geom.tile_bytes();

    uint32_t p = a.p_begin + blockIdx.x;
    if (p >= a.p_end) return;
    uint32_t fill = 0, full_rows = 0, extra8 = 0;
    uint32_t qfill = 0;                       // entries waiting for stage B (wave-uniform)
    uint32_t last_row = 0xFFFFFFFFu;          // row of the last item that reached stage C (wave-uniform)
    uint32_t probed = 0, passed = 0;          // items judged by stage A, items it let through (wave-uniform)
    const QueryRegs<W, PQ> q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);     // qhat, the binary approximation
    const QueryMass mass = a.mass;                                            // of the query itself
    // per unit of a scale copy whose plane's sum was formed from qhat (as in scan_exact_fq_prog_hint<.., true>) ...
    const float slack_all = 2.0f * (mass.y + a.bmass.y) + 0.015875f * a.bmass.x + 1.04f * a.resid;
    // ... and of one whose plane has not been looked at: its table sum is at most the query's own mass
    const float slack_mass = 2.0f * mass.y + 0.015875f * mass.x;
    const uint64_t tau0 = a.tau_ptr[0];
    const float taus0 = threshold_score(tau0);
    const uint32_t hb[3] = {(uint32_t)a.hint_base[0] << 5, (uint32_t)a.hint_base[1] << 5, (uint32_t)a.hint_base[2] << 5};
    auto decode = [&](uint32_t byte, int j) { return __uint_as_float((byte + hb[j]) << 18); };
    // a scale below the smallest copy of its array, 2^(base - 127), is off by up to that much instead (all P arrays here)
    float floor_c = __uint_as_float((uint32_t)a.hint_base_last << 23);
    for (int j = 0; j < F; ++j) floor_c += __uint_as_float((uint32_t)a.hint_base[j] << 23);
    floor_c *= 1.0001f * (a.bmass.x + a.resid + mass.x);
    const float mass_last = mass.x + 2.0f * mass.y;
    const float mass_hint = mass_last + slack_mass;     // what a plane whose scale is known by its copy can add, per unit of the copy
    float floor_j[A];      // (the smallest copy of each streamed plane's array)
#pragma unroll
    for (int j = 0; j < A; ++j) floor_j[j] = 1.0001f * __uint_as_float((uint32_t)a.hint_base[j] << 23);
    const uint32_t hb_last = (uint32_t)a.hint_base_last << 5;

    struct Hints { uint32_t w[NW]; uint32_t last; };
    auto load_hints = [&](Hints& h, uint32_t tile_p) {
        h.last = __builtin_nontemporal_load(a.hints_last + ((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane);
        const uint32_t* src = a.hints + (((size_t)tile_p * kWavesPerBlock + wave) * 64 + lane) * NW;
        if constexpr (NW == 2) {
            const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            h.w[0] = v.x; h.w[1] = v.y;
        } else {
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
            h.w[0] = v.x; h.w[1] = v.y; h.w[2] = v.z; h.w[3] = v.w;
        }
    };

    // Stage B (and C) for the entries [base, base + n) of the wave's queue, one per lane.  All lanes of the wave.
    auto follow_up = [&](uint32_t base, uint32_t n) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const bool act = (uint32_t)lane < n;
        const uint32_t e = base + (act ? (uint32_t)lane : 0u);
        const uint32_t id = s_qid[wave][e], hbytes = s_qhb[wave][e];
        const float h_last = s_qam[wave][e];
        float s = s_qs0[wave][e];
        const uint32_t tp = id >> 10, idx = id & 1023u;
        const char* tile = a.tiles + (size_t)tp * tile_bytes;
        RowRegs<W, P, S> it;          // this lane's item, in slot 0
        bool pass2 = false;
        if (act) {
            float all = 0.0f;
#pragma unroll
            for (int j = 0; j < A; ++j) all += decode((hbytes >> (8 * j)) & 255u, j);
#pragma unroll
            for (int j = A; j < F; ++j) {
                const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
                if constexpr (W == 1) {
                    const u32x2 v = *reinterpret_cast<const u32x2*>(kw);
                    it.w[j][0][0] = v.x; it.w[j][0][1] = v.y;
                } else {
#pragma unroll
                    for (int h = 0; h < W / 2; ++h) {
                        const u32x4 v = reinterpret_cast<const u32x4*>(kw)[h];
                        it.w[j][0][4 * h + 0] = v.x; it.w[j][0][4 * h + 1] = v.y; it.w[j][0][4 * h + 2] = v.z; it.w[j][0][4 * h + 3] = v.w;
                    }
                }
                float t = q0.bias;
#pragma unroll
                for (int i = 0; i < PQ; ++i) {
                    uint32_t pc = 0;
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(it.w[j][0][h] ^ q0.w[i][h]);
                    t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                }
                const float hj = decode((hbytes >> (8 * j)) & 255u, j);
                s = __fmaf_rn(hj, t, s);
                all += hj;
            }
            // the bound of scan_exact_prog_hint, with the item's own last scale (by its copy) for the row's largest
            const float ub = __fmaf_rn(all, slack_all, __fmaf_rn(h_last, mass_hint, s));
            pass2 = !(ub < taus0);
        }
        extra8 += n * (uint32_t)W * (uint32_t)(F - A);
        const uint64_t m2 = __ballot(pass2);
        if (m2) {
            float score = -__builtin_inff();
            uint64_t logical = 0;
            if (pass2) {
                // the rest of the item: the streamed planes again (another lane had them), the last plane, the fp32 scales
#pragma unroll
                for (int jj = 0; jj <= A; ++jj) {
                    const int j = jj < A ? jj : P - 1;
                    const uint32_t* kw = reinterpret_cast<const uint32_t*>(tile + (size_t)j * geom.plane_bytes() + (size_t)idx * 8 * W);
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) it.w[j][0][h] = kw[h];
                }
                const float* sc = reinterpret_cast<const float*>(tile + geom.scales_offset());
#pragma unroll
                for (int j = 0; j < S; ++j) it.a[j][0] = sc[j * kTileItems + idx];
                score = score_item_fq<W, P, MODE>(it, 0, s_lut);
                logical = (uint64_t)phys_to_tile_per_lane(a.layout, tp) * kTileItems + idx;
            }
            bool ok = pass2 && (score >= taus0) && (logical < a.n_items);
            uint64_t key = 0;
            if (ok) { key = make_key(score, (uint32_t)logical); ok = key >= tau0; }
            fill = stage_append1(ok, key, s_keys, fill, a.out, lane);
            const uint32_t n2 = (uint32_t)__builtin_popcountll(m2);
            extra8 += n2 * ((uint32_t)(A + 1) * W + (uint32_t)S / 2u) + (n2 * ((uint32_t)S & 1u)) / 2u;
            // rows that hold such an item: entries leave the queue in the order of their rows, so an item opens a
            // new row if the nearest lower lane with such an item (or, for the lowest, the last batch) holds another one
            const uint64_t below = m2 & ((1ull << lane) - 1ull);
            const int prev = below ? 63 - __builtin_clzll(below) : lane;
            const uint32_t row = id >> 8, row_prev = __shfl(row, prev);
            full_rows += (uint32_t)__builtin_popcountll(__ballot(pass2 && row != (below ? row_prev : last_row)));
            last_row = __shfl(row, 63 - __builtin_clzll(m2));
        }
        __builtin_amdgcn_wave_barrier();
    };

    RowRegs<W, P, S> cur, nxt;
    Hints hc, hn;
    load_row_planes<W, P, S, 0, A>(cur, a.tiles + (size_t)p * tile_bytes, wave, lane);
    load_hints(hc, p);
    bool give_up = false;
    for (;;) {
        if (passed * 10 > probed + 4096) { give_up = true; break; }         // wave-uniform; row p is not done yet
        const uint32_t pn = p + G;
        const bool has_next = pn < a.p_end;
        const uint32_t pl = has_next ? pn : p;          // (unconditional prefetch: see scan_exact_prog_hint)
        load_row_planes<W, P, S, 0, A>(nxt, a.tiles + (size_t)pl * tile_bytes, wave, lane);
        load_hints(hn, pl);
#pragma unroll
        for (int m = 0; m < kItemsPerLane; ++m) {
            uint32_t hbytes = 0;
            float rest = 0.0f;
#pragma unroll
            for (int j = 0; j < F; ++j) {
                const uint32_t c = (hc.w[j] >> (8 * m)) & 255u;
                hbytes |= c << (8 * j);
                if (j >= A) rest += decode(c, j);
            }
            const float h_last = __uint_as_float((((hc.last >> (8 * m)) & 255u) + hb_last) << 18);
            float s0 = floor_c;          // the chain of the one-stage bound after the streamed planes (stage B takes it up)
            float seen = 0.0f;           // what the streamed planes add to this stage's bound
            float h_seen = 0.0f;         // their scale copies, added up
#pragma unroll
            for (int j = 0; j < A; ++j) {
                float t = q0.bias;
#pragma unroll
                for (int i = 0; i < PQ; ++i) {
                    uint32_t pc = 0;
#pragma unroll
                    for (int h = 0; h < 2 * W; ++h) pc += __builtin_popcount(cur.w[j][m][h] ^ q0.w[i][h]);
                    t = __fmaf_rn(q0.m2c[i], (float)pc, t);
                }
                const float hj = decode((hbytes >> (8 * j)) & 255u, j);
                s0 = __fmaf_rn(hj, t, s0);
                seen = __fmaf_rn(__builtin_fabsf(t), __fmaf_rn(0.015875f, hj, floor_j[j]), __fmaf_rn(hj, t, seen));
                h_seen += hj;
            }
            // The first bound of scan_exact_prog2_hint, plane by plane of the stream: a_j t_j <= h_j t_j +
            // (0.015875 h_j + floor_j) |t_j|, every other plane at most (its copy) x (mass + slack).  fp32 query: t_j
            // is qhat's sum; the query's own differs from it by at most a.resid, and the roundings of both sums
            // are allowed for per unit of the streamed planes' copies.
            const float ub = __fmaf_rn(rest + h_last, mass_hint,
                                       __fmaf_rn(2.0f * (mass.y + a.bmass.y) + 1.04f * a.resid, h_seen, seen));
            const bool pass = !(ub < taus0);            // (a NaN bound does not prune)
            const uint64_t mk = __ballot(pass);
            if (mk) {
                if (pass) {
                    const uint32_t at = qfill + (uint32_t)__builtin_popcountll(mk & ((1ull << lane) - 1ull));
                    s_qid[wave][at] = p * (uint32_t)kTileItems + (uint32_t)wave * kRow + lane_item<W>(lane, m);
                    s_qs0[wave][at] = s0;
                    s_qhb[wave][at] = hbytes;
                    s_qam[wave][at] = h_last;
                }
                const uint32_t n = (uint32_t)__builtin_popcountll(mk);
                qfill += n;
                passed += n;
                if (qfill >= 64) {
                    // the 64 oldest entries leave; the rest (fewer than 64) move to the front
                    follow_up(0, 64);
                    qfill -= 64;
                    const bool mv = (uint32_t)lane < qfill;
                    const uint32_t from = 64u + (mv ? (uint32_t)lane : 0u);
                    const uint32_t e_id = s_qid[wave][from], e_hb = s_qhb[wave][from];
                    const float e_s0 = s_qs0[wave][from], e_am = s_qam[wave][from];
                    __builtin_amdgcn_wave_barrier();
                    if (mv) { s_qid[wave][lane] = e_id; s_qhb[wave][lane] = e_hb; s_qs0[wave][lane] = e_s0; s_qam[wave][lane] = e_am; }
                }
            }
        }
        probed += kRow;
        if (!has_next) { p = pn; break; }
        cur = nxt; hc = hn;
        p = pn;
    }
    if (qfill) follow_up(0, qfill);
    if (give_up) {
        fq_prog_hint_rows<W, P, true, P - 1 - A>(a, p, fill, full_rows, extra8, s_keys, s_lut, wave, lane);
        return;
    }
    if (fill) stage_flush1(s_keys, fill, a.out, lane);
    if (a.deep_rows && lane == 0 && full_rows) atomicAdd(a.deep_rows, full_rows);
    if (a.deep_units && lane == 0 && extra8) atomicAdd(a.deep_units, extra8);
}

template <int W, int P, int MODE>
__global__ void dense_scores_fq(const char* __restrict__ tiles, const Layout l, const float* __restrict__ lut,
                                uint64_t first, uint64_t count, float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom g{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const char* tile = tiles + (size_t)tile_to_phys(l, (uint32_t)(z / kTileItems)) * g.tile_bytes();
    const uint32_t o = (uint32_t)(z % kTileItems);
    RowRegs<W, P, S> r;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint32_t* pw = reinterpret_cast<const uint32_t*>(tile + j * g.plane_bytes()) + (size_t)o * 2 * W;
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[j][0][h] = pw[h];
    }
#pragma unroll
    for (int j = 0; j < S; ++j) r.a[j][0] = reinterpret_cast<const float*>(tile + g.scales_offset())[j * kTileItems + o];
    out[t] = score_item_fq<W, P, MODE>(r, 0, reinterpret_cast<const float (*)[256]>(lut));
}

// fp32 score of one query for items first .. first+count (test hook); same arithmetic as the scan.
template <int W, int P, int PQ, int MODE>
__global__ void dense_scores(const char* __restrict__ tiles, const Layout l,
                             const uint32_t* __restrict__ qwords, const float* __restrict__ qcoef,
                             uint64_t first, uint64_t count, float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom g{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const char* tile = tiles + (size_t)tile_to_phys(l, (uint32_t)(z / kTileItems)) * g.tile_bytes();
    const uint32_t o = (uint32_t)(z % kTileItems);
    const QueryRegs<W, PQ> q = load_query<W, PQ>(qwords, qcoef, 0);
    RowRegs<W, P, S> r;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint32_t* pw = reinterpret_cast<const uint32_t*>(tile + j * g.plane_bytes()) + (size_t)o * 2 * W;
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[j][0][h] = pw[h];
    }
#pragma unroll
    for (int j = 0; j < S; ++j) r.a[j][0] = reinterpret_cast<const float*>(tile + g.scales_offset())[j * kTileItems + o];
    out[t] = score_item<W, P, PQ, MODE>(r, 0, q);
}

// ---------------------------------------------------------------- dispatch
namespace {

using ScanFn = void (*)(const ScanArgs);
using DenseFn = void (*)(const char*, const Layout, const uint32_t*, const float*, uint64_t, uint64_t, float*);

template <int W, int P, int PQ>
ScanFn prog_fn_m(int mode, bool single, bool hints, bool two_stage)
{
    if constexpr (P >= 2) {
        if (mode == kModeScaled) {
            if (!single) {
                if constexpr (P >= 3)
                    if (hints && two_stage) return scan_exact_batch_prog2_hint<W, P, PQ, (P >= 4 ? 2 : 1)>;
                return hints ? scan_exact_batch_prog_hint<W, P, PQ> : scan_exact_batch_prog<W, P, PQ, kModeScaled>;
            }
            if constexpr (P >= 3) {
                if (hints && two_stage) return scan_exact_prog2_hint<W, P, PQ, (P >= 4 ? 2 : 1)>;
            }
            return hints ? scan_exact_prog_hint<W, P, PQ> : scan_exact_prog<W, P, PQ, kModeScaled>;
        }
        if constexpr (dyadic_supported(W)) {
            if (mode == kModeDyadicNorm)
                return single ? scan_exact_prog<W, P, PQ, kModeDyadicNorm> : scan_exact_batch_prog<W, P, PQ, kModeDyadicNorm>;
            if (mode == kModeDyadic)
                return single ? scan_exact_prog<W, P, PQ, kModeDyadic> : scan_exact_batch_prog<W, P, PQ, kModeDyadic>;
        }
    }
    return nullptr;
}

template <int W, int P, int PQ>
ScanFn scan_fn_m(int mode, bool single)
{
    if (mode == kModeScaled) return single ? scan_exact<W, P, PQ, true, kModeScaled> : scan_exact<W, P, PQ, false, kModeScaled>;
    if constexpr (dyadic_supported(W)) {
        if (mode == kModeDyadicNorm)
            return single ? scan_exact<W, P, PQ, true, kModeDyadicNorm> : scan_exact<W, P, PQ, false, kModeDyadicNorm>;
        if (mode == kModeDyadic)
            return single ? scan_exact<W, P, PQ, true, kModeDyadic> : scan_exact<W, P, PQ, false, kModeDyadic>;
    }
    return nullptr;
}

template <int W, int P, int PQ>
DenseFn dense_fn_m(int mode)
{
    if (mode == kModeScaled) return dense_scores<W, P, PQ, kModeScaled>;
    if constexpr (dyadic_supported(W)) {
        if (mode == kModeDyadicNorm) return dense_scores<W, P, PQ, kModeDyadicNorm>;
        if (mode == kModeDyadic) return dense_scores<W, P, PQ, kModeDyadic>;
    }
    return nullptr;
}

#define RBE_SWITCH_PQ(FN, P, ...)                       \
    switch (k.PQ) {                                     \
        case 1: return FN<RBE_W, P, 1>(__VA_ARGS__);    \
        case 2: return FN<RBE_W, P, 2>(__VA_ARGS__);    \
        case 3: return FN<RBE_W, P, 3>(__VA_ARGS__);    \
        case 4: return FN<RBE_W, P, 4>(__VA_ARGS__);    \
        default: return nullptr;                        \
    }

ScanFn prog_fn(const KernelSel& k)
{
    switch (k.P) {
        case 2: RBE_SWITCH_PQ(prog_fn_m, 2, k.mode, k.single, k.hints, k.two_stage)
        case 3: RBE_SWITCH_PQ(prog_fn_m, 3, k.mode, k.single, k.hints, k.two_stage)
        case 4: RBE_SWITCH_PQ(prog_fn_m, 4, k.mode, k.single, k.hints, k.two_stage)
        default: return nullptr;
    }
}

ScanFn scan_fn(const KernelSel& k)
{
    if (k.progressive) return prog_fn(k);
    switch (k.P) {
        case 1: RBE_SWITCH_PQ(scan_fn_m, 1, k.mode, k.single)
        case 2: RBE_SWITCH_PQ(scan_fn_m, 2, k.mode, k.single)
        case 3: RBE_SWITCH_PQ(scan_fn_m, 3, k.mode, k.single)
        case 4: RBE_SWITCH_PQ(scan_fn_m, 4, k.mode, k.single)
        default: return nullptr;
    }
}

DenseFn dense_fn(const KernelSel& k)
{
    switch (k.P) {
        case 1: RBE_SWITCH_PQ(dense_fn_m, 1, k.mode)
        case 2: RBE_SWITCH_PQ(dense_fn_m, 2, k.mode)
        case 3: RBE_SWITCH_PQ(dense_fn_m, 3, k.mode)
        case 4: RBE_SWITCH_PQ(dense_fn_m, 4, k.mode)
        default: return nullptr;
    }
}

}  // namespace

namespace {
using FqFn = void (*)(const FqArgs);
using DenseFqFn = void (*)(const char*, const Layout, const float*, uint64_t, uint64_t, float*);

template <int W, int P>
FqFn fq_prog_fn_m(int mode, bool hints, bool binary_bound, bool two_stage)
{
    if constexpr (P >= 2) {
        if (mode == kModeScaled) {
            if (!hints) return scan_exact_fq_prog<W, P, kModeScaled>;
            if constexpr (P >= 3) {
                if (binary_bound && two_stage) return scan_exact_fq_prog2_hint<W, P, (P >= 4 ? 2 : 1)>;
            }
            return binary_bound ? scan_exact_fq_prog_hint<W, P, true> : scan_exact_fq_prog_hint<W, P, false>;
        }
        if constexpr (dyadic_supported(W)) {
            if (mode == kModeDyadicNorm) return scan_exact_fq_prog<W, P, kModeDyadicNorm>;
            if (mode == kModeDyadic) return scan_exact_fq_prog<W, P, kModeDyadic>;
        }
    }
    return nullptr;
}

template <int W, int P>
FqFn fq_fn_m(int mode)
{
    if (mode == kModeScaled) return scan_exact_fq<W, P, kModeScaled>;
    if constexpr (dyadic_supported(W)) {
        if (mode == kModeDyadicNorm) return scan_exact_fq<W, P, kModeDyadicNorm>;
        if (mode == kModeDyadic) return scan_exact_fq<W, P, kModeDyadic>;
    }
    return nullptr;
}

template <int W, int P>
DenseFqFn dense_fq_fn_m(int mode)
{
    if (mode == kModeScaled) return dense_scores_fq<W, P, kModeScaled>;
    if constexpr (dyadic_supported(W)) {
        if (mode == kModeDyadicNorm) return dense_scores_fq<W, P, kModeDyadicNorm>;
        if (mode == kModeDyadic) return dense_scores_fq<W, P, kModeDyadic>;
    }
    return nullptr;
}
}  // namespace

template <>
hipError_t launch_scan_exact_fq_w<RBE_W>(const KernelSel& k, const FqArgs& a, uint32_t n_cu, uint32_t per_cu,
                                         hipStream_t st, uint32_t* grid_out)
{
    FqFn fn = nullptr;
    switch (k.P) {
        case 1: fn = fq_fn_m<RBE_W, 1>(k.mode); break;
        case 2: fn = k.progressive ? fq_prog_fn_m<RBE_W, 2>(k.mode, k.hints, a.qwords != nullptr, k.two_stage && a.hints_last != nullptr) : fq_fn_m<RBE_W, 2>(k.mode); break;
        case 3: fn = k.progressive ? fq_prog_fn_m<RBE_W, 3>(k.mode, k.hints, a.qwords != nullptr, k.two_stage && a.hints_last != nullptr) : fq_fn_m<RBE_W, 3>(k.mode); break;
        case 4: fn = k.progressive ? fq_prog_fn_m<RBE_W, 4>(k.mode, k.hints, a.qwords != nullptr, k.two_stage && a.hints_last != nullptr) : fq_fn_m<RBE_W, 4>(k.mode); break;
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

template <>
hipError_t launch_dense_scores_fq_w<RBE_W>(const KernelSel& k, const char* tiles, const Layout& l, const float* lut,
                                           uint64_t first, uint64_t count, float* out, hipStream_t st)
{
    DenseFqFn fn = nullptr;
    switch (k.P) {
        case 1: fn = dense_fq_fn_m<RBE_W, 1>(k.mode); break;
        case 2: fn = dense_fq_fn_m<RBE_W, 2>(k.mode); break;
        case 3: fn = dense_fq_fn_m<RBE_W, 3>(k.mode); break;
        case 4: fn = dense_fq_fn_m<RBE_W, 4>(k.mode); break;
        default: break;
    }
    if (!fn) return hipErrorInvalidValue;
    fn<<<dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st>>>(tiles, l, lut, first, count, out);
    return hipGetLastError();
}

template <>
hipError_t launch_scan_exact_w<RBE_W>(const KernelSel& k, const ScanArgs& a, uint32_t n_cu, uint32_t per_cu,
                                      hipStream_t st, uint32_t* grid_out)
{
    const ScanFn fn = scan_fn(k);
    if (!fn) return hipErrorInvalidValue;
    if (a.p_end <= a.p_begin) return hipSuccess;
    const size_t dyn_lds = k.single ? 0 : (size_t)kWavesPerBlock * a.stage_entries * sizeof(uint64_t);
    if (!k.single && (a.stage_entries < 512 || a.stage_entries > 4096)) return hipErrorInvalidValue;
    if (dyn_lds > 32768) {   // beyond the default dynamic-LDS limit the kernel must be told
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds);
        if (e != hipSuccess) return e;
    }
    if (per_cu == 0) {
        int nb = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kBlock, dyn_lds);
        if (e != hipSuccess) return e;
        per_cu = (uint32_t)(nb > 0 ? nb : 1);
        // One query is a pure stream: what matters is the bytes in flight per compute unit, and more workgroups
        // than that needs only spread the accesses (measurements at streaming_blocks_per_cu).
        if (k.single) per_cu = std::min(per_cu, streaming_blocks_per_cu(RBE_W, k.P, scale_arrays(k.mode, k.P), k.progressive, k.hints, k.two_stage));
    }
    const uint32_t units = a.p_end - a.p_begin;
    const uint32_t grid = units < n_cu * per_cu ? units : n_cu * per_cu;
    if (grid_out) *grid_out = grid;
    // A batch over a range too short to fill the chip (the coarsest levels of a search: a few tiles, of which most
    // items survive) is bound by the waves' queue flushes -- one returning atomic per 64 survivors, one after the
    // other, for every query in turn.  Rows of workgroups with a slice of the queries each shorten that chain; the
    // tiles they share come from the cache.
    ScanArgs b = a;
    uint32_t rows = 1;
    b.q_slice = 0;
    if (!k.single && !k.progressive && a.calib_repeat == 0 && a.n_queries > 1 && units < n_cu * per_cu) {
        const uint32_t want = (n_cu * per_cu + units - 1) / units;
        rows = want < a.n_queries ? want : a.n_queries;
        b.q_slice = (a.n_queries + rows - 1) / rows;
        rows = (a.n_queries + b.q_slice - 1) / b.q_slice;
    }
    fn<<<dim3(grid, rows), dim3(kBlock), dyn_lds, st>>>(b);
    return hipGetLastError();
}

template <>
hipError_t launch_dense_scores_w<RBE_W>(const KernelSel& k, const char* tiles, const Layout& l, const uint32_t* qwords,
                                        const float* qcoef, uint64_t first, uint64_t count, float* out, hipStream_t st)
{
    const DenseFn fn = dense_fn(k);
    if (!fn) return hipErrorInvalidValue;
    fn<<<dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st>>>(tiles, l, qwords, qcoef, first, count, out);
    return hipGetLastError();
}

}  // namespace rbe
