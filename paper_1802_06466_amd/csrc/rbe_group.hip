// Near-lossless scan kernels (Algorithm 1, queue length 1) for one word count W
// (compile with -DRBE_W=1, 2 or 4).
#include "rbe_internal.hpp"

#ifndef RBE_W
#error "compile with -DRBE_W=1|2|4"
#endif

namespace rbe {

// ---------------------------------------------------------------- near-lossless local selection
// Algorithm 1 with a priority queue of length 1: thread y of block x visits
// items x*256*I + y, + 256, ... (I of them) and forwards only its best one.  In
// rows of 256 items: "super-block" x is rows [x*I, (x+1)*I), and the group of an
// item is (super-block, column = id mod 256).  One workgroup takes one
// super-block per step; wave w scans rows w, w+4, ... keeping, per lane and
// column, the best (score, row) seen; the four waves' partial winners are merged
// through LDS and the group winners that reach the threshold are queued like the
// survivors of the exact scan.

// Physical address of logical row `row` (wave-uniform).
__device__ __forceinline__ const char* row_tile(const GroupArgs& a, const TileGeom& g, uint32_t row)
{
    return a.tiles + (size_t)tile_to_phys(a.layout, row >> 2) * g.tile_bytes();
}

// QL = length of the priority queue of Algorithm 1 (1: the paper's choice; 2: the two best items of a group).
template <int W, int P, int PQ, int QB, int MODE, int QL>
__global__ __launch_bounds__(kBlock) void scan_groupmax(const GroupArgs a)
{
    __shared__ uint64_t s_keys_all[kWavesPerBlock][kStage];
    __shared__ uint32_t s_cnt_all[kWavesPerBlock][17];
    __shared__ float s_best[QB][QL][kWavesPerBlock][kItemsPerLane][64];
    __shared__ uint32_t s_brow[QB][QL][kWavesPerBlock][kItemsPerLane][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // sub-queues for the (at most 4) queries of this launch; 16 counters keep the layout of the batch scan
    const MultiStage ms{s_keys_all[wave], s_cnt_all[wave], (uint32_t)kStage / 16u, a.q_begin, 16u};
    if (lane < 17) s_cnt_all[wave][lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    constexpr int S = scale_arrays(MODE, P);
    const TileGeom geom{(uint32_t)W, (uint32_t)P, (uint32_t)S};
    const float ninf = -__builtin_inff();


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

    for (uint32_t v = a.v_begin + blockIdx.x; v < a.v_end; v += gridDim.x) {
        const uint32_t x = (a.skip ? nth_non_multiple(v, a.skip) : v) * a.stride;
        const uint32_t row0 = x * a.I;
        const uint32_t n_rows = a.rows_total - row0 < a.I ? a.rows_total - row0 : a.I;

        float best[QB][QL][kItemsPerLane];
        uint32_t brow[QB][QL][kItemsPerLane];
#pragma unroll
        for (int b = 0; b < QB; ++b)
#pragma unroll
            for (int e = 0; e < QL; ++e)
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) { best[b][e][m] = ninf; brow[b][e][m] = 0xFFFFFFFFu; }

        uint32_t r = (uint32_t)wave;
        RowRegs<W, P, S> cur, nxt;
        if (r < n_rows) load_row<W, P, S>(cur, row_tile(a, geom, row0 + r), (int)((row0 + r) & 3), lane);
        while (r < n_rows) {
            const uint32_t rn = r + kWavesPerBlock;
            // (prefetch not under a branch: the last step fetches its own row again, and the waits for this row's
            // registers leave the loads just issued in flight)
            const uint32_t rl = rn < n_rows ? rn : r;
            load_row<W, P, S>(nxt, row_tile(a, geom, row0 + rl), (int)((row0 + rl) & 3), lane);
            const uint64_t row_id = (uint64_t)(row0 + r) * kRow;
            const bool tail = row_id + kRow > a.n_items;   // only the corpus' last row can hold missing slots
#pragma unroll
            for (int b = 0; b < QB; ++b) {
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    float s = score_item<W, P, PQ, MODE>(cur, m, qr[b]) + 0.0f;
                    if (tail && row_id + lane_item<W>(lane, m) >= a.n_items) s = ninf;
                    // rows are visited in ascending order: ">" keeps the lowest id among equal scores
                    if (QL == 1) {
                        if (s > best[b][0][m]) { best[b][0][m] = s; brow[b][0][m] = r; }
                    } else {
                        const bool first = s > best[b][0][m];
                        const bool second = !first && s > best[b][QL - 1][m];
                        if (first || second) {
                            best[b][QL - 1][m] = first ? best[b][0][m] : s;
                            brow[b][QL - 1][m] = first ? brow[b][0][m] : r;
                        }
                        if (first) { best[b][0][m] = s; brow[b][0][m] = r; }
                    }
                }
            }
            if (rn < n_rows) cur = nxt;
            r = rn;
        }

        // merge the four waves' queues: wave w finalises item slot m = w of every lane
#pragma unroll
        for (int b = 0; b < QB; ++b)
#pragma unroll
            for (int e = 0; e < QL; ++e)
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    s_best[b][e][wave][m][lane] = best[b][e][m];
                    s_brow[b][e][wave][m][lane] = brow[b][e][m];
                }
        __syncthreads();
        for (int b = 0; b < QB; ++b) {
            if (b >= (int)a.nq) break;
            float ws[QL];
            uint32_t wr[QL];
#pragma unroll
            for (int e = 0; e < QL; ++e) { ws[e] = ninf; wr[e] = 0xFFFFFFFFu; }
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w)
#pragma unroll
                for (int e = 0; e < QL; ++e) {
                    const float s = s_best[b][e][w][wave][lane];
                    const uint32_t rr = s_brow[b][e][w][wave][lane];
                    // insert (s, rr) into the merged queue: better = higher score, then lower row
                    const bool valid = rr != 0xFFFFFFFFu;
                    const bool beats0 = valid && (wr[0] == 0xFFFFFFFFu || s > ws[0] || (s == ws[0] && rr < wr[0]));
                    if (QL == 1) {
                        if (beats0) { ws[0] = s; wr[0] = rr; }
                    } else {
                        const bool beats1 = valid && !beats0 &&
                                            (wr[QL - 1] == 0xFFFFFFFFu || s > ws[QL - 1] || (s == ws[QL - 1] && rr < wr[QL - 1]));
                        if (beats0 || beats1) {
                            ws[QL - 1] = beats0 ? ws[0] : s;
                            wr[QL - 1] = beats0 ? wr[0] : rr;
                        }
                        if (beats0) { ws[0] = s; wr[0] = rr; }
                    }
                }
#pragma unroll
            for (int e = 0; e < QL; ++e) {
                bool ok = (wr[e] != 0xFFFFFFFFu) && (ws[e] >= taus[b]);
                uint64_t key = 0;
                if (ok) {
                    const uint64_t id = (uint64_t)(row0 + wr[e]) * kRow + lane_item<W>(lane, wave);
                    key = make_key(ws[e], (uint32_t)id);
                    ok = key >= tau[b];
                }
                mstage_append(ok, key, (uint32_t)b, ms, a.out, lane);
            }
        }
        __syncthreads();
    }
    mstage_drain(ms, a.out, lane);
}

// ---------------------------------------------------------------- dispatch
namespace {

using GroupFn = void (*)(const GroupArgs);

// Queue length 2 is built for one query per launch (its state doubles the registers of a query).
template <int W, int P, int PQ, int MODE>
GroupFn group_fn_q(bool single, uint32_t qlen)
{
    if (qlen == 2) return scan_groupmax<W, P, PQ, 1, MODE, 2>;
    return single ? scan_groupmax<W, P, PQ, 1, MODE, 1> : scan_groupmax<W, P, PQ, 4, MODE, 1>;
}

template <int W, int P, int PQ>
GroupFn group_fn_m(int mode, bool single, uint32_t qlen)
{
    if (mode == kModeScaled) return group_fn_q<W, P, PQ, kModeScaled>(single, qlen);
    if constexpr (dyadic_supported(W)) {
        if (mode == kModeDyadicNorm) return group_fn_q<W, P, PQ, kModeDyadicNorm>(single, qlen);
        if (mode == kModeDyadic) return group_fn_q<W, P, PQ, kModeDyadic>(single, qlen);
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

GroupFn group_fn(const KernelSel& k)
{
    switch (k.P) {
        case 1: RBE_SWITCH_PQ(group_fn_m, 1, k.mode, k.single, k.qlen)
        case 2: RBE_SWITCH_PQ(group_fn_m, 2, k.mode, k.single, k.qlen)
        case 3: RBE_SWITCH_PQ(group_fn_m, 3, k.mode, k.single, k.qlen)
        case 4: RBE_SWITCH_PQ(group_fn_m, 4, k.mode, k.single, k.qlen)
        default: return nullptr;
    }
}

}  // namespace

template <>
hipError_t launch_scan_groupmax_w<RBE_W>(const KernelSel& k, GroupArgs a, uint32_t n_queries, uint32_t n_cu,
                                         uint32_t per_cu, hipStream_t st, uint32_t* grid_out)
{
    const GroupFn fn = group_fn(k);
    if (!fn) return hipErrorInvalidValue;
    if (a.v_end <= a.v_begin) return hipSuccess;
    if (per_cu == 0) {
        int nb = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kBlock, 0);
        if (e != hipSuccess) return e;
        per_cu = (uint32_t)(nb > 0 ? nb : 1);
    }
    const uint32_t units = a.v_end - a.v_begin;
    const uint32_t grid = units < n_cu * per_cu ? units : n_cu * per_cu;
    if (grid_out) *grid_out = grid;
    const uint32_t QB = (k.single || k.qlen == 2) ? 1 : 4;
    for (uint32_t q0 = 0; q0 < n_queries; q0 += QB) {   // the range is re-read once per block of QB queries
        a.q_begin = q0;
        a.nq = n_queries - q0 < QB ? n_queries - q0 : QB;
        fn<<<dim3(grid), dim3(kBlock), 0, st>>>(a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rbe
