// Launchers of the heavy kernel families.  Each family is compiled once per word
// count W in its own translation unit (rbe_scan.hip / rbe_group.hip with
// -DRBE_W=1|2|4) so that the builds run in parallel; rbe_api.hip only sees these
// declarations.
#pragma once
#include <hip/hip_runtime.h>

#include "rbe_kernels.hpp"

namespace rbe {

struct KernelSel {
    uint32_t P, PQ;   // corpus planes, query planes
    int mode;         // kModeScaled / kModeDyadicNorm / kModeDyadic
    bool single;      // one query per call
    uint32_t qlen = 1;   // near-lossless mode: length of the per-group priority queue (1 or 2)
    bool progressive = false;   // exact mode, last level, P >= 2: read the last plane only where the others cannot rule a row out
    bool hints = false;         // ... one query, general scales: the index holds one-byte copies of the scales
    bool two_stage = false;     // ... and three or more planes: the stream carries plane 0 only (scan_exact_prog2_hint)
};

// Grid = min(units, n_cu * per_cu); per_cu == 0 means "as many workgroups as are
// resident at once" (from the kernel's occupancy).  *grid_out receives the grid.
template <int W>
hipError_t launch_scan_exact_w(const KernelSel& k, const ScanArgs& a, uint32_t n_cu, uint32_t per_cu,
                               hipStream_t st, uint32_t* grid_out);

// One launch per block of 4 queries (1 if single).
template <int W>
hipError_t launch_scan_groupmax_w(const KernelSel& k, GroupArgs a, uint32_t n_queries, uint32_t n_cu,
                                  uint32_t per_cu, hipStream_t st, uint32_t* grid_out);

template <int W>
hipError_t launch_dense_scores_w(const KernelSel& k, const char* tiles, const Layout& l, const uint32_t* qwords,
                                 const float* qcoef, uint64_t first, uint64_t count, float* out, hipStream_t st);

// Hybrid scoring: one launch per query (k.PQ and k.single are ignored).
template <int W>
hipError_t launch_scan_exact_fq_w(const KernelSel& k, const FqArgs& a, uint32_t n_cu, uint32_t per_cu,
                                  hipStream_t st, uint32_t* grid_out);

template <int W>
hipError_t launch_dense_scores_fq_w(const KernelSel& k, const char* tiles, const Layout& l, const float* lut,
                                    uint64_t first, uint64_t count, float* out, hipStream_t st);

// Batched exact scan on the matrix cores; n_query_tiles in {1, 2} (16 queries each, from a.q_begin).  Built for W <= 2.
template <int W>
hipError_t launch_scan_batch_w(const KernelSel& k, const BatchArgs& a, uint32_t n_query_tiles, uint32_t n_cu,
                               uint32_t per_cu, hipStream_t st, uint32_t* grid_out);
template <> hipError_t launch_scan_batch_w<1>(const KernelSel&, const BatchArgs&, uint32_t, uint32_t, uint32_t,
                                              hipStream_t, uint32_t*);
template <> hipError_t launch_scan_batch_w<2>(const KernelSel&, const BatchArgs&, uint32_t, uint32_t, uint32_t,
                                              hipStream_t, uint32_t*);
constexpr bool batch_mfma_supported(uint32_t W) { return W <= 2; }

#define RBE_DECLARE_W(Wv)                                                                                         \
    template <> hipError_t launch_scan_exact_w<Wv>(const KernelSel&, const ScanArgs&, uint32_t, uint32_t,         \
                                                   hipStream_t, uint32_t*);                                       \
    template <> hipError_t launch_scan_groupmax_w<Wv>(const KernelSel&, GroupArgs, uint32_t, uint32_t, uint32_t,  \
                                                      hipStream_t, uint32_t*);                                    \
    template <> hipError_t launch_dense_scores_w<Wv>(const KernelSel&, const char*, const Layout&,                \
                                                     const uint32_t*, const float*, uint64_t, uint64_t, float*,   \
                                                     hipStream_t);                                                \
    template <> hipError_t launch_scan_exact_fq_w<Wv>(const KernelSel&, const FqArgs&, uint32_t, uint32_t,        \
                                                      hipStream_t, uint32_t*);                                    \
    template <> hipError_t launch_dense_scores_fq_w<Wv>(const KernelSel&, const char*, const Layout&,             \
                                                        const float*, uint64_t, uint64_t, float*, hipStream_t);
RBE_DECLARE_W(1)
RBE_DECLARE_W(2)
RBE_DECLARE_W(4)
#undef RBE_DECLARE_W

// Persistent workgroups per compute unit for a one-query streaming scan: about 32 KB of tile stream per compute
// unit and step (a workgroup has this step's tile and the next one's in flight; the progressive scan streams all
// planes and scale arrays but the last).  Measured on 1e9 items (ms of the finest-level scan at 1 / 2 / 3 / 4
// workgroups per unit): 18 KB per tile 2.92 / 2.58 / 2.82 / 2.61, 8 KB 2.57 / 1.56 / 1.25 / 1.28, 24 KB 3.41 / 3.43 /
// 3.43 / 3.47, 36 KB 5.04 / 5.04 / 5.10 / 5.14, 52 KB (1e8 items) 0.69 / 0.70 / 0.71 / 0.72.
inline uint32_t streaming_blocks_per_cu(uint32_t W, uint32_t P, uint32_t S, bool progressive, bool hints, bool two_stage = false)
{
    const bool prog = progressive && P >= 2;
    const bool two = prog && hints && two_stage && P >= 3;
    const uint32_t planes = two ? (P >= 4 ? 2u : 1u) : (prog ? P - 1 : P), scales = prog && S > 0 ? S - 1 : S;     // (see scan_exact_prog2_hint for the planes of its stream)
    const uint32_t tile_stream = kTileItems * (8u * W * planes + (prog && hints ? 1u : 4u) * scales);
    const uint32_t n = (32u * 1024u + tile_stream / 2) / tile_stream;
    return n < 1u ? 1u : (n > 3u ? 3u : n);
}

// Dyadic modes are built for d = 64 and d = 128.
constexpr bool dyadic_supported(uint32_t W) { return W <= 2; }

}  // namespace rbe
