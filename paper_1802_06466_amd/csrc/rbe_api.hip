// Host side of the RBE retrieval library: the C ABI declared in include/rbe.h and include/rbe_debug.h,
// argument checks, device storage, the refinement plan and kernel launches.
#include "rbe.h"
#include "rbe_debug.h"
#include "rbe_internal.hpp"
#include "rbe_misc_kernels.hpp"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

namespace {

thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return (e_ == hipErrorOutOfMemory) ? RBE_ENOMEM : RBE_EHIP;                     \
        }                                                                                   \
    } while (0)

#define ARG_CHECK(cond, ...)                                                                \
    do {                                                                                    \
        if (!(cond)) {                                                                      \
            set_error(__VA_ARGS__);                                                         \
            return RBE_EINVAL;                                                              \
        }                                                                                   \
    } while (0)

constexpr uint32_t kMaxEvents = 2 * RBE_MAX_LEVELS + 2;
// Last level in two parts (see run_search), one binary query per call: split searches in a row that the tighter
// threshold did not help before the level is taken whole, and the searches it then stays whole.
constexpr uint32_t kSplitStreak = 4;
constexpr uint32_t kWholeSearches = 64;
constexpr uint32_t kSplitMinTiles = 4096;     // smaller last levels are not split: a launch and a selection would show
// layout of the block a search sends back (rbe_index::d_result)
constexpr size_t kResultStatusBytes = 256;
constexpr size_t kResultHeaderBytes = kResultStatusBytes + (size_t)RBE_MAX_LEVELS * RBE_MAX_QUERIES * sizeof(uint32_t);

}  // namespace

// Scratch of rbe_search_static: one copy per GPU, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address it yields (per device) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[RBE_STATIC_SCRATCH_BYTES];

struct rbe_index {
    uint64_t n_items = 0;
    uint32_t dim = 0, W = 0, P = 0, flags = 0;
    int mode = rbe::kModeScaled;   // scoring mode of the kernels
    int ready = 0;
    bool loaded_any = false;
    int n_cu = 0;

    char* d_tiles = nullptr;        // n_tiles tiles in nested-sample-major order (rbe_layout.hpp)
    rbe::Layout layout = {};
    rbe::TileGeom geom = {};

    // tuning
    uint32_t cap_override = 0, blocks_per_cu = 0;  // 0 = derived

    // Device scratch of a search (see carve_workspace for the layout of the block it lives in).
    struct DevWs {
        uint64_t* cand = nullptr;       // [Q][cap] candidate keys
        uint32_t* count = nullptr;      // [Q] x kCountStride
        uint64_t* tau = nullptr;        // [Q]
        uint64_t* kmax = nullptr;       // [Q] x kKmaxStride
        // One block holds everything a search sends back, so that one copy fetches it:
        //   [status: kResultStatusBytes][seen: RBE_MAX_LEVELS x RBE_MAX_QUERIES u32][ids: Q x k i64][scores: Q x k f32]
        // (ids and scores packed for the Q and k of the current call).  The pointers below point into it.
        char* result = nullptr;
        uint32_t* status = nullptr;     // 16 words: [0] flags, [1..8] rows read in full per level, [9] (query, row) pairs scored in
                                        // full by the batch progressive scan, [12] [13] first looks of the matrix-core scan, [14] deep units
        uint32_t* seen = nullptr;       // [RBE_MAX_LEVELS][RBE_MAX_QUERIES]
        int64_t* ids = nullptr;
        float* scores = nullptr;
        uint32_t* qwords = nullptr;     // [RBE_MAX_QUERIES][PQ][2W], followed (fixed offset) by
        float* qcoef = nullptr;         // [RBE_MAX_QUERIES][PQ+1] and the query masses
        float* unscale = nullptr;       // [3][RBE_MAX_QUERIES]: matrix-core scan, per query 2^-k, start value, mass
        uint32_t* aops = nullptr;       // matrix-core query operands (BatchArgs::a_ops)
        float* lut = nullptr;           // [Q][8W][256] byte tables of fp32 queries (hybrid scoring)
        uint64_t* gtable = nullptr;     // near-lossless modes: [Q][gslots][2] group table of group_best_build
        uint32_t* gaux = nullptr;       // ... [Q][4] its counters
        uint32_t gslots = 0;
    };
    DevWs ws;                       // the scratch the current search uses: carved from one of the three blocks below
    char* own_ws = nullptr;         // grown on demand by the library (hipMalloc) ...
    size_t own_ws_bytes = 0;
    char* ext_ws = nullptr;         // ... or lent by the caller (rbe_set_workspace): never grown, never freed here
    size_t ext_ws_bytes = 0;
    // pinned host mirrors, allocated once at rbe_index_create for the largest call (RBE_MAX_QUERIES x RBE_MAX_K)
    char* h_result = nullptr;
    uint32_t* h_status = nullptr;
    uint32_t* h_seen = nullptr;
    int64_t* h_ids = nullptr;
    float* h_scores = nullptr;
    uint32_t* h_qwords = nullptr;
    float* h_qcoef = nullptr;
    uint32_t* h_aops = nullptr;
    float* h_unscale = nullptr;
    float* h_lut = nullptr;
    int device = 0;                 // the GPU that owns the index
    // corpus storage lent by the caller (rbe_index_create_in): tiles, side arrays and the scratch of rbe_finalize
    bool borrowed = false;
    char* fin_scratch = nullptr;    // borrowed storage: 256 bytes for rbe_finalize's reductions
    // false if a scale is negative: every bound of the pruning scans assumes a_j >= 0, so they all stay off
    bool nonneg = true;
    float scale_max = 0.0f;         // largest magnitude in the stored scale arrays (general scales), set by rbe_finalize
    int batch_path = 0;             // 0 auto, 1 XOR/popcount kernel always, 2 matrix-core kernel whenever built
    int nl_path = 0;                // near-lossless modes: 0 = exact scans + selection by groups, 1 = the per-thread-queue scan
    uint32_t* d_hints = nullptr;    // general scales, P >= 2: one-byte copies of the scale arrays 0 .. P-2 in lane order (rbe_finalize)
    int hint_base[4] = {1, 1, 1, 1};   // exponent base of each array's hints ([3]: the last array's, see d_hints_last)
    uint32_t* d_hints_last = nullptr;  // three or more planes: one-byte copies of the last scale array (inside the d_hints block)
    float* d_row_amax = nullptr;    // [n_tiles][4] largest value of the last scale array per row (set by rbe_finalize),
                                    // followed by [n_tiles][4] largest scale sum per row
    int plan_split = 0;             // last level in two parts: 0 = if it has kSplitMinTiles tiles (see run_search), 1 = never, 2 = always
    // One binary query per call: the only searches for which the split can cost more than it saves (1 %, where
    // the last level's own threshold already lies inside the query's neighbourhood).  See run_search.
    struct SplitState {
        uint32_t streak = 0;        // split searches in a row whose second part pruned no better than the first
        uint32_t whole_left = 0;    // searches left that take the level whole
    } split1;
    int progressive = 1;            // one query, exact mode, last level: read planes 1.. only where plane 0 leaves a chance
    float batch_margin = 0.0f;      // BatchArgs::margin of the staged batch
    bool batch_i8 = false;          // the staged operands are eight-bit integers (BatchArgs::operand = 1)
    float fq_mass[RBE_MAX_QUERIES][2] = {};   // fp32 queries: {x, 2^-19 x}, x >= sum_d |q_d| (1 + 2^-18): bounds any plane's table sum
    // fp32 queries, one scan per query, general scales with scale copies: a 4-plane binary approximation of each
    // query is staged as well (stage_float_approximations) and the last level's bound is formed from it
    bool fq_binary = false;
    float fq_bmass[RBE_MAX_QUERIES][2] = {};  // its mass (query_mass)
    float fq_resid[RBE_MAX_QUERIES] = {};     // >= sum_d |q_d - qhat_d|

    int profiling = 0;
    hipEvent_t ev[kMaxEvents] = {};
    bool ev_ok = false;
    rbe_search_stats stats = {};
};

namespace {

using namespace rbe;

// ---------------------------------------------------------------- kernel dispatch (per word count W)
hipError_t launch_scan_exact(uint32_t W, const KernelSel& k, const ScanArgs& a, uint32_t n_cu, uint32_t per_cu,
                             hipStream_t st, uint32_t* grid)
{
    switch (W) {
        case 1: return launch_scan_exact_w<1>(k, a, n_cu, per_cu, st, grid);
        case 2: return launch_scan_exact_w<2>(k, a, n_cu, per_cu, st, grid);
        default: return launch_scan_exact_w<4>(k, a, n_cu, per_cu, st, grid);
    }
}

hipError_t launch_scan_groupmax(uint32_t W, const KernelSel& k, const GroupArgs& a, uint32_t Q, uint32_t n_cu,
                                uint32_t per_cu, hipStream_t st, uint32_t* grid)
{
    switch (W) {
        case 1: return launch_scan_groupmax_w<1>(k, a, Q, n_cu, per_cu, st, grid);
        case 2: return launch_scan_groupmax_w<2>(k, a, Q, n_cu, per_cu, st, grid);
        default: return launch_scan_groupmax_w<4>(k, a, Q, n_cu, per_cu, st, grid);
    }
}

hipError_t launch_scan_exact_fq(uint32_t W, const KernelSel& k, const FqArgs& a, uint32_t n_cu, uint32_t per_cu,
                                hipStream_t st, uint32_t* grid)
{
    switch (W) {
        case 1: return launch_scan_exact_fq_w<1>(k, a, n_cu, per_cu, st, grid);
        case 2: return launch_scan_exact_fq_w<2>(k, a, n_cu, per_cu, st, grid);
        default: return launch_scan_exact_fq_w<4>(k, a, n_cu, per_cu, st, grid);
    }
}

hipError_t launch_dense_scores_fq(uint32_t W, const KernelSel& k, const char* tiles, const Layout& l, const float* lut,
                                  uint64_t first, uint64_t count, float* out, hipStream_t st)
{
    switch (W) {
        case 1: return launch_dense_scores_fq_w<1>(k, tiles, l, lut, first, count, out, st);
        case 2: return launch_dense_scores_fq_w<2>(k, tiles, l, lut, first, count, out, st);
        default: return launch_dense_scores_fq_w<4>(k, tiles, l, lut, first, count, out, st);
    }
}

hipError_t launch_dense_scores(uint32_t W, const KernelSel& k, const char* tiles, const Layout& l,
                               const uint32_t* qwords, const float* qcoef, uint64_t first, uint64_t count,
                               float* out, hipStream_t st)
{
    switch (W) {
        case 1: return launch_dense_scores_w<1>(k, tiles, l, qwords, qcoef, first, count, out, st);
        case 2: return launch_dense_scores_w<2>(k, tiles, l, qwords, qcoef, first, count, out, st);
        default: return launch_dense_scores_w<4>(k, tiles, l, qwords, qcoef, first, count, out, st);
    }
}

// ---------------------------------------------------------------- workspace
// All device scratch of one search lives in one block, laid out for the call's n_queries, k and candidate
// capacity: fixed-size state first, the large candidate lists (and, for the near-lossless modes, the group tables)
// last, every part 256-byte aligned.  With
// base == nullptr only the size is computed.  The block is the library's own (grown on demand), the caller's
// (rbe_set_workspace) or the static array of rbe_search_static.
constexpr size_t kWsAlign = 256;
constexpr size_t kQueryWordsBytes = (size_t)RBE_MAX_QUERIES * RBE_MAX_PLANES * 8 * sizeof(uint32_t);
constexpr size_t kQueryCoefBytes = (size_t)RBE_MAX_QUERIES * (RBE_MAX_PLANES + 1 + 2) * sizeof(float);
constexpr size_t kHalvesPerQueryTile = (size_t)4 * 4 * 64 * 8;   // copies x parts <= 16, 64 lanes, 8 halves

size_t carve_workspace(rbe_index::DevWs* ws, char* base, uint32_t W, uint32_t Q, uint32_t k, uint32_t cap, bool groups)
{
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base ? base + off : nullptr;
        off += (bytes + kWsAlign - 1) / kWsAlign * kWsAlign;
        return p;
    };
    rbe_index::DevWs w;
    w.count = reinterpret_cast<uint32_t*>(take((size_t)Q * rbe::kCountStride * sizeof(uint32_t)));
    w.tau = reinterpret_cast<uint64_t*>(take((size_t)Q * sizeof(uint64_t)));
    w.kmax = reinterpret_cast<uint64_t*>(take((size_t)Q * rbe::kKmaxStride * sizeof(uint64_t)));
    // query words and coefficients share one block (coefficients at a fixed offset) so that one copy stages both
    w.qwords = reinterpret_cast<uint32_t*>(take(kQueryWordsBytes + kQueryCoefBytes));
    w.qcoef = base ? reinterpret_cast<float*>(reinterpret_cast<char*>(w.qwords) + kQueryWordsBytes) : nullptr;
    w.unscale = reinterpret_cast<float*>(take(3 * RBE_MAX_QUERIES * sizeof(float)));
    w.aops = reinterpret_cast<uint32_t*>(take((size_t)((Q + 15u) / 16u) * kHalvesPerQueryTile * sizeof(uint16_t)));
    w.lut = reinterpret_cast<float*>(take((size_t)Q * 8 * W * 256 * sizeof(float)));
    w.result = take(kResultHeaderBytes + (size_t)Q * k * (sizeof(int64_t) + sizeof(float)));
    w.cand = reinterpret_cast<uint64_t*>(take((size_t)Q * cap * sizeof(uint64_t)));
    if (groups) {       // near-lossless modes: a table of twice as many slots as a query has candidate slots, two keys each
        w.gslots = 1u;
        while (w.gslots < 2u * cap) w.gslots <<= 1;
        w.gaux = reinterpret_cast<uint32_t*>(take((size_t)Q * 4 * sizeof(uint32_t)));
        w.gtable = reinterpret_cast<uint64_t*>(take((size_t)Q * w.gslots * 2 * sizeof(uint64_t)));
    }
    if (base) {
        w.status = reinterpret_cast<uint32_t*>(w.result);
        w.seen = reinterpret_cast<uint32_t*>(w.result + kResultStatusBytes);
        w.ids = reinterpret_cast<int64_t*>(w.result + kResultHeaderBytes);
        w.scores = reinterpret_cast<float*>(w.ids + (size_t)Q * k);   // this call's scores follow its ids directly
        *ws = w;
    }
    return off;
}

// Candidate slots per query of a search for k results.
uint32_t search_capacity(const rbe_index* ix, uint32_t k)
{
    const uint32_t cap = ix->cap_override ? ix->cap_override : std::max<uint32_t>(65536u, 4u * ix->layout.ratio * k);
    return std::max<uint32_t>(cap, k + 2 * kTileItems);
}

// Points ix->ws at scratch for this call: the caller's block if one was set (an error if it is too small),
// else the library's own block, grown when this call needs more than any call before it.
int acquire_workspace(rbe_index* ix, uint32_t Q, uint32_t k, uint32_t cap, bool groups = false)
{
    const size_t need = carve_workspace(nullptr, nullptr, ix->W, Q, k, cap, groups);
    if (ix->ext_ws) {
        if (need > ix->ext_ws_bytes) {
            set_error("the workspace set with rbe_set_workspace holds %zu bytes; this search needs %zu "
                      "(rbe_workspace_bytes)", ix->ext_ws_bytes, need);
            return RBE_EINVAL;
        }
        carve_workspace(&ix->ws, ix->ext_ws, ix->W, Q, k, cap, groups);
        return RBE_OK;
    }
    if (need > ix->own_ws_bytes) {
        (void)hipFree(ix->own_ws);
        ix->own_ws = nullptr; ix->own_ws_bytes = 0;
        ix->ws = rbe_index::DevWs{};
        HIP_TRY(hipMalloc(&ix->own_ws, need));
        ix->own_ws_bytes = need;
    }
    carve_workspace(&ix->ws, ix->own_ws, ix->W, Q, k, cap, groups);
    return RBE_OK;
}

// Points ix->ws into this GPU's copy of the static scratch array.  Allocates nothing: the address of the array is
// looked up once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices] = {};

int acquire_static_scratch(rbe_index* ix, uint32_t Q, uint32_t k, uint32_t cap, bool groups)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != ix->device) {
        set_error("the index lives on device %d but device %d is current", ix->device, dev);
        return RBE_EINVAL;
    }
    if (dev < 0 || dev >= kMaxDevices) { set_error("device %d: no static scratch slot", dev); return RBE_EUNSUPPORTED; }
    const size_t need = carve_workspace(nullptr, nullptr, ix->W, Q, k, cap, groups);
    if (need > (size_t)RBE_STATIC_SCRATCH_BYTES) {
        set_error("rbe_search_static: %u queries with k = %u need %zu bytes of scratch, the static array holds %zu "
                  "(fewer queries per call, a smaller k, or a smaller cand_capacity via rbe_set_tuning)",
                  Q, k, need, (size_t)RBE_STATIC_SCRATCH_BYTES);
        return RBE_EINVAL;
    }
    char* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = static_cast<char*>(p);
        }
        base = g_scratch_ptr[dev];
    }
    carve_workspace(&ix->ws, base, ix->W, Q, k, cap, groups);
    return RBE_OK;
}

// Pinned host mirrors and events: once per index, sized for the largest call.
int allocate_host_side(rbe_index* ix)
{
    const size_t result_bytes = kResultHeaderBytes + (size_t)RBE_MAX_QUERIES * RBE_MAX_K * (sizeof(int64_t) + sizeof(float));
    HIP_TRY(hipHostMalloc(&ix->h_result, result_bytes, hipHostMallocDefault));
    ix->h_status = reinterpret_cast<uint32_t*>(ix->h_result);
    ix->h_seen = reinterpret_cast<uint32_t*>(ix->h_result + kResultStatusBytes);
    ix->h_ids = reinterpret_cast<int64_t*>(ix->h_result + kResultHeaderBytes);
    HIP_TRY(hipHostMalloc(&ix->h_qwords, kQueryWordsBytes + kQueryCoefBytes, hipHostMallocDefault));
    ix->h_qcoef = reinterpret_cast<float*>(reinterpret_cast<char*>(ix->h_qwords) + kQueryWordsBytes);
    HIP_TRY(hipHostMalloc(&ix->h_aops, (RBE_MAX_QUERIES / 16) * kHalvesPerQueryTile * sizeof(uint16_t), hipHostMallocDefault));
    HIP_TRY(hipHostMalloc(&ix->h_unscale, 3 * RBE_MAX_QUERIES * sizeof(float), hipHostMallocDefault));
    HIP_TRY(hipHostMalloc(&ix->h_lut, (size_t)RBE_MAX_QUERIES * 8 * ix->W * 256 * sizeof(float), hipHostMallocDefault));
    for (uint32_t i = 0; i < kMaxEvents; ++i) HIP_TRY(hipEventCreate(&ix->ev[i]));
    ix->ev_ok = true;
    return RBE_OK;
}

// Mass of one query, from which a scan bounds the contribution of planes it has not read (bound_item).  With
// qhat = sum_i c_i rho_i, M = sum_d |qhat_d| is the largest inner sum any plane can reach (attained by the plane
// whose signs are those of qhat).  General scales: out = {x, 2^-19 x}, x >= (M + 2^-20 d sum_i |c_i|) (1 + 2^-20):
// the second term covers the rounding of the inner sums as the kernel forms them (magnitudes up to
// 3 d sum_i |c_i|), the factor the rounding of the scale sums.  Dyadic modes, in units of 2^-(PQ-1): M is an
// integer, a plane's weighted mismatch count is at least h_min = (d (2^PQ - 1) - M) / 2, and out[0] carries h_min
// as an integer (out[1] = 0).
void query_mass(const uint64_t* planes /* [PQ][W] */, const float* scales /* [PQ] or null */, uint32_t PQ, uint32_t dim,
                bool dyadic, float* out)
{
    const uint32_t W = dim / 64;
    double M = 0.0, B = 0.0;
    for (uint32_t i = 0; i < PQ; ++i) B += std::fabs(dyadic ? std::ldexp(1.0, (int)(PQ - 1 - i)) : (double)scales[i]);
    B *= dim;
    for (uint32_t d = 0; d < dim; ++d) {
        double v = 0.0;
        for (uint32_t i = 0; i < PQ; ++i) {
            const double c = dyadic ? std::ldexp(1.0, (int)(PQ - 1 - i)) : (double)scales[i];
            v += ((planes[(size_t)i * W + d / 64] >> (d % 64)) & 1ull) ? c : -c;
        }
        M += std::fabs(v);
    }
    if (dyadic) {
        const uint32_t h_min = (uint32_t)((dim * ((1u << PQ) - 1u) - (uint32_t)M) / 2u);
        std::memcpy(&out[0], &h_min, sizeof(float));
        out[1] = 0.0f;
    } else {
        const double x = (M + std::ldexp(B, -20)) * (1.0 + std::ldexp(1.0, -20));
        float xf = (float)x;
        if ((double)xf < x) xf = std::nextafter(xf, INFINITY);
        out[0] = xf;
        out[1] = std::ldexp(xf, -19);
    }
}

// Stage one batch of queries: words as 32-bit halves, coefficients (-2 c_i ..., dim * sum c_i), and after the
// coefficients of all queries their masses [Q][2].
int stage_queries(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t Q, uint32_t PQ, hipStream_t st)
{
    const uint32_t W = ix->W;
    const bool dyadic = ix->mode != rbe::kModeScaled;
    if (!dyadic && !q_scales) { set_error("q_scales is NULL"); return RBE_EINVAL; }
    for (uint32_t q = 0; q < Q; ++q) {
        float sum = 0.0f;
        for (uint32_t i = 0; i < PQ; ++i) {
            float c = std::ldexp(1.0f, -(int)i);
            if (q_scales) {
                c = q_scales[(size_t)q * PQ + i];
                if (dyadic && c != std::ldexp(1.0f, -(int)i)) {
                    set_error("dyadic index: q_scales[%u][%u] must be 2^-%u (or pass NULL)", q, i, i);
                    return RBE_EINVAL;
                }
            }
            if (!std::isfinite(c)) { set_error("q_scales[%u][%u] is not finite", q, i); return RBE_EINVAL; }
            for (uint32_t w = 0; w < W; ++w) {
                const uint64_t word = q_planes[((size_t)q * PQ + i) * W + w];
                ix->h_qwords[((size_t)q * PQ + i) * 2 * W + 2 * w] = (uint32_t)word;
                ix->h_qwords[((size_t)q * PQ + i) * 2 * W + 2 * w + 1] = (uint32_t)(word >> 32);
            }
            ix->h_qcoef[(size_t)q * (PQ + 1) + i] = -2.0f * c;
            sum += c;
        }
        ix->h_qcoef[(size_t)q * (PQ + 1) + PQ] = (float)ix->dim * sum;
        query_mass(q_planes + (size_t)q * PQ * W, q_scales ? q_scales + (size_t)q * PQ : nullptr, PQ, ix->dim, dyadic,
                   ix->h_qcoef + (size_t)Q * (PQ + 1) + 2 * (size_t)q);
    }
    const size_t staged = kQueryWordsBytes + (size_t)Q * (PQ + 1 + 2) * sizeof(float);
    HIP_TRY(hipMemcpyAsync(ix->ws.qwords, ix->h_qwords, staged, hipMemcpyHostToDevice, st));
    return RBE_OK;
}

// Byte tables of fp32 queries: lut[q][p][v] = sum_{b<8} q[8p+b] * (bit b of v ? +1 : -1), summed in
// double in bit order and rounded to fp32.
int stage_float_queries(rbe_index* ix, const float* q, uint32_t Q, hipStream_t st)
{
    const size_t per_q = (size_t)8 * ix->W * 256;
    for (uint32_t n = 0; n < Q; ++n) {
        const float* x = q + (size_t)n * ix->dim;
        double m_abs = 0.0;
        for (uint32_t i = 0; i < ix->dim; ++i) {
            if (!std::isfinite(x[i])) { set_error("q[%u][%u] is not finite", n, i); return RBE_EINVAL; }
            m_abs += std::fabs((double)x[i]);
        }
        // a plane's table sum: 8W entries rounded to fp32 and 8W - 1 fp32 additions, all at magnitudes <= m_abs
        m_abs *= 1.0 + std::ldexp(1.0, -18);
        float xf = (float)m_abs;
        if ((double)xf < m_abs) xf = std::nextafter(xf, INFINITY);
        ix->fq_mass[n][0] = xf;
        ix->fq_mass[n][1] = std::ldexp(xf, -19);
        for (uint32_t p = 0; p < 8 * ix->W; ++p)
            for (uint32_t v = 0; v < 256; ++v) {
                double acc = 0.0;
                for (uint32_t b = 0; b < 8; ++b) acc += ((v >> b) & 1u) ? (double)x[8 * p + b] : -(double)x[8 * p + b];
                ix->h_lut[n * per_q + (size_t)p * 256 + v] = (float)acc;
            }
    }
    HIP_TRY(hipMemcpyAsync(ix->ws.lut, ix->h_lut, (size_t)Q * per_q * sizeof(float), hipMemcpyHostToDevice, st));
    return RBE_OK;
}

// Binary approximations of fp32 queries for the bound of scan_exact_fq_prog_hint: the residual encoder of
// rbe_encode_query with RBE_MAX_PLANES planes, staged like binary queries; per query the mass of the approximation
// qhat and R >= sum_d |q_d - qhat_d| (in double, rounded up).
int stage_float_approximations(rbe_index* ix, const float* q, uint32_t Q, hipStream_t st)
{
    const uint32_t PQ = RBE_MAX_PLANES, W = ix->W;
    std::vector<uint64_t> planes((size_t)Q * PQ * W);
    std::vector<float> scales((size_t)Q * PQ);
    for (uint32_t n = 0; n < Q; ++n) {
        const float* x = q + (size_t)n * ix->dim;
        uint64_t* pl = planes.data() + (size_t)n * PQ * W;
        float* sc = scales.data() + (size_t)n * PQ;
        const int rc = rbe_encode_query(x, ix->dim, PQ, pl, sc);
        if (rc) return rc;
        double resid = 0.0;
        for (uint32_t d = 0; d < ix->dim; ++d) {
            double v = 0.0;
            for (uint32_t i = 0; i < PQ; ++i) v += ((pl[(size_t)i * W + d / 64] >> (d % 64)) & 1ull) ? (double)sc[i] : -(double)sc[i];
            resid += std::fabs((double)x[d] - v);
        }
        resid *= 1.0 + std::ldexp(1.0, -20);
        float rf = (float)resid;
        if ((double)rf < resid) rf = std::nextafter(rf, INFINITY);
        ix->fq_resid[n] = rf;
        query_mass(pl, sc, PQ, ix->dim, false, ix->fq_bmass[n]);
    }
    return stage_queries(ix, planes.data(), scales.data(), Q, PQ, st);
}

// 16-query tiles of a batch, and how many of them one launch of the matrix-core scan takes (1 or 2): two while
// the query operands of both fit in about 64 registers.  Per tile they take 4 registers per 32-dimension part,
// times the item planes in the dyadic modes (one weighted copy per plane).
uint32_t batch_tiles(uint32_t Q) { return (Q + 15u) / 16u; }
uint32_t batch_tiles_per_launch(const rbe_index* ix, bool float_query)
{
    const uint32_t per_tile = 4u * 2u * ix->W * (ix->mode == rbe::kModeScaled ? 1u : ix->P);
    // fp32 queries at d = 128: every plane stays in the first look, and with two tiles of accumulators on top of
    // the operands the kernel needs 360 registers or more (one wave per SIMD, or spills)
    if (float_query && ix->W == 2) return 1u;
    return 2u * per_tile <= 64u ? 2u : 1u;
}

// General scales: the contraction carries the hi half only and filters; survivors are scored again exactly as the
// one-query scan scores them (see scan_batch_mfma): 1 = binary queries (XOR/popcount), 2 = fp32 queries (byte
// tables).  0 = dyadic modes, whose queries are exact in one half.
uint32_t batch_rescore(const rbe_index* ix, bool float_query)
{
    return ix->mode != rbe::kModeScaled ? 0u : (float_query ? 2u : 1u);
}

// The pruning scans (progressive last level, first look and filter of the matrix-core scan) rest on upper bounds
// of the form "partial score + largest scale x query mass", which hold for scales >= 0 only: an index that holds a
// negative scale is searched by the plain scans alone.
bool can_prune(const rbe_index* ix) { return ix->nonneg; }

bool batch_operand_i8(const rbe_index* ix, bool float_query, uint32_t q_n_planes = 0);

bool use_batch_mfma(const rbe_index* ix, uint32_t Q, uint32_t mode, bool float_query, uint32_t q_n_planes = 0)
{
    if (mode != RBE_SELECT_EXACT || !rbe::batch_mfma_supported(ix->W)) return false;
    if (!can_prune(ix)) return false;   // its filter slack is margin * sum_j a_j
    // full-precision queries need the filter; the dyadic kernels have none (their binary queries are exact)
    if (float_query && ix->mode != rbe::kModeScaled) return false;
    if (ix->batch_path == 1) return false;
    if (ix->batch_path >= 2) return true;
    // Measured crossover, 1e9 items d=64 P=3, whole search, XOR/popcount scan / this scan.  Integer operands
    // (general scales): 4 queries 6.5 / 6.7 ms, 5 queries 8.0 / 6.8 ms; a 16-query tile costs this scan about as
    // much as 4.3 queries cost the other.  The dyadic modes, 1e9 items, 2 / 3 / 4 (6e8 items) planes, half operands:
    // 5 queries 4.9 / 5.0, 7.1 / 6.9, 5.8 / 6.0 ms; 6 queries 5.6 / 5.1, 8.2 / 7.0, 6.6 / 6.1 ms; integer operands
    // (while the query fits them): 4 queries 4.1 / 4.1, 5.7 / 4.9, 4.7 / 4.0 ms, 5 queries 4.8 / 4.2, 6.8 / 5.0,
    // 5.6 / 4.0 ms.  The byte-table scan of fp32 queries reads the corpus once per query (3.0 ms each), so there the
    // matrix cores win from 3 queries on (7.8 ms).
    if (float_query) return Q >= 3u;
    if (ix->mode != rbe::kModeScaled) return Q >= (batch_operand_i8(ix, false, q_n_planes) ? 4u : 6u);
    return Q >= (batch_operand_i8(ix, false) ? 5u : 7u);
}

// Matrix-core operands of a batch (pure host arithmetic).  Each query is reconstructed in double as
// qhat = sum_i c_i b^i and scaled by a power of two so that v = qhat * 2^k lies in (-1, 1).
//
// The kernel's B operand holds, for item bit b, the half whose only set bit is bit 10 + t (t = 0..3):
// 0 or val_t = 2^-14, 2^-13, 2^-11, 2^-7.  With rho = 2b - 1:
//     sum_d v_d rho_d = sum_d (2 v_d / val_t) (b_d val_t) - sum_d v_d,
// so the A operand carries 2 v_d / val_t (below 2^15), rounded to one half, and the accumulator starts at
// -sum_d v_d.  Lane (g, row) of 32-dimension part kp holds slot e = 2t + h; the kernel
// rotates the part's word left by 4g and takes bits 10 + t (h = 0) and 26 + t (h = 1), i.e. original bit
// (10 + 16h + t - 4g) mod 32.  Dyadic modes: one exact half, one copy per item plane j scaled by 2^-j, and
// the start value covers all planes.
// General scales: the half is a rounding (hi); the accumulators then start at minus the sum of what the
// halves actually hold, so that the contraction equals sum_d vhi_d rho_d exactly, and *margin receives a bound,
// valid for every query of the batch, on |sum_d v_d rho_d - sum_d vhi_d rho_d| plus the fp32 rounding of either
// side (worst case, not typical): the contraction adds d + 1 terms of total magnitude <= 3 sum_d |v_d| in fp32,
// possibly truncating (<= 3 (d + 8) 2^-23 sum_d |v_d|, the + 8 for the P FMAs after it); the XOR/popcount
// arithmetic rounds P (PQ + 2) times at magnitudes up to d sum_i |c_i| (<= 2^-20 of that, which can exceed
// sum_d |v_d| when the query's planes cancel); the byte-table arithmetic of fp32 queries rounds 8W table
// entries and adds them (<= 2^-19 sum_d |v_d|):
//     margin = max_q ( sum_d |v_d - vhi_d| + 3 (d + 8) 2^-23 sum_d |v_d| + 2^-20 d sum_i |c_i| 2^k  [+ 2^-19 sum_d |v_d|] ).
// A hi half that would be subnormal is stored as zero (and counted as lost), so that the bound does not depend
// on how the matrix cores treat subnormal inputs.
//   halves  [tile][plane copy][part][lane][8]   (tile = query / 16, lane = 16 g + query % 16)
//   unscale [Q] = 2^-k,   bias [Q] = start value of the accumulators
struct BatchOperandShape { uint32_t tiles, copies, parts; size_t n_halves; };

BatchOperandShape batch_operand_shape(uint32_t W, uint32_t P, bool dyadic, uint32_t Q)
{
    BatchOperandShape sh;
    sh.tiles = batch_tiles(Q);
    sh.copies = dyadic ? P : 1u;
    sh.parts = 2u * W;
    sh.n_halves = (size_t)sh.tiles * sh.copies * sh.parts * 64 * 8;
    return sh;
}

// q_float != nullptr: the queries are given in full precision ([Q][dim], hybrid scoring) and q_planes / q_scales
// are not read; general scales only.
void build_batch_operands(uint32_t W, uint32_t P, bool dyadic, const uint64_t* q_planes, const float* q_scales,
                          uint32_t Q, uint32_t PQ, uint16_t* halves, float* unscale, float* bias,
                          const float* q_float = nullptr, float* margin = nullptr, float* qmass = nullptr)
{
    const BatchOperandShape sh = batch_operand_shape(W, P, dyadic, Q);
    double worst = 0.0;
    const uint32_t dim = 64 * W, KP = sh.parts, PA = sh.copies;
    std::memset(halves, 0, sh.n_halves * sizeof(uint16_t));
    std::vector<double> qhat(dim);
    static const int kValExp[4] = {-14, -13, -11, -7};
    for (uint32_t q = 0; q < Q; ++q) {
        double biggest = 0.0;
        for (uint32_t d = 0; d < dim; ++d) {
            double v = 0.0;
            if (q_float) {
                v = (double)q_float[(size_t)q * dim + d];
            } else {
                for (uint32_t i = 0; i < PQ; ++i) {
                    const double c = dyadic ? std::ldexp(1.0, -(int)i) : (double)q_scales[(size_t)q * PQ + i];
                    const uint64_t word = q_planes[((size_t)q * PQ + i) * W + d / 64];
                    v += ((word >> (d % 64)) & 1ull) ? c : -c;
                }
            }
            qhat[d] = v;
            biggest = std::max(biggest, std::fabs(v));
        }
        const int k = biggest > 0.0 ? -(std::ilogb(biggest) + 1) : 0;
        unscale[q] = std::ldexp(1.0f, -k);
        const uint32_t qt = q / 16, row = q % 16;
        double coef_mass = 0.0;     // d * sum_i |c_i| in the scaled domain
        if (!q_float && !dyadic)
            for (uint32_t i = 0; i < PQ; ++i) coef_mass += std::fabs((double)q_scales[(size_t)q * PQ + i]);
        coef_mass = std::ldexp(coef_mass * dim, k);
        double sum = 0.0, lost = 0.0, mass = 0.0;
        for (uint32_t part = 0; part < KP; ++part)
            for (uint32_t grp = 0; grp < 4; ++grp)
                for (uint32_t e = 0; e < 8; ++e) {
                    const uint32_t t = e >> 1, h = e & 1u;
                    const uint32_t bit = (10u + 16u * h + t + 32u - 4u * grp) & 31u;
                    const double v = std::ldexp(qhat[part * 32 + bit], k);
                    const uint32_t lane = grp * 16 + row;
                    bool drop = false;
                    if (!dyadic) {
                        // what the half really holds, back in the units of v
                        double held = std::ldexp((double)(float)(_Float16)(float)std::ldexp(v, 1 - kValExp[t]), kValExp[t] - 1);
                        drop = std::fabs(std::ldexp(held, 1 - kValExp[t])) < std::ldexp(1.0, -14);
                        if (drop) held = 0.0;
                        sum += held;
                        lost += std::fabs(v - held);
                        mass += std::fabs(v);
                    } else {
                        sum += v;
                    }
                    for (uint32_t pa = 0; pa < PA; ++pa) {
                        const double aval = std::ldexp(v, 1 - kValExp[t] - (int)pa);
                        const _Float16 hi = drop ? (_Float16)0.0f : (_Float16)(float)aval;
                        uint16_t bits;
                        std::memcpy(&bits, &hi, 2);
                        halves[((((size_t)qt * PA + pa) * KP + part) * 64 + lane) * 8 + e] = bits;
                    }
                }
        const double sum_v = sum;
        if (dyadic) sum *= 2.0 - std::ldexp(1.0, 1 - (int)P);   // every plane's term starts from its own -2^-j sum
        bias[q] = (float)-sum;
        if (qmass) {
            double m_abs = 0.0;
            for (uint32_t d = 0; d < dim; ++d) m_abs += std::fabs(std::ldexp(qhat[d], k));
            if (dyadic) {
                // the most the last plane's term can add to an accumulator that already holds its start value:
                // 2^-(P-1) (qhat . rho + sum_d v_d) <= 2^-(P-1) (sum_d |v_d| + sum_d v_d); a short dyadic fraction
                qmass[q] = (float)std::ldexp(m_abs + sum_v, 1 - (int)P);
            } else {
                // sum_d |v_d|, rounded up: the largest value qhat . rho can take in the scaled domain
                float mf = (float)(m_abs * (1.0 + std::ldexp(1.0, -20)));
                if ((double)mf < m_abs * (1.0 + std::ldexp(1.0, -20))) mf = std::nextafter(mf, INFINITY);
                qmass[q] = mf;
            }
        }
        worst = std::max(worst, lost + std::ldexp(mass * 3.0 * (dim + 8), -23) + std::ldexp(coef_mass, -20) +
                                    (q_float ? std::ldexp(mass, -19) : 0.0) + std::fabs(sum - (double)(float)sum));
    }
    if (margin) *margin = dyadic ? 0.0f : (float)(worst * (1.0 + std::ldexp(1.0, -10)));
}

// Eight-bit integer operands of a batch of binary queries on general scales (pure host arithmetic).
// qhat = sum_i c_i b^i is rounded to T_d * 2^e, T_d an integer of magnitude <= 126 (e the least exponent that
// allows it).  The kernel's B operand holds, for item bit b_d, a byte that is 0 or 64 (dimensions 2g of every
// byte of the plane word, lane group g) or 0 or -128 (dimensions 2g + 1); the A operand holds T_d against the
// 64s and M_d = -round(qhat_d / 2^(e+1)) against the -128s (T_d = -2 M_d there: one bit less).  With rho = 2b - 1
//     64 sum_even T_d b_d - 128 sum_odd M_d b_d - 32 sum_d T_d = 32 sum_d T_d rho_d,
// so the accumulators start at (the bit pattern of the float) 1.5 * 2^23 - 32 sum_d T_d and end at the bit
// pattern of 1.5 * 2^23 + 32 sum_d T_d rho_d: scores are formed in units of 2^e / 32 = unscale.
//   bytes   [tile][64-dim part][lane][16]   (tile = query / 16, lane = 16 g + query % 16; byte 4t + m of a lane
//           is dimension 64 part + 32 (t / 2) + 8 m + 2 g + (t % 2))
// *margin bounds, for every query of the batch and per unit of sum_j a_j[item], the distance between the filter's
// value and the score as the XOR/popcount arithmetic forms it, in those units: the rounding of the query
// (sum_d |qhat_d - 2^e T_d|), the multiply-adds through which the start constant leaves again (its product with
// the item's scale sum is rounded once, and each of two multiply-adds rounds at that magnitude: <= 3 units; 4
// are allowed), and the roundings of the XOR/popcount arithmetic (<= 2^-20 d sum_i |c_i|).
// q_float != nullptr: the queries are given in full precision ([Q][dim], hybrid scoring), q_planes / q_scales are
// not read, and the margin allows for the byte-table arithmetic (<= 2^-19 sum_d |q_d|) in place of the XOR/popcount one.
void build_batch_operands_i8(uint32_t W, const uint64_t* q_planes, const float* q_scales, uint32_t Q, uint32_t PQ,
                             int8_t* bytes, float* unscale, float* bias, float* margin, float* qmass,
                             const float* q_float = nullptr)
{
    const uint32_t dim = 64 * W, tiles = batch_tiles(Q);
    std::memset(bytes, 0, (size_t)tiles * W * 64 * 16);
    std::vector<double> qhat(dim);
    double worst = 0.0;
    for (uint32_t q = 0; q < Q; ++q) {
        double biggest = 0.0, coef = 0.0;
        for (uint32_t d = 0; d < dim; ++d) {
            double v = 0.0;
            if (q_float) {
                v = (double)q_float[(size_t)q * dim + d];
            } else {
                for (uint32_t i = 0; i < PQ; ++i) {
                    const double c = (double)q_scales[(size_t)q * PQ + i];
                    const uint64_t word = q_planes[((size_t)q * PQ + i) * W + d / 64];
                    v += ((word >> (d % 64)) & 1ull) ? c : -c;
                }
            }
            qhat[d] = v;
            biggest = std::max(biggest, std::fabs(v));
        }
        if (!q_float)
            for (uint32_t i = 0; i < PQ; ++i) coef += std::fabs((double)q_scales[(size_t)q * PQ + i]);
        int e = 0;
        if (biggest > 0.0) {
            e = std::ilogb(biggest) - 6;                        // biggest / 2^e in [64, 128)
            if (std::ldexp(biggest, -e) > 126.0) ++e;
        }
        const double unit = std::ldexp(1.0, e - 5);             // 2^e / 32
        unscale[q] = (float)unit;
        const uint32_t qt = q / 16, row = q % 16;
        double lost = 0.0, mass = 0.0;
        long sum_t = 0;
        for (uint32_t part = 0; part < W; ++part)
            for (uint32_t grp = 0; grp < 4; ++grp)
                for (uint32_t t = 0; t < 4; ++t)
                    for (uint32_t m = 0; m < 4; ++m) {
                        const uint32_t d = 64 * part + 32 * (t / 2) + 8 * m + 2 * grp + (t % 2);
                        long T, stored;
                        if (t % 2 == 0) { T = std::lrint(std::ldexp(qhat[d], -e)); stored = T; }
                        else { stored = -std::lrint(std::ldexp(qhat[d], -e - 1)); T = -2 * stored; }
                        sum_t += T;
                        lost += std::fabs(qhat[d] - std::ldexp((double)T, e));
                        mass += std::fabs(qhat[d]);
                        bytes[(((size_t)qt * W + part) * 64 + grp * 16 + row) * 16 + 4 * t + m] = (int8_t)stored;
                    }
        bias[q] = (float)(12582912.0 - 32.0 * (double)sum_t);    // exact: |32 sum T| < 2^22
        // sum_d |qhat_d| in the units of the scores, rounded up: the largest value qhat . rho can take
        const double m_abs = mass / unit * (1.0 + std::ldexp(1.0, -20));
        float mf = (float)m_abs;
        if ((double)mf < m_abs) mf = std::nextafter(mf, INFINITY);
        qmass[q] = mf;
        worst = std::max(worst, lost / unit + 4.0 + std::ldexp(coef * dim / unit, -20) + (q_float ? std::ldexp(mass / unit, -19) : 0.0));
    }
    *margin = (float)(worst * (1.0 + std::ldexp(1.0, -10)));
}

// Eight-bit integer operands of a batch of binary queries on a dyadic index (pure host arithmetic; exact).
// qhat_d = sum_i +-2^-i, so T_d = 2^(PQ-1) qhat_d is an odd integer of magnitude below 2^PQ; item plane j weighs
// 2^-j, and its copy of the query operand holds X_d = 2 T_d 2^(P-1-j) against the 64s of the kernel's item operand
// and -X_d / 2 against the -128s (see build_batch_operands_i8; the factor 2 keeps the halves whole).  All planes add
// into one accumulator, which starts at (the bit pattern of the float) 1.5 * 2^23 - 32 sum_j sum_d X_d and ends at
// 1.5 * 2^23 + 2^(P + PQ + 4) s(q, z): no rounding anywhere, unscale = 2^-(P + PQ + 4).
//   bytes   [tile][plane copy][64-dim part][lane][16]
// qmass: the most the last plane's term can add to an accumulator that already holds its start value,
// 32 (sum_d |X_d| + sum_d X_d) for the last plane's copy.
// Fits eight bits while 2 (2^PQ - 1) 2^(P-1) <= 127 (batch_operand_i8).
void build_batch_operands_i8_dyadic(uint32_t W, uint32_t P, const uint64_t* q_planes, uint32_t Q, uint32_t PQ,
                                    int8_t* bytes, float* unscale, float* bias, float* qmass)
{
    const uint32_t dim = 64 * W, tiles = batch_tiles(Q);
    std::memset(bytes, 0, (size_t)tiles * P * W * 64 * 16);
    std::vector<long> T(dim);
    for (uint32_t q = 0; q < Q; ++q) {
        for (uint32_t d = 0; d < dim; ++d) {
            long v = 0;
            for (uint32_t i = 0; i < PQ; ++i) {
                const uint64_t word = q_planes[((size_t)q * PQ + i) * W + d / 64];
                const long c = 1l << (PQ - 1 - i);
                v += ((word >> (d % 64)) & 1ull) ? c : -c;
            }
            T[d] = v;
        }
        const uint32_t qt = q / 16, row = q % 16;
        long sum_all = 0, last_abs = 0, last_sum = 0;
        for (uint32_t pa = 0; pa < P; ++pa)
            for (uint32_t part = 0; part < W; ++part)
                for (uint32_t grp = 0; grp < 4; ++grp)
                    for (uint32_t t = 0; t < 4; ++t)
                        for (uint32_t m = 0; m < 4; ++m) {
                            const uint32_t d = 64 * part + 32 * (t / 2) + 8 * m + 2 * grp + (t % 2);
                            const long X = 2 * T[d] * (1l << (P - 1 - pa));
                            const long stored = (t % 2 == 0) ? X : -X / 2;
                            sum_all += X;
                            if (pa + 1 == P) { last_abs += std::labs(X); last_sum += X; }
                            bytes[((((size_t)qt * P + pa) * W + part) * 64 + grp * 16 + row) * 16 + 4 * t + m] = (int8_t)stored;
                        }
        bias[q] = (float)(12582912.0 - 32.0 * (double)sum_all);      // exact: |32 sum X| < 2^22
        unscale[q] = std::ldexp(1.0f, -(int)(P + PQ + 4));
        qmass[q] = (float)(32.0 * (double)(last_abs + last_sum));    // exact
    }
}

// Integer operands serve general scales (binary and fp32 queries) and, while they fit eight bits, the binary queries
// of the dyadic modes (q_n_planes = 0: not known yet, taken as "no"); path 3 of rbe_debug_set_batch_path keeps the halves.
bool batch_operand_i8(const rbe_index* ix, bool float_query, uint32_t q_n_planes)
{
    if (ix->batch_path == 3) return false;
    if (ix->mode != rbe::kModeScaled)
        return !float_query && q_n_planes >= 1 && 2u * ((1u << q_n_planes) - 1u) * (1u << (ix->P - 1)) <= 127u;
    // (the accumulators' start constant, 1.5 * 2^23, is multiplied by the item's scale sum on its way out: scales
    // beyond 2^80 -- which would bring that product near the end of the fp32 range -- keep the halves)
    return ix->scale_max <= 0x1p80f;
}

int stage_batch_queries(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t Q, uint32_t PQ,
                        hipStream_t st, const float* q_float = nullptr)
{
    const bool dyadic = ix->mode != rbe::kModeScaled;
    ix->batch_i8 = batch_operand_i8(ix, q_float != nullptr, PQ);
    if (ix->batch_i8) {
        const uint32_t copies = dyadic ? ix->P : 1u;
        if (dyadic) {
            build_batch_operands_i8_dyadic(ix->W, ix->P, q_planes, Q, PQ, reinterpret_cast<int8_t*>(ix->h_aops), ix->h_unscale,
                                           ix->h_unscale + RBE_MAX_QUERIES, ix->h_unscale + 2 * RBE_MAX_QUERIES);
            ix->batch_margin = 0.0f;
        } else {
            build_batch_operands_i8(ix->W, q_planes, q_scales, Q, PQ, reinterpret_cast<int8_t*>(ix->h_aops), ix->h_unscale,
                                    ix->h_unscale + RBE_MAX_QUERIES, &ix->batch_margin, ix->h_unscale + 2 * RBE_MAX_QUERIES, q_float);
        }
        HIP_TRY(hipMemcpyAsync(ix->ws.aops, ix->h_aops, (size_t)batch_tiles(Q) * copies * ix->W * 64 * 16, hipMemcpyHostToDevice, st));
        HIP_TRY(hipMemcpyAsync(ix->ws.unscale, ix->h_unscale, 3 * RBE_MAX_QUERIES * sizeof(float), hipMemcpyHostToDevice, st));
        return RBE_OK;
    }
    const BatchOperandShape sh = batch_operand_shape(ix->W, ix->P, dyadic, Q);
    build_batch_operands(ix->W, ix->P, dyadic, q_planes, q_scales, Q, PQ, reinterpret_cast<uint16_t*>(ix->h_aops),
                         ix->h_unscale, ix->h_unscale + RBE_MAX_QUERIES, q_float, &ix->batch_margin,
                         ix->h_unscale + 2 * RBE_MAX_QUERIES);
    HIP_TRY(hipMemcpyAsync(ix->ws.aops, ix->h_aops, sh.n_halves * sizeof(uint16_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(ix->ws.unscale, ix->h_unscale, 3 * RBE_MAX_QUERIES * sizeof(float), hipMemcpyHostToDevice, st));
    return RBE_OK;
}

struct Level { uint32_t p_begin, p_end; };

// Refinement plan for the exact mode.  Thanks to the nested-sample-major tile
// order every level is a contiguous range of physical tiles.  The coarsest
// level (an evenly strided sample of the corpus) is read with no threshold and
// must fit the candidate list whole; each finer level reads `ratio` times more
// tiles, minus those already read, and keeps only items that reach the k-th
// best key found so far -- a proven lower bound for the final k-th best.
// The plan starts at the coarsest sample that still holds at least 4k items
// (its k-th best is then a useful threshold and every selection sees about
// ratio*k candidates); failing that, at the finest one that fits `cap`.
// Returns an empty plan if even the coarsest sample does not fit `cap`.
std::vector<Level> make_plan(const rbe::Layout& l, uint32_t cap, uint32_t k)
{
    std::vector<Level> plan;
    uint32_t cmin = 0;
    while (cmin <= l.top && (uint64_t)l.n_ge[cmin] * kTileItems > cap) ++cmin;
    if (cmin > l.top) return plan;
    uint32_t c0 = cmin;
    for (uint32_t c = l.top; c > cmin; --c)
        if ((uint64_t)l.n_ge[c] * kTileItems >= 4ull * k) { c0 = c; break; }
    plan.push_back(Level{0, l.n_ge[c0]});
    for (uint32_t c = c0; c-- > 0;) plan.push_back(Level{l.n_ge[c + 1], l.n_ge[c]});
    return plan;
}

}  // namespace

// =========================================================================== C ABI
extern "C" {

const char* rbe_strerror(int code)
{
    switch (code) {
        case RBE_OK: return "ok";
        case RBE_EINVAL: return "invalid argument";
        case RBE_ENOMEM: return "out of memory";
        case RBE_EHIP: return "HIP runtime error";
        case RBE_ESTATE: return "index is in the wrong state for this call";
        case RBE_EUNSUPPORTED: return "unsupported configuration";
        default: return "unknown error code";
    }
}

const char* rbe_last_error(void) { return g_err; }

uint64_t rbe_n_items(const rbe_index* ix) { return ix ? ix->n_items : 0; }
uint32_t rbe_dim(const rbe_index* ix) { return ix ? ix->dim : 0; }
uint32_t rbe_n_planes(const rbe_index* ix) { return ix ? ix->P : 0; }

// Device memory of an index: [tiles][row maxima: 2 floats per row of 256 items, if the items carry scales]
// [one-byte scale copies, general scales with 2 or more planes][256 bytes for rbe_finalize's reductions], every
// part 256-byte aligned.  With base == nullptr only the size is computed.
struct IndexStorage { char* tiles; float* row_amax; uint32_t* hints; char* fin_scratch; size_t bytes; };

static size_t hint_bytes(const rbe_index* ix)
{
    if (!(ix->mode == rbe::kModeScaled && ix->P >= 2)) return 0;
    const uint32_t nw = ix->P - 1 == 3 ? 4u : ix->P - 1;
    return (size_t)ix->layout.n_tiles * (kTileItems / 4) * (nw + (ix->P >= 3 ? 1u : 0u)) * sizeof(uint32_t);
}

// The copies of the last scale array follow those of the others in the same block.
static uint32_t* last_hints_of(const rbe_index* ix, uint32_t* hints)
{
    if (!hints || ix->P < 3) return nullptr;
    const uint32_t nw = ix->P - 1 == 3 ? 4u : ix->P - 1;
    return hints + (size_t)ix->layout.n_tiles * (kTileItems / 4) * nw;
}

static IndexStorage carve_index_storage(const rbe_index* ix, char* base)
{
    IndexStorage st{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base && bytes ? base + off : nullptr;
        off += (bytes + kWsAlign - 1) / kWsAlign * kWsAlign;
        return p;
    };
    st.tiles = take((size_t)ix->layout.n_tiles * ix->geom.tile_bytes());
    const size_t n_rows = (size_t)ix->layout.n_tiles * (kTileItems / kRow);
    st.row_amax = reinterpret_cast<float*>(take(ix->geom.S > 0 ? 2 * n_rows * sizeof(float) : 0));
    st.hints = reinterpret_cast<uint32_t*>(take(hint_bytes(ix)));
    st.fin_scratch = take(256);
    st.bytes = off;
    return st;
}

static int check_shape(uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags, uint32_t ratio, uint32_t allowed_flags)
{
    ARG_CHECK(dim == 64 || dim == 128 || dim == 256, "dim must be 64, 128 or 256 (got %u)", dim);
    ARG_CHECK(n_planes >= 1 && n_planes <= RBE_MAX_PLANES, "n_planes must be 1..%u (got %u)", RBE_MAX_PLANES, n_planes);
    ARG_CHECK(n_items >= 1 && n_items <= RBE_MAX_ITEMS, "n_items must be 1..%llu", (unsigned long long)RBE_MAX_ITEMS);
    ARG_CHECK((flags & ~allowed_flags) == 0, "unknown or misplaced flags 0x%x", flags & ~allowed_flags);
    if ((flags & RBE_DYADIC) && !rbe::dyadic_supported(dim / 64)) {
        set_error("RBE_DYADIC is built for dim 64 and 128 only (got %u)", dim);
        return RBE_EUNSUPPORTED;
    }
    ARG_CHECK(ratio >= 2 && ratio <= 4096, "sample ratio must be 2..4096 (got %u)", ratio);
    return RBE_OK;
}

static void describe_shape(rbe_index* ix, uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags, uint32_t ratio)
{
    ix->n_items = n_items;
    ix->dim = dim;
    ix->W = dim / 64;
    ix->P = n_planes;
    ix->flags = flags;
    ix->mode = (flags & RBE_DYADIC) ? ((flags & RBE_COSINE) ? rbe::kModeDyadicNorm : rbe::kModeDyadic) : rbe::kModeScaled;
    ix->geom = rbe::TileGeom{ix->W, ix->P, (uint32_t)rbe::scale_arrays(ix->mode, (int)ix->P)};
    ix->layout = rbe::make_layout((uint32_t)((n_items + kTileItems - 1) / kTileItems), ratio);
}

// storage == nullptr: the library allocates the tiles (and, at rbe_finalize, the side arrays) itself.
static int create_with_ratio(rbe_index** out, uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags, uint32_t ratio,
                             void* storage = nullptr, size_t storage_bytes = 0)
{
    ARG_CHECK(out != nullptr, "out is NULL");
    int rc = check_shape(n_items, dim, n_planes, flags, ratio, (uint32_t)(RBE_COSINE | RBE_DYADIC) | (storage ? (uint32_t)RBE_BORROW : 0u));
    if (rc) return rc;

    rbe_index* ix = new (std::nothrow) rbe_index();
    if (!ix) { set_error("host allocation failed"); return RBE_ENOMEM; }
    describe_shape(ix, n_items, dim, n_planes, flags & ~(uint32_t)RBE_BORROW, ratio);

    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&ix->device);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, ix->device);
    if (e != hipSuccess) {
        set_error("no usable HIP device: %s", hipGetErrorString(e));
        delete ix;
        return RBE_EHIP;
    }
    ix->n_cu = prop.multiProcessorCount;

    const size_t bytes = (size_t)ix->layout.n_tiles * ix->geom.tile_bytes();
    if (storage) {
        const IndexStorage need = carve_index_storage(ix, nullptr);
        if (storage_bytes < need.bytes || ((uintptr_t)storage % kWsAlign) != 0) {
            set_error("storage must be 256-byte aligned and hold %zu bytes (rbe_index_bytes); got %zu", need.bytes, storage_bytes);
            delete ix;
            return RBE_EINVAL;
        }
        const IndexStorage st = carve_index_storage(ix, static_cast<char*>(storage));
        ix->borrowed = true;
        ix->d_tiles = st.tiles;
        ix->fin_scratch = st.fin_scratch;
        e = hipMemset(ix->d_tiles, 0, bytes);
    } else {
        e = hipMalloc(&ix->d_tiles, bytes);
        if (e == hipSuccess) e = hipMemset(ix->d_tiles, 0, bytes);
    }
    if (e != hipSuccess) {
        set_error("device allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        if (!ix->borrowed) (void)hipFree(ix->d_tiles);
        delete ix;
        return e == hipErrorOutOfMemory ? RBE_ENOMEM : RBE_EHIP;
    }
    rc = allocate_host_side(ix);
    if (rc) { rbe_free(ix); return rc; }
    *out = ix;
    return RBE_OK;
}

int rbe_index_create(rbe_index** out, uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags)
{
    return create_with_ratio(out, n_items, dim, n_planes, flags, 64);
}

int rbe_index_create_ex(rbe_index** out, uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags,
                        uint32_t sample_ratio)
{
    return create_with_ratio(out, n_items, dim, n_planes, flags, sample_ratio ? sample_ratio : 64);
}

size_t rbe_index_bytes(uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags, uint32_t sample_ratio)
{
    const uint32_t ratio = sample_ratio ? sample_ratio : 64;
    if (check_shape(n_items, dim, n_planes, flags, ratio, (uint32_t)(RBE_COSINE | RBE_DYADIC | RBE_BORROW))) return 0;
    rbe_index shape;
    describe_shape(&shape, n_items, dim, n_planes, flags & ~(uint32_t)RBE_BORROW, ratio);
    return carve_index_storage(&shape, nullptr).bytes;
}

int rbe_index_create_in(rbe_index** out, uint64_t n_items, uint32_t dim, uint32_t n_planes, uint32_t flags,
                        uint32_t sample_ratio, void* storage_dev, size_t storage_bytes)
{
    ARG_CHECK(flags & RBE_BORROW, "rbe_index_create_in takes caller-owned storage: pass RBE_BORROW in flags");
    ARG_CHECK(storage_dev != nullptr, "storage_dev is NULL");
    return create_with_ratio(out, n_items, dim, n_planes, flags, sample_ratio ? sample_ratio : 64, storage_dev, storage_bytes);
}

uint32_t rbe_debug_tile_to_phys(uint32_t n_tiles, uint32_t sample_ratio, uint32_t tile)
{
    const rbe::Layout l = rbe::make_layout(n_tiles, sample_ratio);
    return rbe::tile_to_phys(l, tile);
}

uint32_t rbe_debug_phys_to_tile(uint32_t n_tiles, uint32_t sample_ratio, uint32_t phys)
{
    const rbe::Layout l = rbe::make_layout(n_tiles, sample_ratio);
    const uint32_t t = rbe::phys_to_tile(l, phys);
    return t == rbe::phys_to_tile_per_lane(l, phys) ? t : 0xFFFFFFFFu;     // (the two forms must agree)
}

int rbe_debug_exact_plan(uint64_t n_items, uint32_t sample_ratio, uint32_t cand_capacity, uint32_t k,
                         uint32_t* n_levels, uint32_t* first_tile, uint32_t* end_tile)
{
    ARG_CHECK(n_levels && first_tile && end_tile, "NULL argument");
    ARG_CHECK(n_items >= 1 && n_items <= RBE_MAX_ITEMS, "n_items out of range");
    ARG_CHECK(sample_ratio >= 2 && sample_ratio <= 4096, "sample_ratio out of range");
    const rbe::Layout l = rbe::make_layout((uint32_t)((n_items + kTileItems - 1) / kTileItems), sample_ratio);
    const std::vector<Level> plan = make_plan(l, cand_capacity, k);
    ARG_CHECK(plan.size() <= RBE_MAX_LEVELS, "plan longer than RBE_MAX_LEVELS");
    *n_levels = (uint32_t)plan.size();
    for (size_t i = 0; i < plan.size(); ++i) { first_tile[i] = plan[i].p_begin; end_tile[i] = plan[i].p_end; }
    return RBE_OK;
}

int rbe_debug_batch_operands(const uint64_t* q_planes, const float* q_scales, const float* q_float, uint32_t n_queries,
                             uint32_t q_n_planes, uint32_t dim, uint32_t n_planes, uint32_t dyadic, uint16_t* halves_out,
                             size_t halves_capacity, float* unscale_out, float* start_out, uint32_t* shape_out)
{
    ARG_CHECK(halves_out && unscale_out && start_out && shape_out, "NULL argument");
    ARG_CHECK(dyadic <= 1, "dyadic must be 0 or 1");
    ARG_CHECK(q_float ? dyadic == 0 : (q_planes && (dyadic == 1 || q_scales)), "queries missing (or fp32 queries on a dyadic index)");
    ARG_CHECK(dim == 64 || dim == 128, "dim must be 64 or 128");
    ARG_CHECK(n_planes >= 1 && n_planes <= RBE_MAX_PLANES, "n_planes out of range");
    ARG_CHECK(q_float || (q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES), "q_n_planes out of range");
    ARG_CHECK(n_queries >= 1 && n_queries <= RBE_MAX_QUERIES, "n_queries out of range");
    if (q_float)
        for (size_t i = 0; i < (size_t)n_queries * dim; ++i) ARG_CHECK(std::isfinite(q_float[i]), "q_float[%zu] is not finite", i);
    const BatchOperandShape sh = batch_operand_shape(dim / 64, n_planes, dyadic == 1, n_queries);
    ARG_CHECK(halves_capacity >= sh.n_halves, "halves_out too small: %zu needed", sh.n_halves);
    float margin = 0.0f;
    build_batch_operands(dim / 64, n_planes, dyadic == 1, q_planes, q_scales, n_queries, q_n_planes, halves_out,
                         unscale_out, start_out, q_float, &margin);
    shape_out[0] = sh.tiles; shape_out[1] = sh.copies; shape_out[2] = sh.parts;
    std::memcpy(&shape_out[3], &margin, sizeof(float));
    return RBE_OK;
}

int rbe_debug_batch_operands_i8(const uint64_t* q_planes, const float* q_scales, const float* q_float, uint32_t n_queries,
                                uint32_t q_n_planes, uint32_t dim, int8_t* bytes_out, size_t bytes_capacity,
                                float* unscale_out, float* start_out, float* mass_out, float* margin_out)
{
    ARG_CHECK(bytes_out && unscale_out && start_out && mass_out && margin_out, "NULL argument");
    ARG_CHECK(q_float || (q_planes && q_scales), "queries missing");
    ARG_CHECK(dim == 64 || dim == 128, "dim must be 64 or 128");
    ARG_CHECK(q_float || (q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES), "q_n_planes out of range");
    ARG_CHECK(n_queries >= 1 && n_queries <= RBE_MAX_QUERIES, "n_queries out of range");
    if (q_float)
        for (size_t i = 0; i < (size_t)n_queries * dim; ++i) ARG_CHECK(std::isfinite(q_float[i]), "q_float[%zu] is not finite", i);
    else
        for (size_t i = 0; i < (size_t)n_queries * q_n_planes; ++i) ARG_CHECK(std::isfinite(q_scales[i]), "q_scales[%zu] is not finite", i);
    const size_t need = (size_t)batch_tiles(n_queries) * (dim / 64) * 64 * 16;
    ARG_CHECK(bytes_capacity >= need, "bytes_out too small: %zu needed", need);
    build_batch_operands_i8(dim / 64, q_planes, q_scales, n_queries, q_n_planes, bytes_out, unscale_out, start_out,
                            margin_out, mass_out, q_float);
    return RBE_OK;
}

int rbe_debug_batch_operands_i8_dyadic(const uint64_t* q_planes, uint32_t n_queries, uint32_t q_n_planes, uint32_t dim,
                                       uint32_t n_item_planes, int8_t* bytes_out, size_t bytes_capacity,
                                       float* unscale_out, float* start_out, float* mass_out)
{
    ARG_CHECK(q_planes && bytes_out && unscale_out && start_out && mass_out, "NULL argument");
    ARG_CHECK(dim == 64 || dim == 128, "dim must be 64 or 128");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes out of range");
    ARG_CHECK(n_item_planes >= 1 && n_item_planes <= RBE_MAX_PLANES, "n_item_planes out of range");
    ARG_CHECK(n_queries >= 1 && n_queries <= RBE_MAX_QUERIES, "n_queries out of range");
    ARG_CHECK(2u * ((1u << q_n_planes) - 1u) * (1u << (n_item_planes - 1)) <= 127u,
              "%u query planes against %u item planes do not fit eight-bit integer operands", q_n_planes, n_item_planes);
    const size_t need = (size_t)batch_tiles(n_queries) * n_item_planes * (dim / 64) * 64 * 16;
    ARG_CHECK(bytes_capacity >= need, "bytes_out too small: %zu needed", need);
    build_batch_operands_i8_dyadic(dim / 64, n_item_planes, q_planes, n_queries, q_n_planes, bytes_out, unscale_out,
                                   start_out, mass_out);
    return RBE_OK;
}

int rbe_load_chunk(rbe_index* ix, uint64_t first_item, uint64_t count, const uint64_t* planes,
                   const float* scales, int mem_kind, void* hip_stream)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    if (ix->ready) { set_error("rbe_load_chunk after rbe_finalize"); return RBE_ESTATE; }
    ARG_CHECK(count == 0 || planes != nullptr, "planes is NULL");
    const bool want_scales = ix->mode == rbe::kModeScaled;
    ARG_CHECK(count == 0 || !want_scales || scales != nullptr, "scales is NULL");
    ARG_CHECK(mem_kind == RBE_MEM_HOST || mem_kind == RBE_MEM_DEVICE, "bad mem_kind %d", mem_kind);
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item,
              "items [%llu, +%llu) outside the index of %llu items", (unsigned long long)first_item,
              (unsigned long long)count, (unsigned long long)ix->n_items);
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    const uint64_t* src_planes = planes;
    const float* src_scales = scales;
    uint64_t* tmp_planes = nullptr;
    float* tmp_scales = nullptr;
    const size_t pbytes = (size_t)ix->P * count * ix->W * sizeof(uint64_t);
    const size_t sbytes = (size_t)ix->P * count * sizeof(float);
    if (mem_kind == RBE_MEM_HOST) {  // stage the chunk on the device, then scatter it into tiles
        hipError_t e = hipMalloc(&tmp_planes, pbytes);
        if (e == hipSuccess && want_scales) e = hipMalloc(&tmp_scales, sbytes);
        if (e == hipSuccess) e = hipMemcpyAsync(tmp_planes, planes, pbytes, hipMemcpyHostToDevice, st);
        if (e == hipSuccess && want_scales) e = hipMemcpyAsync(tmp_scales, scales, sbytes, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) {
            set_error("staging a chunk of %zu bytes failed: %s", pbytes + sbytes, hipGetErrorString(e));
            (void)hipFree(tmp_planes);
            (void)hipFree(tmp_scales);
            return e == hipErrorOutOfMemory ? RBE_ENOMEM : RBE_EHIP;
        }
        src_planes = tmp_planes;
        src_scales = tmp_scales;
    }
    hipLaunchKernelGGL(rbe::scatter_chunk, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st, ix->d_tiles,
                       ix->layout, ix->geom, src_planes, src_scales, first_item, count);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && mem_kind == RBE_MEM_HOST) e = hipStreamSynchronize(st);
    (void)hipFree(tmp_planes);
    (void)hipFree(tmp_scales);
    if (e != hipSuccess) { set_error("rbe_load_chunk: %s", hipGetErrorString(e)); return RBE_EHIP; }
    ix->loaded_any = true;
    return RBE_OK;
}

int rbe_encode_chunk(rbe_index* ix, uint64_t first_item, uint64_t count, const float* x, int mem_kind,
                     void* hip_stream)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    if (ix->ready) { set_error("rbe_encode_chunk after rbe_finalize"); return RBE_ESTATE; }
    ARG_CHECK(count == 0 || x != nullptr, "x is NULL");
    ARG_CHECK(mem_kind == RBE_MEM_HOST || mem_kind == RBE_MEM_DEVICE, "bad mem_kind %d", mem_kind);
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item,
              "items [%llu, +%llu) outside the index of %llu items", (unsigned long long)first_item,
              (unsigned long long)count, (unsigned long long)ix->n_items);
    if (ix->mode != rbe::kModeScaled) {
        set_error("rbe_encode_chunk produces per-plane scales; a dyadic index takes planes from the model");
        return RBE_EUNSUPPORTED;
    }
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    const float* src = x;
    float* tmp = nullptr;
    const size_t bytes = (size_t)count * ix->dim * sizeof(float);
    if (mem_kind == RBE_MEM_HOST) {
        hipError_t e = hipMalloc(&tmp, bytes);
        if (e == hipSuccess) e = hipMemcpyAsync(tmp, x, bytes, hipMemcpyHostToDevice, st);
        if (e != hipSuccess) {
            set_error("staging %zu bytes of vectors failed: %s", bytes, hipGetErrorString(e));
            (void)hipFree(tmp);
            return e == hipErrorOutOfMemory ? RBE_ENOMEM : RBE_EHIP;
        }
        src = tmp;
    }
    const uint32_t per_block = 256 / ix->W;
    const dim3 grid((uint32_t)((count + per_block - 1) / per_block));
    switch (ix->W) {
        case 1: hipLaunchKernelGGL(rbe::encode_chunk<1>, grid, dim3(256), 0, st, ix->d_tiles, ix->layout, ix->geom, src, first_item, count); break;
        case 2: hipLaunchKernelGGL(rbe::encode_chunk<2>, grid, dim3(256), 0, st, ix->d_tiles, ix->layout, ix->geom, src, first_item, count); break;
        default: hipLaunchKernelGGL(rbe::encode_chunk<4>, grid, dim3(256), 0, st, ix->d_tiles, ix->layout, ix->geom, src, first_item, count); break;
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && mem_kind == RBE_MEM_HOST) e = hipStreamSynchronize(st);
    (void)hipFree(tmp);
    if (e != hipSuccess) { set_error("rbe_encode_chunk: %s", hipGetErrorString(e)); return RBE_EHIP; }
    ix->loaded_any = true;
    return RBE_OK;
}

int rbe_encode_corpus(rbe_index** out, const float* x, uint64_t n_items, uint32_t dim, uint32_t n_planes,
                      int mem_kind, uint32_t flags, void* hip_stream)
{
    ARG_CHECK(out != nullptr, "out is NULL");
    rbe_index* ix = nullptr;
    int rc = rbe_index_create(&ix, n_items, dim, n_planes, flags);
    if (rc) return rc;
    rc = rbe_encode_chunk(ix, 0, n_items, x, mem_kind, hip_stream);
    if (!rc) rc = rbe_finalize(ix, hip_stream);
    if (rc) { rbe_free(ix); return rc; }
    *out = ix;
    return RBE_OK;
}

int rbe_finalize(rbe_index* ix, void* hip_stream)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    if (ix->ready) { set_error("rbe_finalize called twice"); return RBE_ESTATE; }
    hipStream_t st = (hipStream_t)hip_stream;
    const IndexStorage lent = ix->borrowed ? carve_index_storage(ix, ix->d_tiles) : IndexStorage{};

    // What the caller's scales look like (general scales only; the dyadic modes store none of the caller's):
    // per array the largest magnitude, and whether any sign bit is set.
    static_assert(RBE_MAX_PLANES == 4, "scale_array_max writes its sign flags at out[4 + j]");
    uint32_t h_max[2 * RBE_MAX_PLANES] = {};
    auto measure_scales = [&]() -> int {
        uint32_t* d_max = reinterpret_cast<uint32_t*>(ix->fin_scratch);
        if (!ix->borrowed) HIP_TRY(hipMalloc(&d_max, sizeof(h_max)));
        hipError_t e = hipMemsetAsync(d_max, 0, sizeof(h_max), st);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(rbe::scale_array_max, dim3(ix->layout.n_tiles), dim3(256), 0, st, ix->d_tiles, ix->geom, d_max);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpyAsync(h_max, d_max, sizeof(h_max), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (!ix->borrowed) (void)hipFree(d_max);
        HIP_TRY(e);
        uint32_t top = 0;
        for (uint32_t j = 0; j < ix->P; ++j) top = std::max(top, h_max[j]);
        std::memcpy(&ix->scale_max, &top, sizeof(float));
        return RBE_OK;
    };
    if (ix->mode == rbe::kModeScaled) {
        const int rc = measure_scales();
        if (rc != RBE_OK) return rc;
        ix->nonneg = true;
        for (uint32_t j = 0; j < ix->P; ++j) {
            if (h_max[j] >= 0x7f800000u) {
                set_error("scale array %u holds a value that is not finite", j);
                return RBE_EINVAL;      // the index stays in the loading state: the chunk can be loaded again
            }
            ix->nonneg = ix->nonneg && h_max[RBE_MAX_PLANES + j] == 0;
        }
    }
    if (ix->flags & RBE_COSINE) {
        const uint64_t n_slots = (uint64_t)ix->layout.n_tiles * kTileItems;
        hipLaunchKernelGGL(rbe::fold_cosine, dim3((uint32_t)((n_slots + 255) / 256)), dim3(256), 0, st,
                           ix->d_tiles, ix->geom, n_slots);
        HIP_TRY(hipGetLastError());
        if (ix->mode == rbe::kModeScaled) {     // the scales the scans will see are the folded ones
            const int rc = measure_scales();
            if (rc != RBE_OK) return rc;
        }
    }
    // Side arrays of the pruning scans.  Their bounds hold for scales >= 0 only, so an index with a negative scale
    // gets none and is searched by the plain scans (see can_prune).
    if (ix->geom.S > 0 && ix->nonneg) {
        const size_t n_rows = (size_t)ix->layout.n_tiles * (kTileItems / kRow);
        if (ix->borrowed) ix->d_row_amax = lent.row_amax;
        else HIP_TRY(hipMalloc(&ix->d_row_amax, 2 * n_rows * sizeof(float)));
        hipLaunchKernelGGL(rbe::row_scale_max, dim3(ix->layout.n_tiles), dim3(256), 0, st, ix->d_tiles, ix->geom, ix->d_row_amax,
                           ix->d_row_amax + n_rows);
        HIP_TRY(hipGetLastError());
    }
    if (ix->mode == rbe::kModeScaled && ix->P >= 2 && ix->nonneg) {
        if (ix->borrowed) {
            ix->d_hints = lent.hints;
        } else {
            // optional: without them the one-query scan streams the fp32 scale arrays 0 .. P-2 instead
            const hipError_t eh = hipMalloc(&ix->d_hints, hint_bytes(ix));
            if (eh == hipErrorOutOfMemory) { (void)hipGetLastError(); ix->d_hints = nullptr; }
            else HIP_TRY(eh);
        }
    }
    if (ix->d_hints) {
        // exponent base per array, from the array's largest value (the cosine fold has changed the scales: take the
        // maxima again)
        if (ix->flags & RBE_COSINE) {
            uint32_t* d_max = reinterpret_cast<uint32_t*>(ix->fin_scratch);
            if (!ix->borrowed) HIP_TRY(hipMalloc(&d_max, sizeof(h_max)));
            hipError_t e = hipMemsetAsync(d_max, 0, sizeof(h_max), st);
            if (e == hipSuccess) {
                hipLaunchKernelGGL(rbe::scale_array_max, dim3(ix->layout.n_tiles), dim3(256), 0, st, ix->d_tiles, ix->geom, d_max);
                e = hipGetLastError();
            }
            if (e == hipSuccess) e = hipMemcpyAsync(h_max, d_max, sizeof(h_max), hipMemcpyDeviceToHost, st);
            if (e == hipSuccess) e = hipStreamSynchronize(st);
            if (!ix->borrowed) (void)hipFree(d_max);
            HIP_TRY(e);
        }
        // the largest value, rounded as scale_hints rounds it, gets the largest exponent field (7)
        for (uint32_t j = 0; j + 1 < ix->P; ++j)
            ix->hint_base[j] = std::max(1, (int)((h_max[j] + (1u << 17)) >> 23) - 7);
        ix->hint_base[3] = std::max(1, (int)((h_max[ix->P - 1] + (1u << 17)) >> 23) - 7);
        ix->d_hints_last = last_hints_of(ix, ix->d_hints);
        int* d_base = reinterpret_cast<int*>(ix->fin_scratch ? ix->fin_scratch + 128 : nullptr);
        if (!ix->borrowed) HIP_TRY(hipMalloc(&d_base, 4 * sizeof(int)));
        hipError_t e = hipMemcpyAsync(d_base, ix->hint_base, 4 * sizeof(int), hipMemcpyHostToDevice, st);
        if (e == hipSuccess) {
            if (ix->W == 1) hipLaunchKernelGGL(rbe::scale_hints<1>, dim3(ix->layout.n_tiles), dim3(256), 0, st, ix->d_tiles, ix->geom, d_base, ix->d_hints, ix->d_hints_last);
            else hipLaunchKernelGGL(rbe::scale_hints<2>, dim3(ix->layout.n_tiles), dim3(256), 0, st, ix->d_tiles, ix->geom, d_base, ix->d_hints, ix->d_hints_last);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (!ix->borrowed) (void)hipFree(d_base);
        HIP_TRY(e);
    }
    HIP_TRY(hipStreamSynchronize(st));
    ix->ready = 1;
    return RBE_OK;
}

int rbe_load_corpus(rbe_index** out, const uint64_t* planes, const float* scales, uint64_t n_items,
                    uint32_t dim, uint32_t n_planes, int mem_kind, uint32_t flags, void* hip_stream)
{
    ARG_CHECK(out != nullptr, "out is NULL");
    rbe_index* ix = nullptr;
    int rc = rbe_index_create(&ix, n_items, dim, n_planes, flags);
    if (rc) return rc;
    rc = rbe_load_chunk(ix, 0, n_items, planes, scales, mem_kind, hip_stream);
    if (!rc) rc = rbe_finalize(ix, hip_stream);
    if (rc) { rbe_free(ix); return rc; }
    *out = ix;
    return RBE_OK;
}

void rbe_free(rbe_index* ix)
{
    if (!ix) return;
    (void)hipFree(ix->own_ws);
    if (!ix->borrowed) {
        (void)hipFree(ix->d_tiles);
        (void)hipFree(ix->d_row_amax);
        (void)hipFree(ix->d_hints);
    }
    (void)hipHostFree(ix->h_result);
    (void)hipHostFree(ix->h_aops);
    (void)hipHostFree(ix->h_unscale);
    (void)hipHostFree(ix->h_lut);
    (void)hipHostFree(ix->h_qwords);
    if (ix->ev_ok)
        for (uint32_t i = 0; i < kMaxEvents; ++i) (void)hipEventDestroy(ix->ev[i]);
    delete ix;
}

int rbe_encode_query(const float* x, uint32_t dim, uint32_t n_planes, uint64_t* planes_out, float* scales_out)
{
    ARG_CHECK(x && planes_out && scales_out, "NULL argument");
    ARG_CHECK(dim >= 64 && dim % 64 == 0 && dim <= 4096, "dim must be a multiple of 64 up to 4096 (got %u)", dim);
    ARG_CHECK(n_planes >= 1 && n_planes <= RBE_MAX_PLANES, "n_planes must be 1..%u", RBE_MAX_PLANES);
    const uint32_t W = dim / 64;
    std::vector<float> r(x, x + dim);
    for (uint32_t i = 0; i < dim; ++i)
        if (!std::isfinite(r[i])) { set_error("x[%u] is not finite", i); return RBE_EINVAL; }
    for (uint32_t t = 0; t < n_planes; ++t) {
        double acc = 0.0;
        for (uint32_t i = 0; i < dim; ++i) acc += std::fabs((double)r[i]);
        const float scale = (float)(acc / (double)dim);
        uint64_t* words = planes_out + (size_t)t * W;
        std::fill(words, words + W, (uint64_t)0);
        for (uint32_t i = 0; i < dim; ++i) {
            const bool positive = r[i] > 0.0f;
            if (positive) words[i >> 6] |= 1ull << (i & 63);
            const double step = positive ? (double)scale : -(double)scale;
            r[i] = (float)((double)r[i] - step);
        }
        scales_out[t] = scale;
    }
    return RBE_OK;
}

int rbe_set_profiling(rbe_index* ix, int enabled)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ix->profiling = enabled ? 1 : 0;
    return RBE_OK;
}

int rbe_get_search_stats(const rbe_index* ix, rbe_search_stats* out)
{
    ARG_CHECK(ix != nullptr && out != nullptr, "NULL argument");
    *out = ix->stats;
    return RBE_OK;
}

int rbe_set_tuning(rbe_index* ix, uint32_t cand_capacity, uint32_t blocks_per_cu)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ARG_CHECK(cand_capacity == 0 || (cand_capacity >= 2u * kTileItems && cand_capacity <= (1u << 24)),
              "cand_capacity must be %d..2^24", 2 * kTileItems);
    ARG_CHECK(blocks_per_cu <= 16, "blocks_per_cu must be <= 16");
    if (cand_capacity) ix->cap_override = cand_capacity;
    if (blocks_per_cu) ix->blocks_per_cu = blocks_per_cu;
    return RBE_OK;
}

// One scan + select round.  Exact mode: physical tiles [begin, end).  Near-lossless
// mode: super-block ranks [begin, end) with unit = rank (skip == 0) or the rank-th
// non-multiple of `skip`, super-block = unit * stride.
struct Round { uint32_t begin, end, stride, skip; };

struct SearchCtx {
    rbe_index* ix; hipStream_t st; uint32_t Q, PQ, k, cap, mode, I;
    uint32_t qlen;      // near-lossless: entries per group queue (1 or 2); mode holds RBE_SELECT_NEARLOSSLESS for both
    // near-lossless result through the scans and the plan of the exact mode (mode holds RBE_SELECT_EXACT): before each
    // selection the candidates are reduced to the best qlen per group of Algorithm 1 (group_best_build / _compact)
    bool group_select = false;
    bool float_query;   // hybrid scoring: fp32 queries through byte tables
    bool batch_mfma;    // exact mode, several queries: matrix-core scan
    bool float_batch;   // ... of full-precision queries
    uint32_t look_from = 0;   // matrix-core scan: the levels from this one on report how their first looks went
    uint32_t calib_repeat = 0;   // rbe_debug_issue_rate: the batch scans go over what they loaded this many more times
};

// dense: a coarse level of the plan, where a large share of the items passes the (still loose) threshold.
// The matrix-core scan spends such a level in its survivor path; unless it was asked for explicitly, batches of
// binary queries take the XOR/popcount scan there and the matrix cores for the last, large level only (both
// produce the same scores bit for bit, so the levels of one search may mix them).
static int launch_scan_round(const SearchCtx& c, const Round& r, bool dense, uint32_t level_slot)
{
    rbe_index* ix = c.ix;
    if (r.end <= r.begin) return RBE_OK;
    KernelSel sel{ix->P, c.PQ, ix->mode, c.Q == 1, c.qlen};
    const CandList out{ix->ws.cand, ix->ws.count, ix->ws.kmax, c.cap};
    uint32_t grid = 0;
    hipError_t e;
    if (c.float_query) {
        e = hipSuccess;
        sel.progressive = !dense && ix->P >= 2 && ix->progressive != 0 && can_prune(ix);
        sel.hints = ix->d_hints != nullptr && ix->progressive != 2;
        sel.two_stage = ix->progressive == 1 && ix->P >= 3 && ix->d_hints_last != nullptr && ix->fq_binary;
        const size_t per_q = (size_t)8 * ix->W * 256;
        for (uint32_t q = 0; q < c.Q && e == hipSuccess; ++q) {   // one pass over the range per query
            FqArgs fa;
            fa.tiles = ix->d_tiles; fa.layout = ix->layout; fa.n_items = ix->n_items;
            fa.lut = ix->ws.lut + q * per_q; fa.tau_ptr = ix->ws.tau + q;
            fa.mass = rbe::QueryMass{ix->fq_mass[q][0], ix->fq_mass[q][1]}; fa.deep_rows = ix->ws.status + 1 + level_slot; fa.row_amax = ix->d_row_amax; fa.hints = ix->d_hints; fa.deep_units = ix->ws.status + 14;
            for (int j = 0; j < 3; ++j) fa.hint_base[j] = ix->hint_base[j];
            fa.hints_last = ix->d_hints_last; fa.hint_base_last = ix->hint_base[3];
            fa.qwords = nullptr; fa.qcoef = nullptr; fa.bmass = rbe::QueryMass{0.0f, 0.0f}; fa.resid = 0.0f;
            if (ix->fq_binary) {
                fa.qwords = ix->ws.qwords + (size_t)q * RBE_MAX_PLANES * 2 * ix->W;
                fa.qcoef = ix->ws.qcoef + (size_t)q * (RBE_MAX_PLANES + 1);
                fa.bmass = rbe::QueryMass{ix->fq_bmass[q][0], ix->fq_bmass[q][1]};
                fa.resid = ix->fq_resid[q];
            }
            fa.out = CandList{ix->ws.cand + (size_t)q * c.cap, ix->ws.count + q * rbe::kCountStride, ix->ws.kmax + q * rbe::kKmaxStride, c.cap};
            fa.p_begin = r.begin; fa.p_end = r.end;
            e = launch_scan_exact_fq(ix->W, sel, fa, (uint32_t)ix->n_cu, ix->blocks_per_cu, c.st, &grid);
        }
    } else if (c.batch_mfma && !(dense && !c.float_batch && ix->batch_path == 0)) {
        BatchArgs ba;
        ba.tiles = ix->d_tiles; ba.layout = ix->layout; ba.n_items = ix->n_items;
        ba.a_ops = ix->ws.aops; ba.q_unscale = ix->ws.unscale; ba.q_bias = ix->ws.unscale + RBE_MAX_QUERIES; ba.q_mass = ix->ws.unscale + 2 * RBE_MAX_QUERIES; ba.tau = ix->ws.tau;
        ba.look_stats = level_slot >= c.look_from ? ix->ws.status + 12 : nullptr;
        ba.row_amax = ix->d_row_amax; ba.row_asum = ix->d_row_amax ? ix->d_row_amax + (size_t)ix->layout.n_tiles * (kTileItems / kRow) : nullptr; ba.n_queries = c.Q;
        ba.out = out; ba.p_begin = r.begin; ba.p_end = r.end; ba.calib_repeat = c.calib_repeat;
        // (the lean stream prunes like the progressive scans, and goes by their switch)
        ba.lean = (ix->progressive == 1 && can_prune(ix) && !dense) ? 1u : 0u;
        ba.hints = ba.lean ? ix->d_hints : nullptr;
        for (int j = 0; j < 3; ++j) ba.hint_base[j] = (uint8_t)ix->hint_base[j];
        ba.deep_units = ix->ws.status + 14;
        ba.rescore = batch_rescore(ix, c.float_batch); ba.operand = ix->batch_i8 ? 1u : 0u;
        ba.PQ = c.PQ; ba.qwords = ix->ws.qwords; ba.qcoef = ix->ws.qcoef; ba.lut = ix->ws.lut; ba.margin = ix->batch_margin;
        e = hipSuccess;
        const uint32_t tiles = batch_tiles(c.Q), per_launch = batch_tiles_per_launch(ix, c.float_batch);
        for (uint32_t t0 = 0; t0 < tiles && e == hipSuccess; t0 += per_launch) {   // one pass over the range per launch
            const uint32_t nt = std::min(per_launch, tiles - t0);
            ba.q_begin = 16u * t0;
            e = ix->W == 1 ? launch_scan_batch_w<1>(sel, ba, nt, (uint32_t)ix->n_cu, ix->blocks_per_cu, c.st, &grid)
                           : launch_scan_batch_w<2>(sel, ba, nt, (uint32_t)ix->n_cu, ix->blocks_per_cu, c.st, &grid);
        }
    } else if (c.mode == RBE_SELECT_EXACT) {
        ScanArgs sa;
        sa.tiles = ix->d_tiles; sa.layout = ix->layout; sa.n_items = ix->n_items;
        sa.qwords = ix->ws.qwords; sa.qcoef = ix->ws.qcoef; sa.n_queries = c.Q;
        sa.tau = ix->ws.tau; sa.out = out;
        sa.p_begin = r.begin; sa.p_end = r.end;
        // one query against a level that has a threshold: plane 0 and the scales decide which rows need the rest
        sel.progressive = !dense && ix->P >= 2 && ix->progressive != 0 && can_prune(ix);
        // (several queries: the scan that streams the scale copies is ahead up to four queries per call, 4.3 against
        // 5.2 ms for two, level with the one that streams the fp32 scales at five, behind from six on)
        sel.hints = ix->d_hints != nullptr && ix->progressive != 2 && c.Q <= 4;
        sel.two_stage = ix->progressive == 1 && c.Q <= 4 && ix->P >= 3 && ix->d_hints_last != nullptr;
        sa.deep_rows = ix->ws.status + 1 + level_slot; sa.row_amax = ix->d_row_amax; sa.hints = ix->d_hints; sa.deep_units = ix->ws.status + 14;
        sa.deep_pairs = level_slot >= c.look_from ? ix->ws.status + 9 : nullptr;
        for (int j = 0; j < 3; ++j) sa.hint_base[j] = ix->hint_base[j];
        sa.hints_last = ix->d_hints_last; sa.hint_base_last = ix->hint_base[3];
        // survivor queues in LDS: small batches keep the occupancy the HBM-bound scan wants, large ones trade
        // it for sub-queues of 32..64 entries (fewer, larger flushes)
        sa.stage_entries = c.Q <= 8 ? 512u : (c.Q <= 16 ? 1024u : 2048u);
        sa.calib_repeat = c.calib_repeat;
        e = launch_scan_exact(ix->W, sel, sa, (uint32_t)ix->n_cu, ix->blocks_per_cu, c.st, &grid);
    } else {
        GroupArgs ga;
        ga.tiles = ix->d_tiles; ga.layout = ix->layout; ga.n_items = ix->n_items;
        ga.rows_total = (uint32_t)((ix->n_items + kRow - 1) / kRow); ga.I = c.I;
        ga.qwords = ix->ws.qwords; ga.qcoef = ix->ws.qcoef; ga.q_begin = 0; ga.nq = 0;
        ga.tau = ix->ws.tau; ga.out = out;
        ga.v_begin = r.begin; ga.v_end = r.end; ga.stride = r.stride; ga.skip = r.skip;
        e = launch_scan_groupmax(ix->W, sel, ga, c.Q, (uint32_t)ix->n_cu, ix->blocks_per_cu, c.st, &grid);
    }
    if (e != hipSuccess) { set_error("scan launch failed: %s", hipGetErrorString(e)); return RBE_EHIP; }
    if (level_slot < RBE_MAX_LEVELS) {
        uint32_t which = RBE_KERNEL_SCAN_GROUPMAX;
        if (c.float_query)
            which = !sel.progressive ? RBE_KERNEL_SCAN_FLOAT
                                     : (sel.hints && sel.two_stage && ix->mode == rbe::kModeScaled ? RBE_KERNEL_SCAN_FLOAT_PROG2 : RBE_KERNEL_SCAN_FLOAT_PROG);
        else if (c.batch_mfma && !(dense && !c.float_batch && ix->batch_path == 0)) which = RBE_KERNEL_SCAN_BATCH_MFMA;
        else if (c.mode == RBE_SELECT_EXACT)
            which = !sel.progressive ? RBE_KERNEL_SCAN_EXACT
                                     : (sel.hints ? (sel.two_stage && ix->mode == rbe::kModeScaled ? RBE_KERNEL_SCAN_PROG2_HINT : RBE_KERNEL_SCAN_PROG_HINT)
                                                  : RBE_KERNEL_SCAN_PROG);
        ix->stats.scan_kernel[level_slot] = which;
    }
    ix->stats.grid_blocks = std::max(ix->stats.grid_blocks, grid);
    return RBE_OK;
}

static int run_round(const SearchCtx& c, const Round& r, int final_pass, uint32_t level_slot, bool record,
                     bool dense = false)
{
    rbe_index* ix = c.ix;
    int rc = launch_scan_round(c, r, dense, level_slot);
    if (rc) return rc;
    if (record) HIP_TRY(hipEventRecord(ix->ev[2 * level_slot + 1], c.st));

    if (c.group_select) {
        GroupBestArgs ga;
        ga.cand = ix->ws.cand; ga.count = ix->ws.count; ga.cap = c.cap; ga.table = ix->ws.gtable; ga.slots = ix->ws.gslots;
        ga.aux = ix->ws.gaux; ga.group_span = kRow * c.I; ga.qlen = c.qlen; ga.status = ix->ws.status;
        const uint32_t blocks = std::min<uint32_t>((uint32_t)ix->n_cu * 4u, (c.cap + 255u) / 256u);
        hipLaunchKernelGGL(rbe::group_best_build, dim3(blocks, c.Q), dim3(256), 0, c.st, ga);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(rbe::group_best_compact, dim3(std::min<uint32_t>((uint32_t)ix->n_cu * 2u, (ga.slots + 2047u) / 2048u), c.Q),
                           dim3(256), 0, c.st, ga);
        HIP_TRY(hipGetLastError());
    }

    SelectArgs se;
    se.cand = ix->ws.cand; se.count = ix->ws.count; se.tau = ix->ws.tau; se.kmax = ix->ws.kmax; se.cap = c.cap; se.k = c.k;
    se.status = ix->ws.status; se.count_seen = ix->ws.seen + (size_t)level_slot * RBE_MAX_QUERIES;
    se.final_pass = final_pass; se.ids_out = ix->ws.ids; se.scores_out = ix->ws.scores;
    se.group_aux = c.group_select ? ix->ws.gaux : nullptr;
    hipLaunchKernelGGL(rbe::select_topk, dim3(c.Q), dim3(kSelBlock), 0, c.st, se);
    HIP_TRY(hipGetLastError());
    if (record) HIP_TRY(hipEventRecord(ix->ev[2 * level_slot + 2], c.st));
    return RBE_OK;
}

// Rounds of the near-lossless mode: the same nested-sample idea over super-blocks.
// Every super-block forwards at most 256 group winners; the coarsest sample is
// read with no threshold and must fit the candidate list.
static std::vector<Round> make_group_plan(uint32_t n_super, uint32_t ratio, uint32_t cap, uint32_t per_super)
{
    std::vector<uint32_t> strides{1};
    while ((uint64_t)((n_super + strides.back() - 1) / strides.back()) * per_super > cap &&
           strides.size() < RBE_MAX_LEVELS && strides.back() < n_super)
        strides.push_back(strides.back() * ratio);
    std::vector<Round> plan;
    if ((uint64_t)((n_super + strides.back() - 1) / strides.back()) * per_super > cap) return plan;
    for (size_t l = strides.size(); l-- > 0;) {
        Round r;
        r.stride = strides[l];
        const uint32_t units = (n_super + r.stride - 1) / r.stride;
        r.skip = (l + 1 == strides.size()) ? 0u : ratio;
        r.begin = 0;
        r.end = r.skip ? units - (units + ratio - 1) / ratio : units;
        plan.push_back(r);
    }
    return plan;
}

// Common part of the search entry points: plan, enqueue, wait, copy out.  The queries have
// been staged on the stream already.
static int run_search(SearchCtx& c, int64_t* ids_out, float* scores_out)
{
    rbe_index* ix = c.ix;
    const uint32_t k = c.k, mode = c.mode;
    int rc;
    // units of the slow path: tiles (exact) or super-blocks (near-lossless), `per_unit` candidates each at most
    const uint32_t rows_total = (uint32_t)((ix->n_items + kRow - 1) / kRow);
    const uint32_t n_units = mode == RBE_SELECT_EXACT ? ix->layout.n_tiles : (rows_total + c.I - 1) / c.I;
    const uint32_t per_unit = mode == RBE_SELECT_EXACT ? kTileItems : kRow * c.qlen;
    std::vector<Round> plan;
    bool split = false;
    rbe_index::SplitState& ss = ix->split1;
    const bool pruning = ix->progressive != 0 && ix->P >= 2 && can_prune(ix);
    if (mode == RBE_SELECT_EXACT) {
        for (const Level& lv : make_plan(ix->layout, c.cap, k)) plan.push_back(Round{lv.p_begin, lv.p_end, 1, 0});
        // A batch on the matrix cores: the level before the last starts from the k-th best of a 1/ratio sample of
        // itself, is dense by the rule below, and would go to the XOR/popcount scan at n_queries times the cost of
        // one query (a tenth of a 16-query search at 1e9 items).  Taken in two parts, only its first eighth is
        // dense; the rest starts from the k-th best of an eighth of it and runs on the matrix cores.
        if (c.batch_mfma && !c.float_batch && ix->batch_path == 0 && ix->plan_split != 1 && plan.size() >= 2 &&
            plan.size() + 2 <= RBE_MAX_LEVELS) {
            const size_t l2 = plan.size() - 2;
            const Round lv = plan[l2];
            if (lv.end - lv.begin >= 4096u) {
                const uint32_t mid = lv.begin + (lv.end - lv.begin) / 8;
                plan[l2] = Round{lv.begin, mid, 1, 0};
                plan.insert(plan.begin() + (std::ptrdiff_t)l2 + 1, Round{mid, lv.end, 1, 0});
            }
        }
        c.look_from = plan.empty() ? 0u : (uint32_t)plan.size() - 1;     // the last level (both parts of it, if it is split below)
        // The pruning scans of the last level need a threshold that lies inside the query's neighbourhood, and the
        // level's own threshold (the k-th best of a 1/ratio sample of the corpus) often does not: the level is taken
        // in two parts, an eighth of it first, after which the rest starts from the k-th best of about an eighth of
        // the corpus.  Costs a launch and a selection; measured whole / split: 16 queries over 1e9 items 7.97 / 7.20
        // ms, 8 queries k = 4000 9.2 / 7.7, 64 queries over 1e8 items (d = 128) 11.8 / 7.1, one query there 1.35 /
        // 1.03, the 1.2e9-item dyadic point 1.95 / 1.80 (mean), 3 queries and one fp32 query over 1e9 items 5.26 /
        // 5.23 and 3.03 / 3.02 -- and one binary query over 1e9 items 2.87 / 2.90, the one case that loses.  So the
        // split is the rule, and no search's plan depends on earlier searches, except that one-binary-query
        // searches take the level whole for kWholeSearches searches after kSplitStreak split searches in a row
        // whose second part let through no fewer rows than the first (rate for rate); then they ask again.
        // (a one-query scan in two stages gains from every tightening of the threshold: no exception there)
        const bool two_stage = ix->progressive == 1 && ix->P >= 3 && ix->d_hints_last != nullptr;
        const bool one_binary = c.Q == 1 && !c.float_query && !c.batch_mfma && !two_stage;
        split = ix->plan_split == 2 || (ix->plan_split == 0 && pruning && !(one_binary && ss.whole_left > 0));
        const uint32_t min_tiles = ix->plan_split == 2 ? 16u : kSplitMinTiles;
        if (split && plan.size() >= 2 && plan.size() < RBE_MAX_LEVELS && plan.back().end - plan.back().begin >= min_tiles) {
            const Round last = plan.back();
            const uint32_t mid = last.begin + (last.end - last.begin) / 8;
            plan.back() = Round{last.begin, mid, 1, 0};
            plan.push_back(Round{mid, last.end, 1, 0});
        } else {
            split = false;
        }
    } else {
        plan = make_group_plan(n_units, ix->layout.ratio, c.cap, per_unit);
    }

    // this call's scores follow its ids directly, so that the results are one contiguous range (carve_workspace)
    ix->h_scores = reinterpret_cast<float*>(ix->h_ids + (size_t)c.Q * k);

    ix->stats = rbe_search_stats{};
    const bool prof = ix->profiling != 0;
    bool fallback = plan.empty();

    for (int attempt = 0; attempt < 2; ++attempt) {
        hipLaunchKernelGGL(rbe::init_state, dim3(1), dim3(64), 0, c.st, ix->ws.count, ix->ws.tau, ix->ws.kmax, ix->ws.status, c.Q);
        HIP_TRY(hipGetLastError());
        if (c.group_select) {
            // the group tables start empty (group_best_compact leaves them so after every level) and so do the
            // counters that sit in front of them; both parts are multiples of 256 bytes
            const size_t bytes = (size_t)((char*)ix->ws.gtable - (char*)ix->ws.gaux) + (size_t)c.Q * ix->ws.gslots * 2 * sizeof(uint64_t);
            hipLaunchKernelGGL(rbe::fill_zero16, dim3((uint32_t)std::min<size_t>((size_t)ix->n_cu * 8, (bytes / 16 + 255) / 256)), dim3(256),
                               0, c.st, reinterpret_cast<rbe::u32x4*>(ix->ws.gaux), bytes / 16);
            HIP_TRY(hipGetLastError());
        }
        if (!fallback) {
            if (prof) HIP_TRY(hipEventRecord(ix->ev[0], c.st));
            for (size_t l = 0; l < plan.size(); ++l) {
                // A level is "dense" while a large share of its items passes the threshold it starts with: the k-th
                // best of the items read so far, so about k * (its items) / (items before it) survive.  Above one
                // survivor per 500 items the pruning scans (progressive, matrix-core) spend their time in their
                // survivor paths (measured: at one per 1500 they are still well ahead, at one per 250 well behind).
                const uint64_t before = mode == RBE_SELECT_EXACT ? (uint64_t)plan[l].begin * kTileItems : 0;
                const bool dense = l == 0 || (uint64_t)k * 500u > before;
                rc = run_round(c, plan[l], l + 1 == plan.size(), (uint32_t)l, prof, dense);
                if (rc) return rc;
                ix->stats.items_scanned[l] = (uint64_t)(plan[l].end - plan[l].begin) *
                                             (mode == RBE_SELECT_EXACT ? (uint64_t)kTileItems : (uint64_t)c.I * kRow);
            }
            ix->stats.n_levels = (uint32_t)plan.size();
        } else {
            // Slow path that cannot overflow: segments that add at most cap - k candidates, each
            // followed by a selection that compacts the list back to k entries.
            const uint32_t seg = std::max<uint32_t>(1u, (c.cap - k) / per_unit);
            for (uint64_t u0 = 0; u0 < n_units; u0 += seg) {
                const uint32_t u1 = (uint32_t)std::min<uint64_t>(n_units, u0 + seg);
                rc = run_round(c, Round{(uint32_t)u0, u1, 1, 0}, u1 == n_units, 0, false, u0 == 0);
                if (rc) return rc;
            }
            ix->stats.n_levels = 1;
            ix->stats.fallback = 1;
            ix->stats.items_scanned[0] = (uint64_t)ix->layout.n_tiles * kTileItems;
        }
        HIP_TRY(hipMemcpyAsync(ix->h_result, ix->ws.result,
                               kResultHeaderBytes + (size_t)c.Q * k * (sizeof(int64_t) + sizeof(float)),
                               hipMemcpyDeviceToHost, c.st));
        if (prof && !fallback) HIP_TRY(hipEventRecord(ix->ev[kMaxEvents - 1], c.st));
        HIP_TRY(hipStreamSynchronize(c.st));
        if (!(*ix->h_status & rbe::kStatusOverflow)) break;
        if (fallback) { set_error("candidate list overflowed in the bounded-segment path"); return RBE_EHIP; }
        fallback = true;  // a level produced more survivors than the list holds: redo on the slow path
    }

    ix->stats.deep_units = ix->h_status[14];
    ix->stats.deep_rows = 0;
    for (uint32_t l = 0; l < RBE_MAX_LEVELS; ++l) {
        ix->stats.deep_rows_level[l] = ix->h_status[1 + l];
        ix->stats.deep_rows += ix->h_status[1 + l];
    }
    ix->stats.last_level_parts = (!fallback && split) ? 2u : 1u;
    // one binary query, the pruning scan in use (see the plan above): did the second part of the last level let
    // through a smaller share of its rows than the first?
    if (!fallback && mode == RBE_SELECT_EXACT && c.Q == 1 && !c.float_query && !c.batch_mfma && pruning && ix->plan_split == 0 &&
        !(ix->progressive == 1 && ix->P >= 3 && ix->d_hints_last != nullptr)) {
        if (!split) {
            if (ss.whole_left > 0) --ss.whole_left;
        } else {
            const size_t L = plan.size();
            const uint64_t rows1 = (uint64_t)(plan[L - 2].end - plan[L - 2].begin), rows2 = (uint64_t)(plan[L - 1].end - plan[L - 1].begin);
            const uint64_t deep1 = ix->h_status[1 + (L - 2)], deep2 = ix->h_status[1 + (L - 1)];
            const bool helped = deep2 * rows1 * 4 < deep1 * rows2 * 3;       // a quarter fewer, rate for rate
            ss.streak = helped ? 0u : ss.streak + 1u;
            if (ss.streak >= kSplitStreak) { ss.streak = 0; ss.whole_left = kWholeSearches; }
        }
    }
    if (!fallback) {
        for (uint32_t l = 0; l < ix->stats.n_levels; ++l) {
            uint32_t mx = 0;
            for (uint32_t q = 0; q < c.Q; ++q) mx = std::max(mx, ix->h_seen[(size_t)l * RBE_MAX_QUERIES + q]);
            ix->stats.candidates_max[l] = mx;
            if (prof) {
                HIP_TRY(hipEventElapsedTime(&ix->stats.scan_ms[l], ix->ev[2 * l], ix->ev[2 * l + 1]));
                HIP_TRY(hipEventElapsedTime(&ix->stats.select_ms[l], ix->ev[2 * l + 1], ix->ev[2 * l + 2]));
            }
        }
        if (prof) HIP_TRY(hipEventElapsedTime(&ix->stats.total_gpu_ms, ix->ev[0], ix->ev[kMaxEvents - 1]));
    }
    std::memcpy(ids_out, ix->h_ids, (size_t)c.Q * k * sizeof(int64_t));
    std::memcpy(scores_out, ix->h_scores, (size_t)c.Q * k * sizeof(float));
    return RBE_OK;
}

static int search_prologue(rbe_index* ix, SearchCtx& c, uint32_t n_queries, uint32_t k, uint32_t mode,
                           uint32_t group_size_I, const void* ids_out, const void* scores_out, void* hip_stream,
                           bool static_scratch = false)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    if (!ix->ready) { set_error("search before rbe_finalize"); return RBE_ESTATE; }
    ARG_CHECK(ids_out && scores_out, "NULL output argument");
    ARG_CHECK(n_queries >= 1 && n_queries <= RBE_MAX_QUERIES, "n_queries must be 1..%u (got %u)", RBE_MAX_QUERIES, n_queries);
    ARG_CHECK(k >= 1 && k <= RBE_MAX_K, "k must be 1..%u (got %u)", RBE_MAX_K, k);
    ARG_CHECK(mode == RBE_SELECT_EXACT || mode == RBE_SELECT_NEARLOSSLESS || mode == RBE_SELECT_NEARLOSSLESS_Q2,
              "unknown mode %u", mode);
    ARG_CHECK(group_size_I <= 65535, "group_size_I must be <= 65535");
    c.ix = ix; c.st = (hipStream_t)hip_stream; c.Q = n_queries; c.PQ = 1; c.k = k;
    c.group_select = mode != RBE_SELECT_EXACT && ix->nl_path == 0;
    c.mode = c.group_select ? (uint32_t)RBE_SELECT_EXACT : (mode == RBE_SELECT_NEARLOSSLESS_Q2 ? (uint32_t)RBE_SELECT_NEARLOSSLESS : mode);
    c.qlen = mode == RBE_SELECT_NEARLOSSLESS_Q2 ? 2u : 1u;
    c.I = group_size_I ? group_size_I : 256;
    c.float_query = false;
    c.batch_mfma = false;
    c.float_batch = false;
    c.cap = search_capacity(ix, k);
    const bool groups = mode != RBE_SELECT_EXACT;
    return static_scratch ? acquire_static_scratch(ix, c.Q, k, c.cap, groups) : acquire_workspace(ix, c.Q, k, c.cap, groups);
}

static int search_binary(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t n_queries,
                         uint32_t q_n_planes, uint32_t k, uint32_t mode, uint32_t group_size_I,
                         int64_t* ids_out, float* scores_out, void* hip_stream, bool static_scratch)
{
    SearchCtx c;
    int rc = search_prologue(ix, c, n_queries, k, mode, group_size_I, ids_out, scores_out, hip_stream, static_scratch);
    if (rc) return rc;
    ARG_CHECK(q_planes != nullptr, "q_planes is NULL");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes must be 1..%u (got %u)", RBE_MAX_PLANES, q_n_planes);
    c.PQ = q_n_planes;
    rc = stage_queries(ix, q_planes, q_scales, c.Q, c.PQ, c.st);
    if (rc) return rc;
    c.batch_mfma = use_batch_mfma(ix, c.Q, c.mode, false, c.PQ);
    if (c.batch_mfma) {
        rc = stage_batch_queries(ix, q_planes, q_scales, c.Q, c.PQ, c.st);
        if (rc) return rc;
    }
    return run_search(c, ids_out, scores_out);
}

int rbe_search(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t n_queries,
               uint32_t q_n_planes, uint32_t k, uint32_t mode, uint32_t group_size_I,
               int64_t* ids_out, float* scores_out, void* hip_stream)
{
    return search_binary(ix, q_planes, q_scales, n_queries, q_n_planes, k, mode, group_size_I, ids_out, scores_out,
                         hip_stream, false);
}

int rbe_search_static(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t n_queries,
                      uint32_t q_n_planes, uint32_t k, uint32_t mode, uint32_t group_size_I,
                      int64_t* ids_out, float* scores_out, void* hip_stream)
{
    return search_binary(ix, q_planes, q_scales, n_queries, q_n_planes, k, mode, group_size_I, ids_out, scores_out,
                         hip_stream, true);
}

size_t rbe_workspace_bytes(const rbe_index* ix, uint32_t n_queries, uint32_t k, uint32_t mode)
{
    if (!ix || n_queries < 1 || n_queries > RBE_MAX_QUERIES || k < 1 || k > RBE_MAX_K || mode > RBE_SELECT_NEARLOSSLESS_Q2)
        return 0;
    return carve_workspace(nullptr, nullptr, ix->W, n_queries, k, search_capacity(ix, k), mode != RBE_SELECT_EXACT);
}

int rbe_set_workspace(rbe_index* ix, void* dev_ptr, size_t bytes)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ARG_CHECK(dev_ptr != nullptr || bytes == 0, "NULL workspace with a size");
    ARG_CHECK(((uintptr_t)dev_ptr % kWsAlign) == 0, "the workspace must be 256-byte aligned");
    ix->ext_ws = static_cast<char*>(dev_ptr);
    ix->ext_ws_bytes = dev_ptr ? bytes : 0;
    ix->ws = rbe_index::DevWs{};
    if (dev_ptr) {          // the library's own block is not needed while the caller's is in use
        (void)hipFree(ix->own_ws);
        ix->own_ws = nullptr; ix->own_ws_bytes = 0;
    }
    return RBE_OK;
}

int rbe_search_float(rbe_index* ix, const float* q, uint32_t n_queries, uint32_t k, uint32_t mode,
                     uint32_t group_size_I, int64_t* ids_out, float* scores_out, void* hip_stream)
{
    SearchCtx c;
    int rc = search_prologue(ix, c, n_queries, k, mode, group_size_I, ids_out, scores_out, hip_stream);
    if (rc) return rc;
    ARG_CHECK(q != nullptr, "q is NULL");
    if (c.mode != RBE_SELECT_EXACT) {
        set_error("fp32 queries have no per-thread-queue scan: use the default near-lossless path (rbe_debug_set_nearlossless_path 0)");
        return RBE_EUNSUPPORTED;
    }
    for (size_t i = 0; i < (size_t)c.Q * ix->dim; ++i)
        if (!std::isfinite(q[i])) { set_error("q[%zu][%zu] is not finite", i / ix->dim, i % ix->dim); return RBE_EINVAL; }
    c.batch_mfma = use_batch_mfma(ix, c.Q, c.mode, true);
    if (c.batch_mfma) {
        // several queries: the same dense contraction as for binary queries, with the query itself as operand
        c.float_batch = true;
        rc = stage_batch_queries(ix, nullptr, nullptr, c.Q, 0, c.st, q);
        if (!rc) rc = stage_float_queries(ix, q, c.Q, c.st);   // the byte tables survivors are scored from
    } else {
        c.float_query = true;
        rc = stage_float_queries(ix, q, c.Q, c.st);
        ix->fq_binary = !rc && ix->mode == rbe::kModeScaled && ix->P >= 2 && ix->d_hints != nullptr;
        if (ix->fq_binary) rc = stage_float_approximations(ix, q, c.Q, c.st);
    }
    if (rc) return rc;
    return run_search(c, ids_out, scores_out);
}

int rbe_debug_scores_float(rbe_index* ix, const float* q, uint64_t first_item, uint64_t count, float* out,
                           void* hip_stream)
{
    ARG_CHECK(ix && q && out, "NULL argument");
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item, "item range outside the index");
    ARG_CHECK(count <= (1ull << 28), "count too large for a debug dump");
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = acquire_workspace(ix, 1, 1, search_capacity(ix, 1));
    if (rc) return rc;
    rc = stage_float_queries(ix, q, 1, st);
    if (rc) return rc;
    float* d_out = nullptr;
    HIP_TRY(hipMalloc(&d_out, (size_t)count * sizeof(float)));
    hipError_t e = launch_dense_scores_fq(ix->W, KernelSel{ix->P, 1, ix->mode, true}, ix->d_tiles, ix->layout,
                                          ix->ws.lut, first_item, count, d_out, st);
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, (size_t)count * sizeof(float), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_out);
    if (e != hipSuccess) { set_error("rbe_debug_scores_float: %s", hipGetErrorString(e)); return RBE_EHIP; }
    return RBE_OK;
}

int rbe_debug_query_mass(const uint64_t* q_planes, const float* q_scales, uint32_t q_n_planes, uint32_t dim,
                         uint32_t dyadic, float* mass_out)
{
    ARG_CHECK(q_planes && mass_out && (dyadic || q_scales), "NULL argument");
    ARG_CHECK(dim >= 64 && dim <= 256 && dim % 64 == 0 && dim != 192, "dim must be 64, 128 or 256");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes out of range");
    if (!dyadic)
        for (uint32_t i = 0; i < q_n_planes; ++i) ARG_CHECK(std::isfinite(q_scales[i]), "q_scales[%u] is not finite", i);
    query_mass(q_planes, dyadic ? nullptr : q_scales, q_n_planes, dim, dyadic != 0, mass_out);
    return RBE_OK;
}

int rbe_debug_issue_rate(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t n_queries,
                         uint32_t q_n_planes, uint32_t kernel, uint32_t repeat, float* ms_out, uint64_t* pairs_out,
                         void* hip_stream)
{
    ARG_CHECK(ms_out && pairs_out, "NULL output argument");
    ARG_CHECK(kernel <= 1, "kernel must be 0 (XOR/popcount batch scan) or 1 (matrix-core scan)");
    ARG_CHECK(repeat >= 1 && repeat <= 100000, "repeat must be 1..100000");
    SearchCtx c;
    int64_t ids_dummy = 0;
    float scores_dummy = 0.0f;
    int rc = search_prologue(ix, c, n_queries, 1, RBE_SELECT_EXACT, 0, &ids_dummy, &scores_dummy, hip_stream);
    if (rc) return rc;
    ARG_CHECK(q_planes != nullptr, "q_planes is NULL");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes must be 1..%u", RBE_MAX_PLANES);
    ARG_CHECK(n_queries >= 3, "the batch scans take 3 or more queries here");
    if (kernel == 1 && (!rbe::batch_mfma_supported(ix->W) || !can_prune(ix))) {
        set_error("no matrix-core scan for this index");
        return RBE_EUNSUPPORTED;
    }
    c.PQ = q_n_planes;
    rc = stage_queries(ix, q_planes, q_scales, c.Q, c.PQ, c.st);
    if (rc) return rc;
    c.batch_mfma = kernel == 1;
    if (c.batch_mfma) {
        rc = stage_batch_queries(ix, q_planes, q_scales, c.Q, c.PQ, c.st);
        if (rc) return rc;
    }
    c.calib_repeat = repeat;
    hipLaunchKernelGGL(rbe::init_state, dim3(1), dim3(64), 0, c.st, ix->ws.count, ix->ws.tau, ix->ws.kmax, ix->ws.status, c.Q);
    HIP_TRY(hipGetLastError());
    // thresholds no score reaches: the launch runs the scoring arithmetic and queues nothing
    hipLaunchKernelGGL(rbe::fill_u64, dim3(1), dim3(64), 0, c.st, ix->ws.tau, (uint32_t)c.Q, 0xFF800000FFFFFFFFull);   // the key of +infinity
    HIP_TRY(hipGetLastError());
    // one tile per workgroup of a full grid (fewer if the corpus is smaller), each gone over 1 + repeat times
    const uint32_t want = (uint32_t)ix->n_cu * 4u;
    const Round r{0u, std::min(ix->layout.n_tiles, want), 1u, 0u};
    const int saved_path = ix->batch_path, saved_prog = ix->progressive;
    ix->batch_path = kernel == 1 ? 2 : 1;
    ix->progressive = 0;            // the plain batch form of scan_exact (every plane of every pair)
    ix->stats = rbe_search_stats{};
    hipError_t e = hipEventRecord(ix->ev[0], c.st);
    if (e == hipSuccess) { rc = launch_scan_round(c, r, false, 0); }
    if (e == hipSuccess && !rc) e = hipEventRecord(ix->ev[1], c.st);
    if (e == hipSuccess && !rc) e = hipStreamSynchronize(c.st);
    ix->batch_path = saved_path; ix->progressive = saved_prog;
    if (rc) return rc;
    HIP_TRY(e);
    HIP_TRY(hipEventElapsedTime(ms_out, ix->ev[0], ix->ev[1]));
    *pairs_out = (uint64_t)(r.end - r.begin) * kTileItems * (1ull + repeat) * c.Q;
    return RBE_OK;
}

int rbe_debug_index_info(const rbe_index* ix, uint32_t* out)
{
    ARG_CHECK(ix != nullptr && out != nullptr, "NULL argument");
    out[0] = can_prune(ix) ? 1u : 0u;
    out[1] = ix->d_hints ? 1u : 0u;
    out[2] = ix->borrowed ? 1u : 0u;
    out[3] = ix->ext_ws ? 1u : 0u;
    return RBE_OK;
}

int rbe_debug_set_plan_split(rbe_index* ix, int mode)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ARG_CHECK(mode >= 0 && mode <= 2, "mode must be 0 (automatic), 1 (never) or 2 (always)");
    ix->plan_split = mode;
    if (mode == 0) ix->split1 = rbe_index::SplitState{};
    return RBE_OK;
}

int rbe_debug_set_progressive(rbe_index* ix, int enabled)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ix->progressive = (enabled == 2 || enabled == 3) ? enabled : (enabled ? 1 : 0);
    return RBE_OK;
}

int rbe_debug_set_nearlossless_path(rbe_index* ix, int path)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ARG_CHECK(path == 0 || path == 1, "path must be 0 (exact scans + selection by groups) or 1 (per-thread-queue scan)");
    ix->nl_path = path;
    return RBE_OK;
}

int rbe_debug_set_batch_path(rbe_index* ix, int path)
{
    ARG_CHECK(ix != nullptr, "index is NULL");
    ARG_CHECK(path >= 0 && path <= 3, "path must be 0 (auto), 1 (XOR/popcount), 2 (matrix cores) or 3 (matrix cores, half operands)");
    ix->batch_path = path;
    return RBE_OK;
}

int rbe_debug_popcounts(rbe_index* ix, const uint64_t* q_planes, uint32_t q_n_planes, uint64_t first_item,
                        uint64_t count, int32_t* out, void* hip_stream)
{
    ARG_CHECK(ix && q_planes && out, "NULL argument");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes must be 1..%u", RBE_MAX_PLANES);
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item, "item range outside the index");
    ARG_CHECK(count <= (1ull << 26), "count too large for a debug dump");
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    uint64_t* d_q = nullptr;
    int32_t* d_out = nullptr;
    const size_t qbytes = (size_t)q_n_planes * ix->W * sizeof(uint64_t);
    const size_t obytes = (size_t)count * ix->P * q_n_planes * sizeof(int32_t);
    HIP_TRY(hipMalloc(&d_q, qbytes));
    hipError_t e = hipMalloc(&d_out, obytes);
    if (e == hipSuccess) e = hipMemcpyAsync(d_q, q_planes, qbytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(rbe::dense_popcounts, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st,
                           ix->d_tiles, ix->layout, ix->geom, d_q, q_n_planes, first_item, count, d_out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, obytes, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_q);
    (void)hipFree(d_out);
    if (e != hipSuccess) { set_error("rbe_debug_popcounts: %s", hipGetErrorString(e)); return RBE_EHIP; }
    return RBE_OK;
}

int rbe_debug_scores(rbe_index* ix, const uint64_t* q_planes, const float* q_scales, uint32_t q_n_planes,
                     uint64_t first_item, uint64_t count, float* out, void* hip_stream)
{
    ARG_CHECK(ix && q_planes && out, "NULL argument");
    ARG_CHECK(q_n_planes >= 1 && q_n_planes <= RBE_MAX_PLANES, "q_n_planes must be 1..%u", RBE_MAX_PLANES);
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item, "item range outside the index");
    ARG_CHECK(count <= (1ull << 28), "count too large for a debug dump");
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = acquire_workspace(ix, 1, 1, search_capacity(ix, 1));
    if (rc) return rc;
    rc = stage_queries(ix, q_planes, q_scales, 1, q_n_planes, st);
    if (rc) return rc;
    float* d_out = nullptr;
    HIP_TRY(hipMalloc(&d_out, (size_t)count * sizeof(float)));
    hipError_t e = launch_dense_scores(ix->W, KernelSel{ix->P, q_n_planes, ix->mode, true}, ix->d_tiles, ix->layout,
                                       ix->ws.qwords, ix->ws.qcoef, first_item, count, d_out, st);
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, (size_t)count * sizeof(float), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_out);
    if (e != hipSuccess) { set_error("rbe_debug_scores: %s", hipGetErrorString(e)); return RBE_EHIP; }
    return RBE_OK;
}

int rbe_debug_read_scales(rbe_index* ix, uint64_t first_item, uint64_t count, float* out, void* hip_stream)
{
    ARG_CHECK(ix && out, "NULL argument");
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item, "item range outside the index");
    ARG_CHECK(count <= (1ull << 28), "count too large for a debug dump");
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    float* d_out = nullptr;
    const size_t bytes = (size_t)ix->P * count * sizeof(float);
    HIP_TRY(hipMalloc(&d_out, bytes));
    hipLaunchKernelGGL(rbe::gather_scales, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st, ix->d_tiles,
                       ix->layout, ix->geom, first_item, count, d_out);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, bytes, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_out);
    if (e != hipSuccess) { set_error("rbe_debug_read_scales: %s", hipGetErrorString(e)); return RBE_EHIP; }
    return RBE_OK;
}

int rbe_debug_read_planes(rbe_index* ix, uint64_t first_item, uint64_t count, uint64_t* out, void* hip_stream)
{
    ARG_CHECK(ix && out, "NULL argument");
    ARG_CHECK(first_item <= ix->n_items && count <= ix->n_items - first_item, "item range outside the index");
    ARG_CHECK(count <= (1ull << 26), "count too large for a debug dump");
    if (count == 0) return RBE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    uint64_t* d_out = nullptr;
    const size_t bytes = (size_t)ix->P * count * ix->W * sizeof(uint64_t);
    HIP_TRY(hipMalloc(&d_out, bytes));
    hipLaunchKernelGGL(rbe::gather_planes, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st, ix->d_tiles,
                       ix->layout, ix->geom, first_item, count, d_out);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, bytes, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_out);
    if (e != hipSuccess) { set_error("rbe_debug_read_planes: %s", hipGetErrorString(e)); return RBE_EHIP; }
    return RBE_OK;
}

int rbe_debug_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream)
{
    ARG_CHECK(dst_dev && src_dev, "NULL argument");
    ARG_CHECK(bytes % 16 == 0 && ((uintptr_t)dst_dev % 16) == 0 && ((uintptr_t)src_dev % 16) == 0,
              "size and pointers must be multiples of 16 bytes");
    if (bytes == 0) return RBE_OK;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    const size_t n_vec = bytes / 16;
    const uint32_t grid = (uint32_t)std::min<size_t>((n_vec + 255) / 256, (size_t)prop.multiProcessorCount * 8);
    hipLaunchKernelGGL(rbe::calib_copy, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream,
                       (const rbe::u32x4*)src_dev, (rbe::u32x4*)dst_dev, n_vec);
    HIP_TRY(hipGetLastError());
    return RBE_OK;
}

int rbe_debug_read(const void* src_dev, size_t bytes, void* sink_dev, size_t sink_bytes, void* hip_stream)
{
    ARG_CHECK(src_dev && sink_dev, "NULL argument");
    ARG_CHECK(bytes % 16 == 0 && ((uintptr_t)src_dev % 16) == 0 && ((uintptr_t)sink_dev % 16) == 0,
              "size and pointers must be multiples of 16 bytes");
    if (bytes == 0) return RBE_OK;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    const size_t n_vec = bytes / 16;
    const uint32_t grid = (uint32_t)std::min<size_t>((n_vec + 2047) / 2048, (size_t)prop.multiProcessorCount * 3);
    ARG_CHECK(sink_bytes >= (size_t)grid * 256 * 16, "sink must hold %zu bytes", (size_t)grid * 256 * 16);
    hipLaunchKernelGGL(rbe::calib_read, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream,
                       (const rbe::u32x4*)src_dev, n_vec, (rbe::u32x4*)sink_dev);
    HIP_TRY(hipGetLastError());
    return RBE_OK;
}

}  // extern "C"
