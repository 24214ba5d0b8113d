// Device code of the RBE retrieval library for gfx950 (MI355X).
//
// Kernels:
//   scan_exact<W,P,PQ,SINGLE>  streaming exhaustive match (Eq. 14 by XOR/popcount,
//                              Sec. 5.1) fused with threshold pruning: an item whose
//                              (score, id) key reaches the query's proven lower bound
//                              is appended to the query's candidate list.
//   select_topk                per query: k-th largest candidate key by radix
//                              descent, compaction of the k best to the front of the
//                              list, bitonic sort, new threshold (the per-GPU global
//                              selection of Sec. 5 / Sec. 6).
//   dense_popcounts / dense_scores / fold_cosine / init_state   small helpers.
//
// Wavefronts are 64 wide.  One wave reads a "row" of 256 consecutive items per
// step: every plane with 16-byte loads per lane (1 KiB contiguous per wave
// instruction), every scale array with the matching 8- or 4-byte loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rbe {

constexpr int kBlock = 256;             // threads per workgroup of the scan
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kRow = 256;               // items one wave handles per step
constexpr int kTile = kRow * kWavesPerBlock;  // items one workgroup handles per step
constexpr int kItemsPerLane = 4;

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

template <int W, int P>
__device__ __forceinline__ void load_row(RowRegs<W, P>& r, const uint64_t* __restrict__ planes,
                                         const float* __restrict__ scales, size_t plane_stride,
                                         size_t row_base, int lane)
{
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint64_t* pj = planes + (size_t)j * plane_stride * W;
        const float* sj = scales + (size_t)j * plane_stride;
        if (W == 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const size_t it = row_base + s * 128 + 2 * lane;
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + it));
                r.w[j][2 * s][0] = v.x; r.w[j][2 * s][1] = v.y;
                r.w[j][2 * s + 1][0] = v.z; r.w[j][2 * s + 1][1] = v.w;
                const f32x2 a = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sj + it));
                r.a[j][2 * s] = a.x; r.a[j][2 * s + 1] = a.y;
            }
        } else {
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                const size_t it = row_base + m * 64 + lane;
#pragma unroll
                for (int h = 0; h < W / 2; ++h) {
                    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pj + it * W) + h);
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

// Wave-cooperative append of the lanes with ok == true: one atomic per wave.
// Must be reached by all lanes of the wave.
__device__ __forceinline__ void append_keys(bool ok, uint64_t key, uint64_t* __restrict__ cand_q,
                                            uint32_t* __restrict__ count_q, uint32_t cap, int lane)
{
    const uint64_t mask = __ballot(ok);
    if (mask == 0) return;
    const int leader = __ffsll((long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(count_q, (uint32_t)__popcll(mask));
    base = __shfl(base, leader);
    if (ok) {
        const uint32_t pos = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        if (pos < cap) cand_q[pos] = key;  // the count keeps running so that overflow is seen
    }
}

// Map the v-th unit that is NOT a multiple of `skip` to its unit number
// (skip == 0: identity).  Units that are multiples of `skip` were scanned by
// the previous, coarser level.
__device__ __forceinline__ uint32_t unit_of(uint32_t v, uint32_t skip)
{
    if (skip == 0) return v;
    return (v / (skip - 1)) * skip + (v % (skip - 1)) + 1;
}

struct ScanArgs {
    const uint64_t* planes;   // [P][plane_stride][W]
    const float* scales;      // [P][plane_stride]
    size_t plane_stride;      // items per plane array (multiple of kTile)
    uint64_t n_items;
    const uint32_t* qwords;   // [Q][PQ][2W]
    const float* qcoef;       // [Q][PQ+1]
    uint32_t n_queries;
    const uint64_t* tau;      // [Q] threshold keys
    uint64_t* cand;           // [Q][cap]
    uint32_t* count;          // [Q]
    uint32_t cap;
    uint32_t v_begin, v_end;  // range of valid-unit indices this launch covers
    uint32_t stride;          // tile = unit * stride
    uint32_t skip;            // see unit_of
};

// Streaming exhaustive match + threshold pruning.  Persistent workgroups:
// workgroup b takes valid units b, b + grid, ...; the next tile's loads are
// issued before the current tile is scored.
template <int W, int P, int PQ, bool SINGLE>
__global__ __launch_bounds__(kBlock) void scan_exact(const ScanArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const uint32_t G = gridDim.x;
    uint32_t v = a.v_begin + blockIdx.x;
    if (v >= a.v_end) return;

    QueryRegs<W, PQ> q0;
    uint64_t tau0 = 0;
    float taus0 = 0.f;
    if (SINGLE) {
        q0 = load_query<W, PQ>(a.qwords, a.qcoef, 0);
        tau0 = a.tau[0];
        taus0 = threshold_score(tau0);
    }

    RowRegs<W, P> cur, nxt;
    size_t row = ((size_t)unit_of(v, a.skip) * a.stride) * kTile + (size_t)wave * kRow;
    load_row<W, P>(cur, a.planes, a.scales, a.plane_stride, row, lane);

    for (;;) {
        const uint32_t vn = v + G;
        const bool has_next = vn < a.v_end;
        size_t row_n = 0;
        if (has_next) {
            row_n = ((size_t)unit_of(vn, a.skip) * a.stride) * kTile + (size_t)wave * kRow;
            load_row<W, P>(nxt, a.planes, a.scales, a.plane_stride, row_n, lane);
        }

        const uint32_t nq = SINGLE ? 1u : a.n_queries;
        for (uint32_t q = 0; q < nq; ++q) {
            QueryRegs<W, PQ> qr;
            uint64_t tau;
            float taus;
            if (SINGLE) { qr = q0; tau = tau0; taus = taus0; }
            else {
                qr = load_query<W, PQ>(a.qwords, a.qcoef, q);
                tau = a.tau[q];
                taus = threshold_score(tau);
            }
            float s[kItemsPerLane];
            bool any = false;
#pragma unroll
            for (int m = 0; m < kItemsPerLane; ++m) {
                s[m] = score_item<W, P, PQ>(cur, m, qr);
                any |= (s[m] >= taus);
            }
            if (__ballot(any)) {   // rare: at least one lane of the wave has a survivor
#pragma unroll
                for (int m = 0; m < kItemsPerLane; ++m) {
                    const uint64_t id = row + lane_item<W>(lane, m);
                    bool ok = (s[m] >= taus) && (id < a.n_items);
                    uint64_t key = 0;
                    if (ok) { key = make_key(s[m], (uint32_t)id); ok = key >= tau; }
                    append_keys(ok, key, a.cand + (size_t)q * a.cap, a.count + q, a.cap, lane);
                }
            }
        }

        if (!has_next) break;
        cur = nxt;
        row = row_n;
        v = vn;
    }
}

// ---------------------------------------------------------------- selection
constexpr int kSelBlock = 1024;
constexpr int kSelMaxK = 4096;

enum : uint32_t { kStatusOverflow = 1u };

struct SelectArgs {
    uint64_t* cand;      // [Q][cap], in/out: on return the best min(n,k) keys, sorted, at the front
    uint32_t* count;     // [Q] in: appended so far; out: number kept
    uint64_t* tau;       // [Q] out: k-th best key if at least k candidates, else unchanged... see kernel
    uint32_t cap;
    uint32_t k;
    uint32_t* status;    // bit 0 set if any query's count exceeded cap
    uint32_t* count_seen;  // [Q] out: candidate count before selection (for statistics)
    int final_pass;
    int64_t* ids_out;    // [Q][k]   (final pass)
    float* scores_out;   // [Q][k]
};

// One workgroup per query.
__global__ __launch_bounds__(kSelBlock) void select_topk(const SelectArgs a)
{
    __shared__ uint64_t skeys[kSelMaxK];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_digit, s_remaining, s_fill;

    const uint32_t q = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    uint64_t* keys = a.cand + (size_t)q * a.cap;
    const uint32_t appended = a.count[q];
    const uint32_t n = appended < a.cap ? appended : a.cap;
    if (tid == 0) {
        a.count_seen[q] = appended;
        if (appended > a.cap) atomicOr(a.status, kStatusOverflow);
    }
    const uint32_t k = a.k;

    uint64_t kth = 0;  // keys >= kth are kept
    if (n > k) {
        uint64_t prefix = 0, mask = 0;
        uint32_t remaining = k;
        for (int shift = 56; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (uint32_t i = tid; i < n; i += kSelBlock) {
                const uint64_t key = keys[i];
                if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid < 64) {
                // lane l owns digits 255-4l .. 252-4l (descending); find where the running
                // count from the top reaches `remaining`
                const int top = 255 - 4 * (int)tid;
                const uint32_t c0 = hist[top], c1 = hist[top - 1], c2 = hist[top - 2], c3 = hist[top - 3];
                const uint32_t mine = c0 + c1 + c2 + c3;
                uint32_t incl = mine;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const uint32_t o = __shfl_up(incl, d);
                    if ((int)tid >= d) incl += o;
                }
                const uint32_t before = incl - mine;   // keys with larger digits than this lane's
                if (before < remaining && incl >= remaining) {
                    uint32_t acc = before;
                    int dsel = top;
                    if (acc + c0 >= remaining) dsel = top;
                    else { acc += c0;
                        if (acc + c1 >= remaining) dsel = top - 1;
                        else { acc += c1;
                            if (acc + c2 >= remaining) dsel = top - 2;
                            else { acc += c2; dsel = top - 3; } } }
                    s_digit = (uint32_t)dsel;
                    s_remaining = remaining - acc;
                }
            }
            __syncthreads();
            prefix |= (uint64_t)s_digit << shift;
            mask |= (uint64_t)0xFFu << shift;
            remaining = s_remaining;
            __syncthreads();
        }
        kth = prefix;
    }

    // gather the kept keys into LDS (keys are distinct, so exactly min(n,k) qualify)
    const uint32_t m = n < k ? n : k;
    uint32_t pow2 = 1;
    while (pow2 < m) pow2 <<= 1;
    if (tid == 0) s_fill = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += kSelBlock) {
        const uint64_t key = keys[i];
        if (key >= kth) {
            const uint32_t pos = atomicAdd(&s_fill, 1u);
            if (pos < (uint32_t)kSelMaxK) skeys[pos] = key;
        }
    }
    __syncthreads();
    for (uint32_t i = m + tid; i < pow2; i += kSelBlock) skeys[i] = 0;
    __syncthreads();

    // bitonic sort, descending
    for (uint32_t size = 2; size <= pow2; size <<= 1) {
        for (uint32_t st = size >> 1; st > 0; st >>= 1) {
            for (uint32_t i = tid; i < pow2 / 2; i += kSelBlock) {
                const uint32_t lo = 2 * i - (i & (st - 1));
                const uint32_t hi = lo + st;
                const bool desc = ((lo & size) == 0);
                const uint64_t x = skeys[lo], y = skeys[hi];
                if ((x < y) == desc) { skeys[lo] = y; skeys[hi] = x; }
            }
            __syncthreads();
        }
    }

    for (uint32_t i = tid; i < m; i += kSelBlock) keys[i] = skeys[i];
    if (tid == 0) {
        a.count[q] = m;
        if (n >= k && m > 0) a.tau[q] = skeys[m - 1];   // k-th best of everything seen so far
    }
    if (a.final_pass) {
        for (uint32_t i = tid; i < k; i += kSelBlock) {
            int64_t id = -1;
            float sc = -__builtin_inff();
            if (i < m) {
                const uint64_t key = skeys[i];
                id = (int64_t)(uint32_t)(~(uint32_t)key);
                sc = ordered_to_score((uint32_t)(key >> 32));
            }
            a.ids_out[(size_t)q * k + i] = id;
            a.scores_out[(size_t)q * k + i] = sc;
        }
    }
}

__global__ void init_state(uint32_t* count, uint64_t* tau, uint32_t* status, uint32_t n_queries)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_queries) { count[i] = 0; tau[i] = 0; }
    if (i == 0) *status = 0;
}

// ---------------------------------------------------------------- dense helpers (tests, cosine fold)
__global__ void dense_popcounts(const uint64_t* __restrict__ planes, size_t plane_stride, uint32_t W, uint32_t P,
                                const uint64_t* __restrict__ qplanes, uint32_t PQ,
                                uint64_t first, uint64_t count, int32_t* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    for (uint32_t j = 0; j < P; ++j)
        for (uint32_t i = 0; i < PQ; ++i) {
            int32_t pc = 0;
            for (uint32_t w = 0; w < W; ++w)
                pc += __popcll(planes[((size_t)j * plane_stride + z) * W + w] ^ qplanes[i * W + w]);
            out[(t * P + j) * PQ + i] = pc;
        }
}

template <int W, int P, int PQ>
__global__ void dense_scores(const uint64_t* __restrict__ planes, const float* __restrict__ scales,
                             size_t plane_stride, const uint32_t* __restrict__ qwords,
                             const float* __restrict__ qcoef, uint64_t first, uint64_t count,
                             float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const QueryRegs<W, PQ> q = load_query<W, PQ>(qwords, qcoef, 0);
    RowRegs<W, P> r;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const uint32_t* pw = reinterpret_cast<const uint32_t*>(planes + ((size_t)j * plane_stride + z) * W);
#pragma unroll
        for (int h = 0; h < 2 * W; ++h) r.w[j][0][h] = pw[h];
        r.a[j][0] = scales[(size_t)j * plane_stride + z];
    }
    out[t] = score_item<W, P, PQ>(r, 0, q);
}

// Divide each item's scales by the norm of its reconstructed vector:
// ||sum_j a_j b_j||^2 = dim * sum_j a_j^2 + 2 sum_{j<j'} a_j a_j' (dim - 2 popcount(K_j ^ K_j')).
__global__ void fold_cosine(const uint64_t* __restrict__ planes, float* __restrict__ scales,
                            size_t plane_stride, uint32_t W, uint32_t P, uint64_t n_items)
{
    const uint64_t z = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (z >= n_items) return;
    const double dim = 64.0 * W;
    double a[4];
    for (uint32_t j = 0; j < P; ++j) a[j] = (double)scales[(size_t)j * plane_stride + z];
    double n2 = 0.0;
    for (uint32_t j = 0; j < P; ++j) {
        n2 += dim * a[j] * a[j];
        for (uint32_t jj = j + 1; jj < P; ++jj) {
            int pc = 0;
            for (uint32_t w = 0; w < W; ++w)
                pc += __popcll(planes[((size_t)j * plane_stride + z) * W + w] ^
                               planes[((size_t)jj * plane_stride + z) * W + w]);
            n2 += 2.0 * a[j] * a[jj] * (dim - 2.0 * pc);
        }
    }
    if (n2 > 0.0) {
        const double nrm = sqrt(n2);
        for (uint32_t j = 0; j < P; ++j) scales[(size_t)j * plane_stride + z] = (float)(a[j] / nrm);
    }
}

}  // namespace rbe
