// Small kernels of the RBE retrieval library: global selection, state reset, load
// scatter, cosine fold, calibration copy and dense test dumps.
#pragma once
#include "rbe_kernels.hpp"

namespace rbe {

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
    uint64_t* tau;       // [Q] in: threshold the candidates were collected with; out: k-th best key once at
                         //     least k candidates exist
    const uint64_t* kmax;  // [Q] largest key ever appended
    uint32_t cap;
    uint32_t k;
    uint32_t* status;    // bit 0 set if any query's count exceeded cap
    uint32_t* count_seen;  // [Q] out: candidate count before selection (for statistics)
    int final_pass;
    int64_t* ids_out;    // [Q][k]   (final pass; sorted)
    float* scores_out;   // [Q][k]
    uint32_t* group_aux; // near-lossless modes: [Q][4], [0] = entries group_best_compact left in the list (read in place of
                         // `count` and zeroed here); null otherwise
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
// Pair index i of a stage is owned by thread i % 1024, so while the stride is at most
// 64 every wave works inside its own 128-key blocks and only needs to order its own LDS
// traffic; workgroup barriers are needed around the stages with stride >= 128 only.
__device__ __forceinline__ void bitonic_desc(uint64_t* keys, uint32_t pow2)
{
    bool prev_wide = true;   // data written by other threads before the call
    for (uint32_t size = 2; size <= pow2; size <<= 1) {
        for (uint32_t st = size >> 1; st > 0; st >>= 1) {
            const bool wide = st >= 128;
            if (wide || prev_wide) __syncthreads();
            else { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); }
            for (uint32_t i = threadIdx.x; i < pow2 / 2; i += kSelBlock) {
                const uint32_t lo = 2 * i - (i & (st - 1));
                const uint32_t hi = lo + st;
                const bool desc = ((lo & size) == 0);
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
            prev_wide = wide;
        }
    }
    __syncthreads();
}

// One workgroup per query.
__global__ __launch_bounds__(kSelBlock) void select_topk(const SelectArgs a)
{
    __shared__ uint64_t skeys[kSelMaxK];    // keys known to be kept
    __shared__ uint64_t sbound[kSelBound];  // keys of the boundary bin
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t s_wave[16];
    __shared__ uint32_t s_digit, s_remaining, s_binpop, s_fill_keep, s_fill_bound;

    const uint32_t q = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    uint64_t* keys = a.cand + (size_t)q * a.cap;
    const uint32_t appended = a.group_aux ? a.group_aux[q * 4] : a.count[q * kCountStride];
    const uint32_t n = appended < a.cap ? appended : a.cap;
    const uint32_t k = a.k;
    if (a.group_aux) {
        __syncthreads();                          // every thread has read the counter
        if (tid == 0) { a.group_aux[q * 4] = 0; a.count[q * kCountStride] = n; }
    }
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
        // ---- every key lies in [threshold used by the scan, largest key appended]: the bits
        //      these two have in common are common to all keys and need no radix round
        const uint64_t lo_key = a.tau[q], hi_key = a.kmax[q * kKmaxStride];
        const uint64_t diff = lo_key ^ hi_key;
        int pos = diff ? 64 - __clzll((long long)diff) : 0;   // low `pos` bits are undetermined
        uint64_t mask = pos >= 64 ? 0ull : ~((1ull << pos) - 1ull);
        uint64_t prefix = hi_key & mask;
        __syncthreads();                           // everyone has read tau before it is rewritten below
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
        if (tid == 0) a.count[q * kCountStride] = m;
        return;
    }

    // ---- final round: sort the kept keys and emit ids and scores
    uint32_t pow2 = 1;
    while (pow2 < m) pow2 <<= 1;
    for (uint32_t i = m + tid; i < pow2; i += kSelBlock) skeys[i] = 0;
    __syncthreads();
    bitonic_desc(skeys, pow2);
    if (tid == 0) a.count[q * kCountStride] = m;
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

// ---------------------------------------------------------------- near-lossless selection by groups
// Algorithm 1 (Sec. 6.2) forwards, from every group of ids g(z) = (z div (256 I)) * 256 + (z mod 256), only the
// best QL items (QL = 1 in the paper) and returns the best k of what was forwarded.  An item below a lower bound
// tau of the k-th best forwarded item can be neither in the result nor change what another group forwards, so the
// candidates of the exact scans (every item >= tau) hold everything that matters, and the selector reduces to:
// keep the best QL candidates of every group, then select as usual.  Two kernels do the first part on the
// candidate list of each query, in place:
//   group_best_build    every candidate goes into an open-addressing table keyed by its group (the group follows
//                       from the id inside the key); a slot keeps the largest and second largest key of its group
//   group_best_compact  the table's entries become the new candidate list (its length goes to select_topk through a
//                       counter); slots are zeroed on the way, so the table is clean for the next level
// Keys are distinct and ordered by (score desc, id asc), so "largest key" is the group's best item with the lowest
// id among equal scores, as the per-thread queue of Algorithm 1 keeps it.
struct GroupBestArgs {
    uint64_t* cand;        // [Q][cap]
    uint32_t* count;       // [Q] x kCountStride: in: appended so far; out: entries after the reduction
    uint32_t cap;
    uint64_t* table;       // [Q][slots][2]: best, second best key of the group that owns the slot (0 = empty)
    uint32_t slots;        // power of two, at least 2 x cap
    uint32_t* aux;         // [Q][4]: [0] entries written by group_best_compact (select_topk takes the count from there)
    uint32_t group_span;   // 256 x I
    uint32_t qlen;         // 1 or 2
    uint32_t* status;      // bit 0 set if a query's count exceeded cap
};

__device__ __forceinline__ uint32_t key_group(uint64_t key, uint32_t span)
{
    const uint32_t id = ~(uint32_t)key;
    return (id / span) * 256u + (id & 255u);
}

// Slots of the table that a level with n candidates uses: the least power of two that is at least 2 n (and 1024),
// never more than the table has.  The table is empty between levels, so any prefix of it serves; both kernels
// derive the same number from the candidate count, and the second then has only that prefix to go through
// (k = 4000, 8 queries: 2^21 slots per query, of which a level with 30 000 candidates needs 2^16).
__device__ __forceinline__ uint32_t group_slots_in_use(uint32_t n, uint32_t slots)
{
    uint32_t e = 1024u;
    while (e < slots && e < 2u * n) e <<= 1;
    return e < slots ? e : slots;
}

__global__ __launch_bounds__(256) void group_best_build(const GroupBestArgs a)
{
    const uint32_t q = blockIdx.y;
    const uint32_t appended = a.count[q * kCountStride];
    const uint32_t n = appended < a.cap ? appended : a.cap;
    if (blockIdx.x == 0 && threadIdx.x == 0 && appended > a.cap) atomicOr(a.status, kStatusOverflow);
    const uint64_t* keys = a.cand + (size_t)q * a.cap;
    unsigned long long* tbl = reinterpret_cast<unsigned long long*>(a.table + (size_t)q * a.slots * 2);
    const uint32_t in_use = group_slots_in_use(n, a.slots);
    const uint32_t mask = in_use - 1u;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const unsigned long long key = keys[i];
        const uint32_t g = key_group(key, a.group_span);
        uint32_t slot = (g * 2654435761u) >> 7 & mask;
        // at most `in_use` probes: the part in use has twice as many slots as there are candidates
        for (uint32_t probe = 0; probe < in_use; ++probe, slot = (slot + 1u) & mask) {
            unsigned long long cur = *reinterpret_cast<volatile unsigned long long*>(&tbl[2 * (size_t)slot]);
            if (cur == 0ull) {
                cur = atomicCAS(&tbl[2 * (size_t)slot], 0ull, key);
                if (cur == 0ull) break;                                   // claimed the slot for this group
            }
            if (key_group(cur, a.group_span) != g) continue;              // another group's slot (it never changes hands)
            const unsigned long long old = atomicMax(&tbl[2 * (size_t)slot], key);
            // every key of the group except its largest is offered to the second place exactly once: here when it
            // loses on arrival, or when a later key displaces it
            if (a.qlen == 2) atomicMax(&tbl[2 * (size_t)slot + 1], old < key ? old : key);
            break;
        }
    }
}

__global__ __launch_bounds__(256) void group_best_compact(const GroupBestArgs a)
{
    constexpr int kPer = 8;                      // slots per thread and step: 2048 per workgroup
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_start;
    const uint32_t q = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t* keys = a.cand + (size_t)q * a.cap;
    uint64_t* tbl = a.table + (size_t)q * a.slots * 2;
    uint32_t* aux = a.aux + q * 4;
    const uint32_t appended = a.count[q * kCountStride];
    const uint32_t in_use = group_slots_in_use(appended < a.cap ? appended : a.cap, a.slots);     // (as group_best_build)
    // one returning atomic per 2048 slots: with one per wave, the 8192 atomics on this one counter were the
    // kernel's whole run time
    for (uint32_t base = blockIdx.x * (256u * kPer); base < in_use; base += gridDim.x * (256u * kPer)) {
        uint64_t k0[kPer], k1[kPer];
        uint32_t mine = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const uint32_t slot = base + (uint32_t)i * 256u + threadIdx.x;
            k0[i] = 0; k1[i] = 0;
            if (slot < in_use) {
                k0[i] = tbl[2 * (size_t)slot];
                if (k0[i]) {
                    tbl[2 * (size_t)slot] = 0;
                    if (a.qlen == 2) { k1[i] = tbl[2 * (size_t)slot + 1]; tbl[2 * (size_t)slot + 1] = 0; }
                }
            }
            mine += (k0[i] ? 1u : 0u) + (k1[i] ? 1u : 0u);
        }
        uint32_t incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d);
            if (lane >= d) incl += o;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) { before += w < wave ? s_wave[w] : 0u; total += s_wave[w]; }
        if (threadIdx.x == 0) s_start = total ? atomicAdd(&aux[0], total) : 0u;
        __syncthreads();
        uint32_t pos = s_start + before + incl - mine;      // never beyond cap: at most one entry per candidate read
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (k0[i]) keys[pos++] = k0[i];
            if (k1[i]) keys[pos++] = k1[i];
        }
        __syncthreads();                                    // s_wave and s_start are reused by the next step
    }
    // (no hand-off inside the kernel: a device-wide fence per workgroup costs a write-back of the whole L2 on this
    // chip; the selection that follows reads aux[0] as the new count and zeroes it)
}

__global__ void fill_u64(uint64_t* __restrict__ dst, uint32_t n, uint64_t value)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

// Zeroes `n` 16-byte units (the group tables and their counters at the start of a search).
__global__ __launch_bounds__(256) void fill_zero16(u32x4* __restrict__ dst, size_t n)
{
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = z;
}

__global__ void init_state(uint32_t* count, uint64_t* tau, uint64_t* kmax, uint32_t* status, uint32_t n_queries)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_queries) { count[i * kCountStride] = 0; tau[i] = 0; kmax[i * kKmaxStride] = 0; }
    if (i < 16) status[i] = 0;    // flags; rows read in full by the progressive scan, per level
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
    }
    if (g.S == g.P)   // general mode: one scale per plane.  Dyadic modes take no scales from the caller.
        for (uint32_t j = 0; j < g.P; ++j)
            reinterpret_cast<float*>(tile + g.scales_offset())[j * kTileItems + o] = scales[(size_t)j * count + t];
}

// Stand-in encoder on the device (greedy residual sign binarisation, see rbe.h):
// x [count][dim] fp32 -> planes and per-plane scales written straight into the tiles.
// One thread encodes one item with the same sequential arithmetic as the host
// encoder (absolute values summed in double in dimension order), so both produce
// the same bits.  A workgroup first stages its 256 / W items in LDS with coalesced
// loads; rows are padded by one float against bank conflicts.
template <int W>
__global__ __launch_bounds__(256) void encode_chunk(char* __restrict__ tiles, const Layout l, const TileGeom g,
                                                    const float* __restrict__ x, uint64_t first, uint64_t count)
{
    constexpr int D = 64 * W;
    constexpr int IB = 256 / W;           // items per workgroup
    __shared__ float sx[IB][D + 1];
    const uint64_t t0 = (uint64_t)blockIdx.x * IB;
    const uint32_t n_here = (uint32_t)(count - t0 < (uint64_t)IB ? count - t0 : (uint64_t)IB);
    for (uint32_t e = threadIdx.x; e < n_here * D; e += 256) sx[e / D][e % D] = x[t0 * D + e];
    __syncthreads();
    if (threadIdx.x >= n_here) return;
    float* r = sx[threadIdx.x];
    const uint64_t z = first + t0 + threadIdx.x;
    char* tile = item_tile(tiles, l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    for (uint32_t p = 0; p < g.P; ++p) {
        double acc = 0.0;
        for (int i = 0; i < D; ++i) acc += fabs((double)r[i]);
        const float scale = (float)(acc / (double)D);
        uint64_t* dst = reinterpret_cast<uint64_t*>(tile + p * g.plane_bytes()) + (size_t)o * W;
        for (int w = 0; w < W; ++w) {
            uint64_t word = 0;
            for (int b = 0; b < 64; ++b) {
                const float v = r[w * 64 + b];
                const bool positive = v > 0.0f;
                word |= (uint64_t)positive << b;
                r[w * 64 + b] = (float)((double)v - (positive ? (double)scale : -(double)scale));
            }
            dst[w] = word;
        }
        reinterpret_cast<float*>(tile + g.scales_offset())[p * kTileItems + o] = scale;
    }
}

// out[j][t][w] = plane words of item first + t (test hook)
__global__ void gather_planes(const char* __restrict__ tiles, const Layout l, const TileGeom g,
                              uint64_t first, uint64_t count, uint64_t* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const char* tile = item_tile(const_cast<char*>(tiles), l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    for (uint32_t j = 0; j < g.P; ++j)
        for (uint32_t w = 0; w < g.W; ++w)
            out[((size_t)j * count + t) * g.W + w] =
                reinterpret_cast<const uint64_t*>(tile + j * g.plane_bytes())[(size_t)o * g.W + w];
}

// ---------------------------------------------------------------- calibration
// Plain 16-byte-per-lane copy of a known size: the yardstick that hardware
// counter readings of the scan are scaled by.
__global__ __launch_bounds__(256) void calib_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

// Read-only counterpart: a persistent grid in which every workgroup streams contiguous 32 KiB
// chunks (eight 16-byte non-temporal loads in flight per lane, the access shape of the scan) and
// folds them into one value per lane, stored once at the end.  What this reaches is the practical
// ceiling for a kernel that only reads.
__global__ __launch_bounds__(256) void calib_read(const u32x4* __restrict__ src, size_t n_vec, u32x4* __restrict__ sink)
{
    constexpr int kUnroll = 8;
    const size_t per_iter = (size_t)kUnroll * 256;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t base = (size_t)blockIdx.x * per_iter;
    for (; base + per_iter <= n_vec; base += (size_t)gridDim.x * per_iter) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + base + u * 256 + threadIdx.x);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    for (size_t i = base + threadIdx.x; i < n_vec && base < n_vec; i += 256) {   // the one ragged chunk at the end
        if (i >= base + per_iter) break;
        const u32x4 a = __builtin_nontemporal_load(src + i);
        acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
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

// out[j][t] = effective scale of plane j of item first + t
__global__ void gather_scales(const char* __restrict__ tiles, const Layout l, const TileGeom g,
                              uint64_t first, uint64_t count, float* __restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const uint64_t z = first + t;
    const char* tile = item_tile(const_cast<char*>(tiles), l, g, z);
    const uint32_t o = (uint32_t)(z % kTileItems);
    const float* sc = reinterpret_cast<const float*>(tile + g.scales_offset());
    for (uint32_t j = 0; j < g.P; ++j) {
        float v;
        if (g.S == g.P) v = sc[j * kTileItems + o];
        else v = (g.S == 1 ? sc[o] : 1.0f) / (float)(1u << j);   // dyadic: 2^-j times the item's scale
        out[(size_t)j * count + t] = v;
    }
}

// Cosine fold.  With a_j the plane weights of an item (its stored scales, or 2^-j in
// the dyadic mode), ||sum_j a_j b_j||^2 = dim * sum_j a_j^2 + 2 sum_{j<j'} a_j a_j' (dim - 2 popcount(K_j ^ K_j')).
// General mode: every scale of the item is divided by that norm.  Dyadic mode with one
// scale array: the inverse norm is stored there (the keyword magnitude that Sec. 5.1
// precomputes and keeps with the embedding).  One thread per physical slot; in the
// general mode slots never loaded have scale 0 and are left alone.
__global__ void fold_cosine(char* __restrict__ tiles, const TileGeom g, uint64_t n_slots)
{
    const uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_slots) return;
    char* tile = tiles + (size_t)(s / kTileItems) * g.tile_bytes();
    const uint32_t o = (uint32_t)(s % kTileItems);
    float* sc = reinterpret_cast<float*>(tile + g.scales_offset());
    const bool dyadic = g.S != g.P;
    const double dim = 64.0 * g.W;
    double a[4];
    for (uint32_t j = 0; j < g.P; ++j) a[j] = dyadic ? 1.0 / (double)(1u << j) : (double)sc[j * kTileItems + o];
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
        if (dyadic) sc[o] = (float)(1.0 / nrm);
        else for (uint32_t j = 0; j < g.P; ++j) sc[j * kTileItems + o] = (float)(a[j] / nrm);
    }
}

// Largest value of the last scale array over each row of 256 items: out[physical tile][row]; out_sum: largest
// sum of an item's scales over the row.  One workgroup of
// 256 threads per tile, one wave per row.  The one-query progressive scans bound the last plane's contribution
// with it instead of reading that array.
__global__ void row_scale_max(const char* __restrict__ tiles, const TileGeom g, float* __restrict__ out,
                              float* __restrict__ out_sum)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* sc0 = reinterpret_cast<const float*>(tiles + (size_t)blockIdx.x * g.tile_bytes() + g.scales_offset()) + wave * kRow;
    const float* sc = sc0 + (size_t)(g.S - 1) * kTileItems;
    float mx = 0.0f, ms = 0.0f;      // ms: largest sum of an item's scales (summed upwards: never below the fp32 sum
                                     // a kernel forms in any order)
    for (int m = 0; m < kRow / 64; ++m) {
        mx = fmaxf(mx, sc[m * 64 + lane]);
        double sum = 0.0;
        for (uint32_t j = 0; j < g.S; ++j) sum += (double)sc0[(size_t)j * kTileItems + m * 64 + lane];
        ms = fmaxf(ms, __double2float_ru(sum * (1.0 + 1e-6)));
    }
    for (int d = 32; d > 0; d >>= 1) { mx = fmaxf(mx, __shfl_xor(mx, d)); ms = fmaxf(ms, __shfl_xor(ms, d)); }
    if (lane == 0) {
        out[(size_t)blockIdx.x * kWavesPerBlock + wave] = mx;
        out_sum[(size_t)blockIdx.x * kWavesPerBlock + wave] = ms;
    }
}

// What each scale array holds, over the whole corpus: out[j] = largest magnitude as an fp32 bit pattern (sign bit
// cleared; >= 0x7f800000 means that the array holds an infinity or a NaN), out[4 + j] = 1 if any value is below
// zero.  out[0..7] zero-initialised by the caller.
__global__ void scale_array_max(const char* __restrict__ tiles, const TileGeom g, uint32_t* __restrict__ out)
{
    const float* sc = reinterpret_cast<const float*>(tiles + (size_t)blockIdx.x * g.tile_bytes() + g.scales_offset());
    for (uint32_t j = 0; j < g.S; ++j) {
        uint32_t mx = 0, neg = 0;
        for (uint32_t i = threadIdx.x; i < kTileItems; i += blockDim.x) {
            const uint32_t b = __float_as_uint(sc[(size_t)j * kTileItems + i]);
            const uint32_t mag = b & 0x7fffffffu;
            mx = mag > mx ? mag : mx;
            neg |= (b >> 31) & (mag != 0u ? 1u : 0u);
        }
        for (int d = 32; d > 0; d >>= 1) { const uint32_t o = __shfl_xor(mx, d); mx = o > mx ? o : mx; neg |= __shfl_xor(neg, d); }
        // (most waves find the maximum already there: a plain look first keeps the atomics few)
        if ((threadIdx.x & 63) == 0) {
            if (mx > *reinterpret_cast<const volatile uint32_t*>(&out[j])) atomicMax(&out[j], mx);
            if (neg && *reinterpret_cast<const volatile uint32_t*>(&out[4 + j]) == 0u) atomicOr(&out[4 + j], 1u);
        }
    }
}

// One-byte copies ("hints") of the scale arrays 0 .. S-2, in the order in which the lanes of the one-query
// progressive scan want them: out[physical tile][wave][lane][NW words], word j = array j, byte m = the lane's item
// m (lane_item); NW = S - 1, or 4 when S - 1 = 3.  A hint c stands for the fp32 number with the bit pattern
// (c + 32 base_j) << 18: a 3-bit exponent above base_j (a biased fp32 exponent, at least 1, chosen so that the
// array's largest value fits) and the top 5 mantissa bits, rounded to nearest.  So hint = scale (1 +- 2^-6) for
// scales of at least 2^(base_j - 127); smaller ones, zeros and subnormals become that smallest hint.  The scan's
// bound allows for both; the fp32 arrays are read only for the items the bound cannot rule out.
// Scales are finite and not negative here (the caller has looked at scale_array_max).
template <int W>
__global__ void scale_hints(const char* __restrict__ tiles, const TileGeom g, const int* __restrict__ base,
                            uint32_t* __restrict__ out, uint32_t* __restrict__ out_last)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* sc = reinterpret_cast<const float*>(tiles + (size_t)blockIdx.x * g.tile_bytes() + g.scales_offset()) + wave * kRow;
    const uint32_t nw = g.S - 1u == 3u ? 4u : g.S - 1u;
    uint32_t* dst = out + (((size_t)blockIdx.x * kWavesPerBlock + wave) * 64 + lane) * nw;
    for (uint32_t j = 0; j + 1 < g.S; ++j) {
        uint32_t word = 0;
        const int lo = base[j] << 5;
        for (int m = 0; m < kItemsPerLane; ++m) {
            const uint32_t b = __float_as_uint(sc[(size_t)j * kTileItems + lane_item<W>(lane, m)]);
            int c = (int)((b + (1u << 17)) >> 18) - lo;       // exponent and 5 mantissa bits, nearest (a carry moves up a binade)
            c = c < 0 ? 0 : (c > 255 ? 255 : c);               // (above 255 cannot happen: base leaves room for the maximum)
            word |= (uint32_t)c << (8 * m);
        }
        dst[j] = word;
    }
    if (nw == 4u) dst[3] = 0;
    if (out_last) {     // the last array, one word per lane (base[3] is its exponent base)
        uint32_t word = 0;
        const int lo = base[3] << 5;
        for (int m = 0; m < kItemsPerLane; ++m) {
            const uint32_t b = __float_as_uint(sc[(size_t)(g.S - 1u) * kTileItems + lane_item<W>(lane, m)]);
            int c = (int)((b + (1u << 17)) >> 18) - lo;
            c = c < 0 ? 0 : (c > 255 ? 255 : c);
            word |= (uint32_t)c << (8 * m);
        }
        out_last[((size_t)blockIdx.x * kWavesPerBlock + wave) * 64 + lane] = word;
    }
}

}  // namespace rbe
