// Physical layout of an RBE corpus in HBM (host + device code).
//
// Items are grouped into tiles of 1024 consecutive ids.  A tile is stored as
// one contiguous block, structure-of-arrays by ingredient vector inside the
// block (the grouping of Sec. 6.1, applied per tile so that one workgroup step
// reads a single contiguous region):
//
//     [plane 0: 1024 x W words][plane 1] ... [plane P-1][scales 0: 1024 floats] ... [scales S-1]
//
// with S = P scale arrays in the general mode, S = 1 (one inverse norm per item)
// or S = 0 in the dyadic modes, where the plane weights are the constants 2^-j.
//
// Tile ORDER in memory is "nested-sample major".  With ratio r, the class of
// logical tile t is the largest c <= L with r^c | t (tile 0 has class L).
// Tiles are stored by descending class, ascending t within a class.  Hence for
// every c the first ceil(T / r^c) physical tiles are exactly the logical tiles
// that are multiples of r^c: an evenly strided sample of the corpus is a
// contiguous prefix of memory, and the part of a finer sample not contained in
// the coarser one is a contiguous range.  The exact search reads such ranges
// from coarse to fine (see rbe_api.hip).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define RBE_HD __host__ __device__ __forceinline__
#else
#define RBE_HD inline
#endif

namespace rbe {

constexpr int kTileItems = 1024;
constexpr int kMaxClasses = 8;  // L + 1

struct Layout {
    uint32_t n_tiles;               // T
    uint32_t ratio;                 // r >= 2
    uint32_t top;                   // L: highest class
    uint32_t n_ge[kMaxClasses + 1]; // n_ge[c] = ceil(T / r^c) for c <= L; n_ge[L+1] = 0
    uint32_t pow_r[kMaxClasses];    // r^c (saturating at 2^31 is never reached: r^L < T)
};

inline Layout make_layout(uint32_t n_tiles, uint32_t ratio)
{
    Layout l{};
    l.n_tiles = n_tiles;
    l.ratio = ratio;
    uint64_t p = 1;
    uint32_t c = 0;
    for (;; ++c) {
        l.pow_r[c] = (uint32_t)p;
        l.n_ge[c] = (uint32_t)((n_tiles + p - 1) / p);
        // stop once the coarsest sample is at most 32 tiles, or no further split is possible
        if (l.n_ge[c] <= 32 || c + 1 == kMaxClasses || p * ratio >= n_tiles) break;
        p *= ratio;
    }
    l.top = c;
    l.n_ge[c + 1] = 0;
    return l;
}

// v-th (0-based) non-multiple of r  ->  its value
RBE_HD uint32_t nth_non_multiple(uint32_t v, uint32_t r) { return (v / (r - 1)) * r + (v % (r - 1)) + 1; }

RBE_HD uint32_t tile_to_phys(const Layout& l, uint32_t t)
{
    uint32_t c = 0;
    while (c < l.top && t % l.pow_r[c + 1] == 0) ++c;
    const uint32_t u = t / l.pow_r[c];
    if (c == l.top) return u;
    return l.n_ge[c + 1] + (u - u / l.ratio - 1);
}

RBE_HD uint32_t phys_to_tile(const Layout& l, uint32_t p)
{
    uint32_t c = l.top;
    while (c > 0 && p >= l.n_ge[c]) --c;
    if (c == l.top) return p * l.pow_r[c];
    return nth_non_multiple(p - l.n_ge[c + 1], l.ratio) * l.pow_r[c];
}

// phys_to_tile for a physical tile that differs from lane to lane: the same class, found by a loop whose trip
// count is the same for all lanes (n_ge decreases with the class, so the class of p is the number of classes
// c >= 1 with p < n_ge[c]).
RBE_HD uint32_t phys_to_tile_per_lane(const Layout& l, uint32_t p)
{
    uint32_t c = 0;
    for (uint32_t i = 1; i <= l.top; ++i) c += p < l.n_ge[i] ? 1u : 0u;
    if (c == l.top) return p * l.pow_r[c];
    return nth_non_multiple(p - l.n_ge[c + 1], l.ratio) * l.pow_r[c];
}

// Scoring modes (compile-time parameter of the kernels).
enum : int {
    kModeScaled = 0,      // per-item fp32 scale per plane, fp32 query scales
    kModeDyadicNorm = 1,  // plane weights 2^-j on both sides (integer shift-adds), one fp32 scale per item
    kModeDyadic = 2       // plane weights 2^-j on both sides, no per-item scale: scores are exact
};
RBE_HD constexpr int scale_arrays(int mode, int P) { return mode == kModeScaled ? P : (mode == kModeDyadicNorm ? 1 : 0); }

// Byte geometry of a tile.
struct TileGeom {
    uint32_t W, P, S;   // words per plane, planes, scale arrays
    RBE_HD size_t plane_bytes() const { return (size_t)kTileItems * W * 8; }
    RBE_HD size_t scales_offset() const { return plane_bytes() * P; }
    RBE_HD size_t tile_bytes() const { return scales_offset() + (size_t)kTileItems * 4 * S; }
};

}  // namespace rbe
