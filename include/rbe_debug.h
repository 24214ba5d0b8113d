/*
 * rbe_debug.h -- test and measurement hooks of the RBE retrieval library.
 *
 * Not part of the product interface (include/rbe.h): dense dumps that parity
 * tests compare with a reference, switches that force a particular kernel so
 * that two kernels can be compared on the same search, pure host functions that
 * expose intermediate quantities, and two calibration kernels for measurements.
 * Conventions as in rbe.h.
 */
#ifndef RBE_DEBUG_H
#define RBE_DEBUG_H

#include "rbe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------
 * Dense dumps for parity checks (small ranges only).
 * ------------------------------------------------------------------------- */

/* popcount(Q_i XOR K_j[z]) for z in [first_item, first_item+count):
 *   q_planes [q_n_planes][dim/64] (host) -> out [count][n_planes][q_n_planes]
 *   int32 (host).                                                            */
int rbe_debug_popcounts(rbe_index *ix, const uint64_t *q_planes, uint32_t q_n_planes,
                        uint64_t first_item, uint64_t count, int32_t *out, void *hip_stream);

/* fp32 scores s(q, z) of one query for z in [first_item, first_item+count):
 *   out [count] float (host).  Same arithmetic as rbe_search.                */
int rbe_debug_scores(rbe_index *ix, const uint64_t *q_planes, const float *q_scales,
                     uint32_t q_n_planes, uint64_t first_item, uint64_t count,
                     float *out, void *hip_stream);

/* Calls that do not go to the matrix cores (see rbe_debug_set_batch_path), exact mode, 2 or more planes:
 * the last (largest) level of the search streams every plane but the last (one query: with one-byte
 * copies of their scales and the row's largest last scale in place of the fp32
 * arrays) and reads an item's last plane and fp32 scales only where its upper
 * bound -- the exact contribution of the other planes plus the largest value the
 * last plane could add -- reaches the threshold; such items are then scored in
 * full, so the results are those of the plain scan bit for bit.
 * With three or more planes a scan of one to four queries goes one step further:
 * its stream carries plane 0 and the scale copies alone, items that a bound from
 * plane 0 cannot rule out (for some query) are gathered 64 at a time, and only
 * those have their planes 1 .. P-2 read (then the last plane, as above).
 * Larger batches on general scales (the matrix-core scan, up to 16 queries per
 * launch) stream planes 0 .. P-2 and the scale copies and read the last plane
 * and the fp32 scales for the blocks of 32 items their first look cannot rule out.
 * enabled = 0 switches all of it off (every plane of every item is read); default 1;
 * 2 = on, but without the one-byte scale copies (what an index uses whose
 * copies did not fit in device memory; the matrix-core scan then streams whole
 * rows); 3 = on, with planes 0 .. P-2 in the stream (no first stage on plane 0
 * alone; the matrix-core scan streams whole rows).                              */
int rbe_debug_set_progressive(rbe_index *ix, int enabled);

/* The last level of an exact search in two parts (an eighth of its items, a
 * selection, then the rest, which starts from a much tighter threshold, so that
 * the pruning scans rule out more).  mode 0 = the library's rule: every search on
 * an index that can prune whose last level has 4096 tiles or more -- except that
 * searches of ONE binary query, the one case where the split can cost more than
 * it saves (1 %), take the level whole for 64 searches after 4 split searches in a
 * row whose second part let through no smaller a share of its rows than the
 * first, and then ask again (setting mode 0 also forgets that count);
 * 1 = never split; 2 = always (from 16 tiles on).  Results do not depend on any
 * of it.                                                                         */
int rbe_debug_set_plan_split(rbe_index *ix, int mode);

/* The mass of one query as the progressive scan uses it (pure host function, for
 * tests).  With qhat = sum_i c_i rho_i (rho = +-1 per bit), M = sum_d |qhat_d| is the
 * largest value sum_i c_i (rho_i . rho) can take over all sign vectors rho.
 * dyadic = 0: mass_out[0] >= M, larger by a few 2^-20 of dim * sum_i |c_i| (rounding
 * allowance), mass_out[1] = 2^-19 mass_out[0].  dyadic = 1 (c_i = 2^-i, q_scales not
 * read): the bits of mass_out[0] are the integer h_min = (dim (2^Pq - 1) - M') / 2 with
 * M' = 2^(Pq-1) M, the least weighted mismatch count sum_i 2^(Pq-1-i) popcount(Q_i XOR K)
 * any plane K can have; mass_out[1] = 0.
 *   q_planes [q_n_planes][dim/64], q_scales [q_n_planes], mass_out [2]: host.    */
int rbe_debug_query_mass(const uint64_t *q_planes, const float *q_scales, uint32_t q_n_planes,
                         uint32_t dim, uint32_t dyadic, float *mass_out);

/* Which kernel rbe_search uses in exact mode: 0 = automatic (matrix cores from 5
 * queries per call on; RBE_DYADIC: from 4 while the query fits eight-bit
 * integer operands, 2 (2^q_n_planes - 1) 2^(n_planes - 1) <= 127, else from 6;
 * dim <= 128), 1 = always the XOR/popcount kernel, 2 = the matrix-core kernel
 * for any number of queries (dim <= 128), 3 = as 2, with half operands also
 * where eight-bit integer operands are the default.                            */
int rbe_debug_set_batch_path(rbe_index *ix, int path);

/* How the near-lossless modes are computed.  0 (default): the scans and the
 * refinement plan of the exact mode, with the candidates reduced to the best item
 * (or two) of every group of Algorithm 1 before each selection -- the same result,
 * since an item below a lower bound of the k-th best forwarded item can neither be
 * returned nor change what another group forwards.  1: a scan that keeps one queue
 * per thread as Algorithm 1 is written (every plane of every item read; binary
 * queries only).  Both are tested against the oracle and against each other.     */
int rbe_debug_set_nearlossless_path(rbe_index *ix, int path);

/* fp32 hybrid scores (rbe_search_float arithmetic) of one fp32 query q [dim] for z in
 * [first_item, first_item+count): out [count] float (host).                  */
int rbe_debug_scores_float(rbe_index *ix, const float *q, uint64_t first_item,
                           uint64_t count, float *out, void *hip_stream);

/* Copies the (possibly cosine-folded) scales of items [first_item,
 * first_item+count) back: out [n_planes][count] float (host).                */
int rbe_debug_read_scales(rbe_index *ix, uint64_t first_item, uint64_t count,
                          float *out, void *hip_stream);

/* Copies the plane words of items [first_item, first_item+count) back:
 * out [n_planes][count][dim/64] uint64 (host).                               */
int rbe_debug_read_planes(rbe_index *ix, uint64_t first_item, uint64_t count,
                          uint64_t *out, void *hip_stream);

/* Tile order (pure host functions, for tests): physical position of logical
 * tile `tile` in a corpus of n_tiles tiles with the given sample ratio, and the
 * inverse.                                                                     */
uint32_t rbe_debug_tile_to_phys(uint32_t n_tiles, uint32_t sample_ratio, uint32_t tile);
uint32_t rbe_debug_phys_to_tile(uint32_t n_tiles, uint32_t sample_ratio, uint32_t phys);

/* Refinement plan of the exact mode (pure host function, for tests): the levels
 * rbe_search would run for such a corpus, each a range [first_tile, end_tile) of
 * PHYSICAL tile positions; arrays of RBE_MAX_LEVELS entries.  n_levels = 0 means
 * that no plan fits cand_capacity (the bounded-segment path is used instead).    */
int rbe_debug_exact_plan(uint64_t n_items, uint32_t sample_ratio, uint32_t cand_capacity, uint32_t k,
                         uint32_t *n_levels, uint32_t *first_tile, uint32_t *end_tile);

/* Query operands of the matrix-core batch scan (pure host function, for tests).
 * The queries are binary (q_planes [Q][Pq][W] and, unless dyadic, q_scales
 * [Q][Pq]; q_float NULL) or fp32 (q_float [Q][dim]; general scales only, the
 * other two are not read).
 * halves_out [tile][plane copy][part][lane][8] fp16 bit patterns, where
 * tile = query / 16, lane = 16 g + query % 16, part = 32-dimension part of the
 * query and slot e = 2t + h of lane group g stands for bit (10 + 16h + t - 4g)
 * mod 32 of that part, weighted by 2 / val_t with val_t = 2^-14, 2^-13, 2^-11,
 * 2^-7 (the value of a half whose only set bit is bit 10 + t: the form in which
 * the kernel feeds item bits), times 2^-j in plane copy j (dyadic only; one copy
 * otherwise).  dyadic = 1: every half is exact and the contraction is the score.
 * dyadic = 0 (general scales): every component is rounded to one half and the
 * contraction is a filter whose distance from the score is at most
 * margin * sum_j a_j[item]; survivors are scored again exactly.
 * unscale_out[q] = 2^-k undoes the power-of-two scaling of query q; start_out[q]
 * is where its accumulators start (minus the weighted sum of what the halves hold).
 * shape_out = {tiles, plane copies, parts, margin (float bits)}: 4 entries.
 * halves_capacity in halves.                                                    */
int rbe_debug_batch_operands(const uint64_t *q_planes, const float *q_scales, const float *q_float,
                             uint32_t n_queries, uint32_t q_n_planes, uint32_t dim, uint32_t n_planes,
                             uint32_t dyadic, uint16_t *halves_out, size_t halves_capacity,
                             float *unscale_out, float *start_out, uint32_t *shape_out);

/* The eight-bit integer operands the matrix-core scan filters queries on
 * general scales with (Eq. 14 as a dense contraction; pure host arithmetic, no GPU
 * needed).  qhat = sum_i c_i b_q^i is rounded to T_d 2^e with integers |T_d| <= 126;
 * bytes_out [tile = query / 16][dim / 64 parts][lane = 16 g + query % 16][16]: byte
 * 4 t + m of a lane belongs to dimension 64 part + 32 (t / 2) + 8 m + 2 g + (t % 2)
 * and holds T_d for even t, -T_d / 2 for odd t (T_d is even there).  unscale_out [Q]
 * = 2^e / 32, the unit of the filter's scores; start_out [Q] = the float 1.5 * 2^23
 * - 32 sum_d T_d whose bit pattern the accumulators start from; mass_out [Q] =
 * sum_d |qhat_d| in those units, rounded up; *margin_out = the bound, per unit of
 * an item's scale sum and in those units, on |filter value - score| for every
 * query of the batch.  q_float != NULL: [n_queries][dim] fp32 queries (hybrid
 * scoring) take the place of qhat and q_planes / q_scales / q_n_planes are not
 * read.  bytes_capacity: bytes available at bytes_out (EINVAL and the count needed
 * in rbe_last_error() if too small).  All pointers: host.                        */
int rbe_debug_batch_operands_i8(const uint64_t *q_planes, const float *q_scales, const float *q_float,
                                uint32_t n_queries, uint32_t q_n_planes, uint32_t dim,
                                int8_t *bytes_out, size_t bytes_capacity, float *unscale_out,
                                float *start_out, float *mass_out, float *margin_out);

/* The same for a dyadic index (host only): binary queries with the weights 2^-i,
 * n_item_planes item planes with the weights 2^-j; every number is an exact
 * integer.  bytes_out [tile = query / 16][item plane j][dim / 64 parts][lane][16],
 * laid out within a lane as above, holds X_d = 2 T_d 2^(n_item_planes - 1 - j)
 * (T_d = 2^(q_n_planes - 1) qhat_d, an odd integer) for even t and -X_d / 2 for
 * odd t; unscale_out [Q] = 2^-(n_item_planes + q_n_planes + 4); start_out [Q] =
 * the float 1.5 * 2^23 - 32 sum_j sum_d X_d; mass_out [Q] = the most the last
 * item plane can add to an accumulator that holds the start value already.
 * EINVAL if 2 (2^q_n_planes - 1) 2^(n_item_planes - 1) exceeds 127 (such queries
 * keep half operands).                                                          */
int rbe_debug_batch_operands_i8_dyadic(const uint64_t *q_planes, uint32_t n_queries, uint32_t q_n_planes,
                                       uint32_t dim, uint32_t n_item_planes, int8_t *bytes_out,
                                       size_t bytes_capacity, float *unscale_out, float *start_out,
                                       float *mass_out);

/* Measurement yardstick: enqueues a plain copy kernel ("calib_copy") of `bytes`
 * bytes from src_dev to dst_dev (DEVICE pointers, 16-byte aligned, bytes a
 * multiple of 16, non-overlapping).  It reads and writes exactly `bytes` each,
 * so hardware-counter readings of other kernels can be scaled by what the same
 * counters report for it.  Asynchronous on the stream.                         */
int rbe_debug_copy(void *dst_dev, const void *src_dev, size_t bytes, void *hip_stream);

/* Measurement yardstick: enqueues a read-only kernel ("calib_read") that streams
 * `bytes` bytes from src_dev (DEVICE pointer, 16-byte aligned, bytes a multiple
 * of 16) with the scan's access shape and writes 16 bytes per thread to
 * sink_dev (DEVICE, 16-byte aligned, at least 3 * 256 * 16 bytes per compute
 * unit: 3 MiB covers 256 units; EINVAL if too small).  Its rate is the practical
 * read ceiling the scan is compared with.  Asynchronous on the stream.         */
int rbe_debug_read(const void *src_dev, size_t bytes, void *sink_dev, size_t sink_bytes, void *hip_stream);

/* Measurement yardstick for the batch scans: the instruction mix of a scan free of
 * memory traffic.  Launches the last-level kernel of a batched exact search --
 * kernel 0: the XOR/popcount scan, every plane of every pair; kernel 1: the
 * matrix-core scan (its first look; general scales leave the last plane out) --
 * with one tile per workgroup of a full grid, thresholds that no score reaches (so
 * nothing is queued), and every tile gone over 1 + repeat times from registers / LDS
 * without being loaded again.  *ms_out = HIP-event time of the launch(es) on the
 * stream, *pairs_out = (query, item) pairs scored.  The rate is the ceiling that
 * vector- and matrix-instruction issue put on that kernel; the same kernel over a
 * corpus in HBM is compared with it.  Queries as for rbe_search (3..64 of them).   */
int rbe_debug_issue_rate(rbe_index *ix, const uint64_t *q_planes, const float *q_scales,
                         uint32_t n_queries, uint32_t q_n_planes, uint32_t kernel,
                         uint32_t repeat, float *ms_out, uint64_t *pairs_out, void *hip_stream);

/* What rbe_finalize decided for an index: out[0] = 1 if the pruning scans may be
 * used (no negative scale), out[1] = 1 if it holds the one-byte scale copies,
 * out[2] = 1 if it lives in caller-owned storage, out[3] = 1 if a caller-owned
 * workspace is set.  out: 4 entries (host).                                     */
int rbe_debug_index_info(const rbe_index *ix, uint32_t *out);

#ifdef __cplusplus
}
#endif
#endif /* RBE_DEBUG_H */
