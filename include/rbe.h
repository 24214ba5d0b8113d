/*
 * rbe.h -- C ABI of the MI355X (gfx950) library for exhaustive retrieval over
 * Recurrent Binary Embedding (RBE) vectors.
 *
 * What it computes (paper: "Recurrent Binary Embedding for GPU-Enabled
 * Exhaustive Retrieval from Billion-Scale Semantic Vectors", Sec. 5 and 6):
 * every item of a corpus resident in GPU memory is scored against each query
 * and the k best items per query are returned.
 *
 * Representation (Sec. 4.1, Eq. 8-11).  An item z is P "ingredient vectors"
 * (a base vector and P-1 residual vectors) in {-1,+1}^dim, each packed one bit
 * per dimension -- dimension i is bit (i % 64) of 64-bit word (i / 64), bit 1
 * means +1, bit 0 means -1 (the binarisation of Eq. 12 maps x <= 0 to -1) --
 * and each with a non-negative fp32 scale a_j[z].  The paper's fixed residual
 * weights 2^-j and its stored keyword norm (Sec. 4.3, Sec. 5.1) are the
 * special case a_j[z] = 2^-j / ||b_z||.  A query has Pq ingredient vectors
 * with scales c_i; Pq need not equal P (asymmetric design, Sec. 5.2).
 *
 * Score (Eq. 14 with the bit-wise identity of Sec. 5.1, sign corrected):
 *     s(q, z) = sum_{j<P} a_j[z] * sum_{i<Pq} c_i * (dim - 2 * popcount(Q_i XOR K_j[z]))
 * The popcounts are exact integers; the combination is evaluated in fp32 in
 * the order written (i inner, j outer), each inner sum starting from
 * dim * sum_i c_i and accumulating -2 c_i * popcount with fused multiply-adds.
 * With 5 or more queries per call (RBE_DYADIC: 4 or more, 6 or more with 4 query
 * and 4 item planes; exact mode, dim <= 128)
 * the pairs are first filtered on the matrix cores: sum_j a_j[z] * (qhat . b_z^j),
 * qhat = sum_i c_i b_q^i reconstructed on the host in double and carried as eight-bit
 * integers times a power of two (half-precision numbers for indexes whose scales
 * exceed 2^80), with a slack that covers the rounding; what
 * can reach the threshold is then scored by the formula above, so the results do
 * not depend on the number of queries per call.  (RBE_DYADIC: the integer form --
 * half precision with 4 + 4 planes -- is exact and is the score.)  Such a call reads the corpus once per 32
 * queries (once per 16 for RBE_DYADIC with dim 128 and 3 or 4 planes).
 * With fewer queries per call (exact mode, 2 or more planes) the last pass
 * over the corpus reads an item's last plane only where an upper bound on its score -- the
 * exact contribution of the other planes plus the largest value the last plane
 * could add -- reaches the current threshold; such items are then scored in full
 * by the formula above, so the results are unchanged.
 *
 * Selection (Sec. 6).  Results are ordered by (score descending, id
 * ascending).  RBE_SELECT_EXACT returns exactly the k best under that order.
 * RBE_SELECT_NEARLOSSLESS reproduces Algorithm 1 with a priority queue of
 * length 1: items are grouped as thread y = z mod 256 of block
 * x = z div (256 * I) would visit them, every group forwards only its best
 * item, and the k best forwarded items are returned (Appendix A gives the
 * probability that this loses any of the true top k).
 * RBE_SELECT_NEARLOSSLESS_Q2 is the same with priority queues of length 2: every
 * group forwards its two best items, so a true top-k item is lost only where
 * three or more of them share a group.
 *
 * Conventions.  Every function returns RBE_OK (0) or a negative error code and
 * never aborts; rbe_last_error() gives a message for the calling thread's last
 * failure.  Output arguments are untouched on error unless stated.  Pointers
 * are HOST pointers unless the argument description says otherwise.  A
 * `hip_stream` argument is a hipStream_t passed as void* (NULL = the default
 * stream); all device work of the call is enqueued on it.  An index may be
 * used by one thread at a time.  One GPU: the device current at
 * rbe_index_create() owns the index.
 */
#ifndef RBE_H
#define RBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rbe_index rbe_index; /* opaque; owns its device memory unless created with RBE_BORROW */

enum {
    RBE_OK = 0,
    RBE_EINVAL = -1,    /* bad argument (range, alignment, NULL)               */
    RBE_ENOMEM = -2,    /* host or device allocation failed                    */
    RBE_EHIP = -3,      /* a HIP runtime call failed; see rbe_last_error()     */
    RBE_ESTATE = -4,    /* call not valid in the index's current state         */
    RBE_EUNSUPPORTED = -5 /* valid request this build has no kernel for        */
};

enum { RBE_MEM_HOST = 0, RBE_MEM_DEVICE = 1 }; /* where a caller's array lives */

enum {
    RBE_BORROW = 1u << 0, /* rbe_index_create_in() only: the index lives in device memory
                            that the caller owns (e.g. a torch tensor) and never frees it  */
    RBE_COSINE = 1u << 1, /* at rbe_finalize(): divide every item's scales by the
                            norm of its reconstructed vector sum_j a_j b_j, so that
                            scores become the cosine of Eq. 14 up to the query's own
                            norm (which Sec. 5.1 drops as constant per query)      */
    RBE_DYADIC = 1u << 2  /* the paper's own representation (Sec. 4.3, Sec. 5.1):
                            plane j of every item has the fixed weight 2^-j and plane
                            i of every query the weight 2^-i; no per-plane scales are
                            stored.  The weighted sum of the binary dot products is
                            formed with integer shift-adds in Horner order (Sec. 5.1,
                            footnote) and is exact.  With RBE_COSINE one fp32 inverse
                            norm per item is computed at rbe_finalize() and kept with
                            the item (dim/8 * P + 4 bytes per item: 20 at dim 64, P = 2);
                            without it nothing but the bits is stored (16 bytes) and
                            scores are exact dyadic rationals.  The `scales` arguments
                            of the load calls are ignored (may be NULL); q_scales of
                            rbe_search must be NULL or exactly 2^-i.  dim 64 or 128.   */
};

enum { RBE_SELECT_EXACT = 0, RBE_SELECT_NEARLOSSLESS = 1, RBE_SELECT_NEARLOSSLESS_Q2 = 2 };

/* Limits */
#define RBE_MAX_PLANES 4u     /* P and Pq                                        */
#define RBE_MAX_QUERIES 64u   /* queries per rbe_search call                     */
#define RBE_MAX_K 4096u
#define RBE_MAX_ITEMS 4294966272ull /* ids are kept in 32 bits on the device     */

/* ---------------------------------------------------------------------------
 * Corpus (the offline keyword side of Fig. 3: embeddings are produced ahead of
 * time and uploaded once, Sec. 5).  On the device, items are kept in tiles of
 * 1024 consecutive ids; inside a tile storage is structure-of-arrays by
 * ingredient vector (the grouping of Sec. 6.1): all base vectors of the tile,
 * then all first residuals, ..., then the scale arrays in the same order.
 * Tiles are stored in "nested-sample-major" order, so that every evenly
 * strided sample of tiles (stride = a power of the sample ratio) is a
 * contiguous prefix of memory.  Callers never see this order: the arrays they
 * pass are plain [plane][item][word] and ids are item numbers.
 * ------------------------------------------------------------------------- */

/* Allocates device storage for n_items items of `dim` dimensions and
 * `n_planes` ingredient vectors.  dim in {64, 128, 256}; 1 <= n_planes <= 4;
 * 1 <= n_items <= RBE_MAX_ITEMS.  flags: 0 or any of RBE_COSINE, RBE_DYADIC.  The index starts
 * in the "loading" state.  Device memory: n_items * n_planes * (dim/8 + 4)
 * bytes (see RBE_DYADIC for its smaller footprint), rounded up to a multiple of
 * 1024 items.                           */
int rbe_index_create(rbe_index **out, uint64_t n_items, uint32_t dim,
                     uint32_t n_planes, uint32_t flags);

/* Same, with an explicit sample ratio r (2..4096; 0 = the default 64): level c
 * of the exact search reads every r^c-th tile, so each refinement round reads r
 * times more of the corpus than the one before and hands about r*k survivors
 * per query to its selection.  The ratio fixes the tile order, hence it is a
 * property of the index.                                                      */
int rbe_index_create_ex(rbe_index **out, uint64_t n_items, uint32_t dim,
                        uint32_t n_planes, uint32_t flags, uint32_t sample_ratio);

/* Caller-owned corpus storage.  The scans depend on the tile order described
 * above, so a caller's plain [plane][item][word] arrays cannot be searched in
 * place (every search would pay strided reads at about a tenth of the streaming
 * rate); what a caller CAN own is the memory itself.  rbe_index_bytes() gives the
 * device bytes an index of this shape needs (tiles plus the side arrays that
 * rbe_finalize derives; 0 for an invalid shape; sample_ratio 0 = 64), and
 * rbe_index_create_in() builds the index inside `storage_dev` (DEVICE pointer,
 * 256-byte aligned, at least that many bytes; flags must include RBE_BORROW).
 * The library then allocates no device memory for this index at create, finalize
 * or free (rbe_load_chunk / rbe_encode_chunk from HOST arrays still stage through
 * a temporary device buffer; from DEVICE arrays they allocate nothing), writes
 * the storage only through its own calls, and never frees it: keep it alive and
 * untouched until after rbe_free().                                             */
size_t rbe_index_bytes(uint64_t n_items, uint32_t dim, uint32_t n_planes,
                       uint32_t flags, uint32_t sample_ratio);
int rbe_index_create_in(rbe_index **out, uint64_t n_items, uint32_t dim,
                        uint32_t n_planes, uint32_t flags, uint32_t sample_ratio,
                        void *storage_dev, size_t storage_bytes);

/* Copies items [first_item, first_item + count) into the index.
 *   planes: [n_planes][count][dim/64] uint64, scales: [n_planes][count] float,
 *   both in host memory (mem_kind = RBE_MEM_HOST) or both in device memory
 *   (RBE_MEM_DEVICE; e.g. torch tensors).  The caller keeps ownership; the
 *   arrays may be released once the stream has passed the copies (host arrays:
 *   on return).  Scales must be finite (checked at rbe_finalize) and should be
 *   >= 0, as the method produces them: an index that holds a negative scale is
 *   searched correctly, but by the plain scans only (see rbe_finalize).
 * Only valid while loading.                                                   */
int rbe_load_chunk(rbe_index *ix, uint64_t first_item, uint64_t count,
                   const uint64_t *planes, const float *scales,
                   int mem_kind, void *hip_stream);

/* Encodes items [first_item, first_item + count) on the GPU with the stand-in
 * encoder described at rbe_encode_query() (same arithmetic, same bits) and
 * stores them in the index: the offline "keyword side" step of Fig. 3.
 *   x: [count][dim] float, row-major, in host or device memory (mem_kind).
 * Not available for RBE_DYADIC indexes (their planes come from the model).
 * Only valid while loading.                                                   */
int rbe_encode_chunk(rbe_index *ix, uint64_t first_item, uint64_t count,
                     const float *x, int mem_kind, void *hip_stream);

/* rbe_index_create + rbe_encode_chunk of all n_items vectors + rbe_finalize.   */
int rbe_encode_corpus(rbe_index **out, const float *x, uint64_t n_items,
                      uint32_t dim, uint32_t n_planes, int mem_kind,
                      uint32_t flags, void *hip_stream);

/* Ends loading: applies RBE_COSINE if requested, derives the side arrays of the
 * one-query search (per row of 256 items the largest value of the last scale
 * array; for general scales with 2 or more planes also one-byte copies of the
 * other scale arrays: n_planes - 1 bytes of device memory per item, 4 at 4
 * planes), waits for the stream, and makes the index searchable.  Items never
 * loaded score as all-(-1) vectors with scale 0.  If the one-byte copies do not
 * fit in device memory the index works without them (the one-query search then
 * reads the fp32 arrays they stand for).
 * Scales are looked at here.  A scale that is not finite: RBE_EINVAL, and the
 * index stays in the loading state (load the chunk again, then finalize).  A
 * negative scale: every upper bound the pruning searches use (last plane left
 * out, matrix-core filter) assumes scales >= 0, so such an index gets no side
 * arrays and every search on it reads every plane of every item with the plain
 * XOR/popcount (or byte-table) scans; results stay exact, searches are slower. */
int rbe_finalize(rbe_index *ix, void *hip_stream);

/* rbe_index_create + one rbe_load_chunk of the whole corpus + rbe_finalize.
 *   planes: [n_planes][n_items][dim/64], scales: [n_planes][n_items].         */
int rbe_load_corpus(rbe_index **out, const uint64_t *planes, const float *scales,
                    uint64_t n_items, uint32_t dim, uint32_t n_planes,
                    int mem_kind, uint32_t flags, void *hip_stream);

/* Releases the index and everything it owns.  NULL is allowed.                */
void rbe_free(rbe_index *ix);

/* ---------------------------------------------------------------------------
 * Query side.  The paper's learned RBE layers (Eq. 8-11) need trained matrices;
 * this stand-in produces vectors of the same form by greedy residual
 * binarisation: r_0 = x; for t < n_planes: scale_t = mean_i |r_t[i]| (summed in
 * double, stored as fp32), bit_t[i] = (r_t[i] > 0), r_{t+1} = fp32(r_t -
 * scale_t * (2 bit_t - 1)).  Pure host function; no GPU involved.
 *   x: [dim] float; planes_out: [n_planes][dim/64]; scales_out: [n_planes].
 * ------------------------------------------------------------------------- */
int rbe_encode_query(const float *x, uint32_t dim, uint32_t n_planes,
                     uint64_t *planes_out, float *scales_out);

/* ---------------------------------------------------------------------------
 * Search: exhaustive match + selection (Sec. 5-6, Algorithm 1).
 *   q_planes : [n_queries][q_n_planes][dim/64] uint64 (host)
 *   q_scales : [n_queries][q_n_planes] float (host), finite
 *   1 <= n_queries <= RBE_MAX_QUERIES, 1 <= q_n_planes <= 4, 1 <= k <= RBE_MAX_K
 *   mode     : RBE_SELECT_EXACT, RBE_SELECT_NEARLOSSLESS or RBE_SELECT_NEARLOSSLESS_Q2
 *   group_size_I : items per group for the near-lossless mode (the paper's I,
 *                  1..65535; 0 means 256); ignored in exact mode
 *   ids_out  : [n_queries][k] int64 (host), scores_out: [n_queries][k] float
 *              (host).  Per query sorted by (score desc, id asc).  If fewer
 *              than k results exist (k > n_items, or k > number of groups) the
 *              tail holds id = -1, score = -INFINITY.
 * The call returns after the results are in the host arrays (it waits for the
 * stream).  Device scratch (candidate lists, counters, staged queries, results):
 * the block set with rbe_set_workspace() if there is one -- then the call
 * allocates nothing and fails with RBE_EINVAL if the block is too small -- else a
 * block of the library's own, allocated when a call needs more than any call
 * before it (steady-state searches allocate nothing).                          */
int rbe_search(rbe_index *ix, const uint64_t *q_planes, const float *q_scales,
               uint32_t n_queries, uint32_t q_n_planes, uint32_t k,
               uint32_t mode, uint32_t group_size_I,
               int64_t *ids_out, float *scores_out, void *hip_stream);

/* Caller-owned scratch (Sec. 5: everything a query touches stays in GPU memory;
 * here the caller's allocator, e.g. a torch tensor, can own all of it).
 * rbe_workspace_bytes(): device bytes that a search of up to n_queries queries
 * for k results in `mode` needs on this index with its current tuning (0 for
 * arguments out of range; the near-lossless modes need about three times the
 * exact mode's); the figure covers rbe_search and rbe_search_float.
 * rbe_set_workspace(): every later search carves its scratch from dev_ptr (DEVICE
 * pointer, 256-byte aligned, `bytes` long) instead of library-owned memory, which
 * is released; the caller keeps ownership and must keep the block alive and
 * otherwise unused while searches run.  dev_ptr = NULL returns to library-owned
 * scratch.  A search that needs more than `bytes` fails with RBE_EINVAL and the
 * required size in rbe_last_error().                                            */
size_t rbe_workspace_bytes(const rbe_index *ix, uint32_t n_queries, uint32_t k, uint32_t mode);
int rbe_set_workspace(rbe_index *ix, void *dev_ptr, size_t bytes);

/* rbe_search for callers that cannot allocate device memory at all -- code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: same
 * arguments, same results, but the device scratch is a fixed array inside the
 * library (RBE_STATIC_SCRATCH_BYTES per GPU, held until the process ends) and the
 * call makes no allocation of any kind on the device or in pinned host memory.
 * Limit: rbe_workspace_bytes(ix, n_queries, k, mode) <= RBE_STATIC_SCRATCH_BYTES
 * (exact mode at the default tuning: e.g. 4 queries for k = 1000, or 1 query for
 * k = 4096; near-lossless modes: 2 queries for k = 1000),
 * else RBE_EINVAL.  The device that owns the index must be current.  All calls on
 * one GPU share the array: calls that overlap in time on one GPU -- from several
 * threads, or for several indexes -- race; serialise them.  What a call needs
 * cleared it clears itself.                                                     */
#define RBE_STATIC_SCRATCH_BYTES 16777216u
int rbe_search_static(rbe_index *ix, const uint64_t *q_planes, const float *q_scales,
                      uint32_t n_queries, uint32_t q_n_planes, uint32_t k,
                      uint32_t mode, uint32_t group_size_I,
                      int64_t *ids_out, float *scores_out, void *hip_stream);

/* Hybrid scoring: full-precision queries against the binary items (the paper's
 * "hybrid rbe" model, Sec. 8.1, which bounds the accuracy of every RBE model with
 * the same keyword bits):
 *     s(q, z) = sum_j a_j[z] * sum_i q[i] * b_z^j[i],      q in R^dim (fp32).
 * Evaluated through per-byte tables: t_j = sum over the dim/8 bytes p of plane j of
 * T[p][byte], T[p][v] = sum_{b<8} q[8p+b] * (bit b of v ? +1 : -1) (built in double,
 * stored as fp32, added in fp32 in byte order), then fp32 fused multiply-adds over j.
 * For RBE_DYADIC indexes a_j = 2^-j (times the stored inverse norm with RBE_COSINE).
 * With 3 or more queries per call on an index with general scales (dim <= 128) the
 * pairs are first filtered on the matrix cores, exactly as rbe_search does with the
 * reconstructed binary queries (q itself, rounded to eight-bit integers times a power
 * of two, is the left operand),
 * what can reach the threshold is scored through the tables as above, so the results
 * do not depend on the number of queries per call, and the corpus is read once per
 * 32 queries; otherwise it is read once per query.
 *   q: [n_queries][dim] float (host), finite.  Other arguments as rbe_search.
 * Every selection mode of rbe_search is available.                              */
int rbe_search_float(rbe_index *ix, const float *q, uint32_t n_queries, uint32_t k,
                     uint32_t mode, uint32_t group_size_I,
                     int64_t *ids_out, float *scores_out, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Measurement.  With profiling on, rbe_search brackets each kernel with HIP
 * events on the search stream and fills rbe_search_stats after the call.
 * ------------------------------------------------------------------------- */
#define RBE_MAX_LEVELS 8

typedef struct rbe_search_stats {
    uint32_t n_levels;        /* scan+select rounds of the last search           */
    uint32_t fallback;        /* 1 if the bounded-segment slow path was taken    */
    uint32_t grid_blocks;     /* workgroups of the widest scan launch            */
    uint32_t deep_rows;       /* exact mode, pruning scans: rows of 256 items whose
                                 last plane had to be read (the others were ruled
                                 out by the other planes and the scales), all rounds */
    uint64_t items_scanned[RBE_MAX_LEVELS];   /* items read by each scan         */
    uint64_t candidates_max[RBE_MAX_LEVELS];  /* largest per-query candidate
                                                 count handed to each select     */
    float scan_ms[RBE_MAX_LEVELS];            /* kernel time of each scan        */
    float select_ms[RBE_MAX_LEVELS];          /* kernel time of each select      */
    float total_gpu_ms;       /* first enqueue to results ready, on the stream   */
    uint32_t deep_units;      /* one query per scan: what the lanes of the
                                 last scan asked for beyond its stream (last plane
                                 and fp32 scales of items that could still reach
                                 the threshold, whole rows in the fallback), in
                                 units of 8 bytes                                 */
    uint32_t scan_kernel[RBE_MAX_LEVELS];     /* which scan each level ran: RBE_KERNEL_* */
    uint32_t last_level_parts;                /* 1, or 2 if the last (largest) level was taken
                                                 in two parts, the last two rounds       */
    uint32_t deep_rows_level[RBE_MAX_LEVELS]; /* deep_rows, round by round               */
    uint32_t reserved;
} rbe_search_stats;

enum {                        /* rbe_search_stats.scan_kernel                      */
    RBE_KERNEL_NONE = 0,
    RBE_KERNEL_SCAN_EXACT = 1,        /* XOR/popcount, every plane of every item    */
    RBE_KERNEL_SCAN_PROG = 2,         /* ... last plane only where the bound passes */
    RBE_KERNEL_SCAN_PROG_HINT = 3,    /* ... streaming one-byte scale copies        */
    RBE_KERNEL_SCAN_BATCH_MFMA = 4,   /* matrix-core filter + XOR/popcount rescoring */
    RBE_KERNEL_SCAN_GROUPMAX = 5,     /* near-lossless group maxima (Algorithm 1)   */
    RBE_KERNEL_SCAN_FLOAT = 6,        /* fp32 query through byte tables, every plane */
    RBE_KERNEL_SCAN_FLOAT_PROG = 7,   /* ... last plane only where the bound passes */
    RBE_KERNEL_SCAN_PROG2_HINT = 8,   /* as PROG_HINT with plane 0 alone in the stream (1-4 queries) */
    RBE_KERNEL_SCAN_FLOAT_PROG2 = 9   /* the same for an fp32 query                    */
};

int rbe_set_profiling(rbe_index *ix, int enabled);
int rbe_get_search_stats(const rbe_index *ix, rbe_search_stats *out);

/* Tuning knobs (0 keeps the current value):
 *   cand_capacity   : candidate slots per query (default max(65536, 4*ratio*k));
 *                     2048..2^24
 *   blocks_per_cu   : persistent workgroups per compute unit for the scan
 *                     (default: as many as the kernel's occupancy allows)      */
int rbe_set_tuning(rbe_index *ix, uint32_t cand_capacity, uint32_t blocks_per_cu);

const char *rbe_strerror(int code);
const char *rbe_last_error(void);
/* n_items / dim / n_planes of an index (0 for NULL). */
uint64_t rbe_n_items(const rbe_index *ix);
uint32_t rbe_dim(const rbe_index *ix);
uint32_t rbe_n_planes(const rbe_index *ix);

#ifdef __cplusplus
}
#endif
#endif /* RBE_H */
