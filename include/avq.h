/*
 * avq.h -- C ABI of the MI355X (gfx950) library for score-aware / anisotropic
 * quantized maximum inner product search, after "Accelerating Large-Scale
 * Inference with Anisotropic Vector Quantization" (arXiv 1908.10396).
 *
 * The problem (paper, Section 1): a database X = {x_i}, i < n, of points in R^d;
 * for a query q return the points with the largest <q, x_i>. The library
 * answers approximately: product-quantization codes assigned under the
 * anisotropic loss eta*||r_par||^2 + ||r_perp||^2 (Sections 3.1, 3.2, 4.1) are
 * scored through per-query lookup tables (Section 4.1), the best reorder_k
 * candidates are re-scored exactly in fp32 and the best k returned.
 *
 * Conventions that hold for every call
 *  - One GPU. All work runs on the HIP device that is current when avq_create
 *    is called, on the stream passed in (NULL = the default stream). Calls are
 *    asynchronous with respect to the host except where stated; outputs are
 *    valid after the stream has been synchronised.
 *  - "device pointer" = memory on that GPU allocated by the caller (e.g. a
 *    torch tensor's data_ptr()); the library never frees it. "host or device"
 *    = either; such arguments are copied with hipMemcpyDefault and the call
 *    synchronises the stream.
 *  - Matrices are row-major, dense. Floats are IEEE fp32, finite; behaviour
 *    for NaN/Inf inputs is undefined.
 *  - Every function returns AVQ_OK (0) or a negative avq_status; no C++
 *    exception crosses the boundary. avq_last_error() gives a message for the
 *    last failing call on the calling thread.
 *  - A single avq_index must not be used from two threads at once, nor by two
 *    overlapping calls on different streams: calls share per-index scratch.
 */
#ifndef AVQ_H
#define AVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AVQ_OK = 0,
    AVQ_EINVAL = -1, /* bad argument (shape, range, NULL)                   */
    AVQ_ESTATE = -2, /* call out of order (search before codes exist, ...)   */
    AVQ_ENOMEM = -3, /* device or host allocation failed                     */
    AVQ_EHIP = -4    /* a HIP runtime call or kernel launch failed           */
} avq_status;

enum { AVQ_LUT_F32 = 0, AVQ_LUT_U8 = 1 };
enum { AVQ_ETA_LIMIT = 0, AVQ_ETA_EXACT = 1, AVQ_ETA_EXPLICIT = 2 };

/* Largest reorder_k / k / leaves_to_search the wave-level selection supports. */
#define AVQ_MAX_SELECT 512

typedef struct avq_index avq_index; /* opaque; owned by the library */

typedef struct {
    int32_t d;    /* dimension, >= 2                                            */
    int32_t M;    /* number of PQ subspaces; d % M == 0 (Section 4.1)           */
    int32_t bits; /* 4 or 8; codewords per subspace k_c = 1 << bits             */
    float T;      /* threshold of the weight w(t) = I(t >= T), T >= 0 (Sec 3.2) */
    int32_t eta_mode; /* AVQ_ETA_LIMIT: eta = max(1, (d-1) u/(1-u)), u = (T/||x_i||)^2
                         (Eq. 3 used as a proxy, floored at 1 as Theorem 3.3 requires);
                         AVQ_ETA_EXACT: h_par/h_perp of Section 3.2;
                         AVQ_ETA_EXPLICIT: eta_explicit for every point.
                         In the first two modes eta is evaluated per point from
                         its own norm; u is clamped to 0.999; ||x|| = 0 -> 1.   */
    float eta_explicit;
    int32_t kmeans_iters;       /* Lloyd iterations for the PQ dictionaries      */
    int32_t encode_passes;      /* max coordinate-descent passes in avq_encode   */
    int32_t n_leaves;           /* 0 = flat index; > 0 = partition into leaves,
                                   PQ on residuals to the leaf centers          */
    int32_t leaf_kmeans_iters;  /* Lloyd iterations for the leaf centers         */
    int32_t borrow_x;           /* 0: avq_encode/avq_set_data copy x;
                                   1: keep the caller's device pointer, which
                                   must stay valid and unchanged for the life
                                   of the index                                  */
    uint64_t seed;              /* seeds the draw of the initial codewords       */
    int32_t leaf_aniso_iters;   /* partitioned index: 0 = the leaves are an l2 vector
                                   quantizer (Lloyd, nearest-center assignment);
                                   > 0: an anisotropic one (Section 4, Definition 4.1):
                                   after Lloyd, this many rounds of (assignment of the
                                   training rows to the center of smallest anisotropic
                                   loss, Theorem 4.2's center update), and avq_train /
                                   avq_encode assign every point to the leaf of smallest
                                   anisotropic loss                                  */
} avq_config;

/* Validates cfg and allocates an empty index on the current device.
 * AVQ_EINVAL: d < 2, M < 1, d % M != 0, bits not 4/8, T < 0, negative counts,
 * eta_mode out of range, eta_explicit < 1 in explicit mode. */
int avq_create(const avq_config *cfg, avq_index **out);
void avq_destroy(avq_index *idx);

/* Section 4 / 4.1, dictionary learning. x: device pointer [n_train][d].
 * Learns the leaf centers (if n_leaves > 0; Lloyd's algorithm on the full
 * vectors) and then the M dictionaries by Lloyd's algorithm per subspace
 * under the l2 loss -- the dictionary of Section 5.1, which the paper also
 * offers as the initialisation of Section 4.1 -- on x, or on the residuals to
 * the nearest leaf center. Initial codeword j of a dictionary is the datapoint
 * at index lo_j + h mod (hi_j - lo_j), [lo_j, hi_j) the j-th of k equal strata
 * of the n_train rows and h a splitmix64 hash of (seed, dictionary, j).
 * Distances and means are fp64; an empty cluster keeps its center.
 * Needs n_train >= max(k_c, n_leaves). Synchronises the stream. */
int avq_train(avq_index *idx, const float *x, int64_t n_train, void *hip_stream);

/* Section 4.1, partition-assignment step, for every row of x (device pointer
 * [n][d]): start from the l2-nearest codeword in each subspace, then cyclic
 * coordinate descent over the subspaces, each time taking the codeword that
 * minimises eta*||r_par||^2 + ||r_perp||^2 of the whole vector (Section 3.2)
 * with the others fixed, lowest index on equal loss, until a pass changes
 * nothing or encode_passes passes are done. Arithmetic is fp64. With leaves,
 * x~ = center(leaf(x)) + PQ(residual) and the loss is taken against x itself.
 * Replaces any previous database: stores the codes in the library's private
 * blocked layout and x (copied or borrowed) for exact re-scoring.
 * Needs dictionaries (avq_train or avq_set_codebooks). 0 < n < 2^31 - 512.
 * Synchronises the stream. */
int avq_encode(avq_index *idx, const float *x, int64_t n, void *hip_stream);

/* Section 4.2, codeword-update step for all dictionaries at once, with the
 * codes of the last avq_encode / avq_set_database held fixed (Appendix 7.5):
 * the anisotropic loss sum_i eta_i*||r_par,i||^2 + ||r_perp,i||^2 is a convex
 * quadratic in the stacked codewords; its normal equations
 *   (diag(count) + sum_i w_i s_i s_i^T) c = sum_i eta_i s_i,
 *   w_i = (eta_i - 1)/||x_i||^2, s_i = x_i's coordinates placed at the slots
 *   of the codewords point i uses,
 * are solved by conjugate gradients from the current dictionaries, without
 * forming the matrix (one pass over x per iteration), in fp64, until
 * ||residual|| <= tol*||rhs|| or max_iters iterations. A codeword no point
 * uses keeps its value. x: device [n][d], the rows the codes were made from
 * (n must equal avq_size). The dictionaries are replaced in place (rounded to
 * fp32); the stored codes stay as they are, so alternate with avq_encode to
 * iterate Section 4.2. iters_out / rel_residual_out (host, may be NULL):
 * iterations done and ||residual||/||rhs|| at exit.
 * On a partitioned index x~_i = center(leaf(i)) + codewords, the loss still
 * taken against x_i: same matrix, right-hand side sum_i B_i^T A_i (x_i - center),
 * A_i v = v + w_i x_i (x_i^T v). AVQ_ESTATE: no codes yet.
 * Allocates scratch with hipMalloc; synchronises the stream. */
int avq_update_codebooks(avq_index *idx, const float *x, int64_t n, int32_t max_iters, double tol,
                         int32_t *iters_out, double *rel_residual_out, void *hip_stream);

/* Theorem 4.2 for the leaf centers of a partitioned index, with the leaf
 * assignment of the last avq_encode / avq_set_database held fixed: every center
 * becomes the minimiser of the anisotropic loss of its members,
 *   c* = (sum_i A_i)^-1 sum_i eta_i x_i,  A_i = I + w_i x_i x_i^T,
 * (the joint update of Appendix 7.5 with one dictionary whose codewords are the
 * centers and whose codes are the assignments; same conjugate-gradient solve,
 * fp64). A leaf without members keeps its center. x: device [n][d], n must equal
 * avq_size. The stored residual codes refer to the old centers: follow with
 * avq_encode (and avq_train's dictionaries may be refreshed with
 * avq_update_codebooks afterwards) to iterate Section 4. AVQ_EINVAL on a flat
 * index; AVQ_ESTATE without a database. Allocates scratch; synchronises. */
int avq_update_leaf_centers(avq_index *idx, const float *x, int64_t n, int32_t max_iters, double tol,
                            int32_t *iters_out, double *rel_residual_out, void *hip_stream);

/* The query path (Sections 2.2.2 and 4.1 plus exact re-scoring).
 * queries: device [nq][d]; ids_out: device int32 [nq][k]; scores_out: device
 * fp32 [nq][k]. Steps, all on the GPU:
 *  (leaves only) score every leaf center by <q, center> and keep the
 *    leaves_to_search best;
 *  build the tables L[m][j] = <q^(m), c_j^(m)> in fp32 (fma chain over the
 *    subspace's dimensions in index order);
 *  lut_mode AVQ_LUT_U8: quantise them per query to 8 bits: lo_m = min_j L,
 *    R = max_m(max_j L - lo_m), code = clamp(rne((L - lo_m) * (255/R)), 0, 255),
 *    scale = R/255, bias = sum_m lo_m (R = 0: all codes 0, scale 0);
 *  ADC: score every scanned point by the sum of its M table entries (fp32:
 *    the two entries of a packed 4-bit byte are added first, then bytes are
 *    accumulated in order; 8-bit tables: exact integer sum). With leaves the
 *    score is s + <q, center> (fp32) or fma(acc, scale, bias + <q, center>);
 *  keep the R = reorder_k best by (score descending, id ascending). Batches
 *    (36 queries or more) with fp32 tables on a flat index of 4-bit codes do
 *    not score every point in fp32: the 8-bit tables are built as well, the
 *    integer sums of all points are formed on the matrix cores, every point
 *    whose sum is within M + slack units of the R-th best sum is kept (the
 *    rounding of the 8-bit tables moves a sum by at most M/2 units, so no
 *    other point can be among the R best by fp32 score), and only those are
 *    scored in fp32, in the order of additions given above. The R best and
 *    their scores are exactly those of a full fp32 scan. (On large indexes
 *    that scan, also when the search itself uses 8-bit tables, does not keep
 *    sorted lists: it compares against a bound guessed from a sample of the
 *    points and checked afterwards; a query whose guess fails is scanned
 *    again, so results never depend on it.) Large batches on a partitioned
 *    index of 4-bit codes (100000 (query, probed leaf) pairs or more, 16
 *    leaves or more per query; see avq_set_tuning) are regrouped by leaf: a leaf's codes are scored once per 32 of the queries
 *    that probe it (8-bit tables, matrix cores), every point whose estimate
 *    fma(sum, scale, bias + <q, center>) can reach the R-th best score of the
 *    query's first few leaves is kept, and the kept points are scored per
 *    query as above (fp32 tables: fp32 sums of the points within the rounding
 *    margin); same results. A handful of queries on a flat index (up to 35 with
 *    4-bit codes, up to 8 with 8-bit codes) and batches on a flat index of 8-bit
 *    codes do not score every point either, where the code size has the kernels
 *    for it (8, 13, 25 or 32 code bytes per point): the full scan sums 8-bit
 *    (batches: 6-bit) images of the table entries, whose distance from the score is
 *    bounded, and records the largest sum of every block of 256 points; the blocks
 *    whose largest sum is within that bound of the R-th largest block maximum are
 *    scored exactly (same order of additions), and the points at or above the lower
 *    bound of the R-th best score are ranked. Up to 80 queries on a partitioned
 *    index of 4-bit codes (same code sizes) score the blocks of their probed leaves
 *    exactly, keep every block's best key, and score the R blocks with the largest
 *    of those again for the points at or above the R-th largest. Same results,
 *    whatever the data;
 *  re-score those exactly, <q, x_i> as an fp32 fma chain in index order, and
 *    return the k best in the same order.
 * reorder_k == 0: no re-scoring; the k best ADC candidates are returned with
 * their ADC scores (8-bit tables, flat index: fma(acc, scale, bias)).
 * Rows with fewer than k candidates are padded with id -1, score -inf.
 * AVQ_EINVAL: nq < 1, k < 1, reorder_k != 0 and < k, k or reorder_k >
 * AVQ_MAX_SELECT, k > n, bad lut_mode, leaves_to_search outside
 * [1, min(n_leaves, AVQ_MAX_SELECT)] on a partitioned index.
 * AVQ_ESTATE: no codes yet. Does not synchronise (scratch may be grown with
 * hipMalloc on the first call of a given size). */
int avq_search(avq_index *idx, const float *queries, int32_t nq, int32_t k, int32_t reorder_k,
               int32_t lut_mode, int32_t leaves_to_search, int32_t *ids_out, float *scores_out,
               void *hip_stream);

/* avq_search for callers that cannot allocate device memory: code that runs under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same
 * results as avq_search for the same arguments, on a flat index, for a handful
 * of queries per call: it runs the launches avq_search uses for up to 35 queries
 * (block maxima or block bounds of the whole code array, selection of the blocks
 * that matter, exact scores of those, exact re-scoring), and takes every scratch
 * buffer of those kernels (tables, block maxima, listed blocks, candidate keys) from one array of
 * AVQ_NOALLOC_SCRATCH_BYTES that is part of the library's code object: each GPU
 * the library is loaded on holds its own copy from load time until the process
 * ends. The call itself allocates nothing, frees nothing, records no events and
 * does not synchronise; the array's address on the current device is looked up
 * once, on the first call. queries / ids_out / scores_out: device pointers as
 * for avq_search.
 * AVQ_EINVAL: a partitioned index; nq > AVQ_NOALLOC_MAX_QUERIES; a request whose
 * scratch (8 to 16 bytes per query and 256 stored points, plus 2 KiB per query
 * and unit of reorder_k, plus the tables) exceeds the array -- the message
 * states the bytes needed; the argument errors of avq_search.
 * All calls on one GPU share that GPU's array, whatever the index or stream: two
 * calls that overlap in time on one GPU race; issue them on one stream or order
 * them with events. The array keeps the previous call's contents; nothing in it
 * needs clearing between calls (every kernel writes what the next one reads). */
#define AVQ_NOALLOC_SCRATCH_BYTES (64u << 20)
#define AVQ_NOALLOC_MAX_QUERIES 32
int avq_search_noalloc(avq_index *idx, const float *queries, int32_t nq, int32_t k, int32_t reorder_k,
                       int32_t lut_mode, int32_t *ids_out, float *scores_out, void *hip_stream);

/* Section 1's definition, exactly: the k points with the largest <q, x_i>
 * (fp32 fma chain in index order; ties by lower id) among all n stored
 * points. Same argument layout as avq_search. Ground truth for recall. */
int avq_brute_force(avq_index *idx, const float *queries, int32_t nq, int32_t k,
                    int32_t *ids_out, float *scores_out, void *hip_stream);

/* ---- injection and inspection (used to test every stage on its own) ---- */

/* Dictionaries [M][k_c][d/M] fp32, host or device. */
int avq_set_codebooks(avq_index *idx, const float *codebooks);
int avq_get_codebooks(avq_index *idx, float *codebooks_out);
/* Leaf centers [n_leaves][d] fp32, host or device (partitioned index only). */
int avq_set_leaf_centers(avq_index *idx, const float *centers);
int avq_get_leaf_centers(avq_index *idx, float *centers_out);
/* Install a database without encoding it. x: device [n][d] (copied or
 * borrowed as cfg.borrow_x says; may be NULL, then reorder_k must be 0 and
 * avq_brute_force is unavailable). packed: host or device [n][ceil(M*bits/8)],
 * the logical code layout: 8-bit codes one byte per subspace; 4-bit codes two
 * per byte, subspace m in byte m/2, even m in the low nibble. leaf_assign:
 * host or device int32 [n] (partitioned index) or NULL (flat). */
int avq_set_database(avq_index *idx, const float *x, const uint8_t *packed,
                     const int32_t *leaf_assign, int64_t n, void *hip_stream);
/* Codes in the logical layout above / the leaf of every point. Host or device. */
int avq_get_codes(avq_index *idx, uint8_t *packed_out);
int avq_get_leaf_assign(avq_index *idx, int32_t *assign_out);
int64_t avq_size(const avq_index *idx); /* n, or 0 */

/* The tables avq_search would use. lut_out: device fp32 [nq][M][k_c]
 * (AVQ_LUT_F32) or uint8 [nq][M][k_c] (AVQ_LUT_U8); scale_out/bias_out: device
 * fp32 [nq], written in U8 mode only (may be NULL otherwise). */
int avq_debug_lut(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode,
                  void *lut_out, float *scale_out, float *bias_out, void *hip_stream);
/* ADC score of every stored point, flat index only, produced by the scan
 * kernels that form these sums in avq_search (fp32: the kernel over fp32
 * tables, whose order of additions every fp32 score avq_search returns
 * follows; 8-bit tables: the matrix-core kernel where it applies).
 * scores_out: device [nq][n], fp32 (AVQ_LUT_F32) or int32 integer sums
 * (AVQ_LUT_U8). */
int avq_debug_adc_scores(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode,
                         void *scores_out, void *hip_stream);
/* Leaf selection alone: leaf_ids_out int32 [nq][L], leaf_ip_out fp32 [nq][L],
 * device pointers; best leaf first. Up to 32 queries run the kernels that
 * avq_search uses for a few queries, more run those of its batch path. */
int avq_debug_leaf_select(avq_index *idx, const float *queries, int32_t nq, int32_t L,
                          int32_t *leaf_ids_out, float *leaf_ip_out, void *hip_stream);

/* Measurement aid: reads the stored code array once (flat or partitioned), with
 * the loads and the launch shape of the single-query ADC scan of Section 4.1 and
 * none of its table lookups. words_out: device uint32 [ceil(n_slots/256)], one
 * per block of 256 stored points: the xor of the block's 64*NB code words (a
 * word holds the same code byte of four consecutive points). Its duration is
 * the floor for a scan of this index on this machine. *n_blocks_out (host, may
 * be NULL) receives the number of blocks; words_out may be NULL to query it. */
int avq_debug_stream_codes(avq_index *idx, uint32_t *words_out, int64_t *n_blocks_out, void *hip_stream);

/* Measurement aid: launches one kernel of the single-query / small-batch search `reps` times back to back on
 * the stream, after the tables it needs (so that one event pair around the call times reps launches and nothing
 * else). part 0: the full scan of Section 4.1's sums as avq_search runs it for nq <= 35 queries (block maxima of
 * 8-bit table sums, or of the scores where the code size has no such kernel); part 1: the code stream alone
 * (avq_debug_stream_codes' kernel); part 2: the scan's table lookups and additions alone, in its launch shape,
 * on made-up code words (specialised code sizes only: AVQ_EINVAL otherwise). Results go to scratch. Flat index,
 * nq <= 64. May allocate scratch. */
int avq_debug_scan_parts(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode, int32_t part,
                         int32_t reps, void *hip_stream);

/* Measurement aid: after an avq_search with fp32 tables that took its candidates
 * from the 8-bit-table scan (see "scan_prefilter" below): counts_out[0] = the
 * number of queries of that call that were scanned again with fp32 tables
 * (-1 if no such search has happened), of which counts_out[1] because the scan
 * kept more points than the refinement holds, counts_out[2] because the bound
 * guessed from the sample was too high, counts_out[3] for other reasons (no
 * usable margin, the "scan_prefilter" = 2 test mode). Synchronises the device. */
int avq_debug_unverified_queries(avq_index *idx, int32_t *counts_out /* [4] */);

/* eta of Section 3.2 for one norm, on the host (no GPU needed):
 * mode AVQ_ETA_LIMIT or AVQ_ETA_EXACT as in avq_config. */
double avq_eta(int32_t d, double T, double norm, int32_t eta_mode);

/* Launch-shape overrides for experiments; 0 restores the built-in choice.
 * name: "scan_target_wgs" (workgroups the batch scan aims for; for small batches
 * the most workgroups per query of the block-maxima scan), "scan_waves"
 * (waves per scan workgroup), "scan_qt" (queries per tile), "small_batch_max"
 * (v > 0: batches of fewer than v queries on a flat index take the block-maxima
 * path; 1 disables that path; built in with 4-bit codes: from measured costs of the two paths, about 44 at 1.2 million
 * points, 21 at 10 million, 200 at 100000, thousands on indexes of a few thousand points; with 8-bit codes 9, or where batches take their block
 * bounds sixteen queries at a time, up to 33 while queries x blocks of 256 points stay below 120000, and three in any case; on a partitioned index: fewer than v
 * queries take the block maxima of their probed leaves; built in: 81), "small_batch_impl" (0: built in: where
 * the code size has the kernels for it (8, 13, 25 or 32 code bytes per point) the full scan records, per block
 * of 256 points, the largest sum of 8-bit images of the table entries -- a bound of the block's scores -- and
 * only the blocks whose bound can reach the R-th best score are scored exactly; 2: the full scan always records
 * exact block maxima; 1: that algorithm as three separate kernels, and on a partitioned index the scan with one
 * workgroup per query whatever the batch size), "scan_mfma"
 * (1: batches with 8-bit tables on 4-bit codes use the LDS-table scan instead
 * of the matrix-core scan; for that scan "scan_target_wgs" counts waves),
 * "scan_prefilter" (1: batches with fp32 tables on a flat index of 4-bit codes
 * are scanned with the fp32 tables directly instead of taking candidates from
 * the matrix-core scan over the 8-bit tables and re-scoring them in fp32;
 * 2: candidates are taken as usual, but every odd query is treated as one
 * whose candidates cannot be used and is scanned again with fp32 tables),
 * "prefilter_cap" (candidate keys that scan may keep per query and chunk of
 * the index; a query that needs more is scanned again with fp32 tables),
 * "scan_sample" (1: that candidate scan keeps lists and raises its bounds as
 * it goes, instead of scanning against bounds guessed from a sample of the
 * index and checked afterwards; 2: the sample itself is scanned with sorted
 * lists instead of per-class maxima), "bound_leaves" (batches on a partitioned
 * index: how many of a query's best leaves are scanned first, one query at a
 * time, for the bound that the scan of all leaves, regrouped by leaf, runs
 * against; "scan_prefilter" = 1 also switches that regrouped scan off,
 * "prefilter_cap" is its kept keys per query), "group_min_pairs" (queries x
 * probed leaves from which a batch on a partitioned index is regrouped by
 * leaf; built in: 100000, below that one workgroup per query is faster),
 * "select_split" (block-maxima path: 1: one workgroup per query selects the
 * blocks to score exactly; v >= 2: several workgroups per query do, v blocks
 * of the index each; built in: 8192 each for up to 16 queries on an index of
 * 32768 blocks of 256 points or more), "rerank_split" (1: the exact
 * re-scoring of a query's candidates is done by one workgroup; v >= 2: by
 * several, v candidates each; built in: 64 each for up to 16 queries whose
 * reorder_k rows do not fit one workgroup's LDS at once), "bound_bits" (batches
 * of 8-bit codes: 6, 7 or 8 bits per entry of the byte tables whose sums bound
 * a block's scores; built in: 7), "stream_loads" (the scan of the whole code
 * array for one or a few queries: 1 = plain loads, 2 = nontemporal loads and
 * one block of 256 points per wave; built in: 2 when the code array exceeds
 * 256 MB, the Infinity Cache, and the call has one or two queries, or up to
 * eight over more than 1 GiB of codes; else 1).
 * Results never depend on these. Returns
 * AVQ_EINVAL for an unknown name. */
int avq_set_tuning(avq_index *idx, const char *name, int32_t value);

/* Per-stage GPU time of avq_search, measured with HIP events recorded on the
 * caller's stream around each stage's kernel (one event pair per stage per
 * call while enabled; off by default). avq_profile_read waits for the recorded
 * events, then writes the summed milliseconds and the number of launches per
 * stage into ms_out[AVQ_N_STAGES] / launches_out[AVQ_N_STAGES] (host pointers);
 * reset != 0 forgets the records. */
enum { AVQ_STAGE_LEAF = 0,   /* leaf selection                                           */
       AVQ_STAGE_LUT = 1,    /* table build                                              */
       AVQ_STAGE_SCAN = 2,   /* the scan over all codes (batch: with candidate lists;
                                small batch: block maxima only)                          */
       AVQ_STAGE_MERGE = 3,  /* merge of per-chunk lists / selection of the best blocks  */
       AVQ_STAGE_FINAL = 4,  /* exact re-scoring and final top-k                         */
       AVQ_STAGE_RESCAN = 5, /* small batch: scan of the selected blocks; batches: scoring
                                of the kept points and the queries scanned again         */
       AVQ_STAGE_SAMPLE = 6, /* batches through the candidate scan: margins, the launch
                                over a sample of the blocks and the bounds guessed from it;
                                partitioned batches regrouped by leaf: margins, bounds from
                                each query's first leaves, regrouping                     */
       AVQ_N_STAGES = 7 };
int avq_profile_enable(avq_index *idx, int32_t on);
int avq_profile_read(avq_index *idx, double *ms_out, int64_t *launches_out, int32_t reset);

const char *avq_last_error(void);
const char *avq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AVQ_H */
