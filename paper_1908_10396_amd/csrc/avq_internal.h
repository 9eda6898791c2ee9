// Host-side declarations shared by the translation units of libavq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <string>
#include <vector>

#include "../../include/avq.h"

namespace avq {

typedef unsigned long long u64;

// Points are stored in blocks of 256: 64 lanes x 4 points per lane.
constexpr int kBlockPoints = 256;
// Dynamic LDS a kernel may ask for: the CU's 160 KiB less room for small static arrays.
constexpr size_t kMaxDynLds = 159 * 1024;

void set_error(const char *fmt, ...);

#define AVQ_HIP(call)                                                                   \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess) {                                                         \
            ::avq::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),     \
                             __FILE__, __LINE__);                                       \
            return e_ == hipErrorOutOfMemory ? AVQ_ENOMEM : AVQ_EHIP;                    \
        }                                                                               \
    } while (0)

#define AVQ_TRY(call)              \
    do {                           \
        int rc_ = (call);          \
        if (rc_ != AVQ_OK) return rc_; \
    } while (0)

// Raises a kernel's dynamic-LDS limit once per device; safe to call from several threads
// (the attribute is per device and setting it twice is harmless).
struct LdsLimitOnce { std::atomic<uint64_t> devices{0}; };
inline int set_lds_limit(const void *kernel, size_t bytes, LdsLimitOnce *once)
{
    int dev = 0;
    AVQ_HIP(hipGetDevice(&dev));
    const uint64_t bit = 1ull << (dev & 63);
    if (once->devices.load(std::memory_order_acquire) & bit) return AVQ_OK;
    AVQ_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    once->devices.fetch_or(bit, std::memory_order_release);
    return AVQ_OK;
}

// Grow-only device buffer.
struct DevBuf {
    void *p = nullptr;
    size_t cap = 0;
    int reserve(size_t bytes);
    void release();
    template <class T> T *as() const { return (T *)p; }
};

// ---- lut.hip ---------------------------------------------------------------
// L[q][m][j] = <q^(m), c_j^(m)> (fp32 fma chain); u8 mode also writes the
// quantised tables and per-query scale / bias.
int launch_lut(const float *queries, int nq, const float *codebooks, int d, int M, int kc,
               float *lut_f32, uint8_t *lut_u8, float *scale, float *bias, hipStream_t st);

// ---- scan.hip --------------------------------------------------------------
// What relates the 8-bit sums of the block-bound kernel to fp32 scores (see scan.hip): the sum of the byte
// positions' smallest entries, the sum of their largest magnitudes, and the units per score unit.
struct BoundMeta { double sum_lo, amax; float c; int32_t pad; };
struct ScanParams {
    const uint8_t *codes; // blocked layout
    int64_t n_blocks;     // blocks in the whole index
    int32_t n_valid;      // flat: ids >= n_valid are padding
    const int32_t *perm;  // partitioned: slot -> id, -1 = padding
    const float *lut;     // [B][M][kc]
    // single-query kernels over 16-entry fp32 tables: when set, every workgroup computes the
    // table entries itself (paper Section 4.1: <q^(m), c_j^(m)>, the same fma chain as the
    // table kernel) and lut is not read
    const float *fuse_queries;   // [B][fuse_d]
    const float *fuse_codebooks; // [M][16][fuse_d / M]
    int32_t fuse_d;
    const uint8_t *lut8;  // [B][M][kc]
    const float *scale;   // [B]
    const float *bias;    // [B]
    int32_t B, M, bits, NB;
    int32_t R, ns;
    int32_t n_chunks, blocks_per_chunk, n_tiles; // flat
    const int32_t *leaf_ids;                     // partitioned: [B][Lp]
    const float *leaf_ip;                        // [B][Lp]
    const int32_t *leaf_blk;                     // [n_leaves + 1] first block of each leaf
    int32_t Lp;
    const u64 *block_keys; // block-list mode: [B][64*ns], the keys of the blocks to scan
    u64 *block_max;        // block-max kernel: [B][n_blocks]; rescan of listed blocks: best key of the j-th listed block
    // block-bound scan (small batches, specialised code sizes): [B][n_blocks] block maxima of the 8-bit sums;
    // [B] what the margin of those sums follows from (fp32 tables); lut_out (may be NULL): when the table kernel of
    // that scan computes the fp32 tables itself (fuse_queries), [B][M][16] receives them
    uint32_t *block_bound;
    struct BoundMeta *bound_meta;
    float *lut_out;
    uint8_t *bound_tbl;    // [B][NB][256] the byte tables of the block-bound scan (made by launch_bound_tables);
                           // bound_tile = 16: [ceil(B / 16)][NB][256][16], the tables of 16 queries side by side
    int32_t bound_tile;    // 0 or 16
    int32_t bound_levels;  // largest table entry: 255 (0: 255), or 63 for the batch scan, which adds entries as packed bytes
    int32_t bound_shift;   // 8-bit tables on 8-bit codes: the byte tables are the 8-bit tables >> bound_shift (0 or 2)
    // selection of the blocks over several workgroups per query (a few queries on a large index), else NULL:
    // sel_hist [B][8192] scratch, sel_split_per blocks per workgroup (1 .. 8192)
    uint32_t *sel_hist;
    int32_t sel_split_per;
    u64 *partial;         // [n_tiles*QT][n_chunks][64*ns]
    u64 *lists_ws;        // NULL: candidate lists in LDS; else scratch [grid][waves][QT][64*ns]
    // matrix-core kernel, both zeroed before the launch: [B] best known bound of the R-th best
    // ordering value per query; [B][n_chunks] every wave's ceil(R/group)-th best
    uint32_t *thr_shared, *kth_shared;
    int32_t group;        // chunks per threshold group
    int32_t bounds_only;  // matrix-core kernel: publish bounds in thr_shared, write no lists (sampling launch)
    int32_t block_stride; // matrix-core kernel: > 1: visit only every block_stride-th block of a chunk
    // matrix-core kernel, sampling launch without lists: [B][n_chunks][32] ordering values (0: none), the best sum of
    // each of the 32 disjoint point classes (lane half x accumulator) of every wave; nothing else is written
    uint32_t *sample_max;
    int32_t fixed_bound;  // matrix-core kernel, candidate mode: thr_shared holds bounds that are not raised; no lists
    // matrix-core kernel, candidate mode (cand_keys != NULL): every point whose sum is within
    // cand_margin[q] (< 0, or no array: 0) of the bound is appended, as a 32-bit chunk-local key, to
    // cand_keys[q][chunk][cand_cap]; cand_cnt[q][chunk] = how many (cand_cap + 1: overflowed)
    uint32_t *cand_keys, *cand_cnt;
    const int32_t *cand_margin;
    int32_t cand_cap;
    // matrix-core kernel over a partitioned index (item_list != NULL; fixed bounds, no lists): wave w
    // takes item_list[w] = leaf << 11 | tile, i.e. the blocks of that leaf against the 32 entries from
    // qlist[leaf_off[leaf] + 32 * tile] on (leaf_cnt[leaf] of them in all; an entry is query << 9 | slot
    // of the leaf in the query's probe list). A point is kept when fma(sum, scale[q], bias[q] +
    // leaf_ip[q][slot]) can still reach item_bound[q] (less cand_margin[q] units when given): its key goes
    // to kept[q][kept_cap] as (slot << 21 | leaf) << 32 | 32-bit key (ids count from the leaf's first
    // slot), kept_cnt[q] counts them (beyond kept_cap: overflowed). max_items bounds *n_items.
    const uint32_t *item_list, *n_items, *qlist, *leaf_off, *leaf_cnt;
    const uint32_t *item_bound; // [B] ordering values of fp32 scores (ord_from_f32), 0: no bound
    u64 *kept;
    uint32_t *kept_cnt;
    int32_t kept_cap, max_items;
    int32_t leaf_stride;  // partitioned scans: row stride of leaf_ids / leaf_ip when it is not Lp (0: Lp)
    int32_t nt_loads;     // single-query block bounds: the code stream with nontemporal loads (arrays beyond the Infinity Cache)
    int32_t max_wgs;      // block-max kernels: workgroups per query at most (0 = built-in); waves loop beyond it
    // flat scan of a compacted query list whose length only the device knows (NULL: all B
    // queries are live): the kernel derives tiles and chunks from *active_queries, n_chunks is
    // then the most chunks a tile may be cut into, and the grid is scan_dynamic_grid()
    const uint32_t *active_queries;
    void *scores_out;     // debug: [B][score_stride] fp32 or int32, else NULL
    int64_t score_stride;
};
// A launch whose number of live query tiles is known only on the device: about kDynamicItems
// workgroups share the work, so a few tiles are cut into many chunks (every one of them still
// spreads over the chip) and many tiles into few; never more than max_chunks, never fewer than 1.
// tiles * chunks <= max(kDynamicItems, tiles): a grid of max(kDynamicItems, all tiles) covers it.
constexpr int kDynamicItems = 1024;
__host__ __device__ inline int scan_dynamic_chunks(int tiles, int max_chunks)
{
    int c = tiles > 0 ? kDynamicItems / tiles : 1;
    c = c < max_chunks ? c : max_chunks;
    return c > 1 ? c : 1;
}
struct ScanShape { int qt; int waves; size_t lds_bytes; bool lists_global; };
// Picks query-tile size and waves per workgroup that fit LDS. qt_hint/waves_hint 0 = auto.
int scan_pick_shape(int NB, int bits, bool u8, int ns, int B, bool single, int qt_hint, int waves_hint,
                    ScanShape *out);
// SCAN_CHUNK: flat index, grid = query tiles x chunks; SCAN_LEAVES: partitioned index, one
// workgroup per query over its probed leaves; SCAN_BLOCKLIST: flat index, one workgroup per
// query over the blocks named by block_keys.
enum { SCAN_CHUNK = 0, SCAN_LEAVES = 1, SCAN_BLOCKLIST = 2 };
int launch_scan(const ScanParams &p, bool u8, int mode, const ScanShape &shape, hipStream_t st);
// The same flat scan for 4-bit codes and 8-bit tables on the matrix cores: one wave per
// (32 queries, chunk); fills partial[q][chunk][64*ns]. scan_mfma_plan sets n_tiles, n_chunks
// and blocks_per_chunk (target_waves 0 = built-in); lists_ws needs scan_mfma_lists_bytes.
bool scan_mfma_supported(int NB, int bits);
void scan_mfma_plan(int B, int64_t n_blocks, int target_waves, ScanParams *p);
size_t scan_mfma_lists_bytes(const ScanParams &p);
// Fills *sample with the launch that guesses the bounds of a fixed-bound scan `full` (same
// scratch; run it first, with thr_shared and kth_shared cleared). false: the index is too small.
bool scan_mfma_sample_plan(const ScanParams &full, ScanParams *sample);
int launch_scan_mfma(const ScanParams &p, hipStream_t st);
// Whether the small-batch kernels can compute their own tables (fuse_* above).
bool small_batch_can_fuse_tables(int bits, int M, int d, bool u8);
// Full scan that only records the best key of every block (block_max[q][blk]).
int launch_block_max(const ScanParams &p, bool u8, int waves, hipStream_t st);
// Partitioned index, 4-bit codes, specialised code sizes: bound[q] = ordering value of the R-th best score
// (tables as in `u8`) among the points of the first p.Lp leaves of row q of leaf_ids (row stride
// leaf_stride) that fit its LDS, 0 if fewer than R; needs perm, leaf_blk, leaf_ip, lut / lut8, scale, bias.
// max_leaf_blocks <= kLeafBoundMaxBlocks.
constexpr int kLeafBoundMaxBlocks = 96;
int launch_leaf_bound(const ScanParams &p, bool u8, int max_leaf_blocks, int mean_leaf_blocks, uint32_t *bound,
                      hipStream_t st);
// reads the blocked code array once, in the single-query scan's launch shape; out[blk] = xor of the block's words
int launch_stream_codes(const uint8_t *codes, int64_t n_blocks, int NB, uint32_t *out, hipStream_t st, bool nt = false);
// Small batches, after launch_block_max: block selection, scan of the selected blocks,
// final selection with exact re-scoring and output (three kernels).
struct SmallMeta { u64 t1; uint32_t n_sel; uint32_t n_cand; };
struct FinishParams {
    const float *x;        // [n][d], may be NULL when reorder == 0
    const float *queries;  // [B][d]
    int32_t d, k, reorder;
    int32_t stage_rows;    // rows of x staged in LDS per pass of the re-scoring (small_finish_stage_rows)
    u64 *cand;             // scratch [B][cand_stride], cand_stride >= 256 * R
    int64_t cand_stride;
    int32_t *sel_blk;      // scratch: the selected blocks, [B][R] (block maxima) or [B][n_blocks] (block bounds)
    SmallMeta *meta;       // scratch [B]
    int32_t *ids_out;      // [B][k]
    float *scores_out;     // [B][k]
    // block-bound path only: what the final kernel needs to rebuild a candidate list that overflowed
    // (more than cand_stride points at or above the bound: heavy duplication). NULL block_max: never.
    const u64 *block_max;        // [B][n_blocks], entry j = best key of the j-th listed block
    int64_t n_blocks;
    int32_t n_valid, NB, M, bits, u8;
    const uint8_t *codes_logical; // [n][NB]
    const float *lut;             // [B][M][kc] fp32 tables (u8 == 0)
    const uint8_t *lut8;          // [B][M][kc] 8-bit tables (u8 == 1)
    // exact re-scoring over several workgroups per query (a few queries, many or long rows): rerank_rows > 0
    // candidates per workgroup (at most 1024, their rows must fit LDS), fin_out [B][R] and fin_n [B][2] scratch
    int32_t rerank_rows;
    u64 *fin_out;
    uint32_t *fin_n;
};
int small_finish_stage_rows(const ScanParams &p, int d, bool u8);
// The same search through block maxima of 8-bit sums (bounds, not scores: scan.hip): specialised code
// sizes only. launch_bound_tables -> launch_block_bound -> launch_select_bound_blocks -> launch_rescan_listed -> launch_small_final.
bool block_bound_supported(int NB, int bits);
int launch_bound_tables(const ScanParams &p, bool u8, hipStream_t st);
// lookups_only: the same lookups in the same launch shape on made-up code words, no code stream (measurement)
int launch_block_bound(const ScanParams &p, int waves, hipStream_t st, bool lookups_only = false);
// the batch form: tiles of 16 queries x chunks of p.blocks_per_chunk blocks (block_bound_tile_chunk); needs
// bound_tile = 16, bound_levels = 63 (and bound_shift = 2 with 8-bit tables)
int block_bound_tile_chunk(int64_t n_blocks, int B);
int launch_block_bound_tile(const ScanParams &p, hipStream_t st);
int launch_select_bound_blocks(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st);
int launch_rescan_listed(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st);
int launch_small_select(const ScanParams &p, const FinishParams &f, hipStream_t st);
int launch_small_rescan(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st);
// A handful of queries on a partitioned index (4-bit codes, specialised code sizes): exact block maxima over the
// blocks of the probed leaves (p.leaf_ids / leaf_ip / leaf_blk / perm, p.Lp leaves per query), listed per query in
// probe order; selection of the R blocks with the largest maxima (positions in the list to f.sel_blk[q][R], f.meta);
// the points of those at or above t1 to f.cand. launch_small_final finishes (keys carry fp32 scores and point ids).
struct LeafSmallBuffers {
    u64 *best;          // [B][stride]
    int32_t *blk;       // [B][stride]
    float *ip;          // [B][stride]
    uint32_t *n_listed; // [B]
    int64_t stride;     // at least the blocks of any query's probed leaves
};
bool leaf_small_supported(int NB, int bits);
int launch_leaf_block_max(const ScanParams &p, bool u8, const LeafSmallBuffers &b, hipStream_t st);
int launch_select_listed_blocks(const ScanParams &p, const FinishParams &f, const LeafSmallBuffers &b, hipStream_t st);
int launch_rescan_leaf_blocks(const ScanParams &p, const FinishParams &f, bool u8, const LeafSmallBuffers &b, hipStream_t st);
int launch_small_final(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st);

// ---- select.hip ------------------------------------------------------------
// Merges the per-chunk lists of every query into one sorted list cand[q][64*ns].
// row_of / active (both NULL, or both set): query q's list goes to row row_of[q] of cand, only
// queries below *active are merged, and the lists are those of a scan with active_queries set
// (tile_queries per tile, at most n_chunks chunks; tile_queries 0: exactly n_chunks chunks).
int launch_merge_partials(const u64 *partial, int nq, int n_chunks, int ns, u64 *cand,
                          hipStream_t st, const int32_t *row_of = nullptr, const uint32_t *active = nullptr,
                          int tile_queries = 0);
// The R largest of n unsorted keys per query: out[q][64*ns] sorted descending.
int launch_select_keys(const u64 *keys, int nq, int64_t n, int ns, int R, u64 *out, hipStream_t st);
// Final stage. reorder != 0: exact <q, x_id> for the first R candidates, then top-k.
// reorder == 0: first k candidates; score decoded from the key (kind 0: fp32 key,
// kind 1: integer sum -> fma(acc, scale, bias)).
int launch_finalize(const u64 *cand, int ns, int nq, int R, int k, int reorder, int key_kind,
                    const float *x, int d, const float *queries, const float *scale,
                    const float *bias, int32_t *ids_out, float *scores_out, hipStream_t st);
int launch_brute_force(const float *x, int64_t n, int d, const float *queries, int nq, int k,
                       u64 *partial_ws, int n_chunks, u64 *cand_ws, int32_t *ids_out,
                       float *scores_out, hipStream_t st);
int brute_force_chunks(int64_t n, int nq);

// ---- refine.hip ------------------------------------------------------------
// fp32-table search through the 8-bit-table scan (flat index, 4-bit codes). The matrix-core scan
// in candidate mode (ScanParams::cand_*) keeps every point whose integer sum came within
// margin[q] of its bound for the R-th best; top[q][64*ns] = the R best integer sums of query q
// (merged over the chunks). Every sum differs from the exact one, in units of the query's
// scale, by at most M/2 (rounding of the table entries), so with margin[q] >= M + slack no
// other point can be among the R best by fp32 score: the kernel re-scores the kept points at
// or above (R-th best sum - margin) in fp32 (the scan's own order of additions) and writes the
// R best, sorted, to out[q][64*ns]. Queries without a usable margin or whose buffers
// overflowed are appended to fail_list (count in *fail_count, zeroed by the caller) and left to
// a plain fp32 scan. margin[q] comes from launch_prefilter_margin, before the scan.
struct RefineCandParams {
    // one of the two: top[q][64*ns], the R best integer sums (a scan that kept lists), or bound[q],
    // the ordering value of the fixed bound the scan used (then the kernel checks that R kept points
    // reach it, else the query fails, and finds the R-th best sum itself)
    const u64 *top;
    const uint32_t *bound;
    int32_t R, ns, nq, M, NB;
    int32_t n_chunks, cand_cap;
    int64_t chunk_points;        // points per chunk of the scan (ids in the 32-bit keys count from the chunk's first)
    const uint32_t *cand_keys, *cand_cnt;
    const int32_t *margin;
    const float *lut;            // NULL: rank the integer sums themselves (no margin, no re-scoring; margin and codes unused)
    const uint8_t *codes;        // logical [n][NB]
    u64 *out;
    int32_t *fail_list;
    uint32_t *fail_count;
    int32_t force_fail_odd;
};
int launch_prefilter_margin(const float *lut, const float *scale, int M, int NB, int nq, int32_t *margin, hipStream_t st);
int launch_refine_cand(const RefineCandParams &r, hipStream_t st);
// bound[q] = ordering value of the r-th key of the sorted list lists[q][64*ns] (0: fewer than r keys)
// bound[q] = the r-th largest of the S = n_chunks * 32 ordering values of query q in sample_max (0 if fewer are non-zero)
int launch_sample_bound(const uint32_t *sample_max, int S, int r, int nq, uint32_t *bound, hipStream_t st);
int launch_list_bound(const u64 *lists, int ns, int r, int nq, uint32_t *bound, hipStream_t st);
// The kept keys of the matrix-core scan over a partitioned index (ScanParams::kept): per query the R
// best by score, sorted, to out[q][64*ns]. The score of a kept point is fma(sum, scale, bias + leaf_ip)
// (lut == NULL, 8-bit-table search) or, with fp32 tables, the fp32 table sum plus leaf_ip, formed for
// the points whose 8-bit estimate is within margin[q] units of the R-th best estimate. Padding slots
// (perm < 0) are dropped. Queries whose buffer overflowed go to fail_list.
struct IvfRefineParams {
    const u64 *kept;
    const uint32_t *kept_cnt;
    int32_t kept_cap, R, ns, nq, M, NB, leaf_stride;
    const float *lut, *scale, *bias, *leaf_ip;
    const int32_t *margin, *leaf_blk, *perm;
    const uint8_t *codes; // logical [n][NB]
    u64 *out;
    int32_t *fail_list;
    uint32_t *fail_count;
    int32_t force_fail_odd;
};
int launch_ivf_refine(const IvfRefineParams &r, hipStream_t st);
// dst[c] = src[row[c]] for c < *count (rows of row_floats floats); grid sized for max_rows
int launch_gather_rows(const float *src, float *dst, const int32_t *row, const uint32_t *count, int max_rows,
                       int row_floats, hipStream_t st);

// ---- ivf.hip ---------------------------------------------------------------
// centers_t: [d][n_leaves] (transposed). Writes the L best leaves per query.
// The (query, probed leaf) pairs of a batch regrouped by leaf, for the matrix-core scan (see
// ScanParams::item_list). ws: group_by_leaf_words(...) 32-bit words of device scratch.
struct LeafGroups {
    uint32_t *leaf_cnt, *leaf_off, *item_off, *fill, *n_items, *qlist, *pos, *item_list; // pos[q][Lp]: the pair's place in its leaf's list
    uint32_t *cnt_wide; // the counters leaf selection adds to: leaf l's is cnt_wide[l * cnt_stride]
    int cnt_stride;
    int32_t max_items; // every 32 pairs of a leaf are an item: at most pairs / 32 + n_leaves of them
};
inline size_t group_by_leaf_max_items(int nq, int Lp, int n_leaves) { return ((size_t)nq * Lp + 31) / 32 + (size_t)n_leaves; }
size_t group_by_leaf_words(int nq, int Lp, int n_leaves);
// prepare (lays out ws, clears the counts) -> launch_leaf_select(..., g.cnt_wide, g.pos, g.cnt_stride) -> launch_group_by_leaf
int group_by_leaf_prepare(int nq, int Lp, int n_leaves, uint32_t *ws, LeafGroups *g, hipStream_t st);
int launch_group_by_leaf(const int32_t *leaf_ids, int nq, int Lp, int n_leaves, const LeafGroups &g, hipStream_t st);
// The same selection for a handful of queries (L <= 512): scores by many small workgroups into keys[nq][n_leaves]
// (scratch), then the L best per query.
int launch_leaf_select_few(const float *centers_t, int n_leaves, int d, const float *queries, int nq, int L, u64 *keys,
                           int32_t *leaf_ids, float *leaf_ip, hipStream_t st);
// leaf_cnt (optional): leaf_cnt[leaf * cnt_stride] is incremented once per selected (query, leaf) pair; leaf_pos
// (optional, [nq][L]): the count before the pair's own increment, i.e. its place among the pairs of that leaf
int launch_leaf_select(const float *centers_t, int n_leaves, int d, const float *queries, int nq,
                       int L, int32_t *leaf_ids, float *leaf_ip, hipStream_t st, uint32_t *leaf_cnt = nullptr,
                       uint32_t *leaf_pos = nullptr, int cnt_stride = 1);
int launch_transpose(const float *in, int rows, int cols, float *out, hipStream_t st);

// ---- layout.hip ------------------------------------------------------------
// logical [n][NB] -> blocked; slot_of[i] gives the slot of point i (NULL: slot = i).
int launch_to_blocked(const uint8_t *logical, int64_t n, int NB, const int32_t *slot_of,
                      uint8_t *blocked, int64_t n_slots, hipStream_t st);

// ---- train.hip -------------------------------------------------------------
// Lloyd on columns [col0, col0+dim) of x (row stride ld), optionally on residuals
// to resid_centers[resid_assign[i]]. centers: device [k][dim].
int kmeans_device(const float *x, int64_t n, int ld, int col0, int dim, int k, int iters,
                  uint64_t seed, uint32_t stream_id, const float *resid_centers,
                  const int32_t *resid_assign, float *centers, hipStream_t st);
int launch_assign_nearest(const float *x, int64_t n, int d, const float *centers, int k,
                          int32_t *assign, hipStream_t st);
// every row to the center of smallest anisotropic loss (fp64), lowest index on equal loss
int launch_assign_aniso(const float *x, int64_t n, int d, const float *centers, int k, int eta_mode, double T,
                        double eta_explicit, int32_t *assign, hipStream_t st);
// Joint update of all dictionaries with the codes fixed (anisotropic loss; conjugate gradients on
// the normal equations of the paper's Appendix 7.5, matrix-free, fp64). codes: logical [n][NB].
// scratch: pq_update_scratch_bytes(n, M*kc*ds, M*kc) bytes of device memory. Synchronises the stream.
size_t pq_update_scratch_bytes(int64_t n, int D, int slots);
// centers / assign (both NULL or both set): residual quantization, x~ = centers[assign[i]] + codewords, the loss
// against x itself. bits 32: codes are int32, one per subspace (Theorem 4.2 for leaf centers: M = 1, codes = assign).
int pq_joint_update_device(const float *x, int64_t n, int d, int M, int kc, int bits, const uint8_t *codes,
                           const float *centers, const int32_t *assign,
                           int eta_mode, double T, double eta_explicit, float *codebooks, void *scratch,
                           int max_iters, double tol, int *iters_out, double *rel_residual_out, hipStream_t st);
int launch_encode(const float *x, int64_t n, int d, int M, int kc, int bits,
                  const float *codebooks, const float *leaf_centers, const int32_t *leaf_assign,
                  int eta_mode, double T, double eta_explicit, int passes, uint8_t *packed,
                  hipStream_t st);

double eta_host(int d, double T, double norm, int mode);

} // namespace avq
