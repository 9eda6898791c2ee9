// Host-side declarations shared by the translation units of libavq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/avq.h"

namespace avq {

typedef unsigned long long u64;

// Points are stored in blocks of 256: 64 lanes x 4 points per lane.
constexpr int kBlockPoints = 256;

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
struct ScanParams {
    const uint8_t *codes; // blocked layout
    int64_t n_blocks;     // blocks in the whole index
    int32_t n_valid;      // flat: ids >= n_valid are padding
    const int32_t *perm;  // partitioned: slot -> id, -1 = padding
    const float *lut;     // [B][M][kc]
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
    u64 *partial;         // [n_tiles*QT][n_chunks][64*ns]
    void *scores_out;     // debug: [B][score_stride] fp32 or int32, else NULL
    int64_t score_stride;
};
struct ScanShape { int qt; int waves; size_t lds_bytes; };
// Picks query-tile size and waves per workgroup that fit LDS. qt_hint/waves_hint 0 = auto.
int scan_pick_shape(int NB, bool u8, int ns, int B, bool ivf, int qt_hint, int waves_hint,
                    ScanShape *out);
int launch_scan(const ScanParams &p, bool u8, bool ivf, const ScanShape &shape, hipStream_t st);

// ---- select.hip ------------------------------------------------------------
// Merges the per-chunk lists of every query into one sorted list cand[q][64*ns].
int launch_merge_partials(const u64 *partial, int nq, int n_chunks, int ns, u64 *cand,
                          hipStream_t st);
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

// ---- ivf.hip ---------------------------------------------------------------
// centers_t: [d][n_leaves] (transposed). Writes the L best leaves per query.
int launch_leaf_select(const float *centers_t, int n_leaves, int d, const float *queries, int nq,
                       int L, int32_t *leaf_ids, float *leaf_ip, hipStream_t st);
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
int launch_encode(const float *x, int64_t n, int d, int M, int kc, int bits,
                  const float *codebooks, const float *leaf_centers, const int32_t *leaf_assign,
                  int eta_mode, double T, double eta_explicit, int passes, uint8_t *packed,
                  hipStream_t st);

double eta_host(int d, double T, double norm, int mode);

} // namespace avq
