// ADC scan (paper Section 4.1: the score of a quantized point is the sum of one
// table entry per subspace; Section 2.2.2: O(kd + mn) per query) fused with the
// first stage of the top-R selection.
//
// Data layout. Points are stored in blocks of 256 = 64 lanes x 4 points. A point
// has NB code bytes (one per 8-bit subspace, or one per pair of 4-bit
// subspaces). Byte position b of a block is a 256-byte "plane": lane l owns the
// dword holding byte b of its points 4l..4l+3. Planes are grouped four at a time
// into 1 KiB rows (lane l owns 16 contiguous bytes = planes 4j..4j+3) so a lane
// streams its codes with dwordx4 loads; the NB % 4 left-over planes follow as
// 256-byte dword rows. A block is exactly 256*NB bytes: no padding.
//
// Tables. Whatever the code width, the kernels see NB byte positions with a
// 256-entry table each, held in LDS for a tile of QT queries, entry = QT values
// interleaved (one ds_read fetches a byte's entry for the whole tile):
//   8-bit codes: T[b][v] = L[b][v];
//   4-bit codes: T[b][v] = L[2b][v & 15] + L[2b+1][v >> 4]  (one fp32 add, or an
//   integer add of the two 8-bit table codes).
// Scores accumulate over b = 0..NB-1 in order, which is the summation order the
// fp32 path is defined with.
//
// Two selection schemes.
//  * Batches (adc_scan_kernel, MODE_CHUNK / MODE_LEAVES): each wave keeps, per
//    query, a sorted list of the best 64*ns keys in LDS and a 64-entry pending
//    buffer; a lane whose score beats the current R-th best appends to the
//    buffer, a full buffer is sorted and merged (bitonic networks across lanes).
//    At the end the waves' lists are merged and written out per (query, chunk).
//  * A handful of queries (block_max_kernel, then adc_scan_kernel in
//    MODE_BLOCKLIST): with one query the threshold filter has nothing to work
//    with -- every wave sees only a few hundred points -- so the full scan only
//    records the best key of every 256-point block. The R best points all lie
//    in the R blocks with the largest block maxima (R blocks whose maximum is
//    >= t hold R points >= t, and every point outside them is below its own
//    block's maximum, hence below t), so only those R blocks are scanned again
//    with the list machinery above.
#include "avq_internal.h"
#include "wave_topk.h"
#include "wg_select.h"

namespace avq {

enum { MODE_CHUNK = 0, MODE_LEAVES = 1, MODE_BLOCKLIST = 2 };

template <int W> struct VecW;
template <> struct VecW<1> { typedef uint32_t type; };
template <> struct VecW<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct VecW<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct VecW<8> { typedef uint32_t type __attribute__((ext_vector_type(8))); };

template <int W> __device__ __forceinline__ uint32_t vec_get(const typename VecW<W>::type &v, int i)
{
    if constexpr (W == 1) return v;
    else return v[i];
}

// words per table entry: fp32 -> one float per query; 8-bit tables -> one u16 per query
// (a lone query uses a full word)
template <int QT, bool U8> struct EntryWords { static constexpr int value = U8 ? (QT >= 2 ? QT / 2 : 1) : QT; };

// fp32 tables for a tile of 8 queries keep the 16-entry tables themselves (4-bit codes only):
// table T = 2b + h (byte position b, low or high nibble) of query group g (4 queries) is 16
// entries of 4 floats = 256 bytes, at (T * 2 + g) * 256. A wave's 64 reads of 16 bytes from
// one such table touch every bank once (equal entries are broadcast), so they run at the full
// LDS rate, where 16-byte reads at random into a 256-entry table lose more than half to bank
// conflicts; two reads per byte instead of one still come out ahead, and the tables are
// eight times smaller.
template <int QT, bool U8> struct NibbleTiles { static constexpr bool value = !U8 && QT == 8; };

// The code bytes of one block held by one lane.
template <int NBT> struct BlockRegs {
    uint4 rows[NBT / 4 ? NBT / 4 : 1];
    uint32_t tails[NBT % 4 ? NBT % 4 : 1];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// NT: loads marked nontemporal. A code array larger than the 256 MB Infinity Cache is read once per launch, and
// such a stream runs about a tenth faster when its lines are not kept (pure reads of 1.6 GB: 6.3 -> 7.1 TB/s at
// best); a smaller array stays resident between launches and is loaded the plain way.
template <int NBT, bool NT = false>
__device__ __forceinline__ void load_block(BlockRegs<NBT> &r, const uint8_t *__restrict__ codes, int64_t blk,
                                           int lane)
{
    if constexpr (NBT != 0) {
        const uint8_t *base = codes + (size_t)blk * 256 * NBT;
#pragma unroll
        for (int j = 0; j < NBT / 4; ++j) {
            if constexpr (NT) {
                const u32x4 v = __builtin_nontemporal_load((const u32x4 *)(base + (size_t)j * 1024) + lane);
                r.rows[j] = make_uint4(v.x, v.y, v.z, v.w);
            } else {
                r.rows[j] = ((const uint4 *)(base + (size_t)j * 1024))[lane];
            }
        }
#pragma unroll
        for (int t = 0; t < NBT % 4; ++t) {
            const uint32_t *w = (const uint32_t *)(base + (size_t)(NBT / 4) * 1024 + (size_t)t * 256) + lane;
            r.tails[t] = NT ? __builtin_nontemporal_load(w) : *w;
        }
    }
}

// Fills the byte tables of the query tile starting at q0 (all threads of the workgroup).
template <int QT, bool U8>
__device__ __forceinline__ void build_tables(typename VecW<EntryWords<QT, U8>::value>::type *tbl,
                                             const ScanParams &p, int q0, int NB)
{
    const int kc = 1 << p.bits;
    if constexpr (NibbleTiles<QT, U8>::value) {
        float *t = (float *)tbl;
        for (int it = threadIdx.x; it < 2 * NB * 128; it += blockDim.x) {
            const int qq = it & 3, e = (it >> 2) & 15, g = (it >> 6) & 1, T = it >> 7;
            const int gq = q0 + 4 * g + qq;
            t[it] = (gq < p.B && T < p.M) ? p.lut[((size_t)gq * p.M + T) * 16 + e] : 0.0f;
        }
        return;
    }
    const int items = QT * NB * 16; // (q, b, g): 16 consecutive byte values g*16 .. g*16+15
    for (int it = threadIdx.x; it < items; it += blockDim.x) {
        const int q = it % QT;
        const int g = (it / QT) & 15;
        const int b = it / (QT * 16);
        const int gq = q0 + q;
        const bool live = gq < p.B;
        if constexpr (!U8) {
            float *t = (float *)tbl;
            const float *L = p.lut + (size_t)(live ? gq : 0) * p.M * kc;
            if (p.bits == 8) {
                for (int lo = 0; lo < 16; ++lo)
                    t[(size_t)(b * 256 + g * 16 + lo) * QT + q] = live ? L[b * 256 + g * 16 + lo] : 0.0f;
            } else {
                const bool pair = 2 * b + 1 < p.M;
                const float hi = (pair && live) ? L[(2 * b + 1) * 16 + g] : 0.0f;
                for (int lo = 0; lo < 16; ++lo) {
                    float v = live ? L[2 * b * 16 + lo] : 0.0f;
                    if (pair) v = __fadd_rn(v, hi);
                    t[(size_t)(b * 256 + g * 16 + lo) * QT + q] = v;
                }
            }
        } else {
            const uint8_t *L = p.lut8 + (size_t)(live ? gq : 0) * p.M * kc;
            for (int lo = 0; lo < 16; ++lo) {
                uint32_t v;
                if (p.bits == 8) v = L[b * 256 + g * 16 + lo];
                else v = (uint32_t)L[2 * b * 16 + lo] + ((2 * b + 1 < p.M) ? (uint32_t)L[(2 * b + 1) * 16 + g] : 0u);
                if (!live) v = 0;
                const size_t e = (size_t)(b * 256 + g * 16 + lo);
                if constexpr (QT == 1) ((uint32_t *)tbl)[e] = v;
                else ((uint16_t *)tbl)[e * QT + q] = (uint16_t)v;
            }
        }
    }
}

// Scores of the lane's four points of one block against the query tile:
// acc[i] = sum over byte positions, in order, of the table entries.
template <int QT, bool U8, int NBT>
__device__ __forceinline__ void accumulate_block(const typename VecW<EntryWords<QT, U8>::value>::type *tbl,
                                                 const BlockRegs<NBT> &r, const uint8_t *__restrict__ codes,
                                                 int64_t blk, int NB, int lane,
                                                 typename VecW<EntryWords<QT, U8>::value>::type (&acc)[4])
{
    constexpr int WORDS = EntryWords<QT, U8>::value;
    typedef typename VecW<WORDS>::type entry_t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (WORDS == 1) acc[i] = 0u;
        else acc[i] = (entry_t)(0u);
    }
    auto plane = [&](uint32_t w, int b) {
        if constexpr (NibbleTiles<QT, U8>::value) {
            // both nibbles of the word's four bytes, times 16 (the entry size), masked out once
            uint32_t wl = (w << 4) & 0xf0f0f0f0u, wh = w & 0xf0f0f0f0u;
            asm volatile("" : "+v"(wl), "+v"(wh));
            const unsigned char *tb = (const unsigned char *)tbl + (size_t)b * 1024; // tables 2b, 2b+1 x two groups
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t ol = (wl >> (8 * i)) & 0xffu, oh = (wh >> (8 * i)) & 0xffu;
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const float4 lo = *(const float4 *)(tb + g * 256 + ol);
                    const float4 hi = *(const float4 *)(tb + 512 + g * 256 + oh);
                    const float l4[4] = {lo.x, lo.y, lo.z, lo.w}, h4[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float v = __fadd_rn(l4[k], h4[k]);
                        acc[i][4 * g + k] = __float_as_uint(__fadd_rn(__uint_as_float(acc[i][4 * g + k]), v));
                    }
                }
            }
            return;
        }
        const entry_t *tb = tbl + (size_t)b * 256;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t byte = (w >> (8 * i)) & 0xffu;
            const entry_t e = tb[byte];
            if constexpr (U8) {
                acc[i] += e;
            } else {
#pragma unroll
                for (int k = 0; k < WORDS; ++k) {
                    float a = __uint_as_float(vec_get<WORDS>(acc[i], k));
                    a = __fadd_rn(a, __uint_as_float(vec_get<WORDS>(e, k)));
                    if constexpr (WORDS == 1) acc[i] = __float_as_uint(a);
                    else acc[i][k] = __float_as_uint(a);
                }
            }
        }
    };
    if constexpr (NBT != 0) {
#pragma unroll
        for (int j = 0; j < NBT / 4; ++j) {
            plane(r.rows[j].x, 4 * j + 0);
            plane(r.rows[j].y, 4 * j + 1);
            plane(r.rows[j].z, 4 * j + 2);
            plane(r.rows[j].w, 4 * j + 3);
        }
#pragma unroll
        for (int t = 0; t < NBT % 4; ++t) plane(r.tails[t], (NBT / 4) * 4 + t);
    } else {
        const int nfull = NB / 4, ntail = NB % 4;
        const uint8_t *base = codes + (size_t)blk * 256 * NB;
        for (int j = 0; j < nfull; ++j) {
            const uint4 row = ((const uint4 *)(base + (size_t)j * 1024))[lane];
            plane(row.x, 4 * j + 0);
            plane(row.y, 4 * j + 1);
            plane(row.z, 4 * j + 2);
            plane(row.w, 4 * j + 3);
        }
        for (int t = 0; t < ntail; ++t) {
            const uint32_t w = ((const uint32_t *)(base + (size_t)nfull * 1024 + (size_t)t * 256))[lane];
            plane(w, 4 * nfull + t);
        }
    }
}

// Integer sum of query q from the packed accumulators.
template <int QT, int WORDS>
__device__ __forceinline__ int packed_sum(const typename VecW<WORDS>::type &a, int q)
{
    if constexpr (QT == 1) return (int)vec_get<WORDS>(a, 0);
    else return (int)((vec_get<WORDS>(a, q >> 1) >> (16 * (q & 1))) & 0xffffu);
}

template <int QT, bool U8, int NBT, int MODE>
__global__ void __launch_bounds__(QT > 1 ? 512 : 1024, (NibbleTiles<QT, U8>::value ? 4 : 1))
adc_scan_kernel(const ScanParams p)
{
    constexpr int WORDS = EntryWords<QT, U8>::value;
    typedef typename VecW<WORDS>::type entry_t;
    constexpr bool LEAVES = MODE == MODE_LEAVES;
    // With leaves the ranking key is a float even for 8-bit tables (it includes <q, center>).
    constexpr bool FKEY = !U8 || LEAVES;
    // Ids grow along a wave's scan only in MODE_CHUNK; there a score equal to the current
    // R-th best can never enter the list, so the filter may be strict.
    constexpr bool STRICT = MODE == MODE_CHUNK;
    extern __shared__ __align__(16) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int C = 64 * p.ns;

    int tile, chunk;
    int n_chunks = p.n_chunks, blocks_per_chunk = p.blocks_per_chunk;
    if (MODE == MODE_CHUNK && p.active_queries != nullptr) {
        // only the first *active_queries queries are live, a count the host does not know: the
        // grid is cut to fit it here (see scan_dynamic_chunks)
        const int tiles = ((int)*p.active_queries + QT - 1) / QT;
        n_chunks = scan_dynamic_chunks(tiles, p.n_chunks);
        if (tiles == 0 || (int)blockIdx.x >= tiles * n_chunks) return;
        tile = blockIdx.x % tiles;
        chunk = blockIdx.x / tiles;
        blocks_per_chunk = (int)((p.n_blocks + n_chunks - 1) / n_chunks);
    } else if (MODE == MODE_CHUNK || MODE == MODE_LEAVES) {
        tile = blockIdx.x % p.n_tiles;
        chunk = blockIdx.x / p.n_tiles;
        // partitioned index, compacted query list: only the first *active_queries rows are live
        if (MODE == MODE_LEAVES && p.active_queries != nullptr && (uint32_t)tile >= *p.active_queries) return;
    } else { tile = blockIdx.x; chunk = 0; }
    const int q0 = tile * QT;

    entry_t *tbl = (entry_t *)smem;
    const size_t tbl_bytes = NibbleTiles<QT, U8>::value ? (size_t)NB * QT * 128 : (size_t)NB * 256 * WORDS * 4;
    // candidate lists [n_waves][QT][C]: in LDS, or in a global scratch area when the tables
    // need the LDS (they are touched only when a pending buffer is flushed)
    u64 *lists = p.lists_ws ? p.lists_ws + (size_t)blockIdx.x * n_waves * QT * C : (u64 *)(smem + tbl_bytes);
    u64 *pends = (u64 *)(smem + tbl_bytes) + (p.lists_ws ? 0 : (size_t)n_waves * QT * C); // [n_waves][QT][64]
    u64 *my_lists = lists + (size_t)wave * QT * C;
    u64 *my_pends = pends + (size_t)wave * QT * 64;

    build_tables<QT, U8>(tbl, p, q0, NB);
    for (int i = lane; i < QT * C; i += 64) my_lists[i] = 0ull;
    __syncthreads();

    // per-query filter state, wave-uniform
    float thr_f[QT];
    int thr_i[QT];
    int pend_cnt[QT];
    float q_scale[QT], q_off[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q) {
        thr_f[q] = -INFINITY;
        thr_i[q] = -1;
        pend_cnt[q] = 0;
        q_scale[q] = 0.0f;
        q_off[q] = 0.0f;
        if (LEAVES && U8) {
            const int gq = q0 + q < p.B ? q0 + q : 0;
            q_scale[q] = p.scale[gq];
            q_off[q] = p.bias[gq];
        }
    }

    // The filter of query q lets a point through when it can still be among the R best:
    //  * it must beat the wave's own R-th best. A tie loses where ids only grow (STRICT) -- which
    //    holds from one block to the next, not inside a block, whose points are taken four
    //    interleaved sets of 64 at a time: a bound taken from the list in the middle of a block
    //    lets ties pass (they are ordered by id when merged) and is tightened when the next block starts;
    //  * it must reach the smallest of the workgroup's waves' kw-th best scores, kw = ceil(R / waves):
    //    every wave holds that many points at or above it, R in all (the waves scan disjoint
    //    points for the same queries), so it is a lower bound of the final R-th best -- and a much
    //    tighter one than the own R-th best while the lists are young. Ties must pass here.
    // A list read while its owner merges into it shows an older or the newer kw-th best; both are valid.
    const int kw = (p.R + n_waves - 1) / n_waves;
    uint32_t relaxed = 0u; // queries whose bound was taken in the middle of a block (wave-uniform)
    auto refresh_threshold = [&](int q, bool mid_block) {
        const uint32_t ord_own = key_ord(my_lists[(size_t)q * C + (p.R - 1)]); // 0: fewer than R yet
        uint32_t ord_g = 0xffffffffu;
        for (int w = 0; w < n_waves; ++w) {
            const uint32_t o = key_ord(lists[((size_t)w * QT + q) * C + (kw - 1)]);
            ord_g = o < ord_g ? o : ord_g; // 0 while a wave has fewer than kw
        }
        // "reach v" is "beat v - 1" in ordering values
        if (STRICT && mid_block) relaxed |= 1u << q;
        if (FKEY) {
            const uint32_t own = (STRICT && mid_block && ord_own > 0u) ? ord_own - 1u : ord_own;
            const uint32_t t = STRICT ? (ord_g > 0u && ord_g - 1u > own ? ord_g - 1u : own)
                                      : (ord_g > own ? ord_g : own);
            thr_f[q] = t ? f32_from_ord(t) : -INFINITY;
        } else {
            // integer sums: ordering value = sum + 1
            const int own = (int)ord_own - 1 - ((STRICT && mid_block) ? 1 : 0), grp = (int)ord_g - (STRICT ? 2 : 1);
            thr_i[q] = grp > own ? grp : own;
        }
    };

    // one block of 256 points: accumulate, then filter
    auto process_block = [&](int64_t blk, const BlockRegs<NBT> &regs, float seg_bias) {
        if (STRICT && relaxed != 0u) {
#pragma unroll
            for (int q = 0; q < QT; ++q)
                if ((relaxed >> q) & 1u) refresh_threshold(q, false);
            relaxed = 0u;
        }
        entry_t acc[4];
        accumulate_block<QT, U8, NBT>(tbl, regs, p.codes, blk, NB, lane, acc);
        // score of (query q, point i of this lane)
        auto score_of = [&](int q, int i, float &sf, int &si) {
            sf = 0.0f;
            si = 0;
            if constexpr (!U8) {
                sf = __uint_as_float(vec_get<WORDS>(acc[i], q));
                if (LEAVES) sf = __fadd_rn(sf, seg_bias);
            } else {
                si = packed_sum<QT, WORDS>(acc[i], q);
                if (LEAVES) sf = __fmaf_rn((float)si, q_scale[q], __fadd_rn(q_off[q], seg_bias));
            }
        };
        if (p.scores_out != nullptr) { // inspection mode: store every score, select nothing
#pragma unroll
            for (int q = 0; q < QT; ++q) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float sf;
                    int si;
                    score_of(q, i, sf, si);
                    const int64_t slot = blk * 256 + 4 * lane + i;
                    if (slot < p.n_valid && q0 + q < p.B) {
                        if (U8) ((int32_t *)p.scores_out)[(size_t)(q0 + q) * p.score_stride + slot] = si;
                        else ((float *)p.scores_out)[(size_t)(q0 + q) * p.score_stride + slot] = sf;
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < QT; ++q) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float sf;
                int si;
                score_of(q, i, sf, si);
                bool hit;
                if (FKEY) hit = STRICT ? (sf > thr_f[q]) : (sf >= thr_f[q]);
                else hit = STRICT ? (si > thr_i[q]) : (si >= thr_i[q]);
                if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
                // rare path: some lane has a candidate
                const int64_t slot = blk * 256 + 4 * lane + i;
                int32_t id;
                if (LEAVES) { id = p.perm[slot]; hit = hit && id >= 0; }
                else { id = (int32_t)slot; hit = hit && slot < p.n_valid; }
                const uint32_t ord = FKEY ? ord_from_f32(sf) : (uint32_t)(si + 1);
                if (wave_push(my_lists + (size_t)q * C, p.ns, my_pends + q * 64, pend_cnt[q], hit,
                              make_key(ord, id)))
                    refresh_threshold(q, true);
            }
        }
    };

    // streams blocks first, first + step, ... < end with the next block's loads in flight
    auto scan_range = [&](int64_t first, int64_t end, int64_t step, float seg_bias) {
        if constexpr (NibbleTiles<QT, U8>::value) {
            // sixteen waves per compute unit hide the load latency; no second register buffer
            for (int64_t blk = first; blk < end; blk += step) {
                BlockRegs<NBT> cur;
                load_block<NBT>(cur, p.codes, blk, lane);
                process_block(blk, cur, seg_bias);
            }
            return;
        }
        BlockRegs<NBT> cur, nxt;
        if (first < end) load_block<NBT>(cur, p.codes, first, lane);
        for (int64_t blk = first; blk < end; blk += step) {
            const bool more = blk + step < end;
            if (more) load_block<NBT>(nxt, p.codes, blk + step, lane);
            if (LEAVES && p.scores_out == nullptr) refresh_threshold(0, false); // the other waves' progress (QT == 1 here)
            process_block(blk, cur, seg_bias);
            if (more) cur = nxt;
        }
    };

    if (MODE == MODE_CHUNK) {
        const int64_t first = (int64_t)chunk * blocks_per_chunk;
        int64_t end = first + blocks_per_chunk;
        if (end > p.n_blocks) end = p.n_blocks;
        scan_range(first + wave, end, n_waves, 0.0f);
    } else if (MODE == MODE_LEAVES) {
        // the query's probed leaves, dealt to the waves of its n_chunks workgroups in turn
        const int leaf_stride = p.leaf_stride ? p.leaf_stride : p.Lp; // a scan of the first Lp leaves of longer rows
        for (int j = chunk * n_waves + wave; j < p.Lp; j += p.n_chunks * n_waves) {
            const int leaf = p.leaf_ids[(size_t)q0 * leaf_stride + j];
            if (leaf < 0) continue;
            scan_range(p.leaf_blk[leaf], p.leaf_blk[leaf + 1], 1, p.leaf_ip[(size_t)q0 * leaf_stride + j]);
        }
    } else {
        // the R blocks with the largest block maxima, as keys whose id lies in the block
        for (int j = wave; j < p.R; j += n_waves) {
            const u64 key = p.block_keys[(size_t)q0 * C + j];
            if (key == 0ull) continue;
            const int64_t blk = (int64_t)(key_id(key) >> 8);
            scan_range(blk, blk + 1, 1, 0.0f);
        }
    }
    if (p.scores_out != nullptr) return;

    // ---- drain pending buffers, merge the waves' lists, write out -------------
#pragma unroll
    for (int q = 0; q < QT; ++q)
        if (pend_cnt[q] > 0) wave_list_flush(my_lists + (size_t)q * C, p.ns, my_pends + q * 64, pend_cnt[q]);
    __syncthreads();
    if constexpr (QT == 1) {
        // one query, many waves: the lists are merged pairwise up a tree (log2(waves) merges on the critical
        // path instead of waves - 1), wave 0 ends up with the result
        for (int stride = 1; stride < n_waves; stride *= 2) {
            if ((wave % (2 * stride)) == 0 && wave + stride < n_waves)
                wave_list_merge_from(my_lists, p.ns, lists + (size_t)(wave + stride) * C);
            __syncthreads();
        }
        if (wave == 0) {
            u64 *out = p.partial + ((size_t)q0 * n_chunks + chunk) * C;
            for (int i = lane; i < C; i += 64) out[i] = my_lists[i];
        }
        return;
    }
    for (int q = wave; q < QT; q += n_waves) {
        u64 *mine = my_lists + (size_t)q * C;
        for (int w = 0; w < n_waves; ++w) {
            if (w == wave) continue;
            wave_list_merge_from(mine, p.ns, lists + ((size_t)w * QT + q) * C);
        }
        u64 *out = p.partial + ((size_t)(q0 + q) * n_chunks + chunk) * C;
        for (int i = lane; i < C; i += 64) out[i] = mine[i];
    }
}

// Full scan of one query per grid.y: every wave scores one block and records the
// block's best key (score, then lower id) in block_max[q][blk]. Nothing else is
// written: 8 bytes out per 256 points read.
template <bool U8, int NBT>
__global__ void __launch_bounds__(1024)
block_max_kernel(const ScanParams p)
{
    constexpr int WORDS = EntryWords<1, U8>::value;
    typedef typename VecW<WORDS>::type entry_t;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int q = blockIdx.y;
    entry_t *tbl = (entry_t *)smem;
    // the grid's waves take the blocks in turn: a workgroup builds its tables once for many blocks
    const int64_t step = (int64_t)gridDim.x * n_waves;
    int64_t blk = (int64_t)blockIdx.x * n_waves + wave;

    BlockRegs<NBT> regs, nxt;
    if (blk < p.n_blocks) load_block<NBT>(regs, p.codes, blk, lane); // in flight while the tables are built
    build_tables<1, U8>(tbl, p, q, NB);
    __syncthreads();
    for (; blk < p.n_blocks; blk += step) {
        const bool more = blk + step < p.n_blocks;
        if (more) load_block<NBT>(nxt, p.codes, blk + step, lane);
        entry_t acc[4];
        accumulate_block<1, U8, NBT>(tbl, regs, p.codes, blk, NB, lane, acc);
        // best of the lane's four points: higher ordering value, then lower id (= lower i)
        uint32_t best = 0;
        int best_i = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t slot = blk * 256 + 4 * lane + i;
            uint32_t ord = U8 ? (uint32_t)(acc[i] + 1u) : ord_from_f32(__uint_as_float(acc[i]));
            if (slot >= p.n_valid) ord = 0u;
            if (ord > best) { best = ord; best_i = i; }
        }
        uint32_t wmax = best;
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)wmax, m, 64);
            wmax = o > wmax ? o : wmax;
        }
        const u64 owners = __builtin_amdgcn_ballot_w64(best == wmax);
        const int owner = __builtin_ctzll(owners); // lowest lane = lowest id among equal scores
        if (lane == owner)
            p.block_max[(size_t)q * p.n_blocks + blk] =
                wmax ? make_key(wmax, (int32_t)(blk * 256 + 4 * lane + best_i)) : 0ull;
        if (more) regs = nxt;
    }
}

// 16-entry tables of one query in LDS (4-bit codes): 2*NB tables of 16 entries, fp32
// (U8 = false) or one byte each (U8 = true); for odd M the last table is all zero, so
// that every code byte reads two entries. All threads of the workgroup take part.
template <bool U8>
__device__ __forceinline__ void nibble_tables_fill(unsigned char *tbl, const ScanParams &p, int q, int NB)
{
    const int live = p.M * 16, total = 2 * NB * 16;
    if (U8) {
        const uint8_t *L = p.lut8 + (size_t)q * live;
        for (int e = threadIdx.x; e < total; e += blockDim.x) tbl[e] = e < live ? L[e] : (uint8_t)0;
    } else if (p.fuse_queries != nullptr) {
        // no table kernel ran: <q^(m), c_j^(m)> as an fma chain in index order, as it computes them
        const int ds = p.fuse_d / p.M;
        const float *qv = p.fuse_queries + (size_t)q * p.fuse_d;
        for (int e = threadIdx.x; e < total; e += blockDim.x) {
            float sacc = 0.0f;
            if (e < live) {
                const float *c = p.fuse_codebooks + (size_t)e * ds;
                const float *qm = qv + (e >> 4) * ds;
                for (int l = 0; l < ds; ++l) sacc = __fmaf_rn(qm[l], c[l], sacc);
            }
            ((float *)tbl)[e] = sacc;
        }
    } else {
        const float *L = p.lut + (size_t)q * live;
        for (int e = threadIdx.x; e < total; e += blockDim.x) ((float *)tbl)[e] = e < live ? L[e] : 0.0f;
    }
}

// Scores of the lane's four points of one block against those tables: per code byte
// the two entries are added first, then accumulated, byte positions in order.
// regs holds the block's code bytes (NBT != 0; all of its loads are issued before
// the first lookup, so a wave pays the memory latency once per block); with
// NBT == 0 the rows are read from `base` as they are needed.
template <bool U8, int NBT>
__device__ __forceinline__ void nibble_accumulate(const unsigned char *tbl, const BlockRegs<NBT> &regs,
                                                  const uint8_t *__restrict__ base, int NB, int lane,
                                                  float (&accf)[4], uint32_t (&acci)[4])
{
    constexpr int ES = U8 ? 1 : 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) { accf[i] = 0.0f; acci[i] = 0u; }
    // The empty asm statement pins the accumulators once per row: integer sums may be
    // reassociated freely, and left alone the compiler turns the block into one flat sum,
    // reads every table entry first and spills. A row's 32 table reads stay in flight together.
    auto pin = [&]() {
        if constexpr (U8) asm volatile("" : "+v"(acci[0]), "+v"(acci[1]), "+v"(acci[2]), "+v"(acci[3]));
        else asm volatile("" : "+v"(accf[0]), "+v"(accf[1]), "+v"(accf[2]), "+v"(accf[3]));
    };
    // The low and the high nibbles of the word's four bytes are masked out once, already
    // scaled to table offsets, and pinned, so that each lookup costs one bit-field extract;
    // left alone the compiler folds this back into a shift and a mask per nibble.
    auto plane = [&](uint32_t w, const unsigned char *t) {
        uint32_t lo, hi;
        if constexpr (U8) { lo = w & 0x0f0f0f0fu; hi = (w >> 4) & 0x0f0f0f0fu; }
        else { lo = (w << 2) & 0x3c3c3c3cu; hi = (w >> 2) & 0x3c3c3c3cu; }
        asm volatile("" : "+v"(lo), "+v"(hi));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a = (lo >> (8 * i)) & 0xffu, b = (hi >> (8 * i)) & 0xffu;
            if constexpr (U8) {
                acci[i] += (uint32_t)t[a] + (uint32_t)t[16 + b];
            } else {
                const float v = __fadd_rn(*(const float *)(t + a), *(const float *)(t + 64 + b));
                accf[i] = __fadd_rn(accf[i], v);
            }
        }
    };
    if constexpr (NBT != 0) {
#pragma unroll
        for (int j = 0; j < NBT / 4; ++j) {
            const unsigned char *t = tbl + (size_t)j * 128 * ES;
            plane(regs.rows[j].x, t);
            plane(regs.rows[j].y, t + 32 * ES);
            plane(regs.rows[j].z, t + 64 * ES);
            plane(regs.rows[j].w, t + 96 * ES);
            pin();
        }
#pragma unroll
        for (int tt = 0; tt < NBT % 4; ++tt) plane(regs.tails[tt], tbl + (size_t)((NBT / 4) * 4 + tt) * 32 * ES);
    } else {
        const int nfull = NB / 4, ntail = NB % 4;
        const unsigned char *t = tbl;
        const uint4 *rowp = (const uint4 *)base + lane;
        if (nfull > 0) {
            uint4 cur = rowp[0];
            for (int j = 0; j < nfull; ++j) {
                const uint4 nxt = j + 1 < nfull ? rowp[(size_t)(j + 1) * 64] : cur;
                plane(cur.x, t);
                plane(cur.y, t + 32 * ES);
                plane(cur.z, t + 64 * ES);
                plane(cur.w, t + 96 * ES);
                t += 128 * ES;
                cur = nxt;
                pin();
            }
        }
        for (int tt = 0; tt < ntail; ++tt) {
            plane(((const uint32_t *)(base + (size_t)nfull * 1024 + (size_t)tt * 256))[lane], t);
            t += 32 * ES;
        }
    }
}

// The same for 4-bit codes, with the 16-entry tables themselves in LDS instead of
// the 256-entry byte tables: twice the lookups, but the 16 entries of a table sit
// in 16 different banks, so a wave's reads never conflict (random reads of a
// 256-entry table cost about three times as many LDS cycles each), and there is
// no 6400-entry table to build per workgroup. The two entries of a byte are added
// first, then accumulated, exactly as the byte tables do.
template <bool U8, int NBT>
__global__ void __launch_bounds__(1024)
block_max_nibble_kernel(const ScanParams p)
{
    // With the byte count fixed at compile time the tables are a static array: its LDS
    // address is a constant that folds into the offset field of every table read.
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    __shared__ __align__(16) unsigned char fixed_smem[NBT ? 2 * NBT * 16 * (U8 ? 1 : 4) : 16];
    unsigned char *smem = NBT ? fixed_smem : dyn_smem;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int q = blockIdx.y;
    // the grid's waves take the blocks in turn (one each unless the index is large): a
    // workgroup fills its tables once for all of its blocks
    const int64_t step = (int64_t)gridDim.x * n_waves;
    int64_t blk = (int64_t)blockIdx.x * n_waves + wave;

    BlockRegs<NBT> regs, nxt;
    if (blk < p.n_blocks) load_block<NBT>(regs, p.codes, blk, lane); // in flight while the tables are filled
    nibble_tables_fill<U8>(smem, p, q, NB);
    __syncthreads();
    for (; blk < p.n_blocks; blk += step) {
        const bool more = blk + step < p.n_blocks;
        if (more) load_block<NBT>(nxt, p.codes, blk + step, lane);
        float accf[4];
        uint32_t acci[4];
        nibble_accumulate<U8, NBT>(smem, regs, p.codes + (size_t)blk * 256 * NB, NB, lane, accf, acci);
        uint32_t best = 0;
        int best_i = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t slot = blk * 256 + 4 * lane + i;
            uint32_t ord = U8 ? (acci[i] + 1u) : ord_from_f32(accf[i]);
            if (slot >= p.n_valid) ord = 0u;
            if (ord > best) { best = ord; best_i = i; }
        }
        uint32_t wmax = best;
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)wmax, m, 64);
            wmax = o > wmax ? o : wmax;
        }
        const u64 owners = __builtin_amdgcn_ballot_w64(best == wmax);
        const int owner = __builtin_ctzll(owners);
        if (lane == owner)
            p.block_max[(size_t)q * p.n_blocks + blk] =
                wmax ? make_key(wmax, (int32_t)(blk * 256 + 4 * lane + best_i)) : 0ull;
        if (more) regs = nxt;
    }
}

// The code stream alone: the same loads, in the same launch shape, as the single-query scan,
// with the table lookups left out: every wave folds its blocks' words into one (xor) and
// writes it. Its duration is what reading the code array once costs on the machine, the
// floor a scan of that array can approach.
template <int NBT, bool NT = false>
__global__ void __launch_bounds__(1024)
stream_codes_kernel(const uint8_t *__restrict__ codes, int64_t n_blocks, int NB_rt, uint32_t *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : NB_rt;
    const int64_t step = (int64_t)gridDim.x * n_waves;
    for (int64_t blk = (int64_t)blockIdx.x * n_waves + wave; blk < n_blocks; blk += step) {
        uint32_t x = 0u;
        if constexpr (NBT != 0) {
            BlockRegs<NBT> regs;
            load_block<NBT, NT>(regs, codes, blk, lane);
#pragma unroll
            for (int j = 0; j < NBT / 4; ++j) x ^= regs.rows[j].x ^ regs.rows[j].y ^ regs.rows[j].z ^ regs.rows[j].w;
#pragma unroll
            for (int t = 0; t < NBT % 4; ++t) x ^= regs.tails[t];
        } else {
            const uint32_t *base = (const uint32_t *)(codes + (size_t)blk * 256 * NB);
            for (int j = 0; j < NB; ++j) x ^= base[(size_t)j * 64 + lane];
        }
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) x ^= (uint32_t)__shfl_xor((int)x, m, 64);
        if (lane == 0) out[blk] = x;
    }
}

int launch_stream_codes(const uint8_t *codes, int64_t n_blocks, int NB, uint32_t *out, hipStream_t st, bool nt)
{
    const int waves = 4;
    int64_t gx = std::min<int64_t>((n_blocks + waves - 1) / waves, nt ? INT64_MAX : 2048); // the scan's launch shape
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx), block(waves * 64);
    switch (NB) {
    case 8:
        if (nt) hipLaunchKernelGGL((stream_codes_kernel<8, true>), grid, block, 0, st, codes, n_blocks, NB, out);
        else hipLaunchKernelGGL((stream_codes_kernel<8, false>), grid, block, 0, st, codes, n_blocks, NB, out);
        break;
    case 13:
        if (nt) hipLaunchKernelGGL((stream_codes_kernel<13, true>), grid, block, 0, st, codes, n_blocks, NB, out);
        else hipLaunchKernelGGL((stream_codes_kernel<13, false>), grid, block, 0, st, codes, n_blocks, NB, out);
        break;
    case 25:
        if (nt) hipLaunchKernelGGL((stream_codes_kernel<25, true>), grid, block, 0, st, codes, n_blocks, NB, out);
        else hipLaunchKernelGGL((stream_codes_kernel<25, false>), grid, block, 0, st, codes, n_blocks, NB, out);
        break;
    case 32:
        if (nt) hipLaunchKernelGGL((stream_codes_kernel<32, true>), grid, block, 0, st, codes, n_blocks, NB, out);
        else hipLaunchKernelGGL((stream_codes_kernel<32, false>), grid, block, 0, st, codes, n_blocks, NB, out);
        break;
    default: hipLaunchKernelGGL((stream_codes_kernel<0, false>), grid, block, 0, st, codes, n_blocks, NB, out); break;
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// Bounds for the scan over leaves that is regrouped by leaf: bound[q] = ordering value of the R-th
// best score among the points of query q's first p.Lp probed leaves (as many of them as fit
// cap_blocks blocks; any subset of the query's points gives a valid bound), 0 if they hold fewer
// than R points. Scores as the one-query-per-workgroup scan forms them: fp32 table sum (entries of
// a byte first, bytes in order) + <q, center>, or fma(integer sum, scale, bias + <q, center>). One
// workgroup per query: 16-entry tables in LDS, a wave per block, all scores to LDS, then the R-th
// best by bisection over the ordering values. No lists.
template <bool U8, int NBT>
__global__ void __launch_bounds__(512)
leaf_bound_kernel(const ScanParams p, int cap_blocks, uint32_t *__restrict__ bound)
{
    static_assert(NBT != 0, "specialised code sizes only");
    constexpr int nt = 512, n_waves = 8, kSample = 1024, kShort = 2048;
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    __shared__ __align__(16) unsigned char tables[2 * NBT * 16 * (U8 ? 1 : 4)];
    __shared__ int first_blk[65], blk_of[65]; // probed leaf j: its blocks start at blk_of[j], at position first_blk[j] here
    __shared__ int wave_cnt[2][n_waves], short_n;
    __shared__ uint32_t ord_max; // the largest ordering value: no search needs to look above it
    uint32_t *ords = (uint32_t *)dyn_smem;      // [cap_blocks * 256], 0 = no point
    uint32_t *shortlist = ords + (size_t)cap_blocks * 256; // [kShort]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = blockIdx.x;
    const int stride = p.leaf_stride ? p.leaf_stride : p.Lp;
    const int Lb = p.Lp < 64 ? p.Lp : 64;
    if (tid < Lb) { // the leaves' block ranges, one thread each: the loads overlap
        const int leaf = p.leaf_ids[(size_t)q * stride + tid];
        blk_of[tid] = leaf >= 0 ? p.leaf_blk[leaf] : 0;
        first_blk[tid] = leaf >= 0 ? p.leaf_blk[leaf + 1] - p.leaf_blk[leaf] : 0; // block count for now
    }
    nibble_tables_fill<U8>(tables, p, q, NBT);
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int j = 0; j < Lb; ++j) {
            int nb = first_blk[j];
            if (at + nb > cap_blocks) nb = 0; // does not fit: left out
            first_blk[j] = at;
            at += nb;
        }
        first_blk[Lb] = at;
        short_n = 0;
        ord_max = 0u;
    }
    __syncthreads();
    const int total = first_blk[Lb];
    const float scale = U8 ? p.scale[q] : 0.0f, bias = U8 ? p.bias[q] : 0.0f;
    uint32_t my_max = 0u;
    for (int b = wave; b < total; b += n_waves) {
        int j = 0;
        while (b >= first_blk[j + 1]) ++j;
        const int64_t blk = (int64_t)blk_of[j] + (b - first_blk[j]);
        const float ip = p.leaf_ip[(size_t)q * stride + j];
        BlockRegs<NBT> regs;
        load_block<NBT>(regs, p.codes, blk, lane);
        const int4 ids = ((const int4 *)(p.perm + (size_t)blk * 256))[lane];
        float accf[4];
        uint32_t acci[4];
        nibble_accumulate<U8, NBT>(tables, regs, p.codes + (size_t)blk * 256 * NBT, NBT, lane, accf, acci);
        const int idv[4] = {ids.x, ids.y, ids.z, ids.w};
        uint4 o;
        uint32_t *ov = (uint32_t *)&o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float sc = U8 ? __fmaf_rn((float)(int)acci[i], scale, __fadd_rn(bias, ip)) : __fadd_rn(accf[i], ip);
            ov[i] = idv[i] >= 0 ? ord_from_f32(sc) : 0u;
            my_max = ov[i] > my_max ? ov[i] : my_max;
        }
        ((uint4 *)(ords + (size_t)b * 256))[lane] = o;
    }
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) {
        const uint32_t om = (uint32_t)__shfl_xor((int)my_max, m, 64);
        my_max = om > my_max ? om : my_max;
    }
    if (lane == 0 && my_max) atomicMax(&ord_max, my_max);
    __syncthreads();
    const int n = total * 256;
    // number of a[at(i)], i < m, that are >= v (v >= 1: empty slots never count), known to every thread;
    // one barrier per call: the waves' counts go to alternating halves of wave_cnt
    int parity = 0;
    auto count_ge = [&](const uint32_t *a, int m, uint32_t v, auto at) -> int {
        int cn = 0; // the loop is uniform over the wave: every lane sees every ballot
        for (int base = wave * 64; base < m; base += 4 * nt) {
            uint32_t r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * nt + lane;
                r[u] = i < m ? a[at(i)] : 0u;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) cn += __popcll(__builtin_amdgcn_ballot_w64(r[u] >= v));
        }
        if (lane == 0) wave_cnt[parity][wave] = cn;
        __syncthreads();
        int tot = 0;
#pragma unroll
        for (int w = 0; w < n_waves; ++w) tot += wave_cnt[parity][w];
        parity ^= 1;
        return tot;
    };
    // largest v in [lo, 2^32) with at least R values >= v, given that lo has. No value is above ord_max; and the R-th
    // best of thousands of scores is mostly within a factor of two of the best one: when the ordering value one
    // binade below the maximum still has R values at or above it, the search starts there (23 rounds instead of 32).
    const uint32_t top = ord_max;
    auto rth_best = [&](const uint32_t *a, int m, int R, uint32_t lo, auto at) -> uint32_t {
        uint32_t hi = top == 0xffffffffu ? top : top + 1u; // no value reaches it
        if (top > 0x80800000u && top - 0x00800000u > lo && count_ge(a, m, top - 0x00800000u, at) >= R) lo = top - 0x00800000u;
        while (hi - lo > 1u) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (count_ge(a, m, mid, at) >= R) lo = mid; else hi = mid;
        }
        return lo;
    };
    auto plain = [](int i) { return i; };
    uint32_t result = 0u;
    bool done = false;
    // Most values are far below the answer: a bound T0 from an evenly spread sample (its rank there chosen so
    // that, in all likelihood, at least R values overall reach T0), one pass that copies the values >= T0 to
    // a short list, and the R-th best of that list. When the guess fails, the search over all values below.
    const float mu = (float)p.R * (float)kSample / (float)(n > 0 ? n : 1);
    const int rs = (int)(mu + 3.0f * sqrtf(mu) + 2.0f);
    if (n >= 4 * kSample && rs <= kSample / 2) {
        auto spread = [n](int i) { return (int)(((int64_t)i * n) >> 10); };
        if (count_ge(ords, kSample, 1u, spread) >= rs) {
            const uint32_t t0 = rth_best(ords, kSample, rs, 1u, spread);
            const int reach = count_ge(ords, n, t0, plain);
            if (reach >= p.R && reach <= kShort) {
                for (int i = tid; i < n; i += nt) {
                    const uint32_t v = ords[i];
                    if (v >= t0) shortlist[atomicAdd(&short_n, 1)] = v;
                }
                __syncthreads();
                result = rth_best(shortlist, reach, p.R, t0, plain);
                done = true;
            }
        }
    }
    if (!done && count_ge(ords, n, 1u, plain) >= p.R) result = rth_best(ords, n, p.R, 1u, plain);
    if (tid == 0) bound[q] = result;
}

// After the block-maxima scan, for a handful of queries, three short kernels:
//  A. select_blocks_kernel (one workgroup per query): t1 = the R-th largest block
//     maximum (exact, wg_select_threshold); the blocks whose maximum is >= t1 are listed.
//  B. rescan_blocks_kernel (one wave per listed block, spread over the chip): every
//     point with key >= t1 goes to a candidate buffer (at least R points qualify: the
//     block maxima themselves).
//  C. small_batch_final_kernel (one workgroup per query): t2 = the R-th largest
//     candidate; the R candidates >= t2 are ranked by counting, (reorder) re-scored
//     exactly, <q, x> as an fp32 fma chain, and the k best are written out.

__global__ void __launch_bounds__(1024)
select_blocks_kernel(const u64 *__restrict__ block_max, int64_t n_blocks, int R, int32_t *__restrict__ sel_blk,
                     SmallMeta *__restrict__ meta)
{
    extern __shared__ __align__(16) unsigned char smem[];
    WgSelectScratch *sel = (WgSelectScratch *)smem;
    __shared__ uint32_t n_sel;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.x;
    const u64 *bm = block_max + (size_t)q * n_blocks;
    if (tid == 0) n_sel = 0u;
    const u64 t1 = wg_select_threshold(bm, n_blocks, R, sel);
    __syncthreads();
    for (int64_t b = tid; b < n_blocks; b += nt) {
        const u64 key = bm[b];
        if (key >= t1 && key) sel_blk[(size_t)q * R + atomicAdd(&n_sel, 1u)] = (int32_t)b;
    }
    __syncthreads();
    if (tid == 0) {
        meta[q].t1 = t1;
        meta[q].n_sel = n_sel;
        meta[q].n_cand = 0u;
    }
}

// NIB: 4-bit codes with the 16-entry tables in LDS; else 256-entry byte tables.
template <bool U8, int NBT, bool NIB>
__global__ void __launch_bounds__(256)
rescan_blocks_kernel(const ScanParams p, const FinishParams f)
{
    typedef uint32_t entry_t;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int q = blockIdx.y;
    const int j = blockIdx.x * n_waves + wave;
    const int n_sel = (int)f.meta[q].n_sel;
    if ((int)(blockIdx.x * n_waves) >= n_sel) return; // whole workgroup idle
    const bool have = j < n_sel;
    const int64_t blk = have ? f.sel_blk[(size_t)q * p.R + j] : 0;
    BlockRegs<NBT> regs;
    if (have) load_block<NBT>(regs, p.codes, blk, lane);
    if (NIB) nibble_tables_fill<U8>(smem, p, q, NB);
    else build_tables<1, U8>((entry_t *)smem, p, q, NB);
    __syncthreads();
    if (!have) return;
    float sf[4];
    uint32_t si[4];
    if (NIB) {
        nibble_accumulate<U8, NBT>(smem, regs, p.codes + (size_t)blk * 256 * NB, NB, lane, sf, si);
    } else {
        entry_t acc[4];
        accumulate_block<1, U8, NBT>((const entry_t *)smem, regs, p.codes, blk, NB, lane, acc);
#pragma unroll
        for (int i = 0; i < 4; ++i) { si[i] = acc[i]; sf[i] = __uint_as_float(acc[i]); }
    }
    const u64 t1 = f.meta[q].t1;
    u64 *cand = f.cand + (size_t)q * f.cand_stride;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t slot = blk * 256 + 4 * lane + i;
        const uint32_t ord = U8 ? (si[i] + 1u) : ord_from_f32(sf[i]);
        const u64 key = make_key(ord, (int32_t)slot);
        const bool hit = slot < p.n_valid && key >= t1;
        const u64 mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask == 0ull) continue;
        uint32_t base_pos = 0;
        if (lane == 0) base_pos = atomicAdd(&f.meta[q].n_cand, (uint32_t)__builtin_popcountll(mask));
        base_pos = (uint32_t)__shfl((int)base_pos, 0, 64);
        if (hit) cand[base_pos + __builtin_popcountll(mask & ((1ull << lane) - 1ull))] = key;
    }
}

// ---- a handful of queries on a partitioned index: block maxima over the probed leaves ----
//
// A query's probed leaves hold a few hundred blocks, so the scheme of the first paragraph above runs on all of
// them with exact scores: D. leaf_block_max_kernel (one workgroup per probed leaf and query) scores the leaf's blocks
// and records, for the i-th block of the query's probe list (leaves in probe order, their blocks in order), the
// best key, the block and the leaf's <q, center>; A. select_blocks_kernel finds t1 and the R blocks that reach it;
// E. rescan_leaf_blocks_kernel scores those again and keeps the points at or above t1 (at most 256 R);
// C. small_batch_final_kernel finishes. A point's score is what the one-query scan over leaves forms: the fp32
// table sum (entries of a byte first, bytes in order) + <q, center>, or fma(integer sum, scale, bias + <q, center>);
// its key carries the point's id (perm), padding slots have none.
struct LeafBlockList {
    u64 *best;           // [B][stride] best key of the listed block, 0: no point
    int32_t *blk;        // [B][stride] the block
    float *ip;           // [B][stride] its leaf's <q, center>
    uint32_t *n_listed;  // [B] blocks in the query's list
    int64_t stride;
};

template <bool U8>
__device__ __forceinline__ float leaf_point_score(float accf, uint32_t acci, float ip, float scale, float bias)
{
    if (U8) return __fmaf_rn((float)(int)acci, scale, __fadd_rn(bias, ip));
    return __fadd_rn(accf, ip);
}

template <bool U8, int NBT>
__global__ void __launch_bounds__(256)
leaf_block_max_kernel(const ScanParams p, const LeafBlockList list)
{
    static_assert(NBT != 0, "specialised code sizes only");
    __shared__ __align__(16) unsigned char tables[2 * NBT * 16 * (U8 ? 1 : 4)];
    __shared__ int red_before[4], red_total[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.x, q = blockIdx.y;
    const int stride_l = p.leaf_stride ? p.leaf_stride : p.Lp;
    const int32_t *lids = p.leaf_ids + (size_t)q * stride_l;
    // blocks of the leaves before this one in the probe list, and of all of them
    int before = 0, total = 0;
    for (int t = tid; t < p.Lp; t += 256) {
        const int32_t l = lids[t];
        const int nb = l >= 0 ? p.leaf_blk[l + 1] - p.leaf_blk[l] : 0;
        total += nb;
        if (t < j) before += nb;
    }
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) { before += __shfl_xor(before, m, 64); total += __shfl_xor(total, m, 64); }
    if (lane == 0) { red_before[wave] = before; red_total[wave] = total; }
    const int32_t leaf = lids[j];
    const int64_t b0 = leaf >= 0 ? p.leaf_blk[leaf] : 0, b1 = leaf >= 0 ? p.leaf_blk[leaf + 1] : 0;
    BlockRegs<NBT> regs;
    int64_t blk = b0 + wave;
    if (blk < b1) load_block<NBT>(regs, p.codes, blk, lane); // in flight while the tables are filled
    nibble_tables_fill<U8>(tables, p, q, NBT);
    __syncthreads();
    before = red_before[0] + red_before[1] + red_before[2] + red_before[3];
    total = red_total[0] + red_total[1] + red_total[2] + red_total[3];
    if (j == 0 && tid == 0) list.n_listed[q] = (uint32_t)((int64_t)total < list.stride ? total : list.stride);
    const float ip = leaf >= 0 ? p.leaf_ip[(size_t)q * stride_l + j] : 0.0f;
    const float scale = U8 ? p.scale[q] : 0.0f, bias = U8 ? p.bias[q] : 0.0f;
    for (; blk < b1; blk += 4) {
        float accf[4];
        uint32_t acci[4];
        nibble_accumulate<U8, NBT>(tables, regs, p.codes + (size_t)blk * 256 * NBT, NBT, lane, accf, acci);
        const int64_t next = blk + 4;
        if (next < b1) load_block<NBT>(regs, p.codes, next, lane);
        u64 best = 0ull;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int32_t id = p.perm[blk * 256 + 4 * lane + i];
            const float sc = leaf_point_score<U8>(accf[i], acci[i], ip, scale, bias);
            const u64 key = id >= 0 ? make_key(ord_from_f32(sc), id) : 0ull;
            best = key > best ? key : best;
        }
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) best = umax64(best, shfl_xor_u64(best, m));
        const int64_t at = (int64_t)before + (blk - b0);
        if (lane == 0 && at < list.stride) {
            list.best[(size_t)q * list.stride + at] = best;
            list.blk[(size_t)q * list.stride + at] = (int32_t)blk;
            list.ip[(size_t)q * list.stride + at] = ip;
        }
    }
}

// A. for lists of different lengths: one workgroup per query over best[q][0 .. n_listed[q]); sel_blk[q][R] receives
// positions in the list.
__global__ void __launch_bounds__(1024)
select_listed_blocks_kernel(const LeafBlockList list, int R, int32_t *__restrict__ sel_blk, SmallMeta *__restrict__ meta)
{
    extern __shared__ __align__(16) unsigned char smem[];
    WgSelectScratch *sel = (WgSelectScratch *)smem;
    __shared__ uint32_t n_sel;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.x;
    const u64 *bm = list.best + (size_t)q * list.stride;
    const int64_t n = (int64_t)list.n_listed[q];
    if (tid == 0) n_sel = 0u;
    if (n <= (int64_t)kSelList && nt == 1024) {
        // the usual case, a few hundred blocks: a thread per block ranks its key by counting (keys are distinct)
        __shared__ u64 t1_s;
        const u64 mine = tid < n ? bm[tid] : 0ull;
        if (tid < kSelList) sel->list[tid] = mine; // the list holds kSelList keys; the threads beyond hold none
        if (tid == 0) t1_s = 1ull; // fewer than R blocks with a point: all of them
        __syncthreads();
        int rank = 0;
        for (int i = 0; i < (int)n; ++i) rank += sel->list[i] > mine;
        if (mine && rank < R) sel_blk[(size_t)q * R + atomicAdd(&n_sel, 1u)] = tid;
        if (mine && rank == R - 1) t1_s = mine;
        __syncthreads();
        if (tid == 0) {
            meta[q].t1 = t1_s;
            meta[q].n_sel = n_sel;
            meta[q].n_cand = 0u;
        }
        return;
    }
    const u64 t1 = wg_select_threshold(bm, n, R, sel);
    __syncthreads();
    for (int64_t b = tid; b < n; b += nt) {
        const u64 key = bm[b];
        if (key >= t1 && key) sel_blk[(size_t)q * R + atomicAdd(&n_sel, 1u)] = (int32_t)b;
    }
    __syncthreads();
    if (tid == 0) {
        meta[q].t1 = t1;
        meta[q].n_sel = n_sel;
        meta[q].n_cand = 0u;
    }
}

// E. one wave per selected block: its points at or above t1 go to the query's candidates.
template <bool U8, int NBT>
__global__ void __launch_bounds__(256)
rescan_leaf_blocks_kernel(const ScanParams p, const FinishParams f, const LeafBlockList list)
{
    static_assert(NBT != 0, "specialised code sizes only");
    __shared__ __align__(16) unsigned char tables[2 * NBT * 16 * (U8 ? 1 : 4)];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int q = blockIdx.y;
    const int j = blockIdx.x * n_waves + wave;
    const int n_sel = (int)f.meta[q].n_sel;
    if ((int)(blockIdx.x * n_waves) >= n_sel) return; // whole workgroup idle
    const bool have = j < n_sel;
    const int at = have ? f.sel_blk[(size_t)q * p.R + j] : 0;
    const int64_t blk = have ? list.blk[(size_t)q * list.stride + at] : 0;
    BlockRegs<NBT> regs;
    if (have) load_block<NBT>(regs, p.codes, blk, lane);
    nibble_tables_fill<U8>(tables, p, q, NBT);
    __syncthreads();
    if (!have) return;
    const float ip = list.ip[(size_t)q * list.stride + at];
    const float scale = U8 ? p.scale[q] : 0.0f, bias = U8 ? p.bias[q] : 0.0f;
    float accf[4];
    uint32_t acci[4];
    nibble_accumulate<U8, NBT>(tables, regs, p.codes + (size_t)blk * 256 * NBT, NBT, lane, accf, acci);
    const u64 t1 = f.meta[q].t1;
    u64 *cand = f.cand + (size_t)q * f.cand_stride;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int32_t id = p.perm[blk * 256 + 4 * lane + i];
        const float sc = leaf_point_score<U8>(accf[i], acci[i], ip, scale, bias);
        const u64 key = id >= 0 ? make_key(ord_from_f32(sc), id) : 0ull;
        const bool hit = key >= t1 && key != 0ull;
        const u64 mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask == 0ull) continue;
        uint32_t base_pos = 0;
        if (lane == 0) base_pos = atomicAdd(&f.meta[q].n_cand, (uint32_t)__builtin_popcountll(mask));
        base_pos = (uint32_t)__shfl((int)base_pos, 0, 64);
        const u64 pos = (u64)base_pos + (u64)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
        if (hit && pos < (u64)f.cand_stride) cand[pos] = key;
    }
}

// ---- a handful of queries: block bounds from 8-bit tables, then exact scores of few blocks ----
//
// The full scan of a single query is bound by reading the codes only if a point's score costs
// almost nothing, and a table lookup in LDS costs the same 64 lanes x 4 bytes per instruction
// whatever the entry holds. So the full scan does not form the scores at all: per byte
// position b it holds a 256-entry table of *bytes*, U[b][v], an 8-bit image of the entry (or,
// for 4-bit codes, of the sum of the two entries) that byte value v stands for. 256 bytes are
// 64 LDS words, a quarter of what fp32 entries take (a wave's random byte reads over 64 words
// measure 1.3 clocks of a compute unit, 0.8 over 32 words or fewer): one read and one
// integer add per code byte. The integer sum I of a point determines its score within a margin:
//   fp32 tables:  U[b][v] = rne((t_b(v) - lo_b) * c), t_b(v) the fp32 entry (4-bit codes: the fp32
//     sum of the two entries of byte v, which is also the first step of the defined order of
//     additions), lo_b = min_v t_b(v), c = 255 / max_b(max_v t_b(v) - lo_b). Each term moves by at
//     most 1/2 + 4e-5 units of 1/c (rounding to the nearest integer plus the two fp32 roundings
//     before it), and the fp32 score s (NB - 1 additions in order, each within 2^-24 of the partial
//     sum's magnitude, at most A = sum_b max_v |t_b(v)|) is within rho = NB * 2^-24 * A of the real
//     sum, so  | s - (sum_b lo_b + I / c) | <= E / c + rho,  E = NB * (1/2 + 4e-5).
//   8-bit tables, 4-bit codes: U[b][v] = (Q[2b][v & 15] + Q[2b+1][v >> 4] + 1) >> 1, so the exact
//     integer score lies in [2 I - NB, 2 I];   8-bit tables, 8-bit codes: U = Q, I is the score.
// Let theta be the R-th largest of the block maxima of I. R blocks hold a point with I >= theta each,
// so the R-th best score is at least low(theta), and a point with I < theta - m, m = the margin in
// units of I that makes high(I) < low(theta), is not among the R best. Hence: the blocks whose
// maximum reaches theta - m are scored exactly, and of their points those at or above low(theta)
// become candidates -- a superset of the R best by the exact scores, whatever the data.
// block_bound_kernel writes the block maxima of I; select_bound_blocks_kernel finds theta (a
// histogram: I < 8192) and lists the blocks; rescan_listed_blocks_kernel scores them exactly.

// The byte tables U of one query (one workgroup each), written to bound_tbl[q][NB][256] for the scan to copy
// into LDS: made once here, not once per workgroup of the scan, because a scan of a few microseconds cannot
// hide the making (6400 entries at 25 code bytes: as much work as scanning four blocks) behind its loads.
// U8: the search uses 8-bit tables; WIDE: 8-bit codes (else 4-bit codes, two per byte). With 4-bit codes
// the 16-entry tables are read (p.lut, p.lut8) or, for fp32 tables when p.fuse_queries is set, computed
// here (the fma chain of the table kernel) and left in p.lut_out for the kernels that follow.
constexpr int kBoundBins = 8192; // bins of the selection's histogram: sums of byte table entries are at most 255 * 32

template <bool U8, bool WIDE>
__global__ void __launch_bounds__(1024)
bound_tables_kernel(const ScanParams p)
{
    constexpr int kMaxNB = 32;
    if (p.sel_hist != nullptr && (int)blockIdx.x < p.B) // the split selection adds to these: cleared here, two launches ahead
        for (int b = threadIdx.x; b < kBoundBins; b += blockDim.x) p.sel_hist[(size_t)blockIdx.x * kBoundBins + b] = 0u;
    __shared__ __align__(16) float nib[WIDE ? 4 : 2 * kMaxNB * 16]; // 4-bit codes: the 16-entry tables (8-bit tables: as bytes)
    __shared__ float tmin[2 * kMaxNB], tmax[2 * kMaxNB], lo_s[kMaxNB], c_s;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const int q = blockIdx.x;
    const int NB = p.NB;
    // Word `it` of a query's tables = the entries of byte position it / 64, byte values 4 (it % 64) .. + 3. Plain
    // layout: [q][NB][256] bytes. Tile layout (p.bound_tile = 16, the batch scan): [q / 16][NB][256][16], the
    // sixteen queries of a tile side by side in every entry; the launch covers whole tiles and the queries
    // beyond the batch get zero tables (their bytes share words with live queries' in the scan's sums).
    auto put = [&](int it, uint32_t pack) {
        if (p.bound_tile == 0) {
            ((uint32_t *)(p.bound_tbl + (size_t)q * NB * 256))[it] = pack;
        } else {
            uint8_t *dst = p.bound_tbl + (((size_t)(q >> 4) * NB * 256 + (size_t)it * 4) << 4) + (q & 15);
#pragma unroll
            for (int k = 0; k < 4; ++k) dst[k * 16] = (uint8_t)(pack >> (8 * k));
        }
    };
    if (q >= p.B) {
        for (int it = tid; it < NB * 64; it += nt) put(it, 0u);
        return;
    }
    const float levels = (float)(p.bound_levels > 0 ? p.bound_levels : 255);
    if constexpr (U8 && WIDE) {
        const uint32_t *L = (const uint32_t *)(p.lut8 + (size_t)q * NB * 256);
        const uint32_t keep = 0x01010101u * (0xffu >> p.bound_shift);
        for (int it = tid; it < NB * 64; it += nt) put(it, (L[it] >> p.bound_shift) & keep);
        return;
    }
    if constexpr (U8 && !WIDE) {
        unsigned char *n8 = (unsigned char *)nib;
        const int live = p.M * 16;
        const uint8_t *L = p.lut8 + (size_t)q * live;
        for (int e = tid; e < 2 * NB * 16; e += nt) n8[e] = e < live ? L[e] : (uint8_t)0;
        __syncthreads();
        for (int it = tid; it < NB * 64; it += nt) {
            const int b = it >> 6, v0 = (it & 63) * 4;
            const uint32_t hi = n8[32 * b + 16 + (v0 >> 4)];
            uint32_t pack = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) pack |= (((uint32_t)n8[32 * b + (v0 & 15) + k] + hi + 1u) >> 1) << (8 * k);
            put(it, pack);
        }
        return;
    }
    if constexpr (!U8) {
        const float *Lw = nullptr;
        if constexpr (WIDE) {
            Lw = p.lut + (size_t)q * NB * 256;
            for (int b = wave; b < NB; b += n_waves) {
                const float4 e = ((const float4 *)(Lw + (size_t)b * 256))[lane];
                float mn = fminf(fminf(e.x, e.y), fminf(e.z, e.w)), mx = fmaxf(fmaxf(e.x, e.y), fmaxf(e.z, e.w));
#pragma unroll
                for (int m = 32; m > 0; m >>= 1) {
                    mn = fminf(mn, __shfl_xor(mn, m, 64));
                    mx = fmaxf(mx, __shfl_xor(mx, m, 64));
                }
                if (lane == 0) { tmin[b] = mn; tmax[b] = mx; }
            }
        } else {
            // one entry per thread (2 * NB * 16 <= 1024 = blockDim.x); a table's 16 entries sit in 16 neighbouring
            // lanes: its extremes by four exchanges
            const int live = p.M * 16, e = tid;
            float v = 0.0f;
            if (e < live) {
                if (p.fuse_queries != nullptr) {
                    const int ds = p.fuse_d / p.M;
                    const float *c = p.fuse_codebooks + (size_t)e * ds;
                    const float *qm = p.fuse_queries + (size_t)q * p.fuse_d + (e >> 4) * ds;
                    for (int l = 0; l < ds; ++l) v = __fmaf_rn(qm[l], c[l], v);
                    if (p.lut_out != nullptr) p.lut_out[(size_t)q * live + e] = v;
                } else {
                    v = p.lut[(size_t)q * live + e];
                }
            }
            float mn = v, mx = v;
#pragma unroll
            for (int m = 1; m < 16; m <<= 1) {
                mn = fminf(mn, __shfl_xor(mn, m, 64));
                mx = fmaxf(mx, __shfl_xor(mx, m, 64));
            }
            if (e < 2 * NB * 16) {
                nib[e] = v;
                if ((e & 15) == 0) { tmin[e >> 4] = mn; tmax[e >> 4] = mx; }
            }
        }
        __syncthreads();
        // Range of every byte position's entries (fp32 addition is monotone: the extremes of the sums of two
        // entries are the sums of the extremes), the units per score unit, and what the margin follows from.
        if (wave == 0) {
            float lo = 0.0f, hi = 0.0f;
            if (lane < NB) {
                if constexpr (WIDE) { lo = tmin[lane]; hi = tmax[lane]; }
                else { lo = __fadd_rn(tmin[2 * lane], tmin[2 * lane + 1]); hi = __fadd_rn(tmax[2 * lane], tmax[2 * lane + 1]); }
                lo_s[lane] = lo;
            }
            float range = lane < NB ? __fsub_rn(hi, lo) : 0.0f;
            double sum_lo = (double)lo, amax = (double)fmaxf(fabsf(lo), fabsf(hi));
#pragma unroll
            for (int m = 32; m > 0; m >>= 1) {
                range = fmaxf(range, __shfl_xor(range, m, 64));
                sum_lo += __shfl_xor(sum_lo, m, 64);
                amax += __shfl_xor(amax, m, 64);
            }
            const float c = range > 1e-30f ? __fdiv_rn(levels, range) : 0.0f;
            if (lane == 0) {
                c_s = c;
                BoundMeta bm;
                bm.sum_lo = sum_lo; bm.amax = amax; bm.c = c; bm.pad = 0;
                p.bound_meta[q] = bm;
            }
        }
        __syncthreads();
        const float c = c_s;
        for (int it = tid; it < NB * 64; it += nt) {
            const int b = it >> 6, v0 = (it & 63) * 4;
            const float lo_b = lo_s[b];
            float t[4];
            if constexpr (WIDE) {
                const float4 e = ((const float4 *)(Lw + (size_t)b * 256))[it & 63];
                t[0] = e.x; t[1] = e.y; t[2] = e.z; t[3] = e.w;
            } else {
                const float hi = nib[32 * b + 16 + (v0 >> 4)];
#pragma unroll
                for (int k = 0; k < 4; ++k) t[k] = __fadd_rn(nib[32 * b + (v0 & 15) + k], hi);
            }
            uint32_t pack = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float u = rintf(__fmul_rn(__fsub_rn(t[k], lo_b), c));
                u = fminf(fmaxf(u, 0.0f), levels);
                pack |= (uint32_t)u << (8 * k);
            }
            put(it, pack);
        }
    }
}

// The full scan: block maxima of the sums of the byte tables' entries. A wave's loads come back in the order
// they were issued, so the workgroup's copy of the tables is asked for before the wave's first block of codes.
template <int NBT, bool NT>
__device__ __forceinline__ void block_bound_body(const ScanParams &p)
{
    static_assert(NBT != 0 && NBT <= 32, "specialised code sizes only");
    constexpr int kWords = NBT * 64, kPer = 8; // table words per thread: kWords <= 2048 = kPer * 256 <= kPer * blockDim.x
    __shared__ __align__(16) unsigned char tbl8[NBT * 256];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const int q = blockIdx.y;
    const int64_t step = (int64_t)gridDim.x * n_waves;
    int64_t blk = (int64_t)blockIdx.x * n_waves + wave;
    BlockRegs<NBT> regs, nxt;
    {
        const uint32_t *src = (const uint32_t *)(p.bound_tbl + (size_t)q * NBT * 256);
        uint32_t tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int it = tid + i * nt;
            tv[i] = it < kWords ? src[it] : 0u;
        }
        asm volatile("" ::: "memory");
        if (blk < p.n_blocks) load_block<NBT, NT>(regs, p.codes, blk, lane);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int it = tid + i * nt;
            if (it < kWords) ((uint32_t *)tbl8)[it] = tv[i];
        }
    }
    __syncthreads();

    for (; blk < p.n_blocks; blk += step) {
        const bool more = blk + step < p.n_blocks;
        if (more) load_block<NBT, NT>(nxt, p.codes, blk + step, lane);
        uint32_t acc[4] = {0u, 0u, 0u, 0u};
        auto plane = [&](uint32_t w, const unsigned char *t) {
            acc[0] += t[w & 0xffu];
            acc[1] += t[(w >> 8) & 0xffu];
            acc[2] += t[(w >> 16) & 0xffu];
            acc[3] += t[w >> 24];
        };
#pragma unroll
        for (int j = 0; j < NBT / 4; ++j) {
            const unsigned char *t = tbl8 + (size_t)j * 1024;
            plane(regs.rows[j].x, t);
            plane(regs.rows[j].y, t + 256);
            plane(regs.rows[j].z, t + 512);
            plane(regs.rows[j].w, t + 768);
            // keeps a row's sixteen reads together and the sums in four registers (see nibble_accumulate)
            asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
        }
#pragma unroll
        for (int tt = 0; tt < NBT % 4; ++tt) plane(regs.tails[tt], tbl8 + (size_t)((NBT / 4) * 4 + tt) * 256);
        uint32_t best = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (blk * 256 + 4 * lane + i < p.n_valid) best = acc[i] > best ? acc[i] : best;
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)best, m, 64);
            best = o > best ? o : best;
        }
        if (lane == 0) p.block_bound[(size_t)q * p.n_blocks + blk] = best;
        if (more) regs = nxt;
    }
}

template <int NBT>
__global__ void __launch_bounds__(1024)
block_bound_kernel(const ScanParams p)
{
    block_bound_body<NBT, false>(p);
}

// The same scan over a code array that exceeds the Infinity Cache: nontemporal loads (see load_block), launched
// with one block per wave.
template <int NBT>
__global__ void __launch_bounds__(1024)
block_bound_stream_kernel(const ScanParams p)
{
    block_bound_body<NBT, true>(p);
}

// The same block maxima for a batch: a workgroup holds the byte tables of sixteen queries in LDS, side by side in
// every entry (16 bytes per byte position and byte value: one 16-byte read serves sixteen queries), and its
// waves take the blocks of one chunk of the index in turn. Table entries are at most 63 (six bits, GROUP = 4), so
// that the entries of four byte positions are added as packed bytes before they are spread into 16-bit sums, at
// most 127 (seven bits, GROUP = 2: two positions per packed sum, bounds half as wide, so a third as many blocks
// are scored exactly afterwards) or the full 8 bits (GROUP = 1: every entry spread by itself). One 32-bit store
// per query and block.
typedef unsigned short pk_u16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    const pk_u16 r = __builtin_elementwise_max(*(const pk_u16 *)&a, *(const pk_u16 *)&b);
    return *(const uint32_t *)&r;
}

template <int NBT, int GROUP>
__global__ void __launch_bounds__(1024)
block_bound_tile_kernel(const ScanParams p)
{
    static_assert(GROUP == 4 || GROUP == 2 || GROUP == 1, "packed sums of four or two entries, or none");
    static_assert(NBT != 0 && NBT <= 32, "specialised code sizes only");
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    const uint4 *tbl = (const uint4 *)dyn_smem; // [NBT][256] entries of 16 queries
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const int tile = blockIdx.x, q0 = tile * 16;
    const int64_t c0 = (int64_t)blockIdx.y * p.blocks_per_chunk;
    const int64_t c1 = c0 + p.blocks_per_chunk < p.n_blocks ? c0 + p.blocks_per_chunk : p.n_blocks;
    int64_t blk = c0 + wave;
    BlockRegs<NBT> regs, nxt;
    if (blk < c1) load_block<NBT>(regs, p.codes, blk, lane);
    {
        const uint4 *src = (const uint4 *)(p.bound_tbl + (size_t)tile * NBT * 256 * 16);
        for (int it = tid; it < NBT * 256; it += nt) ((uint4 *)dyn_smem)[it] = src[it];
    }
    __syncthreads();
    for (; blk < c1; blk += n_waves) {
        const bool more = blk + n_waves < c1;
        if (more) load_block<NBT>(nxt, p.codes, blk + n_waves, lane);
        uint32_t even[4][4], odd[4][4]; // [point][word]: 16-bit sums of queries 4w, 4w + 2 (even) and 4w + 1, 4w + 3 (odd)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int w = 0; w < 4; ++w) { even[i][w] = 0u; odd[i][w] = 0u; }
        auto spread = [&](int i, const uint4 &sum) {
            const uint32_t sw[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                even[i][w] += sw[w] & 0x00ff00ffu;
                odd[i][w] += (sw[w] >> 8) & 0x00ff00ffu;
            }
        };
        auto entry = [&](uint32_t word, int i, int b) -> uint4 { return tbl[b * 256 + ((word >> (8 * i)) & 0xffu)]; };
        auto add4 = [](const uint4 &a, const uint4 &b) -> uint4 { return make_uint4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); };
#pragma unroll
        for (int j = 0; j < NBT / 4; ++j) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 lo2 = add4(entry(regs.rows[j].x, i, 4 * j), entry(regs.rows[j].y, i, 4 * j + 1));
                const uint4 hi2 = add4(entry(regs.rows[j].z, i, 4 * j + 2), entry(regs.rows[j].w, i, 4 * j + 3));
                if constexpr (GROUP == 4) {
                    spread(i, add4(lo2, hi2));
                } else if constexpr (GROUP == 2) {
                    spread(i, lo2);
                    spread(i, hi2);
                } else {
                    spread(i, entry(regs.rows[j].x, i, 4 * j));
                    spread(i, entry(regs.rows[j].y, i, 4 * j + 1));
                    spread(i, entry(regs.rows[j].z, i, 4 * j + 2));
                    spread(i, entry(regs.rows[j].w, i, 4 * j + 3));
                }
                // keeps a point's four reads together and the sums where they are: left alone the compiler reads
                // every entry of the block first and spills
                asm volatile("" : "+v"(even[i][0]), "+v"(even[i][1]), "+v"(even[i][2]), "+v"(even[i][3]),
                                  "+v"(odd[i][0]), "+v"(odd[i][1]), "+v"(odd[i][2]), "+v"(odd[i][3]));
            }
        }
        if constexpr (NBT % 4 != 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint4 sum = entry(regs.tails[0], i, (NBT / 4) * 4);
#pragma unroll
                for (int tt = 1; tt < NBT % 4; ++tt) {
                    if ((GROUP == 2 && tt == 2) || GROUP == 1) { // the third of three goes by itself
                        spread(i, sum);
                        sum = entry(regs.tails[tt], i, (NBT / 4) * 4 + tt);
                    } else {
                        sum = add4(sum, entry(regs.tails[tt], i, (NBT / 4) * 4 + tt));
                    }
                }
                spread(i, sum);
            }
        }
        // best of the lane's four points (padding slots of the last block count for nothing), then of the wave
        uint32_t be[4], bo[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) { be[w] = 0u; bo[w] = 0u; }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool valid = blk * 256 + 4 * lane + i < p.n_valid;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                be[w] = pk_max_u16(be[w], valid ? even[i][w] : 0u);
                bo[w] = pk_max_u16(bo[w], valid ? odd[i][w] : 0u);
            }
        }
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                be[w] = pk_max_u16(be[w], (uint32_t)__shfl_xor((int)be[w], m, 64));
                bo[w] = pk_max_u16(bo[w], (uint32_t)__shfl_xor((int)bo[w], m, 64));
            }
        }
        if (lane < 16 && q0 + lane < p.B) {
            // query lane of the tile: byte lane & 3 of word lane >> 2; bytes 0, 2 are in `even`, 1, 3 in `odd`
            const int w = lane >> 2, byte = lane & 3;
            uint32_t v = 0;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww)
                if (ww == w) v = (byte & 1) ? bo[ww] : be[ww];
            v = (byte & 2) ? (v >> 16) : (v & 0xffffu);
            p.block_bound[(size_t)(q0 + lane) * p.n_blocks + blk] = v;
        }
        if (more) regs = nxt;
    }
}

// Measurement aid: the lookups and additions of block_bound_kernel in its launch shape, with no code stream --
// a wave's code words are made up from its block number (a different byte in every position, lane and block)
// instead of being loaded. Its duration is what the table lookups of a scan cost by themselves.
template <int NBT>
__global__ void __launch_bounds__(1024)
lookup_only_kernel(const ScanParams p)
{
    __shared__ __align__(16) unsigned char tbl8[NBT * 256];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const int q = blockIdx.y;
    const int64_t step = (int64_t)gridDim.x * n_waves;
    const uint32_t *src = (const uint32_t *)(p.bound_tbl + (size_t)q * NBT * 256);
    for (int it = tid; it < NBT * 64; it += nt) ((uint32_t *)tbl8)[it] = src[it];
    __syncthreads();
    for (int64_t blk = (int64_t)blockIdx.x * n_waves + wave; blk < p.n_blocks; blk += step) {
        uint32_t acc[4] = {0u, 0u, 0u, 0u};
        uint32_t w = (uint32_t)blk * 2654435761u + (uint32_t)lane * 40503u;
        auto plane = [&](const unsigned char *t) {
            w = w * 1664525u + 1013904223u;
            acc[0] += t[w & 0xffu];
            acc[1] += t[(w >> 8) & 0xffu];
            acc[2] += t[(w >> 16) & 0xffu];
            acc[3] += t[w >> 24];
        };
#pragma unroll
        for (int b = 0; b < NBT; ++b) {
            plane(tbl8 + (size_t)b * 256);
            if ((b & 3) == 3) asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
        }
        uint32_t best = acc[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) best = acc[i] > best ? acc[i] : best;
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)best, m, 64);
            best = o > best ? o : best;
        }
        if (lane == 0) p.block_bound[(size_t)q * p.n_blocks + blk] = best;
    }
}

// fn(block, its maximum) for the blocks [b0, b0 + cnt) of a query's row bb, by the calling workgroup. With
// hundreds of thousands of blocks a pass is all memory latency: 16-byte loads, four of them in flight per thread
// (the few values before the first 16-byte boundary and after the last go one by one).
template <class F>
__device__ __forceinline__ void for_every_block(const uint32_t *__restrict__ bb, int64_t b0, int64_t cnt, int tid, int nt, F fn)
{
    const uint32_t *row = bb + b0;
    const int64_t mis = (int64_t)((4u - (uint32_t)(((size_t)row >> 2) & 3u)) & 3u);
    const int64_t head = mis < cnt ? mis : cnt;
    const int64_t n4 = (cnt - head) / 4;
    const uint4 *b4 = (const uint4 *)(row + head);
    if (tid < head) fn(b0 + tid, row[tid]);
    for (int64_t i0 = tid; i0 < n4; i0 += (int64_t)4 * nt) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { const int64_t i = i0 + (int64_t)u * nt; v[u] = i < n4 ? b4[i] : make_uint4(0u, 0u, 0u, 0u); }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + (int64_t)u * nt;
            if (i >= n4) continue;
            const int64_t b = b0 + head + 4 * i;
            fn(b, v[u].x); fn(b + 1, v[u].y); fn(b + 2, v[u].z); fn(b + 3, v[u].w);
        }
    }
    const int64_t b = head + 4 * n4 + tid;
    if (b < cnt) fn(b0 + b, row[b]);
}

// theta = the largest bin with at least `need` counts at or above it (hist[kBoundBins] in LDS, 1,024 threads; ends
// with a barrier, *theta_s valid afterwards; 0 when fewer than `need` counts exist).
__device__ __forceinline__ int theta_from_hist(const uint32_t *hist, uint32_t need, uint32_t *wave_sum, uint32_t *theta_s, int tid)
{
    const int lane = tid & 63, wave = tid >> 6, n_waves = 16;
    constexpr int per = kBoundBins / 1024; // bins per thread
    uint32_t mine = 0;
    for (int j = 0; j < per; ++j) mine += hist[tid * per + j];
    uint32_t suf = mine;
    for (int m = 1; m < 64; m <<= 1) {
        const uint32_t o = (uint32_t)__shfl_down((int)suf, m, 64);
        if (lane + m < 64) suf += o;
    }
    if (lane == 0) wave_sum[wave] = suf;
    __syncthreads();
    uint32_t above = suf - mine;
    for (int w = wave + 1; w < n_waves; ++w) above += wave_sum[w];
    for (int j = per - 1; j >= 0; --j) {
        const uint32_t h = hist[tid * per + j];
        if (above < need && need <= above + h) *theta_s = (uint32_t)(tid * per + j);
        above += h;
    }
    __syncthreads();
    return (int)*theta_s;
}

// From theta: the smallest block maximum worth a look (returned) and the lower bound of the R-th best exact score
// as a key threshold (*t1). kind 0: fp32 tables (margin and bound from bm, see above), 1: 8-bit tables on 4-bit
// codes (sums halved), 2: 8-bit tables on 8-bit codes (the tables themselves, or without their `shift` low bits).
__device__ __forceinline__ uint32_t cut_from_theta(int theta, int kind, int NB, int shift, const BoundMeta &bm, bool few_blocks, u64 *t1_out)
{
    int margin;
    u64 t1;
    if (kind == 0) {
        const double E = (double)NB * (0.5 + 4e-5);
        const double rho = (double)NB * 5.9604644775390625e-8 * bm.amax * 1.000001;
        const double c = (double)bm.c;
        if (c > 0.0) {
            margin = (int)ceil(2.0 * E + 2.0 * rho * c) + 1;
            const double low = bm.sum_lo + ((double)theta - E) / c - rho;
            float lf = (float)(low - fabs(low) * 1e-7 - 1e-30);
            if ((double)lf > low) lf = nextafterf(lf, -INFINITY);
            t1 = (u64)ord_from_f32(lf) << 32;
        } else {
            margin = kBoundBins; // flat tables: every block, every point
            t1 = 1ull;
        }
    } else if (kind == 1) {
        margin = (NB + 1) / 2;
        const int low = 2 * theta - NB;
        t1 = (u64)(uint32_t)((low > 0 ? low : 0) + 1) << 32;
    } else {
        // the tables are the 8-bit tables less their `shift` low bits: the exact sum lies in [s I, s I + (s - 1) NB]
        const int sc = 1 << shift;
        margin = ((sc - 1) * NB + sc - 1) / sc;
        t1 = (u64)(uint32_t)(sc * theta + 1) << 32;
    }
    if (few_blocks) t1 = 1ull; // fewer blocks than R: no R points are known to reach any bound
    *t1_out = t1;
    return theta > margin ? (uint32_t)(theta - margin) : 0u;
}

// One workgroup per query: theta = the R-th largest block maximum of the 8-bit sums, the list of the blocks
// whose maximum reaches theta - margin, and the key threshold meta[q].t1.
__global__ void __launch_bounds__(1024)
select_bound_blocks_kernel(const uint32_t *__restrict__ block_bound, int64_t n_blocks, int R, int NB, int kind, int shift,
                           const BoundMeta *__restrict__ bound_meta, int32_t *__restrict__ sel_blk,
                           SmallMeta *__restrict__ meta)
{
    __shared__ uint32_t hist[kBoundBins];
    __shared__ uint32_t wave_sum[16];
    __shared__ uint32_t theta_s, n_sel;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.x;
    const uint32_t *bb = block_bound + (size_t)q * n_blocks;
    for (int b = tid; b < kBoundBins; b += nt) hist[b] = 0u;
    if (tid == 0) { theta_s = 0u; n_sel = 0u; }
    __syncthreads();
    for_every_block(bb, 0, n_blocks, tid, nt, [&](int64_t, uint32_t v) { atomicAdd(&hist[v < (uint32_t)kBoundBins ? v : kBoundBins - 1], 1u); });
    __syncthreads();
    const int theta = theta_from_hist(hist, (uint32_t)(n_blocks < R ? n_blocks : R), wave_sum, &theta_s, tid);
    u64 t1;
    const BoundMeta bm = kind == 0 ? bound_meta[q] : BoundMeta{};
    const uint32_t cut = cut_from_theta(theta, kind, NB, shift, bm, n_blocks < R, &t1);
    for_every_block(bb, 0, n_blocks, tid, nt, [&](int64_t b, uint32_t v) {
        if (v >= cut) sel_blk[(size_t)q * n_blocks + atomicAdd(&n_sel, 1u)] = (int32_t)b;
    });
    __syncthreads();
    if (tid == 0) {
        meta[q].t1 = t1;
        meta[q].n_sel = n_sel;
        meta[q].n_cand = 0u;
    }
}

// The same over several compute units, for a few queries on a large index, where one workgroup's two passes
// over the block maxima are bound by what a single compute unit draws from memory. Two launches of one
// workgroup per `per` blocks and query. The first counts its blocks into a histogram in LDS and adds the bins it
// filled to the query's histogram in global memory (sel_hist[q][8192], cleared by bound_tables_kernel). In the
// second every workgroup reads that histogram back, finds theta for itself, and lists those of its blocks that
// reach the cut, taking room in the query's list with one atomic addition to meta[q].n_sel.
constexpr int kSelSplitMaxPer = 8192; // blocks per workgroup (its list in LDS)

__global__ void __launch_bounds__(1024)
select_split_count_kernel(const uint32_t *__restrict__ block_bound, int64_t n_blocks, int per, uint32_t *__restrict__ sel_hist,
                          SmallMeta *__restrict__ meta)
{
    __shared__ uint32_t hist[kBoundBins];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.y;
    const uint32_t *bb = block_bound + (size_t)q * n_blocks;
    uint32_t *gh = sel_hist + (size_t)q * kBoundBins;
    for (int b = tid; b < kBoundBins; b += nt) hist[b] = 0u;
    if (blockIdx.x == 0 && tid == 0) meta[q].n_sel = 0u;
    __syncthreads();
    const int64_t b0 = (int64_t)blockIdx.x * per;
    const int64_t cnt = b0 + per <= n_blocks ? per : (b0 < n_blocks ? n_blocks - b0 : 0);
    for_every_block(bb, b0, cnt, tid, nt, [&](int64_t, uint32_t v) { atomicAdd(&hist[v < (uint32_t)kBoundBins ? v : kBoundBins - 1], 1u); });
    __syncthreads();
    for (int b = tid; b < kBoundBins; b += nt)
        if (hist[b]) atomicAdd(&gh[b], hist[b]);
}

__global__ void __launch_bounds__(1024)
select_split_list_kernel(const uint32_t *__restrict__ block_bound, int64_t n_blocks, int per, int R, int NB, int kind, int shift,
                         const BoundMeta *__restrict__ bound_meta, const uint32_t *__restrict__ sel_hist,
                         int32_t *__restrict__ sel_blk, SmallMeta *__restrict__ meta)
{
    __shared__ __align__(16) uint32_t hist[kBoundBins]; // then the workgroup's list
    __shared__ uint32_t wave_sum[16];
    __shared__ uint32_t theta_s, n_loc, base;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.y;
    const uint32_t *bb = block_bound + (size_t)q * n_blocks;
    {
        const uint4 *gh = (const uint4 *)(sel_hist + (size_t)q * kBoundBins);
        uint4 h[kBoundBins / 4096];
#pragma unroll
        for (int u = 0; u < kBoundBins / 4096; ++u) h[u] = gh[tid + u * 1024];
#pragma unroll
        for (int u = 0; u < kBoundBins / 4096; ++u) ((uint4 *)hist)[tid + u * 1024] = h[u];
    }
    if (tid == 0) { theta_s = 0u; n_loc = 0u; }
    __syncthreads();
    const int theta = theta_from_hist(hist, (uint32_t)(n_blocks < R ? n_blocks : R), wave_sum, &theta_s, tid);
    u64 t1;
    const BoundMeta bm = kind == 0 ? bound_meta[q] : BoundMeta{};
    const uint32_t cut = cut_from_theta(theta, kind, NB, shift, bm, n_blocks < R, &t1);
    if (blockIdx.x == 0 && tid == 0) {
        meta[q].t1 = t1;
        meta[q].n_cand = 0u;
    }
    __syncthreads(); // every thread has read its bins: the array becomes the list
    int32_t *loc = (int32_t *)hist;
    const int64_t b0 = (int64_t)blockIdx.x * per;
    const int64_t cnt = b0 + per <= n_blocks ? per : (b0 < n_blocks ? n_blocks - b0 : 0);
    for_every_block(bb, b0, cnt, tid, nt, [&](int64_t b, uint32_t v) {
        if (v >= cut) loc[atomicAdd(&n_loc, 1u)] = (int32_t)b;
    });
    __syncthreads();
    if (tid == 0) base = n_loc ? atomicAdd(&meta[q].n_sel, n_loc) : 0u;
    __syncthreads();
    int32_t *dst = sel_blk + (size_t)q * n_blocks + base;
    for (uint32_t i = tid; i < n_loc; i += nt) dst[i] = loc[i];
}

// Exact scores of the listed blocks of every query, the waves of a query's workgroups taking the blocks
// in turn: every point whose key reaches meta[q].t1 is appended to the query's candidates (beyond
// f.cand_stride of them the count keeps running and the keys are dropped: the final kernel then
// rebuilds the candidates from block_max), and block_max[q][j] receives the best key of the j-th listed block.
template <bool U8, int NBT, bool NIB>
__global__ void __launch_bounds__(256)
rescan_listed_blocks_kernel(const ScanParams p, const FinishParams f)
{
    typedef uint32_t entry_t;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int q = blockIdx.y;
    const int n_sel = (int)f.meta[q].n_sel;
    if ((int)(blockIdx.x * n_waves) >= n_sel) return; // whole workgroup idle
    const int step = (int)gridDim.x * n_waves;
    int j = blockIdx.x * n_waves + wave;
    const int32_t *sel = f.sel_blk + (size_t)q * p.n_blocks;
    BlockRegs<NBT> regs;
    int64_t blk = j < n_sel ? sel[j] : 0;
    if (j < n_sel) load_block<NBT>(regs, p.codes, blk, lane);
    if (NIB) nibble_tables_fill<U8>(smem, p, q, NB);
    else build_tables<1, U8>((entry_t *)smem, p, q, NB);
    __syncthreads();
    const u64 t1 = f.meta[q].t1;
    u64 *cand = f.cand + (size_t)q * f.cand_stride;
    for (; j < n_sel; j += step) {
        float sf[4];
        uint32_t si[4];
        if (NIB) {
            nibble_accumulate<U8, NBT>(smem, regs, p.codes + (size_t)blk * 256 * NB, NB, lane, sf, si);
        } else {
            entry_t acc[4];
            accumulate_block<1, U8, NBT>((const entry_t *)smem, regs, p.codes, blk, NB, lane, acc);
#pragma unroll
            for (int i = 0; i < 4; ++i) { si[i] = acc[i]; sf[i] = __uint_as_float(acc[i]); }
        }
        const int64_t this_blk = blk;
        if (j + step < n_sel) { // the next block's codes travel while this one's candidates are written
            blk = sel[j + step];
            load_block<NBT>(regs, p.codes, blk, lane);
        }
        u64 best = 0ull;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t slot = this_blk * 256 + 4 * lane + i;
            const uint32_t ord = U8 ? (si[i] + 1u) : ord_from_f32(sf[i]);
            const u64 key = slot < p.n_valid ? make_key(ord, (int32_t)slot) : 0ull;
            best = key > best ? key : best;
            const bool hit = key >= t1 && key != 0ull;
            const u64 mask = __builtin_amdgcn_ballot_w64(hit);
            if (mask == 0ull) continue;
            uint32_t base_pos = 0;
            if (lane == 0) base_pos = atomicAdd(&f.meta[q].n_cand, (uint32_t)__builtin_popcountll(mask));
            base_pos = (uint32_t)__shfl((int)base_pos, 0, 64);
            const u64 at = (u64)base_pos + (u64)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
            if (hit && at < (u64)f.cand_stride) cand[at] = key;
        }
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) best = umax64(best, shfl_xor_u64(best, m));
        if (lane == 0) p.block_max[(size_t)q * p.n_blocks + j] = best;
    }
}

// Number of keys of keys[0..c) above `mine`, counted by four neighbouring lanes (part =
// lane & 3 takes every fourth key); all four must call it together.
__device__ __forceinline__ int rank_by_four(const u64 *keys, int c, u64 mine, int part)
{
    int r = 0;
#pragma unroll 4
    for (int t = part; t < c; t += 4) r += keys[t] > mine;
    r += __shfl_xor(r, 1, 64);
    r += __shfl_xor(r, 2, 64);
    return r;
}

// key_kind 1: the keys carry integer sums of 8-bit table codes (flat index); 0: fp32 scores.
__global__ void __launch_bounds__(1024)
small_batch_final_kernel(const FinishParams f, int R, int key_kind, const float *__restrict__ scale,
                         const float *__restrict__ bias)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.x;

    // LDS: final keys [R] x2 | counter | query [d] | then a region used first for the
    // selection (candidate keys or the selection scratch), later for staging rows of x
    u64 *fin = (u64 *)smem;                                                       // [R] candidates
    u64 *fin2 = fin + R;                                                          // [R] re-scored
    uint32_t *counters = (uint32_t *)(fin2 + R);                                  // [4]
    float *qs = (float *)(counters + 4);                                          // [d]
    // (an offset from smem, not a rounded-up address: through an integer the pointer would lose its address space
    // and every access below would become a flat one)
    unsigned char *region = smem + ((((size_t)R * 16 + 16 + (size_t)f.d * 4) + 15) & ~(size_t)15);
    WgSelectScratch *sel = (WgSelectScratch *)region;
    u64 *clist = (u64 *)region;                                                   // [<= kSelList] candidate keys
    float *stage = (float *)region;                                               // [stage_rows][d + 1]

    int n_cand = (int)f.meta[q].n_cand;
    u64 *cand = f.cand + (size_t)q * f.cand_stride;
    for (int l = tid; l < f.d; l += nt) qs[l] = f.queries[(size_t)q * f.d + l];
    if (tid < 4) counters[tid] = 0u;
    if (f.meta[q].n_cand > (uint32_t)f.cand_stride && f.block_max != nullptr) {
        // More points reached the bound than the buffer holds (a heap of equal scores at the top). The listed
        // blocks' exact maxima are known: the R best points lie in the R blocks with the largest maxima, at or
        // above the R-th largest of them, t. Those blocks are scored again here, point by point from the logical
        // codes and the tables in global memory, in the defined order of additions; at most 256 R keys reach t.
        const int n_sel = (int)f.meta[q].n_sel;
        const u64 *bm = f.block_max + (size_t)q * f.n_blocks;
        const int32_t *selb = f.sel_blk + (size_t)q * f.n_blocks;
        const u64 t = wg_select_threshold(bm, n_sel, R, sel);
        __syncthreads();
        const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
        const int kc = 1 << f.bits;
        for (int j = wave; j < n_sel; j += n_waves) {
            const u64 top = bm[j];
            if (top < t || top == 0ull) continue;
            const int64_t blk = selb[j];
            for (int i = 0; i < 4; ++i) {
                const int64_t id = blk * 256 + 64 * i + lane;
                if (id >= f.n_valid) continue;
                const uint8_t *row = f.codes_logical + (size_t)id * f.NB;
                uint32_t ord;
                if (f.u8) {
                    const uint8_t *L = f.lut8 + (size_t)q * f.M * kc;
                    uint32_t acc = 0;
                    if (f.bits == 8) {
                        for (int b = 0; b < f.NB; ++b) acc += L[b * 256 + row[b]];
                    } else {
                        for (int b = 0; b < f.NB; ++b) {
                            acc += L[2 * b * 16 + (row[b] & 15)];
                            if (2 * b + 1 < f.M) acc += L[(2 * b + 1) * 16 + (row[b] >> 4)];
                        }
                    }
                    ord = acc + 1u;
                } else {
                    const float *L = f.lut + (size_t)q * f.M * kc;
                    float acc = 0.0f;
                    if (f.bits == 8) {
                        for (int b = 0; b < f.NB; ++b) acc = __fadd_rn(acc, L[b * 256 + row[b]]);
                    } else {
                        for (int b = 0; b < f.NB; ++b) {
                            float v = L[2 * b * 16 + (row[b] & 15)];
                            v = __fadd_rn(v, 2 * b + 1 < f.M ? L[(2 * b + 1) * 16 + (row[b] >> 4)] : 0.0f);
                            acc = __fadd_rn(acc, v);
                        }
                    }
                    ord = ord_from_f32(acc);
                }
                const u64 key = make_key(ord, (int32_t)id);
                if (key >= t) {
                    const uint32_t at = atomicAdd(&counters[1], 1u);
                    if ((int64_t)at < f.cand_stride) cand[at] = key;
                }
            }
        }
        __threadfence_block();
        __syncthreads();
        n_cand = (int)(counters[1] < (uint32_t)f.cand_stride ? counters[1] : (uint32_t)f.cand_stride);
        __syncthreads();
    }
    int n_fin;
    if (n_cand <= kSelList) {
        // the usual case, a few hundred candidates: rank them all by counting and keep the
        // R best, already in order
        for (int i = tid; i < n_cand; i += nt) clist[i] = cand[i];
        __syncthreads();
        for (int j0 = 0; j0 < n_cand; j0 += nt / 4) {
            const int j = j0 + (tid >> 2);
            const u64 mine = j < n_cand ? clist[j] : ~0ull;
            const int rank = rank_by_four(clist, n_cand, mine, tid & 3);
            if (j < n_cand && (tid & 3) == 0 && rank < R) fin[rank] = mine;
        }
        n_fin = n_cand < R ? n_cand : R;
        __syncthreads();
    } else {
        const u64 t2 = wg_select_threshold(cand, n_cand, R, sel);
        __syncthreads();
        for (int i = tid; i < n_cand; i += nt) {
            const u64 key = cand[i];
            if (key >= t2) fin[atomicAdd(&counters[0], 1u)] = key;
        }
        __syncthreads();
        n_fin = (int)counters[0]; // min(R, n_cand)
    }
    const int k = f.k;
    const u64 *ranked = fin;
    if (f.reorder && f.rerank_rows > 0) {
        // the exact re-scoring is spread over several workgroups per query (rerank_split_kernel, next launch)
        for (int i = tid; i < n_fin; i += nt) f.fin_out[(size_t)q * R + i] = fin[i];
        if (tid == 0) { f.fin_n[2 * q] = (uint32_t)n_fin; f.fin_n[2 * q + 1] = 0u; }
        return;
    }
    if (f.reorder) {
        // exact re-scoring: the candidates' rows are copied to LDS by the whole workgroup
        // (eight threads per row, all loads in flight at once), then one thread per candidate
        // runs the fma chain in index order. Row stride d + 1 keeps the threads on different banks.
        const int d = f.d, ld = f.d + 1;
        const bool vec = (d & 3) == 0;
        for (int r0 = 0; r0 < n_fin; r0 += f.stage_rows) {
            const int rows = n_fin - r0 < f.stage_rows ? n_fin - r0 : f.stage_rows;
            __syncthreads();
            for (int rb = 0; rb < rows; rb += nt / 8) {
                const int r = rb + (tid >> 3);
                if (r >= rows) continue;
                const float *src = f.x + (size_t)key_id(fin[r0 + r]) * d;
                float *dst = stage + r * ld;
                if (vec) {
                    for (int c4 = tid & 7; c4 < d / 4; c4 += 8) {
                        const float4 v = ((const float4 *)src)[c4];
                        dst[4 * c4] = v.x; dst[4 * c4 + 1] = v.y; dst[4 * c4 + 2] = v.z; dst[4 * c4 + 3] = v.w;
                    }
                } else {
                    for (int l = tid & 7; l < d; l += 8) dst[l] = src[l];
                }
            }
            __syncthreads();
            for (int r = tid; r < rows; r += nt) {
                const float *row = stage + r * ld;
                float sc = 0.0f;
#pragma unroll 20
                for (int l = 0; l < d; ++l) sc = __fmaf_rn(qs[l], row[l], sc);
                fin2[r0 + r] = make_key(ord_from_f32(sc), key_id(fin[r0 + r]));
            }
        }
        __syncthreads();
        ranked = fin2;
    }
    for (int j0 = 0; j0 < n_fin; j0 += nt / 4) {
        const int j = j0 + (tid >> 2);
        const u64 mine = j < n_fin ? ranked[j] : ~0ull;
        const int rank = rank_by_four(ranked, n_fin, mine, tid & 3);
        if (j < n_fin && (tid & 3) == 0 && rank < k) {
            f.ids_out[(size_t)q * k + rank] = key_id(mine);
            float sc;
            if (f.reorder || !key_kind) sc = f32_from_ord(key_ord(mine));
            else sc = __fmaf_rn((float)(int)(key_ord(mine) - 1u), scale[q], bias[q]);
            f.scores_out[(size_t)q * k + rank] = sc;
        }
    }
    for (int j = n_fin + tid; j < k; j += nt) { // fewer than k candidates exist
        f.ids_out[(size_t)q * k + j] = -1;
        f.scores_out[(size_t)q * k + j] = -INFINITY;
    }
}

// The exact re-scoring of a query's R candidates over several workgroups, for a few queries with so many or so
// long rows that one workgroup stages them in several passes through the one compute unit it runs on. Workgroup
// g takes the candidates [g rows, (g + 1) rows) of fin_out[q] (left there in rank order by small_batch_final_kernel,
// fin_n[2 q] of them), copies their rows to LDS (sixteen threads per row), runs the fma chain in index order, one
// thread per row, and writes the key of the exact score over the candidate's. The workgroup that finishes last
// (a ticket in fin_n[2 q + 1]) ranks the keys and writes the k best.
__global__ void __launch_bounds__(1024)
rerank_split_kernel(const FinishParams f, int R)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t last;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.y;
    const int d = f.d, ld = f.d + 1, rows_per = f.rerank_rows;
    float *qs = (float *)smem;               // [d]
    float *stage = qs + ((d + 3) & ~3);      // [rows_per][d + 1]; the last workgroup: keys [R]
    u64 *keys = f.fin_out + (size_t)q * R;
    const int n_fin = (int)f.fin_n[2 * q];
    const int r0 = blockIdx.x * rows_per;
    const int rows = r0 < n_fin ? (n_fin - r0 < rows_per ? n_fin - r0 : rows_per) : 0;
    for (int l = tid; l < d; l += nt) qs[l] = f.queries[(size_t)q * d + l];
    const bool vec = (d & 3) == 0;
    for (int rb = 0; rb < rows; rb += nt / 16) {
        const int r = rb + (tid >> 4);
        if (r >= rows) continue;
        const float *src = f.x + (size_t)key_id(keys[r0 + r]) * d;
        float *dst = stage + r * ld;
        if (vec) {
            for (int c4 = tid & 15; c4 < d / 4; c4 += 16) {
                const float4 v = ((const float4 *)src)[c4];
                dst[4 * c4] = v.x; dst[4 * c4 + 1] = v.y; dst[4 * c4 + 2] = v.z; dst[4 * c4 + 3] = v.w;
            }
        } else {
            for (int l = tid & 15; l < d; l += 16) dst[l] = src[l];
        }
    }
    __syncthreads();
    for (int r = tid; r < rows; r += nt) {
        const float *row = stage + r * ld;
        float sc = 0.0f;
#pragma unroll 20
        for (int l = 0; l < d; ++l) sc = __fmaf_rn(qs[l], row[l], sc);
        keys[r0 + r] = make_key(ord_from_f32(sc), key_id(keys[r0 + r]));
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) last = atomicAdd(&f.fin_n[2 * q + 1], 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (!last) return;
    __threadfence();
    u64 *ranked = (u64 *)stage;
    for (int i = tid; i < n_fin; i += nt) ranked[i] = __hip_atomic_load(&keys[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int k = f.k;
    for (int j0 = 0; j0 < n_fin; j0 += nt / 4) {
        const int j = j0 + (tid >> 2);
        const u64 mine = j < n_fin ? ranked[j] : ~0ull;
        const int rank = rank_by_four(ranked, n_fin, mine, tid & 3);
        if (j < n_fin && (tid & 3) == 0 && rank < k) {
            f.ids_out[(size_t)q * k + rank] = key_id(mine);
            f.scores_out[(size_t)q * k + rank] = f32_from_ord(key_ord(mine));
        }
    }
    for (int j = n_fin + tid; j < k; j += nt) { // fewer than k candidates exist
        f.ids_out[(size_t)q * k + j] = -1;
        f.scores_out[(size_t)q * k + j] = -INFINITY;
    }
}

// ---- host side ---------------------------------------------------------------

static size_t scan_lds_bytes(int NB, bool u8, int qt, int waves, int ns, bool lists_global)
{
    const int words = u8 ? (qt >= 2 ? qt / 2 : 1) : qt;
    const size_t tables = (!u8 && qt == 8) ? (size_t)NB * qt * 128 : (size_t)NB * 256 * words * 4;
    return tables + (size_t)waves * qt * ((lists_global ? 0 : 64 * ns) + 64) * 8;
}

int scan_pick_shape(int NB, int bits, bool u8, int ns, int B, bool single, int qt_hint, int waves_hint,
                    ScanShape *out)
{
    const size_t lds_max = kMaxDynLds;
    int qts_f[] = {8, 4, 1, 0}, qts_u[] = {8, 4, 1, 0};
    const int *qts = u8 ? qts_u : qts_f;
    // First choice: the widest query tile that still leaves room for eight waves (two per
    // SIMD hide the LDS latency of the lookups); failing that, the widest tile that fits.
    for (int pass = 0; pass < 2; ++pass) {
        for (int i = 0; qts[i]; ++i) {
            int qt = qts[i];
            if (single && qt != 1) continue;
            if (!u8 && qt == 8 && bits != 4) continue; // the fp32 tile of 8 keeps 16-entry tables
            if (pass == 0 && qt == 1 && !single) continue;
            if (!single) {
                if (qt_hint) { if (qt != qt_hint) continue; }
                else if (qt > 1 && B < qt) continue; // small batches: one query per workgroup
            }
            int wlist[] = {16, 8, 4, 2, 1, 0};
            for (int j = 0; wlist[j]; ++j) {
                int w = wlist[j];
                if (qt > 1 && w > 8) continue; // the tiled kernels are compiled for <= 512 threads
                if (waves_hint) { if (w != waves_hint) continue; }
                else {
                    if (qt == 1 && w > 4) continue;
                    if (pass == 0 && qt > 1 && w < 8) continue;
                }
                const bool lists_global = qt > 1; // tiled kernels: LDS goes to the tables
                size_t need = scan_lds_bytes(NB, u8, qt, w, ns, lists_global);
                if (need <= lds_max) {
                    out->qt = qt; out->waves = w; out->lds_bytes = need; out->lists_global = lists_global;
                    return AVQ_OK;
                }
            }
        }
    }
    set_error("scan: no launch shape fits LDS (NB=%d ns=%d)", NB, ns);
    return AVQ_EINVAL;
}

template <class K>
static int set_max_lds(K kern, LdsLimitOnce *once)
{
    return set_lds_limit((const void *)kern, kMaxDynLds, once);
}

template <bool U8, int NBT>
static int launch_leaf_bound_one(const ScanParams &p, int cap_blocks, uint32_t *bound, hipStream_t st)
{
    auto kern = leaf_bound_kernel<U8, NBT>;
    static LdsLimitOnce attr_done; // the tables are static LDS on top of this
    AVQ_TRY(set_lds_limit((const void *)kern, kLeafBoundMaxBlocks * 1024 + 8192, &attr_done));
    hipLaunchKernelGGL(kern, dim3(p.B), dim3(512), (size_t)cap_blocks * 1024 + 8192, st, p, cap_blocks, bound);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_leaf_bound(const ScanParams &p, bool u8, int max_leaf_blocks, int mean_leaf_blocks, uint32_t *bound, hipStream_t st)
{
    if (p.bits != 4 || !p.leaf_ids || !p.leaf_ip || !p.leaf_blk || !p.perm || p.Lp < 1 || p.R < 1) {
        set_error("leaf bounds: bad arguments");
        return AVQ_EINVAL;
    }
    const int Lb = std::min(p.Lp, 64);
    // room for leaves half again as large as the mean (probed leaves tend to be the larger ones), never more
    // than the largest ones need; several workgroups per compute unit as long as this stays small
    int64_t cap = (int64_t)Lb * std::max(1, mean_leaf_blocks) * 3 / 2 + 4;
    cap = std::min<int64_t>(cap, (int64_t)Lb * std::max(1, max_leaf_blocks));
    if (max_leaf_blocks > kLeafBoundMaxBlocks) { set_error("leaf bounds: leaves of %d blocks are too large", max_leaf_blocks); return AVQ_EINVAL; }
    const int cap_blocks = (int)std::max<int64_t>(std::max(1, max_leaf_blocks), std::min<int64_t>(kLeafBoundMaxBlocks, cap));
    switch (p.NB) {
    case 8: return u8 ? launch_leaf_bound_one<true, 8>(p, cap_blocks, bound, st) : launch_leaf_bound_one<false, 8>(p, cap_blocks, bound, st);
    case 13: return u8 ? launch_leaf_bound_one<true, 13>(p, cap_blocks, bound, st) : launch_leaf_bound_one<false, 13>(p, cap_blocks, bound, st);
    case 25: return u8 ? launch_leaf_bound_one<true, 25>(p, cap_blocks, bound, st) : launch_leaf_bound_one<false, 25>(p, cap_blocks, bound, st);
    case 32: return u8 ? launch_leaf_bound_one<true, 32>(p, cap_blocks, bound, st) : launch_leaf_bound_one<false, 32>(p, cap_blocks, bound, st);
    default: set_error("leaf bounds: code size %d not specialised", p.NB); return AVQ_EINVAL;
    }
}

template <int QT, bool U8, int NBT, int MODE>
static int launch_one(const ScanParams &p, const ScanShape &s, int grid, hipStream_t st)
{
    auto kern = adc_scan_kernel<QT, U8, NBT, MODE>;
    static LdsLimitOnce attr_done; // per instantiation
    AVQ_TRY(set_max_lds(kern, &attr_done));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(s.waves * 64), s.lds_bytes, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <int QT, bool U8, int MODE>
static int launch_nb(const ScanParams &p, const ScanShape &s, int grid, hipStream_t st)
{
    switch (p.NB) {
    case 8: return launch_one<QT, U8, 8, MODE>(p, s, grid, st);
    case 13: return launch_one<QT, U8, 13, MODE>(p, s, grid, st);
    case 25: return launch_one<QT, U8, 25, MODE>(p, s, grid, st);
    case 32: return launch_one<QT, U8, 32, MODE>(p, s, grid, st);
    default: return launch_one<QT, U8, 0, MODE>(p, s, grid, st);
    }
}

int launch_scan(const ScanParams &p, bool u8, int mode, const ScanShape &s, hipStream_t st)
{
    if (mode == SCAN_LEAVES || mode == SCAN_BLOCKLIST) {
        if (s.qt != 1) { set_error("scan: this mode needs qt == 1"); return AVQ_EINVAL; }
        const int grid = p.B;
        if (mode == SCAN_LEAVES) {
            const int lgrid = p.n_tiles * p.n_chunks; // n_tiles == B
            return u8 ? launch_nb<1, true, MODE_LEAVES>(p, s, lgrid, st) : launch_nb<1, false, MODE_LEAVES>(p, s, lgrid, st);
        }
        return u8 ? launch_nb<1, true, MODE_BLOCKLIST>(p, s, grid, st)
                  : launch_nb<1, false, MODE_BLOCKLIST>(p, s, grid, st);
    }
    const int64_t grid64 = p.active_queries ? std::max<int64_t>(kDynamicItems, p.n_tiles) : (int64_t)p.n_tiles * p.n_chunks;
    if (grid64 > 0x7fffffff) { set_error("scan: grid too large"); return AVQ_EINVAL; }
    const int grid = (int)grid64;
    if (!u8) {
        if (s.qt == 1) return launch_nb<1, false, MODE_CHUNK>(p, s, grid, st);
        if (s.qt == 4) return launch_nb<4, false, MODE_CHUNK>(p, s, grid, st);
        if (s.qt == 8 && p.bits == 4) return launch_nb<8, false, MODE_CHUNK>(p, s, grid, st);
    } else {
        if (s.qt == 1) return launch_nb<1, true, MODE_CHUNK>(p, s, grid, st);
        if (s.qt == 4) return launch_nb<4, true, MODE_CHUNK>(p, s, grid, st);
        if (s.qt == 8) return launch_nb<8, true, MODE_CHUNK>(p, s, grid, st);
    }
    set_error("scan: unsupported query tile %d", s.qt);
    return AVQ_EINVAL;
}

template <bool U8, int NBT>
static int launch_block_max_one(const ScanParams &p, int waves, hipStream_t st)
{
    auto kern = block_max_kernel<U8, NBT>;
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_max_lds(kern, &attr_done));
    const size_t lds = (size_t)p.NB * 256 * 4;
    // at most about four workgroups per compute unit and query: beyond that each one loops
    int64_t gx = (p.n_blocks + waves - 1) / waves;
    const int64_t cap = p.max_wgs > 0 ? p.max_wgs : std::max<int64_t>(1, 1024 / p.B);
    if (gx > cap) gx = cap;
    hipLaunchKernelGGL(kern, dim3((unsigned)gx, p.B), dim3(waves * 64), lds, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <bool U8>
static int launch_block_max_nb(const ScanParams &p, int waves, hipStream_t st)
{
    switch (p.NB) {
    case 8: return launch_block_max_one<U8, 8>(p, waves, st);
    case 13: return launch_block_max_one<U8, 13>(p, waves, st);
    case 25: return launch_block_max_one<U8, 25>(p, waves, st);
    case 32: return launch_block_max_one<U8, 32>(p, waves, st);
    default: return launch_block_max_one<U8, 0>(p, waves, st);
    }
}

template <bool U8, int NBT>
static int launch_block_max_nibble_one(const ScanParams &p, hipStream_t st)
{
    const int waves = 4;
    const size_t lds = (size_t)2 * p.NB * 16 * (U8 ? 1 : 4);
    // at most eight workgroups per compute unit and query; beyond that each wave loops
    int64_t gx = (p.n_blocks + waves - 1) / waves;
    const int64_t cap = p.max_wgs > 0 ? p.max_wgs : std::max<int64_t>(1, 2048 / p.B);
    if (gx > cap) gx = cap;
    hipLaunchKernelGGL((block_max_nibble_kernel<U8, NBT>), dim3((unsigned)gx, p.B), dim3(waves * 64), lds, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <bool U8>
static int launch_block_max_nibble_nb(const ScanParams &p, hipStream_t st)
{
    switch (p.NB) {
    case 8: return launch_block_max_nibble_one<U8, 8>(p, st);
    case 13: return launch_block_max_nibble_one<U8, 13>(p, st);
    case 25: return launch_block_max_nibble_one<U8, 25>(p, st);
    case 32: return launch_block_max_nibble_one<U8, 32>(p, st);
    default: return launch_block_max_nibble_one<U8, 0>(p, st);
    }
}

static bool use_nibble_tables(const ScanParams &p) { return p.bits == 4 && (size_t)p.M * 64 <= 60 * 1024; }

bool small_batch_can_fuse_tables(int bits, int M, int d, bool u8)
{
    // fp32 tables of 4-bit codes with short subspaces: a few fma per entry, cheaper than a launch
    return !u8 && bits == 4 && (size_t)M * 64 <= 60 * 1024 && d / M <= 8;
}

// LDS of the final kernel: keys, query, then max(selection scratch, row staging).
static size_t small_final_fixed_bytes(int R, int d)
{
    return (((size_t)R * 16 + 16 + (size_t)d * 4) + 15) & ~(size_t)15;
}

int small_finish_stage_rows(const ScanParams &p, int d, bool u8)
{
    (void)u8;
    const size_t row = (size_t)(d + 1) * 4;
    const size_t avail = kMaxDynLds - small_final_fixed_bytes(p.R, d) - 256;
    size_t want = (size_t)p.R * row;                       // all candidates at once if they fit
    if (want < sizeof(WgSelectScratch)) want = sizeof(WgSelectScratch);
    if (want > avail) want = avail;
    const int rows = (int)(want / row);
    return rows < 1 ? 1 : (rows > p.R ? p.R : rows);
}

template <bool U8, int NBT, bool NIB>
static int launch_rescan_one(const ScanParams &p, const FinishParams &f, hipStream_t st)
{
    auto kern = rescan_blocks_kernel<U8, NBT, NIB>;
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_max_lds(kern, &attr_done));
    const int waves = 4;
    const size_t lds = NIB ? (size_t)2 * p.NB * 16 * (U8 ? 1 : 4) : (size_t)p.NB * 256 * 4;
    hipLaunchKernelGGL(kern, dim3((p.R + waves - 1) / waves, p.B), dim3(waves * 64), lds, st, p, f);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <bool U8>
static int launch_rescan_u(const ScanParams &p, const FinishParams &f, hipStream_t st)
{
    if (use_nibble_tables(p)) {
        switch (p.NB) {
        case 8: return launch_rescan_one<U8, 8, true>(p, f, st);
        case 13: return launch_rescan_one<U8, 13, true>(p, f, st);
        case 25: return launch_rescan_one<U8, 25, true>(p, f, st);
        case 32: return launch_rescan_one<U8, 32, true>(p, f, st);
        default: return launch_rescan_one<U8, 0, true>(p, f, st);
        }
    }
    if (p.NB == 32) return launch_rescan_one<U8, 32, false>(p, f, st);
    return launch_rescan_one<U8, 0, false>(p, f, st);
}

bool block_bound_supported(int NB, int bits)
{
    return (bits == 4 || bits == 8) && (NB == 8 || NB == 13 || NB == 25 || NB == 32);
}

template <int NBT>
static int launch_block_bound_one(const ScanParams &p, int waves, bool lookups_only, hipStream_t st)
{
    // one block per wave while they all fit the chip at once (the table copy is cheap, and small workgroups
    // spread evenly over the compute units); beyond that the waves take the blocks in turn -- except over an array
    // streamed with nontemporal loads, where one block per wave throughout measured fastest (1.6 GB: 224 us against
    // 246 us at 8,192 workgroups and 267 us at 2,048)
    if (waves <= 0) waves = 4;
    const int64_t cap = p.max_wgs > 0 ? p.max_wgs : (p.nt_loads ? INT64_MAX : std::max<int64_t>(1, 2048 / p.B));
    int64_t gx = std::min<int64_t>((p.n_blocks + waves - 1) / waves, cap);
    if (gx < 1) gx = 1;
    if (lookups_only) hipLaunchKernelGGL((lookup_only_kernel<NBT>), dim3((unsigned)gx, p.B), dim3(waves * 64), 0, st, p);
    else if (p.nt_loads) hipLaunchKernelGGL((block_bound_stream_kernel<NBT>), dim3((unsigned)gx, p.B), dim3(waves * 64), 0, st, p);
    else hipLaunchKernelGGL((block_bound_kernel<NBT>), dim3((unsigned)gx, p.B), dim3(waves * 64), 0, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_bound_tables(const ScanParams &p, bool u8, hipStream_t st)
{
    const dim3 grid(p.bound_tile ? (p.B + p.bound_tile - 1) / p.bound_tile * p.bound_tile : p.B), block(1024);
    if (p.bits == 8) {
        if (u8) hipLaunchKernelGGL((bound_tables_kernel<true, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bound_tables_kernel<false, true>), grid, block, 0, st, p);
    } else {
        if (u8) hipLaunchKernelGGL((bound_tables_kernel<true, false>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((bound_tables_kernel<false, false>), grid, block, 0, st, p);
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_block_bound(const ScanParams &p, int waves, hipStream_t st, bool lookups_only)
{
    if (waves < 0 || waves > 16) waves = 0;
    if (waves > 0 && waves < 4) waves = 4; // the table copy counts on 256 threads
    switch (p.NB) {
    case 8: return launch_block_bound_one<8>(p, waves, lookups_only, st);
    case 13: return launch_block_bound_one<13>(p, waves, lookups_only, st);
    case 25: return launch_block_bound_one<25>(p, waves, lookups_only, st);
    case 32: return launch_block_bound_one<32>(p, waves, lookups_only, st);
    default: set_error("block bounds: unsupported code size %d", p.NB); return AVQ_EINVAL;
    }
}

template <int NBT, int GROUP>
static int launch_block_bound_tile_one(const ScanParams &p, hipStream_t st)
{
    auto kern = block_bound_tile_kernel<NBT, GROUP>;
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_max_lds(kern, &attr_done));
    const int tiles = (p.B + 15) / 16;
    const int chunks = (int)((p.n_blocks + p.blocks_per_chunk - 1) / p.blocks_per_chunk);
    // the tile index runs fastest: the workgroups that are resident together scan the same few chunks, so the
    // codes they stream are shared through the caches beyond a compute unit
    hipLaunchKernelGGL(kern, dim3(tiles, chunks), dim3(1024), (size_t)NBT * 256 * 16, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int block_bound_tile_chunk(int64_t n_blocks, int B)
{
    // about four rounds of one workgroup per compute unit, chunks of at least 128 blocks (eight per wave)
    const int tiles = (B + 15) / 16;
    int64_t chunks = std::max<int64_t>(1, 1024 / tiles);
    chunks = std::min<int64_t>(chunks, std::max<int64_t>(1, n_blocks / 128));
    return (int)((n_blocks + chunks - 1) / chunks);
}

int launch_block_bound_tile(const ScanParams &p, hipStream_t st)
{
    if (p.bound_tile != 16 || (p.bound_levels != 63 && p.bound_levels != 127 && p.bound_levels != 255)) {
        set_error("block bounds: tiles of 16 queries take byte tables of 63, 127 or 255 levels");
        return AVQ_EINVAL;
    }
    const int group = p.bound_levels == 63 ? 4 : (p.bound_levels == 127 ? 2 : 1);
#define AVQ_TILE_CASE(NB_)                                                                     \
    case NB_:                                                                                  \
        return group == 4 ? launch_block_bound_tile_one<NB_, 4>(p, st)                         \
                          : (group == 2 ? launch_block_bound_tile_one<NB_, 2>(p, st) : launch_block_bound_tile_one<NB_, 1>(p, st));
    switch (p.NB) {
        AVQ_TILE_CASE(8)
        AVQ_TILE_CASE(13)
        AVQ_TILE_CASE(25)
        AVQ_TILE_CASE(32)
    default: set_error("block bounds: unsupported code size %d", p.NB); return AVQ_EINVAL;
    }
#undef AVQ_TILE_CASE
}

int launch_select_bound_blocks(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st)
{
    const int kind = !u8 ? 0 : (p.bits == 4 ? 1 : 2);
    const int shift = kind == 2 ? p.bound_shift : 0;
    if (p.sel_hist != nullptr) {
        const int per = p.sel_split_per;
        if (per < 1 || per > kSelSplitMaxPer) { set_error("split selection: bad arguments"); return AVQ_EINVAL; }
        const dim3 grid((unsigned)((p.n_blocks + per - 1) / per), p.B);
        hipLaunchKernelGGL(select_split_count_kernel, grid, dim3(1024), 0, st, p.block_bound, p.n_blocks, per, p.sel_hist, f.meta);
        hipLaunchKernelGGL(select_split_list_kernel, grid, dim3(1024), 0, st, p.block_bound, p.n_blocks, per, p.R, p.NB, kind, shift,
                           p.bound_meta, p.sel_hist, f.sel_blk, f.meta);
        AVQ_HIP(hipGetLastError());
        return AVQ_OK;
    }
    hipLaunchKernelGGL(select_bound_blocks_kernel, dim3(p.B), dim3(1024), 0, st, p.block_bound, p.n_blocks, p.R, p.NB, kind, shift,
                       p.bound_meta, f.sel_blk, f.meta);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <bool U8, int NBT, bool NIB>
static int launch_rescan_listed_one(const ScanParams &p, const FinishParams &f, hipStream_t st)
{
    auto kern = rescan_listed_blocks_kernel<U8, NBT, NIB>;
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_max_lds(kern, &attr_done));
    const int waves = 4;
    const size_t lds = NIB ? (size_t)2 * p.NB * 16 * (U8 ? 1 : 4) : (size_t)p.NB * 256 * 4;
    // a wave per listed block while there are few (the usual case), in turns beyond; every workgroup builds the
    // query's tables for itself, so batches of thousands of queries get one or two workgroups per query
    const int64_t per_query = std::max<int64_t>(256 / p.B, std::min<int64_t>(16, std::max<int64_t>(1, 16384 / p.B)));
    const int64_t gx = std::min<int64_t>((p.n_blocks + waves - 1) / waves, per_query);
    hipLaunchKernelGGL(kern, dim3((unsigned)gx, p.B), dim3(waves * 64), lds, st, p, f);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <bool U8>
static int launch_rescan_listed_u(const ScanParams &p, const FinishParams &f, hipStream_t st)
{
    if (p.bits == 4) {
        switch (p.NB) {
        case 8: return launch_rescan_listed_one<U8, 8, true>(p, f, st);
        case 13: return launch_rescan_listed_one<U8, 13, true>(p, f, st);
        case 25: return launch_rescan_listed_one<U8, 25, true>(p, f, st);
        case 32: return launch_rescan_listed_one<U8, 32, true>(p, f, st);
        }
    } else {
        switch (p.NB) {
        case 8: return launch_rescan_listed_one<U8, 8, false>(p, f, st);
        case 13: return launch_rescan_listed_one<U8, 13, false>(p, f, st);
        case 25: return launch_rescan_listed_one<U8, 25, false>(p, f, st);
        case 32: return launch_rescan_listed_one<U8, 32, false>(p, f, st);
        }
    }
    set_error("rescan of listed blocks: unsupported code size %d", p.NB);
    return AVQ_EINVAL;
}

int launch_rescan_listed(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st)
{
    return u8 ? launch_rescan_listed_u<true>(p, f, st) : launch_rescan_listed_u<false>(p, f, st);
}

int launch_small_select(const ScanParams &p, const FinishParams &f, hipStream_t st)
{
    static LdsLimitOnce attr;
    AVQ_TRY(set_max_lds(select_blocks_kernel, &attr));
    hipLaunchKernelGGL(select_blocks_kernel, dim3(p.B), dim3(1024), sizeof(WgSelectScratch), st, p.block_max,
                       p.n_blocks, p.R, f.sel_blk, f.meta);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_small_rescan(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st)
{
    if ((size_t)p.NB * 256 * 4 > kMaxDynLds && !use_nibble_tables(p)) {
        set_error("small-batch rescan: tables do not fit LDS");
        return AVQ_EINVAL;
    }
    return u8 ? launch_rescan_u<true>(p, f, st) : launch_rescan_u<false>(p, f, st);
}

bool leaf_small_supported(int NB, int bits)
{
    return bits == 4 && (NB == 8 || NB == 13 || NB == 25 || NB == 32);
}

template <bool U8>
static int launch_leaf_small_u(const ScanParams &p, const FinishParams &f, const LeafBlockList &list, bool rescan, hipStream_t st)
{
    const dim3 grid = rescan ? dim3((unsigned)((p.R + 3) / 4), p.B) : dim3((unsigned)p.Lp, p.B);
#define AVQ_LEAF_SMALL(N)                                                                                          \
    case N:                                                                                                        \
        if (rescan) hipLaunchKernelGGL((rescan_leaf_blocks_kernel<U8, N>), grid, dim3(256), 0, st, p, f, list);    \
        else hipLaunchKernelGGL((leaf_block_max_kernel<U8, N>), grid, dim3(256), 0, st, p, list);                  \
        break;
    switch (p.NB) {
        AVQ_LEAF_SMALL(8)
        AVQ_LEAF_SMALL(13)
        AVQ_LEAF_SMALL(25)
        AVQ_LEAF_SMALL(32)
    default: set_error("leaf block maxima: unsupported code size %d", p.NB); return AVQ_EINVAL;
    }
#undef AVQ_LEAF_SMALL
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

static int check_leaf_small(const ScanParams &p, const LeafSmallBuffers &b)
{
    if (!leaf_small_supported(p.NB, p.bits) || !p.perm || !p.leaf_ids || !p.leaf_ip || !p.leaf_blk || p.Lp < 1 || p.B < 1 ||
        p.R < 1 || !b.best || !b.blk || !b.ip || !b.n_listed || b.stride < 1) {
        set_error("leaf block maxima: bad arguments");
        return AVQ_EINVAL;
    }
    return AVQ_OK;
}

int launch_leaf_block_max(const ScanParams &p, bool u8, const LeafSmallBuffers &b, hipStream_t st)
{
    AVQ_TRY(check_leaf_small(p, b));
    const LeafBlockList list{b.best, b.blk, b.ip, b.n_listed, b.stride};
    const FinishParams f{};
    return u8 ? launch_leaf_small_u<true>(p, f, list, false, st) : launch_leaf_small_u<false>(p, f, list, false, st);
}

int launch_select_listed_blocks(const ScanParams &p, const FinishParams &f, const LeafSmallBuffers &b, hipStream_t st)
{
    AVQ_TRY(check_leaf_small(p, b));
    static LdsLimitOnce attr;
    AVQ_TRY(set_max_lds(select_listed_blocks_kernel, &attr));
    const LeafBlockList list{b.best, b.blk, b.ip, b.n_listed, b.stride};
    hipLaunchKernelGGL(select_listed_blocks_kernel, dim3(p.B), dim3(1024), sizeof(WgSelectScratch), st, list, p.R, f.sel_blk, f.meta);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_rescan_leaf_blocks(const ScanParams &p, const FinishParams &f, bool u8, const LeafSmallBuffers &b, hipStream_t st)
{
    AVQ_TRY(check_leaf_small(p, b));
    const LeafBlockList list{b.best, b.blk, b.ip, b.n_listed, b.stride};
    return u8 ? launch_leaf_small_u<true>(p, f, list, true, st) : launch_leaf_small_u<false>(p, f, list, true, st);
}

int launch_small_final(const ScanParams &p, const FinishParams &f, bool u8, hipStream_t st)
{
    static LdsLimitOnce attr;
    AVQ_TRY(set_max_lds(small_batch_final_kernel, &attr));
    size_t region = sizeof(WgSelectScratch);
    const size_t stage = (size_t)f.stage_rows * (f.d + 1) * 4;
    if (stage > region) region = stage;
    const size_t lds = small_final_fixed_bytes(p.R, f.d) + region + 16;
    hipLaunchKernelGGL(small_batch_final_kernel, dim3(p.B), dim3(1024), lds, st, f, p.R, u8 ? 1 : 0, p.scale, p.bias);
    if (f.reorder && f.rerank_rows > 0) {
        if (!f.fin_out || !f.fin_n || f.rerank_rows > 1024) { set_error("split re-scoring: bad arguments"); return AVQ_EINVAL; }
        static LdsLimitOnce attr2;
        AVQ_TRY(set_max_lds(rerank_split_kernel, &attr2));
        const size_t rows_b = (size_t)f.rerank_rows * (f.d + 1) * 4, keys_b = (size_t)p.R * 8;
        const size_t lds2 = (size_t)((f.d + 3) & ~3) * 4 + (rows_b > keys_b ? rows_b : keys_b) + 16;
        if (lds2 > kMaxDynLds) { set_error("split re-scoring: %d rows of %d values do not fit LDS", f.rerank_rows, f.d); return AVQ_EINVAL; }
        hipLaunchKernelGGL(rerank_split_kernel, dim3((p.R + f.rerank_rows - 1) / f.rerank_rows, p.B), dim3(1024), lds2, st, f, p.R);
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_block_max(const ScanParams &p, bool u8, int waves, hipStream_t st)
{
    if (use_nibble_tables(p))
        return u8 ? launch_block_max_nibble_nb<true>(p, st) : launch_block_max_nibble_nb<false>(p, st);
    if ((size_t)p.NB * 256 * 4 > kMaxDynLds) { set_error("block max: tables do not fit LDS"); return AVQ_EINVAL; }
    return u8 ? launch_block_max_nb<true>(p, waves, st) : launch_block_max_nb<false>(p, waves, st);
}

} // namespace avq
