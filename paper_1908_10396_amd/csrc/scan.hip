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
// Tables. Whatever the code width, the kernel sees NB byte positions with a
// 256-entry table each, held in LDS for a tile of QT queries, entry = QT values
// interleaved (one ds_read fetches a byte's entry for the whole tile):
//   8-bit codes: T[b][v] = L[b][v];
//   4-bit codes: T[b][v] = L[2b][v & 15] + L[2b+1][v >> 4]  (one fp32 add, or an
//   integer add of the two 8-bit table codes).
// Scores accumulate over b = 0..NB-1 in order, which is the summation order the
// fp32 path is defined with.
//
// Selection. Each wave keeps, per query, a sorted list of the best 64*ns keys
// in LDS and a 64-entry pending buffer; a lane whose score beats the current
// R-th best appends to the buffer, a full buffer is sorted and merged (bitonic
// networks across lanes). At the end the waves' lists are merged and written
// out per (query, chunk).
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

template <int W> struct VecW;
template <> struct VecW<1> { typedef uint32_t type; };
template <> struct VecW<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct VecW<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

template <int W> __device__ __forceinline__ uint32_t vec_get(const typename VecW<W>::type &v, int i)
{
    if constexpr (W == 1) return v;
    else return v[i];
}

// words per table entry
template <int QT, bool U8> struct EntryWords { static constexpr int value = U8 ? (QT >= 2 ? QT / 2 : 1) : QT; };

template <int QT, bool U8, int NBT, bool IVF>
__global__ void __launch_bounds__(QT > 1 ? 512 : 1024)
adc_scan_kernel(const ScanParams p)
{
    constexpr int WORDS = EntryWords<QT, U8>::value;
    typedef typename VecW<WORDS>::type entry_t;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int NB = NBT ? NBT : p.NB;
    const int kc = 1 << p.bits;
    const int C = 64 * p.ns;

    int tile, chunk;
    if (IVF) { tile = blockIdx.x; chunk = 0; }
    else { tile = blockIdx.x % p.n_tiles; chunk = blockIdx.x / p.n_tiles; }
    const int q0 = tile * QT;

    entry_t *tbl = (entry_t *)smem;
    const size_t tbl_bytes = (size_t)NB * 256 * WORDS * 4;
    u64 *lists = (u64 *)(smem + tbl_bytes);                    // [n_waves][QT][C]
    u64 *pends = lists + (size_t)n_waves * QT * C;             // [n_waves][QT][64]
    u64 *my_lists = lists + (size_t)wave * QT * C;
    u64 *my_pends = pends + (size_t)wave * QT * 64;

    // ---- build the byte tables of this query tile --------------------------
    {
        const int items = QT * NB * 16; // (q, b, g): 16 consecutive byte values g*16 .. g*16+15
        for (int it = tid; it < items; it += blockDim.x) {
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
        for (int i = lane; i < QT * C; i += 64) my_lists[i] = 0ull;
    }
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
        if (IVF && U8) {
            const int gq = q0 + q < p.B ? q0 + q : 0;
            q_scale[q] = p.scale[gq];
            q_off[q] = p.bias[gq];
        }
    }
    // In the partitioned index the ranking key is a float even with 8-bit tables.
    constexpr bool FKEY = !U8 || IVF;

    auto refresh_threshold = [&](int q) {
        const u64 kth = my_lists[(size_t)q * C + (p.R - 1)];
        if (FKEY) thr_f[q] = kth ? f32_from_ord(key_ord(kth)) : -INFINITY;
        else thr_i[q] = (int)key_ord(kth) - 1;
    };

    // one block of 256 points: accumulate, then filter
    auto process_block = [&](int64_t blk, const uint4 *rows, const uint32_t *tails, int nfull,
                             int ntail, float seg_bias) {
        entry_t acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (WORDS == 1) acc[i] = 0u;
            else acc[i] = (entry_t)(0u);
        }
        auto plane = [&](uint32_t w, int b) {
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
                plane(rows[j].x, 4 * j + 0);
                plane(rows[j].y, 4 * j + 1);
                plane(rows[j].z, 4 * j + 2);
                plane(rows[j].w, 4 * j + 3);
            }
#pragma unroll
            for (int t = 0; t < NBT % 4; ++t) plane(tails[t], (NBT / 4) * 4 + t);
        } else {
            const uint8_t *base = p.codes + (size_t)blk * 256 * NB;
            for (int j = 0; j < nfull; ++j) {
                const uint4 r = ((const uint4 *)(base + (size_t)j * 1024))[lane];
                plane(r.x, 4 * j + 0);
                plane(r.y, 4 * j + 1);
                plane(r.z, 4 * j + 2);
                plane(r.w, 4 * j + 3);
            }
            for (int t = 0; t < ntail; ++t) {
                const uint32_t w = ((const uint32_t *)(base + (size_t)nfull * 1024 + (size_t)t * 256))[lane];
                plane(w, 4 * nfull + t);
            }
        }

        // score of (query q, point i of this lane)
        auto score_of = [&](int q, int i, float &sf, int &si) {
            sf = 0.0f;
            si = 0;
            if constexpr (!U8) {
                sf = __uint_as_float(vec_get<WORDS>(acc[i], q));
                if (IVF) sf = __fadd_rn(sf, seg_bias);
            } else {
                if constexpr (QT == 1) si = (int)vec_get<WORDS>(acc[i], 0);
                else si = (int)((vec_get<WORDS>(acc[i], q >> 1) >> (16 * (q & 1))) & 0xffffu);
                if (IVF) sf = __fmaf_rn((float)si, q_scale[q], __fadd_rn(q_off[q], seg_bias));
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
                if (FKEY) hit = IVF ? (sf >= thr_f[q]) : (sf > thr_f[q]);
                else hit = si > thr_i[q];
                if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
                // rare path: some lane has a candidate
                const int64_t slot = blk * 256 + 4 * lane + i;
                int32_t id;
                if (IVF) { id = p.perm[slot]; hit = hit && id >= 0; }
                else { id = (int32_t)slot; hit = hit && slot < p.n_valid; }
                const uint32_t ord = FKEY ? ord_from_f32(sf) : (uint32_t)(si + 1);
                if (wave_push(my_lists + (size_t)q * C, p.ns, my_pends + q * 64, pend_cnt[q], hit,
                              make_key(ord, id)))
                    refresh_threshold(q);
            }
        }
    };

    // ---- stream the code blocks ---------------------------------------------
    const int nfull = NB / 4, ntail = NB % 4;
    constexpr int NROWS = NBT ? (NBT / 4 ? NBT / 4 : 1) : 1;
    constexpr int NTAILS = NBT ? (NBT % 4 ? NBT % 4 : 1) : 1;
    auto load_block = [&](int64_t blk, uint4 *rows, uint32_t *tails) {
        if constexpr (NBT != 0) {
            const uint8_t *base = p.codes + (size_t)blk * 256 * NBT;
#pragma unroll
            for (int j = 0; j < NBT / 4; ++j) rows[j] = ((const uint4 *)(base + (size_t)j * 1024))[lane];
#pragma unroll
            for (int t = 0; t < NBT % 4; ++t)
                tails[t] = ((const uint32_t *)(base + (size_t)(NBT / 4) * 1024 + (size_t)t * 256))[lane];
        }
    };
    auto scan_range = [&](int64_t first, int64_t end, int64_t step, float seg_bias) {
        uint4 cur[NROWS], nxt[NROWS];
        uint32_t cur_t[NTAILS], nxt_t[NTAILS];
        if (first < end) load_block(first, cur, cur_t);
        for (int64_t blk = first; blk < end; blk += step) {
            const bool more = blk + step < end;
            if (more) load_block(blk + step, nxt, nxt_t);
            process_block(blk, cur, cur_t, nfull, ntail, seg_bias);
            if (more) {
#pragma unroll
                for (int j = 0; j < NROWS; ++j) cur[j] = nxt[j];
#pragma unroll
                for (int t = 0; t < NTAILS; ++t) cur_t[t] = nxt_t[t];
            }
        }
    };

    if (!IVF) {
        const int64_t first = (int64_t)chunk * p.blocks_per_chunk;
        int64_t end = first + p.blocks_per_chunk;
        if (end > p.n_blocks) end = p.n_blocks;
        scan_range(first + wave, end, n_waves, 0.0f);
    } else {
        const int gq = q0; // QT == 1
        for (int j = wave; j < p.Lp; j += n_waves) {
            const int leaf = p.leaf_ids[(size_t)gq * p.Lp + j];
            if (leaf < 0) continue;
            scan_range(p.leaf_blk[leaf], p.leaf_blk[leaf + 1], 1, p.leaf_ip[(size_t)gq * p.Lp + j]);
        }
    }
    if (p.scores_out != nullptr) return;

    // ---- drain pending buffers, merge the waves' lists, write out -------------
#pragma unroll
    for (int q = 0; q < QT; ++q)
        if (pend_cnt[q] > 0) wave_list_flush(my_lists + (size_t)q * C, p.ns, my_pends + q * 64, pend_cnt[q]);
    __syncthreads();
    for (int q = wave; q < QT; q += n_waves) {
        u64 *mine = my_lists + (size_t)q * C;
        for (int w = 0; w < n_waves; ++w) {
            if (w == wave) continue;
            wave_list_merge_from(mine, p.ns, lists + ((size_t)w * QT + q) * C);
        }
        u64 *out = p.partial + ((size_t)(q0 + q) * p.n_chunks + chunk) * C;
        for (int i = lane; i < C; i += 64) out[i] = mine[i];
    }
}

// ---- host side ---------------------------------------------------------------

static size_t scan_lds_bytes(int NB, bool u8, int qt, int waves, int ns)
{
    const int words = u8 ? (qt >= 2 ? qt / 2 : 1) : qt;
    return (size_t)NB * 256 * words * 4 + (size_t)waves * qt * (64 * ns + 64) * 8;
}

int scan_pick_shape(int NB, bool u8, int ns, int B, bool ivf, int qt_hint, int waves_hint,
                    ScanShape *out)
{
    const size_t lds_max = 160 * 1024;
    int qts_f[] = {4, 1, 0}, qts_u[] = {8, 1, 0};
    const int *qts = u8 ? qts_u : qts_f;
    for (int i = 0; qts[i]; ++i) {
        int qt = qts[i];
        if (ivf && qt != 1) continue;
        if (qt_hint) { if (qt != qt_hint) continue; }
        else if (qt > 1 && B < qt) continue; // small batches: one query per workgroup
        int wlist[] = {16, 8, 4, 2, 1, 0};
        for (int j = 0; wlist[j]; ++j) {
            int w = wlist[j];
            if (qt > 1 && w > 8) continue; // the tiled kernels are compiled for <= 512 threads
            if (waves_hint) { if (w != waves_hint) continue; }
            else if (qt == 1 && w > 4) continue;
            size_t need = scan_lds_bytes(NB, u8, qt, w, ns);
            if (need <= lds_max) {
                out->qt = qt; out->waves = w; out->lds_bytes = need;
                return AVQ_OK;
            }
        }
    }
    set_error("scan: no launch shape fits LDS (NB=%d ns=%d)", NB, ns);
    return AVQ_EINVAL;
}

template <int QT, bool U8, int NBT, bool IVF>
static int launch_one(const ScanParams &p, const ScanShape &s, int grid, hipStream_t st)
{
    auto kern = adc_scan_kernel<QT, U8, NBT, IVF>;
    static bool attr_done = false; // per instantiation
    if (!attr_done) {
        AVQ_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024));
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(s.waves * 64), s.lds_bytes, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

template <int QT, bool U8, bool IVF>
static int launch_nb(const ScanParams &p, const ScanShape &s, int grid, hipStream_t st)
{
    switch (p.NB) {
    case 8: return launch_one<QT, U8, 8, IVF>(p, s, grid, st);
    case 25: return launch_one<QT, U8, 25, IVF>(p, s, grid, st);
    case 32: return launch_one<QT, U8, 32, IVF>(p, s, grid, st);
    default: return launch_one<QT, U8, 0, IVF>(p, s, grid, st);
    }
}

int launch_scan(const ScanParams &p, bool u8, bool ivf, const ScanShape &s, hipStream_t st)
{
    if (ivf) {
        if (s.qt != 1) { set_error("scan: partitioned scan needs qt == 1"); return AVQ_EINVAL; }
        const int grid = p.B;
        return u8 ? launch_nb<1, true, true>(p, s, grid, st) : launch_nb<1, false, true>(p, s, grid, st);
    }
    const int64_t grid64 = (int64_t)p.n_tiles * p.n_chunks;
    if (grid64 > 0x7fffffff) { set_error("scan: grid too large"); return AVQ_EINVAL; }
    const int grid = (int)grid64;
    if (!u8) {
        if (s.qt == 1) return launch_nb<1, false, false>(p, s, grid, st);
        if (s.qt == 4) return launch_nb<4, false, false>(p, s, grid, st);
    } else {
        if (s.qt == 1) return launch_nb<1, true, false>(p, s, grid, st);
        if (s.qt == 8) return launch_nb<8, true, false>(p, s, grid, st);
    }
    set_error("scan: unsupported query tile %d", s.qt);
    return AVQ_EINVAL;
}

} // namespace avq
