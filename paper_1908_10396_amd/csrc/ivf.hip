// Leaf selection for the partitioned index (paper Sections 2.2.1 and 5.3: a
// vector-quantization tree reduces the number of points that are scored; the
// paper gives no details, the design here is: one level of leaves, a query
// visits the leaves whose centers have the largest inner product with it).
#include "avq_internal.h"
#include "wave_topk.h"
#include "wg_select.h"

namespace avq {

// One workgroup per query; its waves take the leaves 64 at a time in turn, each keeping its
// own list, and the lists are merged pairwise at the end. centers_t is [d][n_leaves] so that
// lane l reads leaf base + l with coalesced loads. The score is the fp32 fma chain in index order.
__global__ void __launch_bounds__(1024)
leaf_select_kernel(const float *__restrict__ centers_t, int n_leaves, int d,
                   const float *__restrict__ queries, int L, int ns,
                   int32_t *__restrict__ leaf_ids, float *__restrict__ leaf_ip, uint32_t *__restrict__ leaf_cnt,
                   uint32_t *__restrict__ leaf_pos, int cnt_stride)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int q = blockIdx.x;
    u64 *lists = (u64 *)smem;                    // [n_waves][C]
    u64 *pends = lists + (size_t)n_waves * C;    // [n_waves][64]
    float *qs = (float *)(pends + (size_t)n_waves * 64);
    u64 *list = lists + (size_t)wave * C;
    u64 *pend = pends + (size_t)wave * 64;
    for (int l = threadIdx.x; l < d; l += blockDim.x) qs[l] = queries[(size_t)q * d + l];
    wave_list_clear(list, ns);
    __syncthreads();
    float thr = -INFINITY;
    int cnt = 0;
    for (int base = wave * 64; base < n_leaves; base += n_waves * 64) {
        const int leaf = base + lane;
        const bool valid = leaf < n_leaves;
        float s = 0.0f;
        if (valid) {
            const float *col = centers_t + leaf;
#pragma unroll 8
            for (int l = 0; l < d; ++l) s = __fmaf_rn(qs[l], col[(size_t)l * n_leaves], s); // eight loads in flight
        }
        const bool hit = valid && s > thr; // a wave visits its leaves in increasing id
        if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
        if (wave_push(list, ns, pend, cnt, hit, make_key(ord_from_f32(s), leaf))) {
            const u64 kth = list[L - 1];
            thr = kth ? f32_from_ord(key_ord(kth)) : -INFINITY;
        }
    }
    if (cnt > 0) wave_list_flush(list, ns, pend, cnt);
    for (int stride = 1; stride < n_waves; stride *= 2) {
        __syncthreads();
        if ((wave % (2 * stride)) == 0 && wave + stride < n_waves)
            wave_list_merge_from(list, ns, lists + (size_t)(wave + stride) * C);
    }
    if (wave != 0) return;
    for (int j = lane; j < L; j += 64) {
        const u64 key = list[j];
        leaf_ids[(size_t)q * L + j] = key ? key_id(key) : -1;
        leaf_ip[(size_t)q * L + j] = key ? f32_from_ord(key_ord(key)) : -INFINITY;
        if (leaf_cnt != nullptr && key) { // how many queries probe each leaf, and this pair's place among them
            const uint32_t at = atomicAdd(&leaf_cnt[(size_t)key_id(key) * cnt_stride], 1u);
            if (leaf_pos != nullptr) leaf_pos[(size_t)q * L + j] = at;
        }
    }
}

// The same for large batches, without lists. A workgroup takes eight queries: every thread scores
// its leaves against all eight (eight fma chains fed by one load of each center value; the kernel
// above loads every value once per query) and the scores go to LDS. Then each wave takes one of the
// queries: the ordering value of the L-th best score by bisection (a lane counts its share of the
// scores, no barriers), the scores at or above it are collected and ranked by counting.
constexpr int kLeafTile = 8;

__global__ void __launch_bounds__(512)
leaf_select_tile_kernel(const float *__restrict__ centers_t, int n_leaves, int d, const float *__restrict__ queries, int nq,
                        int L, int32_t *__restrict__ leaf_ids, float *__restrict__ leaf_ip, uint32_t *__restrict__ leaf_cnt,
                   uint32_t *__restrict__ leaf_pos, int cnt_stride)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int nt = 512, n_waves = 8;
    const int q0 = blockIdx.x * kLeafTile;
    uint32_t *ords = (uint32_t *)smem;                                  // [8][n_leaves] ordering values of the scores
    u64 *fin = (u64 *)(ords + (size_t)kLeafTile * n_leaves);            // [8 waves][n_fin_max]
    const int n_fin_max = L;
    // The eight queries' components are the same for every lane: read straight from memory they are scalar
    // loads and scalar operands of the fma chains, and the loop is vector loads of center values and
    // arithmetic only. (Queries beyond the batch repeat the last one; their scores are never used.)
    const float *qrow[kLeafTile];
#pragma unroll
    for (int t = 0; t < kLeafTile; ++t) qrow[t] = queries + (size_t)(q0 + t < nq ? q0 + t : nq - 1) * d;
    for (int leaf = tid; leaf < n_leaves; leaf += nt) {
        const float *col = centers_t + leaf;
        float s[kLeafTile];
#pragma unroll
        for (int t = 0; t < kLeafTile; ++t) s[t] = 0.0f;
        // sixteen center values at a time, the next sixteen asked for before the current ones are used (the
        // loads take longer than the 128 fused multiply-adds they feed)
        constexpr int kChunk = 16;
        const int full = d / kChunk;
        float c[kChunk];
        if (full > 0) {
#pragma unroll
            for (int i = 0; i < kChunk; ++i) c[i] = col[(size_t)i * n_leaves];
        }
        for (int ch = 0; ch < full; ++ch) {
            float nx[kChunk];
            const bool more = ch + 1 < full;
            if (more) {
#pragma unroll
                for (int i = 0; i < kChunk; ++i) nx[i] = col[(size_t)((ch + 1) * kChunk + i) * n_leaves];
            }
#pragma unroll
            for (int i = 0; i < kChunk; ++i)
#pragma unroll
                for (int t = 0; t < kLeafTile; ++t) s[t] = __fmaf_rn(qrow[t][ch * kChunk + i], c[i], s[t]);
            if (more) {
#pragma unroll
                for (int i = 0; i < kChunk; ++i) c[i] = nx[i];
            }
        }
        for (int l = full * kChunk; l < d; ++l) {
            const float cl = col[(size_t)l * n_leaves];
#pragma unroll
            for (int t = 0; t < kLeafTile; ++t) s[t] = __fmaf_rn(qrow[t][l], cl, s[t]);
        }
#pragma unroll
        for (int t = 0; t < kLeafTile; ++t) ords[(size_t)t * n_leaves + leaf] = ord_from_f32(s[t]);
    }
    __syncthreads();
    const int want = L < n_leaves ? L : n_leaves;
    u64 *my_fin = fin + (size_t)wave * n_fin_max;
    for (int t = wave; t < kLeafTile; t += n_waves) {
        const int q = q0 + t;
        if (q >= nq) break;
        const uint32_t *o = ords + (size_t)t * n_leaves;
        // up to 2048 leaves: a lane's share of the scores stays in registers through the bisection
        constexpr int kReg = 32;
        const bool in_regs = n_leaves <= kReg * 64;
        uint32_t mine[kReg];
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < kReg; ++i) mine[i] = lane + i * 64 < n_leaves ? o[lane + i * 64] : 0u;
        }
        auto count_ge = [&](uint32_t v) -> int {
            if (in_regs) { // v >= 1 in every call, so the zeros that stand for "no leaf" never count
                int cr = 0; // one compare per register; the counting is scalar work on the lane masks
#pragma unroll
                for (int i = 0; i < kReg; ++i) cr += __popcll(__builtin_amdgcn_ballot_w64(mine[i] >= v));
                return cr;
            }
            int cn = 0;
            int leaf = lane;
            for (; leaf + 7 * 64 < n_leaves; leaf += 8 * 64) { // eight reads in flight
                uint32_t r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = o[leaf + i * 64];
#pragma unroll
                for (int i = 0; i < 8; ++i) cn += r[i] >= v;
            }
            for (; leaf < n_leaves; leaf += 64) cn += o[leaf] >= v;
            for (int m = 32; m > 0; m >>= 1) cn += __shfl_xor(cn, m, 64);
            return cn;
        };
        uint32_t lo = 0u, hi = 0xffffffffu; // count_ge(lo) >= want > count_ge(hi)
        if (in_regs) {
            // no score is above the best one, and the L-th best of a few thousand is mostly within a factor of two
            // of it: then the search covers one binade (23 rounds instead of 32)
            uint32_t top = 0u;
#pragma unroll
            for (int i = 0; i < kReg; ++i) top = mine[i] > top ? mine[i] : top;
            for (int m = 32; m > 0; m >>= 1) {
                const uint32_t o_top = (uint32_t)__shfl_xor((int)top, m, 64);
                top = o_top > top ? o_top : top;
            }
            if (top != 0xffffffffu) hi = top + 1u;
            if (top > 0x80800000u && count_ge(top - 0x00800000u) >= want) lo = top - 0x00800000u;
        }
        while (hi - lo > 1u) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (count_ge(mid) >= want) lo = mid; else hi = mid;
        }
        // the `want` best: every score above the L-th best, then scores equal to it in leaf order (equal
        // scores rank by id) until there are `want`
        const int n_gt = count_ge(lo + 1u);
        int at_gt = 0, at_eq = n_gt;
        for (int base = 0; base < n_leaves; base += 64) {
            const int leaf = base + lane;
            const uint32_t ov = leaf < n_leaves ? o[leaf] : 0u;
            const bool gt = leaf < n_leaves && ov > lo, eq = leaf < n_leaves && ov == lo;
            const u64 m_gt = __builtin_amdgcn_ballot_w64(gt), m_eq = __builtin_amdgcn_ballot_w64(eq);
            const u64 below = (1ull << lane) - 1ull;
            if (gt) my_fin[at_gt + __builtin_popcountll(m_gt & below)] = make_key(ov, leaf);
            const int e_at = at_eq + __builtin_popcountll(m_eq & below);
            if (eq && e_at < want) my_fin[e_at] = make_key(ov, leaf);
            at_gt += __builtin_popcountll(m_gt);
            at_eq += __builtin_popcountll(m_eq);
        }
        wave_lds_fence();
        const int nf = want;
        for (int j = lane; j < nf; j += 64) {
            const u64 k = my_fin[j];
            int rank = 0;
            for (int i = 0; i < nf; ++i) rank += my_fin[i] > k;
            if (rank < L) {
                leaf_ids[(size_t)q * L + rank] = key_id(k);
                leaf_ip[(size_t)q * L + rank] = f32_from_ord(key_ord(k));
                if (leaf_cnt != nullptr) {
                    const uint32_t at = atomicAdd(&leaf_cnt[(size_t)key_id(k) * cnt_stride], 1u);
                    if (leaf_pos != nullptr) leaf_pos[(size_t)q * L + rank] = at;
                }
            }
        }
        for (int j = want + lane; j < L; j += 64) { // fewer leaves than asked for
            leaf_ids[(size_t)q * L + j] = -1;
            leaf_ip[(size_t)q * L + j] = -INFINITY;
        }
        wave_lds_fence();
    }
}

// Leaf selection for a handful of queries, where the kernel above is all load latency in one workgroup: first every
// leaf's score by a thread of its own, spread over many small workgroups (the same fma chain in index order, 25 loads
// in flight), as keys (score, then lower leaf id) in keys[q][n_leaves]; then one workgroup per query finds the L-th
// largest key, gathers the keys at or above it and ranks them by counting.
__global__ void __launch_bounds__(64)
leaf_scores_kernel(const float *__restrict__ centers_t, int n_leaves, int d, const float *__restrict__ queries,
                   u64 *__restrict__ keys)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *qs = (float *)smem;
    const int q = blockIdx.y;
    for (int l = threadIdx.x; l < d; l += 64) qs[l] = queries[(size_t)q * d + l];
    __syncthreads();
    const int leaf = blockIdx.x * 64 + threadIdx.x;
    if (leaf >= n_leaves) return;
    const float *col = centers_t + leaf;
    float s = 0.0f;
#pragma unroll 25
    for (int l = 0; l < d; ++l) s = __fmaf_rn(qs[l], col[(size_t)l * n_leaves], s);
    keys[(size_t)q * n_leaves + leaf] = make_key(ord_from_f32(s), leaf);
}

__global__ void __launch_bounds__(1024)
leaf_top_kernel(const u64 *__restrict__ keys, int n_leaves, int L, int32_t *__restrict__ leaf_ids, float *__restrict__ leaf_ip)
{
    __shared__ WgSelectScratch sel;
    __shared__ u64 top[512];
    __shared__ uint32_t n_top;
    const int tid = threadIdx.x, q = blockIdx.x;
    const u64 *row = keys + (size_t)q * n_leaves;
    if (tid == 0) n_top = 0u;
    const u64 t = wg_select_threshold(row, n_leaves, L, &sel);
    __syncthreads();
    for (int i = tid; i < n_leaves; i += 1024) {
        const u64 key = row[i];
        if (key >= t && key) {
            const uint32_t at = atomicAdd(&n_top, 1u);
            if (at < 512u) top[at] = key;
        }
    }
    __syncthreads();
    const int n = (int)(n_top < 512u ? n_top : 512u); // min(L, leaves)
    for (int i = tid; i < n; i += 1024) {
        const u64 mine = top[i];
        int rank = 0;
        for (int j = 0; j < n; ++j) rank += top[j] > mine;
        if (rank < L) {
            leaf_ids[(size_t)q * L + rank] = key_id(mine);
            leaf_ip[(size_t)q * L + rank] = f32_from_ord(key_ord(mine));
        }
    }
    for (int i = n + tid; i < L; i += 1024) { // fewer leaves than asked for
        leaf_ids[(size_t)q * L + i] = -1;
        leaf_ip[(size_t)q * L + i] = -INFINITY;
    }
}

int launch_leaf_select_few(const float *centers_t, int n_leaves, int d, const float *queries, int nq, int L, u64 *keys,
                           int32_t *leaf_ids, float *leaf_ip, hipStream_t st)
{
    if (L < 1 || L > 512 || nq < 1 || n_leaves < 1 || (size_t)d * 4 > 60 * 1024 || !keys) {
        set_error("leaf select: bad arguments (L = %d)", L);
        return AVQ_EINVAL;
    }
    hipLaunchKernelGGL(leaf_scores_kernel, dim3((n_leaves + 63) / 64, nq), dim3(64), (size_t)d * 4, st, centers_t, n_leaves, d,
                       queries, keys);
    hipLaunchKernelGGL(leaf_top_kernel, dim3(nq), dim3(1024), 0, st, keys, n_leaves, L, leaf_ids, leaf_ip);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_leaf_select(const float *centers_t, int n_leaves, int d, const float *queries, int nq,
                       int L, int32_t *leaf_ids, float *leaf_ip, hipStream_t st, uint32_t *leaf_cnt, uint32_t *leaf_pos,
                       int cnt_stride)
{
    const int ns = (L + 63) / 64;
    if (nq >= 768) {
        const size_t lds = (size_t)kLeafTile * n_leaves * 4 + (size_t)8 * L * 8;
        if (lds <= kMaxDynLds) {
            static LdsLimitOnce tile_attr_done;
            AVQ_TRY(set_lds_limit((const void *)leaf_select_tile_kernel, kMaxDynLds, &tile_attr_done));
            hipLaunchKernelGGL(leaf_select_tile_kernel, dim3((nq + kLeafTile - 1) / kLeafTile), dim3(512), lds, st, centers_t, n_leaves,
                               d, queries, nq, L, leaf_ids, leaf_ip, leaf_cnt, leaf_pos, cnt_stride);
            AVQ_HIP(hipGetLastError());
            return AVQ_OK;
        }
    }
    // few queries: as many waves as there are 64-leaf groups (at most 16); batches: four
    int waves = nq >= 1024 ? 4 : 16;
    while (waves > 1 && (waves / 2) * 64 >= n_leaves) waves /= 2;
    const size_t lds = (size_t)waves * (64 * ns + 64) * 8 + (size_t)d * 4;
    if (lds > kMaxDynLds) { set_error("leaf select: L = %d too large", L); return AVQ_EINVAL; }
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_lds_limit((const void *)leaf_select_kernel, kMaxDynLds, &attr_done));
    hipLaunchKernelGGL(leaf_select_kernel, dim3(nq), dim3(waves * 64), lds, st, centers_t, n_leaves, d,
                       queries, L, ns, leaf_ids, leaf_ip, leaf_cnt, leaf_pos, cnt_stride);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- queries grouped by probed leaf ------------------------------------------------------
//
// The matrix-core scan shares a leaf's code stream among 32 queries, so the (query, probed
// leaf) pairs of a batch (Section 5.3: every query scans a few leaves of the partition) are
// regrouped by leaf: leaf_cnt[l] pairs probe leaf l, they are listed from qlist[leaf_off[l]]
// on as query << 9 | slot (slot = position of the leaf in the query's probe list), and every
// 32 of them are one work item, item_list[i] = leaf << 11 | tile. The order of a leaf's pairs
// depends on the order of atomic operations; no result depends on it.

// One workgroup: running sums of the pair counts and of the item counts; clears the fill cursors. The counts
// arrive spread out (cnt_wide[l * cnt_stride], see group_by_leaf_prepare) and leave side by side in leaf_cnt.
__global__ void __launch_bounds__(1024)
group_offsets_kernel(const uint32_t *__restrict__ cnt_wide, int cnt_stride, uint32_t *__restrict__ leaf_cnt, int n_leaves,
                     uint32_t *__restrict__ leaf_off, uint32_t *__restrict__ item_off, uint32_t *__restrict__ fill,
                     uint32_t *__restrict__ n_items)
{
    __shared__ uint32_t part_p[1024], part_i[1024];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int per = (n_leaves + nt - 1) / nt;
    const int lo = tid * per, hi = lo + per < n_leaves ? lo + per : n_leaves;
    uint32_t sp = 0u, si = 0u;
    for (int l = lo; l < hi; ++l) {
        const uint32_t cn = cnt_wide[(size_t)l * cnt_stride];
        leaf_cnt[l] = cn;
        sp += cn;
        si += (cn + 31u) / 32u;
    }
    part_p[tid] = sp;
    part_i[tid] = si;
    __syncthreads();
    for (int d = 1; d < nt; d *= 2) { // inclusive scans
        const uint32_t ap = tid >= d ? part_p[tid - d] : 0u, ai = tid >= d ? part_i[tid - d] : 0u;
        __syncthreads();
        part_p[tid] += ap;
        part_i[tid] += ai;
        __syncthreads();
    }
    uint32_t op = part_p[tid] - sp, oi = part_i[tid] - si; // exclusive
    for (int l = lo; l < hi; ++l) {
        leaf_off[l] = op;
        item_off[l] = oi;
        fill[l] = 0u;
        op += leaf_cnt[l];
        oi += (leaf_cnt[l] + 31u) / 32u;
    }
    if (tid == nt - 1) *n_items = part_i[tid];
}

__global__ void __launch_bounds__(256)
group_fill_kernel(const int32_t *__restrict__ leaf_ids, const uint32_t *__restrict__ leaf_pos, int64_t n_pairs, int Lp,
                  const uint32_t *__restrict__ leaf_off, uint32_t *__restrict__ qlist)
{
    // a pair's place in its leaf's list was taken when leaf selection counted it: a plain scatter, no atomics
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const int32_t leaf = leaf_ids[i];
    if (leaf < 0) return;
    const uint32_t q = (uint32_t)(i / Lp), slot = (uint32_t)(i % Lp);
    qlist[leaf_off[leaf] + leaf_pos[i]] = (q << 9) | slot;
}

__global__ void __launch_bounds__(256)
group_items_kernel(const uint32_t *__restrict__ leaf_cnt, const uint32_t *__restrict__ item_off, int n_leaves,
                   uint32_t *__restrict__ item_list)
{
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_leaves) return;
    const uint32_t tiles = (leaf_cnt[l] + 31u) / 32u;
    for (uint32_t t = 0; t < tiles; ++t) item_list[item_off[l] + t] = ((uint32_t)l << 11) | t;
}

// Counting a batch's pairs is a million atomic additions to a few thousand words, and additions to words of one
// cache line wait for one another: the counters that take them are spread out, one per 128 bytes while that
// stays under a megabyte.
static int leaf_cnt_stride(int n_leaves)
{
    int stride = 32;
    while (stride > 1 && (size_t)n_leaves * stride > ((size_t)1 << 18)) stride /= 2;
    return stride;
}

size_t group_by_leaf_words(int nq, int Lp, int n_leaves)
{
    return (size_t)4 * n_leaves + 4 + (size_t)2 * nq * Lp + group_by_leaf_max_items(nq, Lp, n_leaves) +
           (size_t)n_leaves * leaf_cnt_stride(n_leaves);
}

// Lays the scratch out and clears the pair counts; leaf selection then counts (launch_leaf_select's
// leaf_cnt = g.cnt_wide with g.cnt_stride), and launch_group_by_leaf does the rest.
int group_by_leaf_prepare(int nq, int Lp, int n_leaves, uint32_t *ws, LeafGroups *g, hipStream_t st)
{
    if (Lp > 512 || nq > (1 << 16) || n_leaves > (1 << 21)) { set_error("grouping by leaf: batch or partition too large"); return AVQ_EINVAL; }
    g->leaf_cnt = ws;
    g->leaf_off = g->leaf_cnt + n_leaves;
    g->item_off = g->leaf_off + n_leaves;
    g->fill = g->item_off + n_leaves;
    g->n_items = g->fill + n_leaves;
    g->qlist = g->n_items + 4;
    g->pos = g->qlist + (size_t)nq * Lp;
    g->item_list = g->pos + (size_t)nq * Lp;
    g->max_items = (int32_t)group_by_leaf_max_items(nq, Lp, n_leaves);
    g->cnt_wide = g->item_list + g->max_items;
    g->cnt_stride = leaf_cnt_stride(n_leaves);
    AVQ_HIP(hipMemsetAsync(g->cnt_wide, 0, sizeof(uint32_t) * (size_t)n_leaves * g->cnt_stride, st));
    return AVQ_OK;
}

int launch_group_by_leaf(const int32_t *leaf_ids, int nq, int Lp, int n_leaves, const LeafGroups &g, hipStream_t st)
{
    const int64_t n_pairs = (int64_t)nq * Lp;
    hipLaunchKernelGGL(group_offsets_kernel, dim3(1), dim3(1024), 0, st, g.cnt_wide, g.cnt_stride, g.leaf_cnt, n_leaves, g.leaf_off,
                       g.item_off, g.fill, g.n_items);
    hipLaunchKernelGGL(group_fill_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st, leaf_ids, g.pos, n_pairs, Lp,
                       g.leaf_off, g.qlist);
    hipLaunchKernelGGL(group_items_kernel, dim3((n_leaves + 255) / 256), dim3(256), 0, st, g.leaf_cnt, g.item_off, n_leaves,
                       g.item_list);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

__global__ void transpose_kernel(const float *__restrict__ in, int rows, int cols,
                                 float *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)rows * cols) return;
    const int r = (int)(i / cols), c = (int)(i % cols);
    out[(size_t)c * rows + r] = in[i];
}

int launch_transpose(const float *in, int rows, int cols, float *out, hipStream_t st)
{
    const int64_t total = (int64_t)rows * cols;
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, in,
                       rows, cols, out);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

} // namespace avq
