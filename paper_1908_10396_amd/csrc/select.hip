// Second stage of the top-R selection (merge of the per-chunk lists), exact
// fp32 re-scoring with the final top-k, and brute-force MIPS (paper Section 1:
// argmax over the database of <q, x_i>), which is the ground truth for recall.
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

// ---- merge of per-chunk candidate lists --------------------------------------

// One workgroup per query; wave w merges chunks w, w + W, ...; wave 0 then
// merges the waves' lists. cand[q][C] sorted descending.
__global__ void __launch_bounds__(1024)
merge_partials_kernel(const u64 *__restrict__ partial, int n_chunks, int ns, u64 *__restrict__ cand,
                      const int32_t *__restrict__ row_of, const uint32_t *__restrict__ active, int tile_queries)
{
    if (active != nullptr) {
        if (blockIdx.x >= *active) return;
        if (tile_queries > 0) n_chunks = scan_dynamic_chunks(((int)*active + tile_queries - 1) / tile_queries, n_chunks);
    }
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int q = blockIdx.x;
    u64 *lists = (u64 *)smem;
    u64 *mine = lists + (size_t)wave * C;
    wave_list_clear(mine, ns);
    for (int c = wave; c < n_chunks; c += n_waves)
        wave_list_merge_from(mine, ns, partial + ((size_t)q * n_chunks + c) * C);
    __syncthreads();
    if (wave == 0) {
        for (int w = 1; w < n_waves; ++w) wave_list_merge_from(mine, ns, lists + (size_t)w * C);
        const size_t row = row_of ? (size_t)row_of[q] : (size_t)q;
        for (int i = lane; i < C; i += 64) cand[row * C + i] = mine[i];
    }
}

int launch_merge_partials(const u64 *partial, int nq, int n_chunks, int ns, u64 *cand,
                          hipStream_t st, const int32_t *row_of, const uint32_t *active, int tile_queries)
{
    int waves = 1;
    while (waves < 16 && waves * 4 <= n_chunks) waves *= 2;
    const size_t lds = (size_t)waves * 64 * ns * 8;
    hipLaunchKernelGGL(merge_partials_kernel, dim3(nq), dim3(waves * 64), lds, st, partial,
                       n_chunks, ns, cand, row_of, active, tile_queries);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- top-R of an unsorted key array (block maxima) ---------------------------------

// One workgroup per query: every wave filters its share of the keys into its own
// list, then the lists are merged pairwise up a tree.
__global__ void __launch_bounds__(1024)
select_keys_kernel(const u64 *__restrict__ keys, int64_t n, int ns, int R, u64 *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int q = blockIdx.x;
    u64 *lists = (u64 *)smem;                       // [W][C]
    u64 *pends = lists + (size_t)n_waves * C;       // [W][64]
    u64 *mine = lists + (size_t)wave * C;
    u64 *pend = pends + (size_t)wave * 64;
    wave_list_clear(mine, ns);
    u64 thr = 0ull;
    int cnt = 0;
    const u64 *src = keys + (size_t)q * n;
    for (int64_t base = (int64_t)wave * 64; base < n; base += (int64_t)n_waves * 64) {
        const int64_t i = base + lane;
        const u64 key = i < n ? src[i] : 0ull;
        const bool hit = key > thr;
        if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
        if (wave_push(mine, ns, pend, cnt, hit, key)) thr = mine[R - 1];
    }
    if (cnt > 0) wave_list_flush(mine, ns, pend, cnt);
    for (int stride = 1; stride < n_waves; stride *= 2) {
        __syncthreads();
        if ((wave % (2 * stride)) == 0 && wave + stride < n_waves)
            wave_list_merge_from(mine, ns, lists + (size_t)(wave + stride) * C);
    }
    if (wave == 0)
        for (int i = lane; i < C; i += 64) out[(size_t)q * C + i] = mine[i];
}

int launch_select_keys(const u64 *keys, int nq, int64_t n, int ns, int R, u64 *out, hipStream_t st)
{
    int waves = 16;
    while (waves > 1 && (int64_t)waves * 128 > n) waves /= 2;
    const size_t lds = (size_t)waves * (64 * ns + 64) * 8;
    hipLaunchKernelGGL(select_keys_kernel, dim3(nq), dim3(waves * 64), lds, st, keys, n, ns, R, out);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- exact re-scoring and final top-k -------------------------------------------

// <q, x> as an fp32 fma chain in index order. qs: query in LDS.
__device__ __forceinline__ float dot_chain(const float *qs, const float *__restrict__ row, int d)
{
    float s = 0.0f;
    if ((d & 3) == 0 && (((uintptr_t)row) & 15) == 0) {
        // five 16-byte loads in flight at a time (the chain itself is serial): a row of 100 floats in five rounds
        const float4 *r4 = (const float4 *)row;
        const int n4 = d / 4;
        int l = 0;
        for (; l + 5 <= n4; l += 5) {
            float4 v[5];
#pragma unroll
            for (int u = 0; u < 5; ++u) v[u] = r4[l + u];
#pragma unroll
            for (int u = 0; u < 5; ++u) {
                s = __fmaf_rn(qs[4 * (l + u) + 0], v[u].x, s);
                s = __fmaf_rn(qs[4 * (l + u) + 1], v[u].y, s);
                s = __fmaf_rn(qs[4 * (l + u) + 2], v[u].z, s);
                s = __fmaf_rn(qs[4 * (l + u) + 3], v[u].w, s);
            }
        }
        for (; l < n4; ++l) {
            const float4 v = r4[l];
            s = __fmaf_rn(qs[4 * l + 0], v.x, s);
            s = __fmaf_rn(qs[4 * l + 1], v.y, s);
            s = __fmaf_rn(qs[4 * l + 2], v.z, s);
            s = __fmaf_rn(qs[4 * l + 3], v.w, s);
        }
    } else {
        for (int l = 0; l < d; ++l) s = __fmaf_rn(qs[l], row[l], s);
    }
    return s;
}

// One wave per query.
__global__ void __launch_bounds__(64)
finalize_kernel(const u64 *__restrict__ cand, int ns, int R, int k, int reorder, int key_kind,
                const float *__restrict__ x, int d, const float *__restrict__ queries,
                const float *__restrict__ scale, const float *__restrict__ bias,
                int32_t *__restrict__ ids_out, float *__restrict__ scores_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x;
    const int q = blockIdx.x;
    const u64 *mine = cand + (size_t)q * C;
    if (!reorder) {
        for (int j = lane; j < k; j += 64) {
            const u64 key = mine[j];
            float s = -INFINITY;
            int32_t id = -1;
            if (key) {
                id = key_id(key);
                if (key_kind == 0) s = f32_from_ord(key_ord(key));
                else s = __fmaf_rn((float)(int)(key_ord(key) - 1u), scale[q], bias[q]);
            }
            ids_out[(size_t)q * k + j] = id;
            scores_out[(size_t)q * k + j] = s;
        }
        return;
    }
    u64 *list = (u64 *)smem;              // [C]
    float *qs = (float *)(list + C);      // [d]
    for (int l = lane; l < d; l += 64) qs[l] = queries[(size_t)q * d + l];
    wave_list_clear(list, ns);
    for (int s0 = 0; s0 < R; s0 += 64) {
        const int j = s0 + lane;
        const u64 key = j < R ? mine[j] : 0ull;
        u64 nk = 0ull;
        if (key) {
            const int32_t id = key_id(key);
            const float s = dot_chain(qs, x + (size_t)id * d, d);
            nk = make_key(ord_from_f32(s), id);
        }
        nk = wave_sort_desc(nk);
        wave_list_insert_sorted(list, ns, nk);
    }
    for (int j = lane; j < k; j += 64) {
        const u64 key = list[j];
        ids_out[(size_t)q * k + j] = key ? key_id(key) : -1;
        scores_out[(size_t)q * k + j] = key ? f32_from_ord(key_ord(key)) : -INFINITY;
    }
}

int launch_finalize(const u64 *cand, int ns, int nq, int R, int k, int reorder, int key_kind,
                    const float *x, int d, const float *queries, const float *scale,
                    const float *bias, int32_t *ids_out, float *scores_out, hipStream_t st)
{
    const size_t lds = (size_t)64 * ns * 8 + (size_t)d * 4;
    hipLaunchKernelGGL(finalize_kernel, dim3(nq), dim3(64), lds, st, cand, ns, R, k, reorder,
                       key_kind, x, d, queries, scale, bias, ids_out, scores_out);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- brute force --------------------------------------------------------------------

// grid = (chunks, query tiles of QB). Each lane scores one point against QB
// queries per step (the row is read once per tile), then filters into per-wave
// lists exactly like the ADC scan does.
template <int QB>
__global__ void __launch_bounds__(256)
brute_kernel(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ queries,
             int nq, int ns, int k, int64_t pts_per_chunk, int n_chunks, u64 *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int chunk = blockIdx.x, q0 = blockIdx.y * QB;
    float *qs = (float *)smem;                                   // [QB][d]
    u64 *lists = (u64 *)(smem + (((size_t)QB * d * 4 + 15) & ~(size_t)15)); // [W][QB][C]
    u64 *pends = lists + (size_t)n_waves * QB * C;               // [W][QB][64]
    u64 *my_lists = lists + (size_t)wave * QB * C;
    u64 *my_pends = pends + (size_t)wave * QB * 64;
    for (int i = threadIdx.x; i < QB * d; i += blockDim.x) {
        const int q = q0 + i / d;
        qs[i] = q < nq ? queries[(size_t)q * d + i % d] : 0.0f;
    }
    for (int i = lane; i < QB * C; i += 64) my_lists[i] = 0ull;
    __syncthreads();
    float thr[QB];
    int cnt[QB];
#pragma unroll
    for (int q = 0; q < QB; ++q) { thr[q] = -INFINITY; cnt[q] = 0; }
    const int64_t first = (int64_t)chunk * pts_per_chunk;
    int64_t end = first + pts_per_chunk;
    if (end > n) end = n;
    for (int64_t base = first + (int64_t)wave * 64; base < end; base += (int64_t)n_waves * 64) {
        const int64_t i = base + lane;
        const bool valid = i < end;
        const float *row = x + (size_t)(valid ? i : first) * d;
        float s[QB];
#pragma unroll
        for (int q = 0; q < QB; ++q) s[q] = 0.0f;
        for (int l = 0; l < d; ++l) {
            const float v = row[l];
#pragma unroll
            for (int q = 0; q < QB; ++q) s[q] = __fmaf_rn(qs[q * d + l], v, s[q]);
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const bool hit = valid && s[q] > thr[q]; // ids increase along the scan: strict is exact
            if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
            u64 *list = my_lists + (size_t)q * C;
            if (wave_push(list, ns, my_pends + q * 64, cnt[q], hit, make_key(ord_from_f32(s[q]), (int32_t)i))) {
                const u64 kth = list[k - 1];
                thr[q] = kth ? f32_from_ord(key_ord(kth)) : -INFINITY;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < QB; ++q)
        if (cnt[q] > 0) wave_list_flush(my_lists + (size_t)q * C, ns, my_pends + q * 64, cnt[q]);
    __syncthreads();
    for (int q = wave; q < QB; q += n_waves) {
        u64 *mine = my_lists + (size_t)q * C;
        for (int w = 0; w < n_waves; ++w)
            if (w != wave) wave_list_merge_from(mine, ns, lists + ((size_t)w * QB + q) * C);
        if (q0 + q < nq) {
            u64 *out = partial + ((size_t)(q0 + q) * n_chunks + chunk) * C;
            for (int i = lane; i < C; i += 64) out[i] = mine[i];
        }
    }
}

int brute_force_chunks(int64_t n, int nq)
{
    // enough workgroups to fill the chip even for a handful of queries
    int64_t tiles = (nq + 7) / 8;
    int64_t chunks = (2048 + tiles - 1) / tiles;
    int64_t max_chunks = (n + 1023) / 1024;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    return (int)chunks;
}

int launch_brute_force(const float *x, int64_t n, int d, const float *queries, int nq, int k,
                       u64 *partial_ws, int n_chunks, u64 *cand_ws, int32_t *ids_out,
                       float *scores_out, hipStream_t st)
{
    const int ns = (k + 63) / 64;
    const int C = 64 * ns;
    const int64_t ppc = (n + n_chunks - 1) / n_chunks;
    const int waves = 4;
    auto lds_for = [&](int qb) {
        return (((size_t)qb * d * 4 + 15) & ~(size_t)15) + (size_t)waves * qb * (C + 64) * 8;
    };
    if (lds_for(8) <= 96 * 1024) {
        AVQ_HIP(hipFuncSetAttribute((const void *)brute_kernel<8>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        hipLaunchKernelGGL(brute_kernel<8>, dim3(n_chunks, (nq + 7) / 8), dim3(waves * 64),
                           lds_for(8), st, x, n, d, queries, nq, ns, k, ppc, n_chunks, partial_ws);
    } else if (lds_for(1) <= kMaxDynLds) {
        AVQ_HIP(hipFuncSetAttribute((const void *)brute_kernel<1>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        hipLaunchKernelGGL(brute_kernel<1>, dim3(n_chunks, nq), dim3(waves * 64), lds_for(1), st, x,
                           n, d, queries, nq, ns, k, ppc, n_chunks, partial_ws);
    } else {
        set_error("brute force: d = %d too large", d);
        return AVQ_EINVAL;
    }
    AVQ_HIP(hipGetLastError());
    AVQ_TRY(launch_merge_partials(partial_ws, nq, n_chunks, ns, cand_ws, st));
    return launch_finalize(cand_ws, ns, nq, k, k, 0, 0, nullptr, d, queries, nullptr, nullptr,
                           ids_out, scores_out, st);
}

} // namespace avq
