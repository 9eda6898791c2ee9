// Leaf selection for the partitioned index (paper Sections 2.2.1 and 5.3: a
// vector-quantization tree reduces the number of points that are scored; the
// paper gives no details, the design here is: one level of leaves, a query
// visits the leaves whose centers have the largest inner product with it).
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

// One workgroup per query; its waves take the leaves 64 at a time in turn, each keeping its
// own list, and the lists are merged pairwise at the end. centers_t is [d][n_leaves] so that
// lane l reads leaf base + l with coalesced loads. The score is the fp32 fma chain in index order.
__global__ void __launch_bounds__(1024)
leaf_select_kernel(const float *__restrict__ centers_t, int n_leaves, int d,
                   const float *__restrict__ queries, int L, int ns,
                   int32_t *__restrict__ leaf_ids, float *__restrict__ leaf_ip)
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
    }
}

int launch_leaf_select(const float *centers_t, int n_leaves, int d, const float *queries, int nq,
                       int L, int32_t *leaf_ids, float *leaf_ip, hipStream_t st)
{
    const int ns = (L + 63) / 64;
    // few queries: as many waves as there are 64-leaf groups (at most 16); batches: four
    int waves = nq >= 1024 ? 4 : 16;
    while (waves > 1 && (waves / 2) * 64 >= n_leaves) waves /= 2;
    const size_t lds = (size_t)waves * (64 * ns + 64) * 8 + (size_t)d * 4;
    if (lds > kMaxDynLds) { set_error("leaf select: L = %d too large", L); return AVQ_EINVAL; }
    static bool attr_done = false;
    if (!attr_done) {
        AVQ_HIP(hipFuncSetAttribute((const void *)leaf_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        attr_done = true;
    }
    hipLaunchKernelGGL(leaf_select_kernel, dim3(nq), dim3(waves * 64), lds, st, centers_t, n_leaves, d,
                       queries, L, ns, leaf_ids, leaf_ip);
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
