// Leaf selection for the partitioned index (paper Sections 2.2.1 and 5.3: a
// vector-quantization tree reduces the number of points that are scored; the
// paper gives no details, the design here is: one level of leaves, a query
// visits the leaves whose centers have the largest inner product with it).
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

// One wave per query. centers_t is [d][n_leaves] so that lane l reads leaf
// t*64 + l with coalesced loads. The score is the fp32 fma chain in index order.
__global__ void __launch_bounds__(64)
leaf_select_kernel(const float *__restrict__ centers_t, int n_leaves, int d,
                   const float *__restrict__ queries, int L, int ns,
                   int32_t *__restrict__ leaf_ids, float *__restrict__ leaf_ip)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int C = 64 * ns;
    const int lane = threadIdx.x;
    const int q = blockIdx.x;
    u64 *list = (u64 *)smem;       // [C]
    u64 *pend = list + C;          // [64]
    float *qs = (float *)(pend + 64);
    for (int l = lane; l < d; l += 64) qs[l] = queries[(size_t)q * d + l];
    wave_list_clear(list, ns);
    float thr = -INFINITY;
    int cnt = 0;
    for (int base = 0; base < n_leaves; base += 64) {
        const int leaf = base + lane;
        const bool valid = leaf < n_leaves;
        float s = 0.0f;
        if (valid)
            for (int l = 0; l < d; ++l) s = __fmaf_rn(qs[l], centers_t[(size_t)l * n_leaves + leaf], s);
        const bool hit = valid && s > thr; // leaves are visited in increasing id
        if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
        if (wave_push(list, ns, pend, cnt, hit, make_key(ord_from_f32(s), leaf))) {
            const u64 kth = list[L - 1];
            thr = kth ? f32_from_ord(key_ord(kth)) : -INFINITY;
        }
    }
    if (cnt > 0) wave_list_flush(list, ns, pend, cnt);
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
    const size_t lds = (size_t)(64 * ns + 64) * 8 + (size_t)d * 4;
    hipLaunchKernelGGL(leaf_select_kernel, dim3(nq), dim3(64), lds, st, centers_t, n_leaves, d,
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
