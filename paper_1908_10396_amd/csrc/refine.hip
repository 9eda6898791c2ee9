// fp32-table search by way of the 8-bit-table scan (flat index, 4-bit codes).
//
// The ADC score of Section 4.1 with fp32 tables is s_i = sum_m L[m][code_i[m]]. The 8-bit
// tables hold code[m][j] = rne((L[m][j] - lo_m) * c), c = 255 / R, so with
// u[m][j] = (L[m][j] - lo_m) * c (real numbers) s_i = sum_m lo_m + (1/c) * sum_m u[m][code_i[m]]
// exactly, and the integer sum acc_i the matrix-core scan produces differs from
// U_i = sum_m u[m][code_i[m]] by at most E = M * (1/2 + 4e-5) (rounding to integer, plus the
// fp32 rounding of the two operations inside rne()). The fp32 sum the scan kernels form
// (entries of a byte first, then the bytes in order) differs from the real s_i by at most
// rho = (NB + 2) * 2^-24 * sum_m max_j |L[m][j]|.
//
// Let the candidates be the Rp points of largest acc (ties by lower id), acc_(R) the R-th
// largest and acc_last the smallest of them. The R best candidates by acc all have fp32 score
// >= bound = sum lo + (acc_(R) - E)/c - rho, so the R-th best fp32 score of the whole index
// is >= bound; a point outside the list has acc <= acc_last and fp32 score
// <= sum lo + (acc_last + E)/c + rho. If acc_last < acc_(R) - (2E + 2 rho c) that is
// strictly below bound: no point outside the list is among the R best, and the R best of
// the index are the R best of the candidates, which are then re-scored and ranked exactly.
// Where the condition fails (lists too short for a flat score distribution, or tables with a
// tiny range) the query is handed to the plain fp32 scan instead.
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

__global__ void __launch_bounds__(256)
refine_f32_kernel(const RefineParams r)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int q = blockIdx.x;
    const int Cp = 64 * r.nsp, C = 64 * r.ns;
    const int n_tab = 2 * r.NB; // odd M: one all-zero table, as in the scan kernels
    float *tbl = (float *)smem;                                   // [n_tab][16]
    u64 *keys = (u64 *)(smem + (((size_t)n_tab * 64 + 15) & ~(size_t)15)); // [Rp]
    __shared__ float amax_sum;
    __shared__ int n_cand_s;

    const float *L = r.lut + (size_t)q * r.M * 16;
    for (int e = tid; e < n_tab * 16; e += nt) tbl[e] = e < r.M * 16 ? L[e] : 0.0f;
    if (tid == 0) { amax_sum = 0.0f; n_cand_s = 0; }
    __syncthreads();
    // A = sum_m max_j |L[m][j]| and the number of candidates (the list is sorted, empty slots are 0)
    if (tid < r.M) {
        float a = 0.0f;
        for (int j = 0; j < 16; ++j) a = fmaxf(a, fabsf(tbl[tid * 16 + j]));
        atomicAdd(&amax_sum, a); // order of the additions does not matter: only an upper bound is needed (slack below)
    }
    const u64 *cand = r.cand8 + (size_t)q * Cp;
    int mine = 0;
    for (int i = tid; i < r.Rp; i += nt) mine += cand[i] != 0ull;
    if (mine) atomicAdd(&n_cand_s, mine);
    __syncthreads();
    const int n_cand = n_cand_s;
    bool ok = true;
    if (n_cand == r.Rp) {
        // full list: points outside it exist, the gap between the R-th and the last sum must exceed the margin
        const float scale = r.scale[q];
        const float rho = (float)(r.NB + 2) * 5.9604645e-8f * amax_sum * 1.01f;
        const float marg_f = (float)r.M + 0.01f + (scale > 0.0f ? 2.02f * rho / scale : INFINITY);
        ok = false;
        if (marg_f < 1.0e6f) {
            const int64_t margin = (int64_t)ceilf(marg_f) + 1;
            const int64_t acc_r = (int64_t)key_ord(cand[r.R - 1]);
            const int64_t acc_last = (int64_t)key_ord(cand[r.Rp - 1]);
            ok = acc_last < acc_r - margin;
        }
    }
    if (r.force_fail_odd && (q & 1)) ok = false;
    if (!ok) {
        if (tid == 0) r.fail_list[atomicAdd(r.fail_count, 1u)] = q;
        return;
    }
    // exact fp32 table sums of the candidates: per code byte the two entries first, then the bytes in order
    for (int i = tid; i < n_cand; i += nt) {
        const int32_t id = key_id(cand[i]);
        const uint8_t *row = r.codes + (size_t)id * r.NB;
        float s = 0.0f;
        for (int b = 0; b < r.NB; ++b) {
            const uint32_t byte = row[b];
            const float v = __fadd_rn(tbl[(2 * b) * 16 + (byte & 15u)], tbl[(2 * b + 1) * 16 + (byte >> 4)]);
            s = __fadd_rn(s, v);
        }
        keys[i] = make_key(ord_from_f32(s), id);
    }
    __syncthreads();
    // rank by counting, four lanes per key
    u64 *out = r.out + (size_t)q * C;
    for (int j0 = 0; j0 < n_cand; j0 += nt / 4) {
        const int j = j0 + (tid >> 2);
        const u64 k = j < n_cand ? keys[j] : ~0ull;
        int rank = 0;
        for (int t = tid & 3; t < n_cand; t += 4) rank += keys[t] > k;
        rank += __shfl_xor(rank, 1, 64);
        rank += __shfl_xor(rank, 2, 64);
        if (j < n_cand && (tid & 3) == 0 && rank < r.R) out[rank] = k;
    }
    const int n_fin = n_cand < r.R ? n_cand : r.R;
    for (int i = n_fin + tid; i < C; i += nt) out[i] = 0ull;
}

int launch_refine_f32(const RefineParams &r, hipStream_t st)
{
    if (r.M > 64 || r.Rp <= r.R || r.Rp > 64 * r.nsp || r.R > 64 * r.ns) {
        set_error("refine: bad shape (M %d, R %d, Rp %d)", r.M, r.R, r.Rp);
        return AVQ_EINVAL;
    }
    const size_t lds = (((size_t)2 * r.NB * 64 + 15) & ~(size_t)15) + sizeof(u64) * (size_t)r.Rp;
    hipLaunchKernelGGL(refine_f32_kernel, dim3(r.nq), dim3(256), lds, st, r);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

__global__ void __launch_bounds__(256)
gather_rows_kernel(const float *__restrict__ src, float *__restrict__ dst, const int32_t *__restrict__ row,
                   const uint32_t *__restrict__ count, int row_floats)
{
    if (blockIdx.x >= *count) return;
    const float *s = src + (size_t)row[blockIdx.x] * row_floats;
    float *d = dst + (size_t)blockIdx.x * row_floats;
    for (int e = threadIdx.x; e < row_floats; e += blockDim.x) d[e] = s[e];
}

int launch_gather_rows(const float *src, float *dst, const int32_t *row, const uint32_t *count, int max_rows,
                       int row_floats, hipStream_t st)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3(max_rows), dim3(256), 0, st, src, dst, row, count, row_floats);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

} // namespace avq
