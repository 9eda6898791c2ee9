// Lookup-table build (paper Section 4.1: for every dictionary the partial dot
// product of the query's subspace with every codeword; cost O(kd) per query,
// Section 2.2.2) and its 8-bit quantisation.
//
// One workgroup per query. The contraction is d*kc multiply-adds per query --
// far too small to matter next to the scan -- and its results feed integer
// decisions (the 8-bit table codes), so it is an explicit fp32 fma chain in
// index order rather than an MFMA tile whose internal summation order is not a
// contract.
#include "avq_internal.h"

namespace avq {

__global__ void __launch_bounds__(256)
lut_kernel(const float *__restrict__ queries, const float *__restrict__ codebooks, int d, int M,
           int kc, float *__restrict__ lut_f32, uint8_t *__restrict__ lut_u8,
           float *__restrict__ scale_out, float *__restrict__ bias_out)
{
    extern __shared__ float sm[]; // u8 mode: L[M*kc], lo[M], width[M]
    const int qi = blockIdx.x;
    const int ds = d / M;
    const float *q = queries + (size_t)qi * d;
    const int total = M * kc;
    const bool u8 = lut_u8 != nullptr;
    float *L = sm;
    float *lo_s = sm + total;
    float *wd_s = lo_s + M;

    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        const int m = e / kc;
        const float *c = codebooks + (size_t)e * ds;
        float s = 0.0f;
        for (int l = 0; l < ds; ++l) s = __fmaf_rn(q[m * ds + l], c[l], s);
        if (lut_f32) lut_f32[(size_t)qi * total + e] = s;
        if (u8) L[e] = s;
    }
    if (!u8) return;
    __syncthreads();
    // per subspace: lo = min, width = max - min (sequential compares in index order)
    for (int m = threadIdx.x; m < M; m += blockDim.x) {
        float lo = L[m * kc], hi = lo;
        for (int j = 1; j < kc; ++j) {
            const float v = L[m * kc + j];
            if (v < lo) lo = v;
            if (v > hi) hi = v;
        }
        lo_s[m] = lo;
        wd_s[m] = __fsub_rn(hi, lo);
    }
    __syncthreads();
    // one range for the whole query and the bias, in subspace order
    __shared__ float sh_inv, sh_R;
    if (threadIdx.x == 0) {
        float R = 0.0f, b = 0.0f;
        for (int m = 0; m < M; ++m) {
            if (wd_s[m] > R) R = wd_s[m];
            b = __fadd_rn(b, lo_s[m]);
        }
        sh_R = R;
        sh_inv = R == 0.0f ? 0.0f : __fdiv_rn(255.0f, R);
        scale_out[qi] = R == 0.0f ? 0.0f : __fdiv_rn(R, 255.0f);
        bias_out[qi] = b;
    }
    __syncthreads();
    const float inv = sh_inv;
    const bool flat = sh_R == 0.0f;
    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        uint8_t code = 0;
        if (!flat) {
            float t = __fsub_rn(L[e], lo_s[e / kc]);
            t = __fmul_rn(t, inv);
            t = rintf(t); // round half to even
            t = t < 0.0f ? 0.0f : (t > 255.0f ? 255.0f : t);
            code = (uint8_t)t;
        }
        lut_u8[(size_t)qi * total + e] = code;
    }
}

int launch_lut(const float *queries, int nq, const float *codebooks, int d, int M, int kc,
               float *lut_f32, uint8_t *lut_u8, float *scale, float *bias, hipStream_t st)
{
    const size_t lds = lut_u8 ? ((size_t)M * kc + 2 * (size_t)M) * sizeof(float) : 0;
    if (lds > 60 * 1024) {
        set_error("lut: M*kc = %d too large for the 8-bit table build", M * kc);
        return AVQ_EINVAL;
    }
    hipLaunchKernelGGL(lut_kernel, dim3(nq), dim3(256), lds, st, queries, codebooks, d, M, kc,
                       lut_f32, lut_u8, scale, bias);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

} // namespace avq
