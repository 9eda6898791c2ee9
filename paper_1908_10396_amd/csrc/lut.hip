// Lookup-table build (paper Section 4.1: for every dictionary the partial dot
// product of the query's subspace with every codeword; cost O(kd) per query,
// Section 2.2.2) and its 8-bit quantisation.
//
// One workgroup per query. The contraction is d*kc multiply-adds per query --
// far too small to matter next to the scan -- and its results feed integer
// decisions (the 8-bit table codes), so it is an explicit fp32 fma chain in
// index order rather than an MFMA tile whose internal summation order is not a
// contract.
#include <type_traits>
#include "avq_internal.h"

namespace avq {

// The table build for batches (one workgroup of 256 threads per query, made for throughput: a thread per
// subspace finds its minimum and width, one thread the range and the bias).
__global__ void __launch_bounds__(256)
lut_batch_kernel(const float *__restrict__ queries, const float *__restrict__ codebooks, int d, int M,
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

// The same tables for one query or a few, made for latency.
// First occurrence of the smallest (MIN) or largest value, as a sequential scan with < or > finds it: among equal
// values (+0 and -0 are equal) the lower index wins.
template <bool MIN>
__device__ __forceinline__ bool better(float v, int i, float w, int j)
{
    return (MIN ? v < w : v > w) || (v == w && i < j);
}

__global__ void __launch_bounds__(1024)
lut_kernel(const float *__restrict__ queries, const float *__restrict__ codebooks, int d, int M,
           int kc, float *__restrict__ lut_f32, uint8_t *__restrict__ lut_u8,
           float *__restrict__ scale_out, float *__restrict__ bias_out)
{
    extern __shared__ float sm[]; // q[d]; u8 mode: L[M*kc], lo[M], width[M]
    const int qi = blockIdx.x;
    const int ds = d / M;
    const int total = M * kc;
    const bool u8 = lut_u8 != nullptr;
    const int tid = threadIdx.x, nt = blockDim.x;
    float *qs = sm;
    float *L = sm + d;
    float *lo_s = L + total;
    float *wd_s = lo_s + M;

    // one entry per thread and round; a round is up to eight entries per thread whose codeword loads are all in
    // flight together, the first round's together with the query's
    constexpr int kPer = 8;
    auto entry = [&](int e, const float *cw) {
        const int m = e / kc;
        float s = 0.0f;
        for (int l = 0; l < ds; ++l) s = __fmaf_rn(qs[m * ds + l], cw[l], s);
        if (lut_f32) lut_f32[(size_t)qi * total + e] = s;
        if (u8) L[e] = s;
    };
    // the codeword as 16-byte (8-byte for two dimensions) loads into registers, for the usual subspace sizes
    auto rounds = [&](auto ds_tag) {
        constexpr int DS = decltype(ds_tag)::value;
        for (int e0 = tid; e0 < total || e0 == tid; e0 += kPer * nt) {
            float cw[kPer][DS];
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int e = e0 + i * nt;
                if (e >= total) continue;
                const float *c = codebooks + (size_t)e * DS;
                if (DS == 2) { const float2 v = *(const float2 *)c; cw[i][0] = v.x; cw[i][1] = v.y; }
                else {
#pragma unroll
                    for (int l4 = 0; l4 < DS / 4; ++l4) {
                        const float4 v = *(const float4 *)(c + 4 * l4);
                        cw[i][4 * l4] = v.x; cw[i][4 * l4 + 1] = v.y; cw[i][4 * l4 + 2] = v.z; cw[i][4 * l4 + 3] = v.w;
                    }
                }
            }
            if (e0 == tid) { // first round (every thread has one): the query arrives with the codewords
                for (int l = tid; l < d; l += nt) qs[l] = queries[(size_t)qi * d + l];
                __syncthreads();
            }
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int e = e0 + i * nt;
                if (e >= total) continue;
                const int m = e / kc;
                float sum = 0.0f;
#pragma unroll
                for (int l = 0; l < DS; ++l) sum = __fmaf_rn(qs[m * DS + l], cw[i][l], sum);
                if (lut_f32) lut_f32[(size_t)qi * total + e] = sum;
                if (u8) L[e] = sum;
            }
        }
    };
    if (ds == 2) rounds(std::integral_constant<int, 2>{});
    else if (ds == 4) rounds(std::integral_constant<int, 4>{});
    else if (ds == 8) rounds(std::integral_constant<int, 8>{});
    else {
        for (int l = tid; l < d; l += nt) qs[l] = queries[(size_t)qi * d + l];
        __syncthreads();
        for (int e = tid; e < total; e += nt) entry(e, codebooks + (size_t)e * ds);
    }
    if (!u8) return;
    __syncthreads();
    // per subspace: lo = min, width = max - min, as sequential compares in index order find them; a group of
    // G = min(kc, 64) lanes per subspace, every lane its entries in index order, then the lanes of a group pairwise
    {
        const int G = kc < 64 ? kc : 64; // a power of two (kc is 16 or 256)
        const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
        const int per_wave = 64 / G, g = lane % G;
        for (int m0 = wave * per_wave; m0 < M; m0 += n_waves * per_wave) {
            const int m = m0 + lane / G;
            float lo = 0.0f, hi = 0.0f;
            int li = 0x7fffffff, hi_i = 0x7fffffff;
            if (m < M) {
                for (int j = g; j < kc; j += G) {
                    const float v = L[m * kc + j];
                    if (li == 0x7fffffff || better<true>(v, j, lo, li)) { lo = v; li = j; }
                    if (hi_i == 0x7fffffff || better<false>(v, j, hi, hi_i)) { hi = v; hi_i = j; }
                }
            }
            for (int w = 1; w < G; w <<= 1) {
                const float olo = __shfl_xor(lo, w, 64), ohi = __shfl_xor(hi, w, 64);
                const int oli = __shfl_xor(li, w, 64), ohi_i = __shfl_xor(hi_i, w, 64);
                if (better<true>(olo, oli, lo, li)) { lo = olo; li = oli; }
                if (better<false>(ohi, ohi_i, hi, hi_i)) { hi = ohi; hi_i = ohi_i; }
            }
            if (m < M && g == 0) {
                lo_s[m] = lo;
                wd_s[m] = __fsub_rn(hi, lo);
            }
        }
    }
    __syncthreads();
    // one range for the whole query (the largest width) and the bias, the sum of the minima in subspace order:
    // the first wave, 64 subspaces at a time, lane 0's sum taking the lanes' values one after the other
    __shared__ float sh_inv, sh_R;
    if (tid < 64) {
        float R = 0.0f, b = 0.0f;
        for (int m0 = 0; m0 < M; m0 += 64) {
            const int m = m0 + tid;
            float w = m < M ? wd_s[m] : 0.0f;
            const float lo = m < M ? lo_s[m] : 0.0f;
            for (int x = 1; x < 64; x <<= 1) { const float o = __shfl_xor(w, x, 64); w = o > w ? o : w; }
            if (w > R) R = w;
            const int cnt = M - m0 < 64 ? M - m0 : 64;
            for (int i = 0; i < cnt; ++i) b = __fadd_rn(b, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lo), i)));
        }
        if (tid == 0) {
            sh_R = R;
            sh_inv = R == 0.0f ? 0.0f : __fdiv_rn(255.0f, R);
            scale_out[qi] = R == 0.0f ? 0.0f : __fdiv_rn(R, 255.0f);
            bias_out[qi] = b;
        }
    }
    __syncthreads();
    const float inv = sh_inv;
    const bool flat = sh_R == 0.0f;
    for (int e = tid; e < total; e += nt) {
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
    const size_t lds = ((size_t)d + (lut_u8 ? (size_t)M * kc + 2 * (size_t)M : 0)) * sizeof(float);
    if (lds > 62 * 1024) {
        set_error("lut: d = %d, M*kc = %d too large for the table build", d, M * kc);
        return AVQ_EINVAL;
    }
    if (kc != 16 && kc != 256) { set_error("lut: %d codewords per subspace", kc); return AVQ_EINVAL; }
    if (nq > 32) {
        const size_t lds_b = lut_u8 ? ((size_t)M * kc + 2 * (size_t)M) * sizeof(float) : 0;
        hipLaunchKernelGGL(lut_batch_kernel, dim3(nq), dim3(256), lds_b, st, queries, codebooks, d, M, kc,
                           lut_f32, lut_u8, scale, bias);
    } else {
        const int threads = M * kc > 256 ? 1024 : 256;
        hipLaunchKernelGGL(lut_kernel, dim3(nq), dim3(threads), lds, st, queries, codebooks, d, M, kc,
                           lut_f32, lut_u8, scale, bias);
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

} // namespace avq
