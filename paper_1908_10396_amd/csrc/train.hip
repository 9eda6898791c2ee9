// Dictionary learning and encoding.
//
// Dictionaries: Lloyd's algorithm under the l2 loss, per subspace (paper
// Section 4: the k-means objective; Section 5.1 learns the dictionary this way
// and then assigns codes under the anisotropic loss; Section 4.1 names it as the
// initialisation). Encoding: the partition-assignment step of Section 4.1 under
// the loss eta*||r_par||^2 + ||r_perp||^2 of Section 3.2.
//
// All arithmetic here is fp64: the results are arg-mins, and they have to agree
// with a plain reference evaluation except at exact ties.
#include "avq_internal.h"

namespace avq {

// ---- eta (Section 3.2, Theorem 3.4) --------------------------------------------

__host__ __device__ inline double clamp_ratio_sq(double T, double norm)
{
    const double r = T / norm;
    const double u = r * r;
    return u > 0.999 ? 0.999 : u;
}

// int_0^alpha sin^d by composite Simpson (smooth integrand, fixed fine grid).
__host__ __device__ inline double sin_power_integral(int d, double alpha)
{
    const int N = 8192;
    const double h = alpha / N;
    double s = (d == 0 ? 2.0 : pow(sin(alpha), (double)d));
    for (int i = 1; i < N; ++i) {
        const double f = d == 0 ? 1.0 : pow(sin(i * h), (double)d);
        s += (i & 1) ? 4.0 * f : 2.0 * f;
    }
    return s * h / 3.0;
}

__host__ __device__ inline double eta_of_norm(int d, double T, double norm, int mode, double eta_explicit)
{
    if (mode == AVQ_ETA_EXPLICIT) return eta_explicit;
    if (!(norm > 0.0) || d < 2) return 1.0;
    const double u = clamp_ratio_sq(T, norm);
    if (mode == AVQ_ETA_EXACT) {
        // eta = h_par / h_perp = (d-1) (I_{d-2} / I_d - 1), I_d = int_0^alpha sin^d,
        // alpha = arccos(T / ||x||)
        const double alpha = acos(sqrt(u));
        return (double)(d - 1) * (sin_power_integral(d - 2, alpha) / sin_power_integral(d, alpha) - 1.0);
    }
    // the limit of Theorem 3.4 as a proxy, floored at 1 (Theorem 3.3: h_par >= h_perp)
    const double eta = (double)(d - 1) * u / (1.0 - u);
    return eta < 1.0 ? 1.0 : eta;
}

double eta_host(int d, double T, double norm, int mode) { return eta_of_norm(d, T, norm, mode, 1.0); }

// ---- k-means ----------------------------------------------------------------------

static inline uint64_t mix64(uint64_t z)
{
    // splitmix64 output function
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Stratified draw of the initial codewords: index of codeword j among n rows.
static int64_t init_index(uint64_t seed, uint32_t stream_id, int j, int k, int64_t n)
{
    const int64_t lo = (int64_t)(((__int128)j * n) / k);
    const int64_t hi = (int64_t)(((__int128)(j + 1) * n) / k);
    const uint64_t h = mix64(seed ^ mix64(((uint64_t)stream_id << 32) | (uint32_t)j));
    return lo + (int64_t)(h % (uint64_t)(hi - lo));
}

__device__ __forceinline__ double sub_value(const float *__restrict__ x, int64_t i, int ld, int col,
                                            const float *__restrict__ rc, const int32_t *__restrict__ ra)
{
    double v = (double)x[(size_t)i * ld + col];
    if (rc) v -= (double)rc[(size_t)ra[i] * ld + col];
    return v;
}

__global__ void init_centers_kernel(const float *__restrict__ x, int ld, int col0, int dim, int k,
                                    const int64_t *__restrict__ idx, const float *__restrict__ rc,
                                    const int32_t *__restrict__ ra, float *__restrict__ centers)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= k * dim) return;
    const int j = t / dim, l = t % dim;
    centers[t] = (float)sub_value(x, idx[j], ld, col0 + l, rc, ra);
}

// One thread per point: nearest center in fp64 squared l2 (lowest index on
// ties); the point's values are staged in LDS, transposed, so the inner loop
// reads them conflict-free; every lane reads the same center value.
// ACCUM: add the point into sums/counts; else write the assignment.
// ACCUM with k*dim <= kLdsAccMax: sums are first added up per workgroup in LDS.
constexpr int kLdsAccMax = 4096;

// XT: type of the staged values. float (half the LDS, so twice the waves per compute unit at large dim) holds
// them exactly when no residual is formed (rc == nullptr: the values are the floats of x).
template <bool ACCUM, typename XT = double>
__global__ void __launch_bounds__(256)
nearest_kernel(const float *__restrict__ x, int64_t n, int ld, int col0, int dim, int k,
               const float *__restrict__ rc, const int32_t *__restrict__ ra,
               const float *__restrict__ centers, double *__restrict__ sums,
               unsigned long long *__restrict__ counts, int32_t *__restrict__ assign)
{
    extern __shared__ double xs_raw[]; // XT [dim][blockDim.x], then (ACCUM, small k*dim) double [k*dim] + [k]
    XT *xs = (XT *)xs_raw;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    const int bs = blockDim.x;
    const bool lds_acc = ACCUM && k * dim <= kLdsAccMax;
    double *lsum = (double *)(xs + (size_t)dim * bs); // 8-byte aligned: bs is a multiple of 64
    unsigned long long *lcnt = (unsigned long long *)(lsum + k * dim);
    if (lds_acc) {
        for (int t = threadIdx.x; t < k * dim; t += bs) lsum[t] = 0.0;
        for (int t = threadIdx.x; t < k; t += bs) lcnt[t] = 0ull;
        __syncthreads();
    }
    for (int l = 0; l < dim; ++l) xs[l * bs + threadIdx.x] = valid ? (XT)sub_value(x, i, ld, col0 + l, rc, ra) : (XT)0;
    int best = 0;
    double bestd = INFINITY;
    for (int j = 0; j < k; ++j) {
        const float *c = centers + (size_t)j * dim;
        double dd = 0.0;
        for (int l = 0; l < dim; ++l) {
            const double t = (double)xs[l * bs + threadIdx.x] - (double)c[l];
            dd += t * t;
        }
        if (dd < bestd) { bestd = dd; best = j; }
    }
    if (lds_acc) {
        if (valid) {
            for (int l = 0; l < dim; ++l) atomicAdd(&lsum[best * dim + l], (double)xs[l * bs + threadIdx.x]);
            atomicAdd(&lcnt[best], 1ull);
        }
        __syncthreads();
        for (int t = threadIdx.x; t < k; t += bs) {
            if (lcnt[t] == 0ull) continue;
            atomicAdd(&counts[t], lcnt[t]);
            for (int l = 0; l < dim; ++l) atomicAdd(&sums[(size_t)t * dim + l], lsum[t * dim + l]);
        }
        return;
    }
    if (!valid) return;
    if (ACCUM) {
        for (int l = 0; l < dim; ++l) atomicAdd(&sums[(size_t)best * dim + l], (double)xs[l * bs + threadIdx.x]);
        atomicAdd(&counts[best], 1ull);
    } else {
        assign[i] = best;
    }
}

__global__ void update_centers_kernel(const double *__restrict__ sums,
                                      const unsigned long long *__restrict__ counts, int k, int dim,
                                      float *__restrict__ centers)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= k * dim) return;
    const unsigned long long c = counts[t / dim];
    if (c > 0) centers[t] = (float)(sums[t] / (double)c); // an empty cluster keeps its center
}

static int nearest_block_size(int dim)
{
    int bs = 256;
    while (bs > 64 && (size_t)bs * dim * sizeof(double) > 120 * 1024) bs /= 2;
    return bs;
}

// Values staged as floats (no residual, and doubles would leave room for one small workgroup per compute
// unit only): workgroups of at most 64 KB, so that several share a compute unit.
static bool nearest_stage_floats(int dim, bool residual)
{
    return !residual && (size_t)256 * dim * sizeof(double) > 64 * 1024;
}
static int nearest_block_size_floats(int dim)
{
    int bs = 256;
    while (bs > 64 && (size_t)bs * dim * sizeof(float) > 64 * 1024) bs /= 2;
    return bs;
}

int kmeans_device(const float *x, int64_t n, int ld, int col0, int dim, int k, int iters,
                  uint64_t seed, uint32_t stream_id, const float *resid_centers,
                  const int32_t *resid_assign, float *centers, hipStream_t st)
{
    if (n < k) { set_error("k-means: %lld points for %d centers", (long long)n, k); return AVQ_EINVAL; }
    const bool floats = nearest_stage_floats(dim, resid_centers != nullptr);
    const int bs = floats ? nearest_block_size_floats(dim) : nearest_block_size(dim);
    const size_t stage = (size_t)bs * dim * (floats ? sizeof(float) : sizeof(double));
    if (stage > 150 * 1024) {
        set_error("k-means: dimension %d too large", dim);
        return AVQ_EINVAL;
    }
    std::vector<int64_t> idx(k);
    for (int j = 0; j < k; ++j) idx[j] = init_index(seed, stream_id, j, k, n);
    int64_t *idx_dev = nullptr;
    double *sums = nullptr;
    unsigned long long *counts = nullptr;
    AVQ_HIP(hipMalloc(&idx_dev, sizeof(int64_t) * k));
    AVQ_HIP(hipMalloc(&sums, sizeof(double) * (size_t)k * dim));
    AVQ_HIP(hipMalloc(&counts, sizeof(unsigned long long) * k));
    int rc = AVQ_OK;
    auto body = [&]() -> int {
        AVQ_HIP(hipMemcpyAsync(idx_dev, idx.data(), sizeof(int64_t) * k, hipMemcpyHostToDevice, st));
        hipLaunchKernelGGL(init_centers_kernel, dim3((k * dim + 255) / 256), dim3(256), 0, st, x, ld,
                           col0, dim, k, idx_dev, resid_centers, resid_assign, centers);
        AVQ_HIP(hipGetLastError());
        AVQ_HIP(hipFuncSetAttribute((const void *)nearest_kernel<true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        AVQ_HIP(hipFuncSetAttribute((const void *)nearest_kernel<true, float>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        const unsigned grid = (unsigned)((n + bs - 1) / bs);
        for (int it = 0; it < iters; ++it) {
            AVQ_HIP(hipMemsetAsync(sums, 0, sizeof(double) * (size_t)k * dim, st));
            AVQ_HIP(hipMemsetAsync(counts, 0, sizeof(unsigned long long) * k, st));
            const size_t lds = stage + (k * dim <= kLdsAccMax ? (size_t)(k * dim + k) * sizeof(double) : 0);
            if (floats)
                hipLaunchKernelGGL((nearest_kernel<true, float>), dim3(grid), dim3(bs), lds, st, x, n, ld, col0, dim,
                                   k, resid_centers, resid_assign, centers, sums, counts, (int32_t *)nullptr);
            else
                hipLaunchKernelGGL(nearest_kernel<true>, dim3(grid), dim3(bs), lds,
                                   st, x, n, ld, col0, dim, k, resid_centers, resid_assign, centers, sums,
                                   counts, (int32_t *)nullptr);
            AVQ_HIP(hipGetLastError());
            hipLaunchKernelGGL(update_centers_kernel, dim3((k * dim + 255) / 256), dim3(256), 0, st, sums,
                               counts, k, dim, centers);
            AVQ_HIP(hipGetLastError());
        }
        AVQ_HIP(hipStreamSynchronize(st));
        return AVQ_OK;
    };
    rc = body();
    (void)hipFree(idx_dev);
    (void)hipFree(sums);
    (void)hipFree(counts);
    return rc;
}

int launch_assign_nearest(const float *x, int64_t n, int d, const float *centers, int k,
                          int32_t *assign, hipStream_t st)
{
    const bool floats = nearest_stage_floats(d, false);
    const int bs = floats ? nearest_block_size_floats(d) : nearest_block_size(d);
    const size_t stage = (size_t)bs * d * (floats ? sizeof(float) : sizeof(double));
    if (stage > 150 * 1024) {
        set_error("assign: dimension %d too large", d);
        return AVQ_EINVAL;
    }
    if (floats) {
        AVQ_HIP(hipFuncSetAttribute((const void *)nearest_kernel<false, float>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        hipLaunchKernelGGL((nearest_kernel<false, float>), dim3((unsigned)((n + bs - 1) / bs)), dim3(bs), stage, st,
                           x, n, d, 0, d, k, (const float *)nullptr, (const int32_t *)nullptr, centers,
                           (double *)nullptr, (unsigned long long *)nullptr, assign);
    } else {
        AVQ_HIP(hipFuncSetAttribute((const void *)nearest_kernel<false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        hipLaunchKernelGGL(nearest_kernel<false>, dim3((unsigned)((n + bs - 1) / bs)), dim3(bs), stage, st, x, n, d,
                           0, d, k, (const float *)nullptr, (const int32_t *)nullptr, centers, (double *)nullptr,
                           (unsigned long long *)nullptr, assign);
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// Definition 4.1's assignment step with the leaf centers as codewords: every point to the center of smallest
// anisotropic loss. With r = x - c: ||r||^2 = ||x||^2 - 2<c,x> + ||c||^2 and <r,x> = ||x||^2 - <c,x>, so the
// loss ||r||^2 + (eta - 1) <r,x>^2 / ||x||^2 (Section 3.2) needs <c,x> and ||c||^2 only; fp64. A workgroup
// holds 64 points in LDS; thread (point p, group g of 4) takes the centers j = g, g + 4, ...; lowest index
// on equal loss.
__global__ void __launch_bounds__(256)
assign_aniso_kernel(const float *__restrict__ x, int64_t n, int d, const float *__restrict__ centers, int k,
                    int eta_mode, double T, double eta_explicit, int32_t *__restrict__ assign)
{
    extern __shared__ double xs[]; // [64][d + 1], then best loss [4][64] and best index [4][64]
    const int ld = d + 1;
    double *best_loss = xs + (size_t)64 * ld;
    int *best_idx = (int *)(best_loss + 256);
    const int tid = threadIdx.x, p = tid & 63, g = tid >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * 64;
    for (int e = tid; e < 64 * d; e += 256) {
        const int pp = e / d, l = e - pp * d;
        xs[(size_t)pp * ld + l] = i0 + pp < n ? (double)x[(size_t)(i0 + pp) * d + l] : 0.0;
    }
    __syncthreads();
    const double *xp = xs + (size_t)p * ld;
    double nx2 = 0.0;
    for (int l = 0; l < d; ++l) nx2 += xp[l] * xp[l];
    const double eta = eta_of_norm(d, T, sqrt(nx2), eta_mode, eta_explicit);
    const double w = nx2 > 0.0 ? (eta - 1.0) / nx2 : 0.0;
    double bl = 0.0;
    int bi = -1;
    for (int j = g; j < k; j += 4) {
        const float *c = centers + (size_t)j * d;
        double cx = 0.0, cc = 0.0;
        for (int l = 0; l < d; ++l) {
            const double cv = (double)c[l];
            cx += cv * xp[l];
            cc += cv * cv;
        }
        const double rx = nx2 - cx;
        const double loss = (nx2 - 2.0 * cx + cc) + w * rx * rx;
        if (bi < 0 || loss < bl) { bl = loss; bi = j; }
    }
    best_loss[g * 64 + p] = bl;
    best_idx[g * 64 + p] = bi;
    __syncthreads();
    if (g == 0 && i0 + p < n) {
        for (int gg = 1; gg < 4; ++gg) {
            const double l2 = best_loss[gg * 64 + p];
            const int j2 = best_idx[gg * 64 + p];
            if (j2 >= 0 && (bi < 0 || l2 < bl || (l2 == bl && j2 < bi))) { bl = l2; bi = j2; }
        }
        assign[i0 + p] = bi;
    }
}

int launch_assign_aniso(const float *x, int64_t n, int d, const float *centers, int k, int eta_mode, double T,
                        double eta_explicit, int32_t *assign, hipStream_t st)
{
    const size_t lds = sizeof(double) * ((size_t)64 * (d + 1) + 256) + sizeof(int) * 256;
    if (lds > kMaxDynLds) { set_error("assign: dimension %d too large", d); return AVQ_EINVAL; }
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_lds_limit((const void *)assign_aniso_kernel, kMaxDynLds, &attr_done));
    hipLaunchKernelGGL(assign_aniso_kernel, dim3((unsigned)((n + 63) / 64)), dim3(256), lds, st, x, n, d, centers, k,
                       eta_mode, T, eta_explicit, assign);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- encoding under the anisotropic loss ------------------------------------------

constexpr int kMaxM = 256;

// One thread per point. With r = x - x~, p = <r, x>, e = ||r||^2:
// ||r_par||^2 = p^2/||x||^2 and ||r_perp||^2 = e - p^2/||x||^2, so the loss is
// e + (eta - 1) p^2 / ||x||^2. p and e are sums over subspaces; changing the
// codeword of subspace m only changes that subspace's terms, so the terms of the
// current codewords are kept per subspace and only summed again (every pass forms
// the sums before and after each subspace afresh from the kept terms: no drift).
// DS = dimensions per subspace known at compile time (0: any): the point's sub-vector of the
// subspace at hand then stays in registers while its kc codewords (wave-uniform, read through
// the scalar cache) pass by, instead of being read again for every codeword from a row that
// no neighbouring lane shares.
template <int DS>
__global__ void __launch_bounds__(128)
encode_kernel(const float *__restrict__ x, int64_t n, int d, int M, int kc, int bits,
              const float *__restrict__ codebooks, const float *__restrict__ leaf_centers,
              const int32_t *__restrict__ leaf_assign, int eta_mode, double T, double eta_explicit,
              int passes, uint8_t *__restrict__ packed)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int ds = DS ? DS : d / M;
    const float *xi = x + (size_t)i * d;
    const float *ce = leaf_centers ? leaf_centers + (size_t)leaf_assign[i] * d : nullptr;
    constexpr int kReg = DS ? DS : 1;
    double xv_m[kReg], xr_m[kReg]; // DS != 0: x^(m) and x^(m) - center^(m) of the subspace entered last
    uint8_t code[kMaxM];
    double pm_cur[kMaxM], em_cur[kMaxM]; // terms of the current codeword of every subspace
    double pm_after[kMaxM], em_after[kMaxM]; // their sums over the subspaces after m, as of the start of a pass

    double nx2 = 0.0;
    for (int l = 0; l < d; ++l) nx2 += (double)xi[l] * (double)xi[l];
    const double eta = eta_of_norm(d, T, sqrt(nx2), eta_mode, eta_explicit);
    const double w = nx2 > 0.0 ? (eta - 1.0) / nx2 : 0.0;

    // terms of subspace m for codeword j: pm = <r^(m), x^(m)>, em = ||r^(m)||^2 (fused multiply-adds: one
    // rounding per term instead of two, a third fewer fp64 operations per codeword)
    auto enter = [&](int m) {
        if constexpr (DS != 0) {
#pragma unroll
            for (int l = 0; l < DS; ++l) {
                xv_m[l] = (double)xi[m * DS + l];
                xr_m[l] = xv_m[l] - (ce ? (double)ce[m * DS + l] : 0.0);
            }
        }
    };
    auto terms = [&](int m, int j, double &pm, double &em) {
        const float *c = codebooks + ((size_t)m * kc + j) * ds;
        pm = 0.0;
        em = 0.0;
        if constexpr (DS != 0) {
#pragma unroll
            for (int l = 0; l < DS; ++l) {
                const double r = xr_m[l] - (double)c[l];
                pm = fma(r, xv_m[l], pm);
                em = fma(r, r, em);
            }
        } else {
            for (int l = 0; l < ds; ++l) {
                const double xv = (double)xi[m * ds + l];
                const double r = (xv - (ce ? (double)ce[m * ds + l] : 0.0)) - (double)c[l];
                pm = fma(r, xv, pm);
                em = fma(r, r, em);
            }
        }
    };

    // start: l2-nearest codeword of the (residual) sub-vector in every subspace
    for (int m = 0; m < M; ++m) {
        int best = 0;
        double bestd = INFINITY, bestp = 0.0;
        enter(m);
        for (int j = 0; j < kc; ++j) {
            double pm, em;
            terms(m, j, pm, em);
            if (em < bestd) { bestd = em; bestp = pm; best = j; }
        }
        code[m] = (uint8_t)best;
        pm_cur[m] = bestp;
        em_cur[m] = bestd;
    }
    for (int pass = 0; pass < passes; ++pass) {
        bool changed = false;
        // p and e of the other subspaces = the subspaces before m (running sums of this pass) + those after
        // it (sums formed here, from the last subspace down): M additions per pass instead of M per subspace
        double after_p = 0.0, after_e = 0.0;
        for (int m = M - 1; m >= 0; --m) {
            pm_after[m] = after_p;
            em_after[m] = after_e;
            after_p += pm_cur[m];
            after_e += em_cur[m];
        }
        double before_p = 0.0, before_e = 0.0;
        for (int m = 0; m < M; ++m) {
            const double Pr = before_p + pm_after[m], Er = before_e + em_after[m];
            int best = 0;
            double bestv = INFINITY, bestp = 0.0, beste = 0.0;
            enter(m);
            for (int j = 0; j < kc; ++j) {
                double pm, em;
                terms(m, j, pm, em);
                const double p = Pr + pm, e = Er + em;
                const double v = e + w * p * p;
                if (v < bestv) { bestv = v; best = j; bestp = pm; beste = em; }
            }
            if (best != code[m]) {
                code[m] = (uint8_t)best;
                pm_cur[m] = bestp;
                em_cur[m] = beste;
                changed = true;
            }
            before_p += pm_cur[m];
            before_e += em_cur[m];
        }
        if (!changed) break;
    }
    const int NB = (M * bits + 7) / 8;
    uint8_t *out = packed + (size_t)i * NB;
    if (bits == 8) {
        for (int m = 0; m < M; ++m) out[m] = code[m];
    } else {
        for (int b = 0; b < NB; ++b) {
            uint8_t v = code[2 * b] & 15;
            if (2 * b + 1 < M) v |= (uint8_t)((code[2 * b + 1] & 15) << 4);
            out[b] = v;
        }
    }
}

int launch_encode(const float *x, int64_t n, int d, int M, int kc, int bits,
                  const float *codebooks, const float *leaf_centers, const int32_t *leaf_assign,
                  int eta_mode, double T, double eta_explicit, int passes, uint8_t *packed,
                  hipStream_t st)
{
    if (M > kMaxM) { set_error("encode: M = %d exceeds %d", M, kMaxM); return AVQ_EINVAL; }
    if (M < 1 || d % M != 0) { set_error("encode: d = %d is not a multiple of M = %d", d, M); return AVQ_EINVAL; }
    const dim3 grid((unsigned)((n + 127) / 128)), block(128);
#define AVQ_ENCODE(DS)                                                                                        \
    hipLaunchKernelGGL(encode_kernel<DS>, grid, block, 0, st, x, n, d, M, kc, bits, codebooks, leaf_centers, \
                       leaf_assign, eta_mode, T, eta_explicit, passes, packed)
    switch (d / M) {
    case 2: AVQ_ENCODE(2); break;
    case 4: AVQ_ENCODE(4); break;
    case 8: AVQ_ENCODE(8); break;
    default: AVQ_ENCODE(0); break;
    }
#undef AVQ_ENCODE
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- joint dictionary update under the anisotropic loss ---------------------------------
//
// Section 4.2 alternates assignment and codeword update; with the codes fixed the loss is a
// convex quadratic in the stacked dictionaries c (D = M*kc*ds unknowns) and Appendix 7.5
// gives its normal equations
//     (sum_i B_i^T A_i B_i) c = sum_i h_par,i B_i^T x_i,
//     A_i = h_perp,i I + (h_par,i - h_perp,i) x_i x_i^T / ||x_i||^2,
// where B_i picks codeword code_i[m] of every dictionary m (x~_i = B_i c). With h_perp = 1,
// h_par = eta_i and s_i = B_i^T x_i (x_i's coordinates scattered to its codewords' slots):
//     A = diag(counts) + sum_i w_i s_i s_i^T,  w_i = (eta_i - 1)/||x_i||^2,  b = sum_i eta_i s_i.
// A is never formed: conjugate gradients need only v -> A v, one pass over the points with
// a gather of d values of v, a dot product and a scatter-add. Codewords no point uses keep
// their value (unit diagonal, right-hand side = old value). All in fp64.

// bits 32: one int32 per subspace (the leaf assignment seen as the code of a one-dictionary quantizer)
__device__ __forceinline__ int code_at(const uint8_t *row, int m, int bits)
{
    if (bits == 32) return ((const int32_t *)row)[m];
    return bits == 8 ? (int)row[m] : (int)((row[m >> 1] >> (4 * (m & 1))) & 15);
}

// One wave per point (grid-stride): w_i, counts, right-hand side and the rank-one part of A's diagonal.
__global__ void __launch_bounds__(256)
pq_update_setup_kernel(const float *__restrict__ x, int64_t n, int d, int M, int kc, int bits, int NB,
                       const uint8_t *__restrict__ codes, const float *__restrict__ centers,
                       const int32_t *__restrict__ assign, int eta_mode, double T, double eta_explicit,
                       double *__restrict__ w_out, double *__restrict__ eta_out, double *__restrict__ b,
                       double *__restrict__ dA, unsigned int *__restrict__ cnt)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int ds = d / M;
    for (int64_t i = wave0; i < n; i += n_waves) {
        const float *xi = x + (size_t)i * d;
        const uint8_t *ci = codes + (size_t)i * NB;
        // with leaf centers g: x~ = g + B c, the loss still against x; the right-hand side is B^T A (x - g),
        // A v = v + w x (x^T v); without, A x = eta x
        const float *gi = centers ? centers + (size_t)assign[i] * d : nullptr;
        double part = 0.0, xr = 0.0;
        for (int a = lane; a < d; a += 64) {
            part += (double)xi[a] * (double)xi[a];
            if (gi) xr += (double)xi[a] * ((double)xi[a] - (double)gi[a]);
        }
        for (int m = 32; m > 0; m >>= 1) { part += __shfl_xor(part, m, 64); xr += __shfl_xor(xr, m, 64); }
        const double nx2 = part;
        const double eta = eta_of_norm(d, T, sqrt(nx2), eta_mode, eta_explicit);
        const double wi = nx2 > 0.0 ? (eta - 1.0) / nx2 : 0.0;
        if (lane == 0) {
            w_out[i] = wi;
            eta_out[i] = eta;
        }
        for (int a = lane; a < d; a += 64) {
            const int m = a / ds;
            const int slot = m * kc + code_at(ci, m, bits);
            const double rhs = gi ? ((double)xi[a] - (double)gi[a]) + wi * xr * (double)xi[a] : eta * (double)xi[a];
            unsafeAtomicAdd(&b[(size_t)slot * ds + (a - m * ds)], rhs);
            if (wi != 0.0) unsafeAtomicAdd(&dA[(size_t)slot * ds + (a - m * ds)], wi * (double)xi[a] * (double)xi[a]);
            if (a == m * ds) atomicAdd(&cnt[slot], 1u);
        }
    }
}

// y += sum_i w_i s_i (s_i^T v). One wave per point. With use_lds the sum is accumulated per
// workgroup in LDS (D doubles) and added to y once per workgroup; otherwise (D too large for
// LDS) every term goes to y directly.
__global__ void __launch_bounds__(256)
pq_update_matvec_kernel(const float *__restrict__ x, int64_t n, int d, int M, int kc, int bits, int NB,
                        const uint8_t *__restrict__ codes, const double *__restrict__ w,
                        const double *__restrict__ v, double *__restrict__ y, int D, int use_lds)
{
    extern __shared__ double acc_lds[]; // [D] when use_lds
    double *acc = use_lds ? acc_lds : y;
    if (use_lds) {
        for (int r = threadIdx.x; r < D; r += blockDim.x) acc_lds[r] = 0.0;
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int ds = d / M;
    for (int64_t i = wave0; i < n; i += n_waves) {
        const float *xi = x + (size_t)i * d;
        const uint8_t *ci = codes + (size_t)i * NB;
        double t = 0.0;
        for (int a = lane; a < d; a += 64) {
            const int m = a / ds;
            const int r = (m * kc + code_at(ci, m, bits)) * ds + (a - m * ds);
            t += (double)xi[a] * v[r];
        }
        for (int m = 32; m > 0; m >>= 1) t += __shfl_xor(t, m, 64);
        const double wt = w[i] * t;
        if (wt != 0.0) {
            for (int a = lane; a < d; a += 64) {
                const int m = a / ds;
                const int r = (m * kc + code_at(ci, m, bits)) * ds + (a - m * ds);
                if (use_lds) atomicAdd(&acc_lds[r], wt * (double)xi[a]);
                else unsafeAtomicAdd(&acc[r], wt * (double)xi[a]);
            }
        }
    }
    if (!use_lds) return;
    __syncthreads();
    for (int r = threadIdx.x; r < D; r += blockDim.x)
        if (acc_lds[r] != 0.0) unsafeAtomicAdd(&y[r], acc_lds[r]);
}

// Conjugate gradients with the diagonal of A as preconditioner (exact in one step when every
// eta_i = 1, where A is diagonal). state[0] = r.z, state[1] = b.b, state[2] = iterations done,
// state[3] = r.r. One workgroup.
// mode 0 (start, after y = A c0 is complete): r = b - y, z = r/dA, p = z, y = diag(count) * p.
// mode 1 (step, after y = A p is complete): the usual update, then y = diag(count) * p for the next product.
__global__ void __launch_bounds__(1024)
pq_update_cg_kernel(int mode, int D, int ds, const unsigned int *__restrict__ cnt, const double *__restrict__ b,
                    const double *__restrict__ dA, double *__restrict__ c, double *__restrict__ r,
                    double *__restrict__ p, double *__restrict__ y, double *__restrict__ state, double tol2)
{
    __shared__ double red[1024];
    const int tid = threadIdx.x, nt = blockDim.x;
    auto reduce = [&](double v) -> double {
        red[tid] = v;
        __syncthreads();
        for (int s = nt >> 1; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        const double out = red[0];
        __syncthreads();
        return out;
    };
    auto diag = [&](int e) -> double { const unsigned int k = cnt[e / ds]; return k ? (double)k : 1.0; };
    if (mode == 0) {
        double rz = 0.0, rr = 0.0, bb = 0.0;
        for (int e = tid; e < D; e += nt) {
            const double re = b[e] - y[e];
            const double ze = re / dA[e];
            r[e] = re;
            p[e] = ze;
            rz += re * ze;
            rr += re * re;
            bb += b[e] * b[e];
        }
        rz = reduce(rz);
        rr = reduce(rr);
        bb = reduce(bb);
        for (int e = tid; e < D; e += nt) y[e] = diag(e) * p[e];
        if (tid == 0) { state[0] = rz; state[1] = bb; state[2] = 0.0; state[3] = rr; }
        return;
    }
    const double rz = state[0];
    if (rz == 0.0 || state[3] <= tol2 * state[1]) return; // converged: later steps of a burst do nothing
    double pap = 0.0;
    for (int e = tid; e < D; e += nt) pap += p[e] * y[e];
    pap = reduce(pap);
    const double alpha = rz / pap;
    double rz2 = 0.0, rr2 = 0.0;
    for (int e = tid; e < D; e += nt) {
        c[e] += alpha * p[e];
        const double re = r[e] - alpha * y[e];
        r[e] = re;
        rz2 += re * re / dA[e];
        rr2 += re * re;
    }
    rz2 = reduce(rz2);
    rr2 = reduce(rr2);
    const double beta = rz2 / rz;
    for (int e = tid; e < D; e += nt) {
        const double pe = r[e] / dA[e] + beta * p[e];
        p[e] = pe;
        y[e] = diag(e) * pe;
    }
    if (tid == 0) { state[0] = rz2; state[2] += 1.0; state[3] = rr2; }
}

// c0 (the current dictionaries, as doubles), the right-hand side of unused codewords,
// y = diag(count) * c0, and the counts added to A's diagonal
__global__ void pq_update_init_kernel(int D, int ds, const unsigned int *__restrict__ cnt,
                                      const float *__restrict__ codebooks, double *__restrict__ c,
                                      double *__restrict__ b, double *__restrict__ y, double *__restrict__ dA)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= D) return;
    const double c0 = (double)codebooks[e];
    c[e] = c0;
    const unsigned int k = cnt[e / ds];
    if (k == 0u) b[e] = c0;
    y[e] = (k ? (double)k : 1.0) * c0;
    dA[e] += k ? (double)k : 1.0;
}

__global__ void pq_update_store_kernel(int D, const double *__restrict__ c, float *__restrict__ codebooks)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < D) codebooks[e] = (float)c[e];
}

// scratch: doubles w[n], eta[n], then b, c, r, p, y, dA of D each, state[4]; then cnt[M*kc] unsigned
size_t pq_update_scratch_bytes(int64_t n, int D, int slots)
{
    return sizeof(double) * ((size_t)2 * n + (size_t)6 * D + 4) + sizeof(unsigned int) * (size_t)slots;
}

int pq_joint_update_device(const float *x, int64_t n, int d, int M, int kc, int bits, const uint8_t *codes,
                           const float *centers, const int32_t *assign,
                           int eta_mode, double T, double eta_explicit, float *codebooks, void *scratch,
                           int max_iters, double tol, int *iters_out, double *rel_residual_out, hipStream_t st)
{
    const int ds = d / M, D = M * kc * ds, slots = M * kc, NB = (M * bits + 7) / 8;
    const int use_lds = (size_t)D * sizeof(double) <= 64 * 1024;
    double *w = (double *)scratch, *eta = w + n, *b = eta + n, *c = b + D, *r = c + D, *p = r + D, *y = p + D, *dA = y + D;
    double *state = dA + D;
    unsigned int *cnt = (unsigned int *)(state + 4);
    AVQ_HIP(hipMemsetAsync(b, 0, sizeof(double) * ((size_t)6 * D + 4) + sizeof(unsigned int) * (size_t)slots, st));
    const int grid = (int)std::min<int64_t>(1024, (n + 3) / 4);
    hipLaunchKernelGGL(pq_update_setup_kernel, dim3(grid), dim3(256), 0, st, x, n, d, M, kc, bits, NB, codes,
                       centers, assign, eta_mode, T, eta_explicit, w, eta, b, dA, cnt);
    AVQ_HIP(hipGetLastError());
    const int vgrid = (D + 255) / 256;
    hipLaunchKernelGGL(pq_update_init_kernel, dim3(vgrid), dim3(256), 0, st, D, ds, cnt, codebooks, c, b, y, dA);
    AVQ_HIP(hipGetLastError());
    const size_t lds = use_lds ? sizeof(double) * (size_t)D : 0;
    static LdsLimitOnce attr_done;
    AVQ_TRY(set_lds_limit((const void *)pq_update_matvec_kernel, 64 * 1024, &attr_done));
    // y = A c0
    hipLaunchKernelGGL(pq_update_matvec_kernel, dim3(grid), dim3(256), lds, st, x, n, d, M, kc, bits, NB, codes, w, c, y, D, use_lds);
    AVQ_HIP(hipGetLastError());
    hipLaunchKernelGGL(pq_update_cg_kernel, dim3(1), dim3(1024), 0, st, 0, D, ds, cnt, b, dA, c, r, p, y, state, tol * tol);
    AVQ_HIP(hipGetLastError());
    double host_state[4] = {0, 0, 0, 0};
    int done = 0;
    const int check_every = 16;
    while (done < max_iters) {
        const int burst = std::min(check_every, max_iters - done);
        for (int it = 0; it < burst; ++it) {
            hipLaunchKernelGGL(pq_update_matvec_kernel, dim3(grid), dim3(256), lds, st, x, n, d, M, kc, bits, NB, codes, w, p, y, D, use_lds);
            hipLaunchKernelGGL(pq_update_cg_kernel, dim3(1), dim3(1024), 0, st, 1, D, ds, cnt, b, dA, c, r, p, y, state, tol * tol);
        }
        AVQ_HIP(hipGetLastError());
        done += burst;
        AVQ_HIP(hipMemcpyAsync(host_state, state, sizeof(host_state), hipMemcpyDeviceToHost, st));
        AVQ_HIP(hipStreamSynchronize(st));
        if (host_state[1] == 0.0 || host_state[3] <= tol * tol * host_state[1]) break;
    }
    hipLaunchKernelGGL(pq_update_store_kernel, dim3(vgrid), dim3(256), 0, st, D, c, codebooks);
    AVQ_HIP(hipGetLastError());
    if (iters_out) *iters_out = (int)host_state[2];
    if (rel_residual_out) *rel_residual_out = host_state[1] > 0.0 ? sqrt(host_state[3] / host_state[1]) : 0.0;
    return AVQ_OK;
}

} // namespace avq
