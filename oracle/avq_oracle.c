/*
 * avq_oracle.c -- plain CPU reference for anisotropic (score-aware) product
 * quantization and the query-time asymmetric-distance (ADC) search path.
 *
 * THIS IS TEST INFRASTRUCTURE. It exists so that the GPU library can be
 * checked against something slow and obviously right. Nothing in the product
 * path may include, link or call it. It shares no code with the GPU path.
 *
 * Every function follows a passage of the paper "Accelerating Large-Scale
 * Inference with Anisotropic Vector Quantization" (arXiv 1908.10396); the
 * passage is named above each function. Where the paper is silent the reading
 * taken is stated in the comment.
 *
 * Precision: everything that the paper leaves as real arithmetic (eta, the
 * residual decomposition, the loss, k-means, encoding) is fp64. The query path
 * is fp32 because its definition fixes fp32 (fp32 tables, fp32 re-ranking) and
 * because float decisions (the 8-bit table codes, the top-k) have to be taken
 * in the same precision and operation order by both sides. That order is
 * written out with explicit fmaf/+ and the file is compiled with
 * -ffp-contract=off so the compiler cannot fuse or reorder it.
 *
 * Parity pins (see tests/test_oracle_*.py): eta against numerical quadrature,
 * the printed eta = 4.125, the T = 0 special case; the decomposition against
 * orthogonality identities, the quadratic form of the proof of Theorem 4.2 and
 * a Monte-Carlo estimate of Definition 3.1; encoding against exhaustive
 * enumeration and the eta = 1 reduction; tables and ADC against <q, x~> with
 * x~ rebuilt from the codes; top-k against a full stable sort; search with
 * reorder_k = n against brute-force MIPS. Unpinned: recall figures (the
 * paper's datasets are not available) -- "parity unpinned" for those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOMEM (-3)

/* ------------------------------------------------------------------------ */
/* eta                                                                      */
/* ------------------------------------------------------------------------ */

/* Ratio clamp: T >= ||x|| makes eta infinite (Section 3.2, special cases).
 * Reading: (T/||x||)^2 is clamped to 0.999 so eta stays finite. */
static double clamp_u(double T, double norm)
{
    double u = (T / norm) * (T / norm);
    return u > 0.999 ? 0.999 : u;
}

/* Theorem 3.4 / Eq. 3 used as a proxy for eta (Section 3.2):
 * eta = (d-1) u / (1-u), u = (T/||x||)^2.
 * Reading: Theorem 3.3 requires eta >= 1 and the T = 0 special case must give
 * eta = 1, so the proxy is floored at 1. ||x|| = 0 has no direction: eta = 1. */
double orc_eta_limit(int d, double T, double norm)
{
    if (norm <= 0.0) return 1.0;
    double u = clamp_u(T, norm);
    double eta = (double)(d - 1) * u / (1.0 - u);
    return eta < 1.0 ? 1.0 : eta;
}

/* I_d(alpha) = int_0^alpha sin^d(theta) d theta by composite Simpson with a
 * fixed, fine panel count (the integrand is smooth; 16384 panels resolve the
 * peak of sin^d for every d used here to better than 1e-10). */
double orc_sin_power_integral(int d, double alpha)
{
    const int N = 16384; /* even */
    double h = alpha / N;
    double s = pow(sin(0.0), (double)d) + pow(sin(alpha), (double)d);
    if (d == 0) s = 2.0;
    for (int i = 1; i < N; ++i) {
        double f = d == 0 ? 1.0 : pow(sin(i * h), (double)d);
        s += (i & 1) ? 4.0 * f : 2.0 * f;
    }
    return s * h / 3.0;
}

/* Exact ratio h_par / h_perp for w(t) = I(t >= T), Section 3.2:
 * h_par = (d-1) int_0^alpha (sin^{d-2} - sin^d), h_perp = int_0^alpha sin^d,
 * alpha = arccos(T/||x||); so eta = (d-1) (I_{d-2}/I_d - 1). The integrals are
 * evaluated directly: the paper's recursion
 * d I_d = (d-1) I_{d-2} - cos(alpha) sin^{d-1}(alpha) run upwards multiplies
 * rounding error by 1/sin^2(alpha) per step and loses all digits for larger
 * T/||x||; the tests check that the integrals satisfy it. */
double orc_eta_exact(int d, double T, double norm)
{
    if (norm <= 0.0 || d < 2) return 1.0;
    double ca = sqrt(clamp_u(T, norm));
    if (T < 0) ca = -ca;
    double alpha = acos(ca);
    double Id = orc_sin_power_integral(d, alpha);
    double Idm2 = orc_sin_power_integral(d - 2, alpha);
    return (double)(d - 1) * (Idm2 / Id - 1.0);
}

/* mode 0: limit proxy, 1: exact ratio, 2: explicit constant. */
double orc_eta(int mode, int d, double T, double norm, double eta_explicit)
{
    if (mode == 2) return eta_explicit;
    if (mode == 1) return orc_eta_exact(d, T, norm);
    return orc_eta_limit(d, T, norm);
}

/* ------------------------------------------------------------------------ */
/* residual decomposition and loss                                          */
/* ------------------------------------------------------------------------ */

/* Section 3.1: r_par = <x - x~, x> x / ||x||^2,  r_perp = (x - x~) - r_par.
 * ||x|| = 0: r_par = 0. */
void orc_residual_decompose(const double *x, const double *xt, int d,
                            double *r_par, double *r_perp)
{
    double nx2 = 0.0, p = 0.0;
    for (int l = 0; l < d; ++l) {
        nx2 += x[l] * x[l];
        p += (x[l] - xt[l]) * x[l];
    }
    double c = nx2 > 0.0 ? p / nx2 : 0.0;
    for (int l = 0; l < d; ++l) {
        r_par[l] = c * x[l];
        r_perp[l] = (x[l] - xt[l]) - r_par[l];
    }
}

/* Section 3.2: loss proportional to eta ||r_par||^2 + ||r_perp||^2, evaluated
 * from the two vectors themselves. scratch holds 2*d doubles. */
static double aniso_loss_ws(const double *x, const double *xt, int d, double eta,
                            double *scratch)
{
    double *rp = scratch, *ro = scratch + d;
    orc_residual_decompose(x, xt, d, rp, ro);
    double a = 0.0, b = 0.0;
    for (int l = 0; l < d; ++l) {
        a += rp[l] * rp[l];
        b += ro[l] * ro[l];
    }
    return eta * a + b;
}

double orc_aniso_loss(const double *x, const double *xt, int d, double eta)
{
    double *ws = (double *)malloc(sizeof(double) * 2 * (size_t)d);
    double v = aniso_loss_ws(x, xt, d, eta, ws);
    free(ws);
    return v;
}

/* ------------------------------------------------------------------------ */
/* counter-based index generator for initial codewords                      */
/* ------------------------------------------------------------------------ */

/* splitmix64 output function (Steele, Lea, Flood 2014) applied to a counter. */
static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Section 4, initialization step: codewords start as datapoints drawn from the
 * data. Reading: codeword j of stream s is drawn from the j-th of k equal
 * strata of the n points, at offset mix64(seed, s, j) mod stratum length, so
 * the k indices are distinct. Requires n >= k. */
int64_t orc_init_index(uint64_t seed, uint32_t stream, int j, int k, int64_t n)
{
    int64_t lo = (int64_t)(((__int128)j * n) / k);
    int64_t hi = (int64_t)(((__int128)(j + 1) * n) / k);
    uint64_t h = mix64(seed ^ mix64(((uint64_t)stream << 32) | (uint32_t)j));
    return lo + (int64_t)(h % (uint64_t)(hi - lo));
}

/* ------------------------------------------------------------------------ */
/* k-means (Lloyd) -- the l2 dictionary of Section 4 / Section 5.1          */
/* ------------------------------------------------------------------------ */

/* nearest center in squared l2, fp64, ties to the lowest index.
 * v: dim values with stride 1; optional `sub` is subtracted first. */
static int nearest_center(const float *v, const float *sub, const float *centers,
                          int k, int dim)
{
    int best = 0;
    double bestd = INFINITY;
    for (int j = 0; j < k; ++j) {
        double dd = 0.0;
        for (int l = 0; l < dim; ++l) {
            double a = (double)v[l] - (sub ? (double)sub[l] : 0.0);
            double t = a - (double)centers[(size_t)j * dim + l];
            dd += t * t;
        }
        if (dd < bestd) { bestd = dd; best = j; }
    }
    return best;
}

/* Lloyd's algorithm on columns [col0, col0+dim) of x (row stride ld).
 * If resid_centers != NULL the vector clustered is
 * x_i[col0..] - resid_centers[resid_assign[i]][col0..] (row stride ld).
 * Fixed iteration count (reading of "until convergence or a maximum number
 * of iterations"); an empty cluster keeps its previous center. Centers are
 * stored as fp32 after every update. */
int orc_kmeans(const float *x, int64_t n, int ld, int col0, int dim, int k, int iters,
               uint64_t seed, uint32_t stream, const float *resid_centers,
               const int32_t *resid_assign, float *centers)
{
    if (n < k || k < 1 || dim < 1) return ORC_EINVAL;
    for (int j = 0; j < k; ++j) {
        int64_t i = orc_init_index(seed, stream, j, k, n);
        for (int l = 0; l < dim; ++l) {
            double v = (double)x[(size_t)i * ld + col0 + l];
            if (resid_centers)
                v -= (double)resid_centers[(size_t)resid_assign[i] * ld + col0 + l];
            centers[(size_t)j * dim + l] = (float)v;
        }
    }
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    double *sum = (double *)malloc(sizeof(double) * (size_t)k * dim);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    if (!assign || !sum || !cnt) { free(assign); free(sum); free(cnt); return ORC_ENOMEM; }
    for (int it = 0; it < iters; ++it) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            const float *sub = resid_centers
                ? resid_centers + (size_t)resid_assign[i] * ld + col0 : NULL;
            assign[i] = nearest_center(x + (size_t)i * ld + col0, sub, centers, k, dim);
        }
        memset(sum, 0, sizeof(double) * (size_t)k * dim);
        memset(cnt, 0, sizeof(int64_t) * (size_t)k);
        for (int64_t i = 0; i < n; ++i) {
            int j = assign[i];
            cnt[j]++;
            for (int l = 0; l < dim; ++l) {
                double v = (double)x[(size_t)i * ld + col0 + l];
                if (resid_centers)
                    v -= (double)resid_centers[(size_t)resid_assign[i] * ld + col0 + l];
                sum[(size_t)j * dim + l] += v;
            }
        }
        for (int j = 0; j < k; ++j)
            if (cnt[j] > 0)
                for (int l = 0; l < dim; ++l)
                    centers[(size_t)j * dim + l] = (float)(sum[(size_t)j * dim + l] / (double)cnt[j]);
    }
    free(assign); free(sum); free(cnt);
    return ORC_OK;
}

/* l2-nearest center for every row (leaf assignment of the partitioning tree,
 * Section 5.3; reading: plain nearest center). */
void orc_assign_nearest(const float *x, int64_t n, int d, const float *centers, int k,
                        int32_t *assign)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        assign[i] = nearest_center(x + (size_t)i * d, NULL, centers, k, d);
}

/* PQ dictionaries by k-means per subspace (Section 4.1 with the l2-trained
 * dictionary of Section 5.1): codebooks[M][kc][ds]. */
int orc_train_pq(const float *x, int64_t n, int d, int M, int kc, int iters, uint64_t seed,
                 const float *leaf_centers, const int32_t *leaf_assign, float *codebooks)
{
    if (M < 1 || d % M != 0) return ORC_EINVAL;
    int ds = d / M;
    for (int m = 0; m < M; ++m) {
        int rc = orc_kmeans(x, n, d, m * ds, ds, kc, iters, seed, (uint32_t)(1 + m),
                            leaf_centers, leaf_assign,
                            codebooks + (size_t)m * kc * ds);
        if (rc) return rc;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* encoding under the anisotropic loss (Section 4.1, assignment step)       */
/* ------------------------------------------------------------------------ */

static double norm_d(const float *x, int d)
{
    double s = 0.0;
    for (int l = 0; l < d; ++l) s += (double)x[l] * (double)x[l];
    return sqrt(s);
}

/* Quantized point for a code vector: x~ = center + concatenated codewords. */
static void reconstruct(const uint8_t *code, const float *codebooks, const float *center,
                        int d, int M, int kc, double *xt)
{
    int ds = d / M;
    for (int m = 0; m < M; ++m)
        for (int l = 0; l < ds; ++l)
            xt[m * ds + l] = (center ? (double)center[m * ds + l] : 0.0) +
                             (double)codebooks[((size_t)m * kc + code[m]) * ds + l];
}

void orc_reconstruct(const uint8_t *codes, int64_t n, const float *codebooks,
                     const float *centers, const int32_t *assign, int d, int M, int kc,
                     double *xt)
{
    for (int64_t i = 0; i < n; ++i)
        reconstruct(codes + (size_t)i * M, codebooks,
                    centers ? centers + (size_t)assign[i] * d : NULL, d, M, kc,
                    xt + (size_t)i * d);
}

/* One datapoint. Reading of the one-sentence assignment step: start from the
 * l2-nearest codeword in every subspace; then cyclic coordinate descent over
 * the subspaces m = 0..M-1, replacing code m by the codeword that minimises
 * the full-vector loss with the other subspaces fixed (equal losses go to the
 * lowest codeword index); stop after a pass without change or after `passes`
 * passes. The loss is always taken against the original x. */
static void encode_point(const float *x, const float *center, const float *codebooks,
                         int d, int M, int kc, double eta, int passes, uint8_t *code,
                         double *ws /* 4*d doubles */)
{
    int ds = d / M;
    double *xd = ws, *xt = ws + d, *scr = ws + 2 * d;
    for (int l = 0; l < d; ++l) xd[l] = (double)x[l];
    for (int m = 0; m < M; ++m)
        code[m] = (uint8_t)nearest_center(x + m * ds, center ? center + m * ds : NULL,
                                          codebooks + (size_t)m * kc * ds, kc, ds);
    reconstruct(code, codebooks, center, d, M, kc, xt);
    for (int pass = 0; pass < passes; ++pass) {
        int changed = 0;
        for (int m = 0; m < M; ++m) {
            int best = 0;
            double bestv = INFINITY;
            for (int j = 0; j < kc; ++j) {
                for (int l = 0; l < ds; ++l)
                    xt[m * ds + l] = (center ? (double)center[m * ds + l] : 0.0) +
                                     (double)codebooks[((size_t)m * kc + j) * ds + l];
                double v = aniso_loss_ws(xd, xt, d, eta, scr);
                if (v < bestv) { bestv = v; best = j; }
            }
            if (best != code[m]) { code[m] = (uint8_t)best; changed = 1; }
            for (int l = 0; l < ds; ++l)
                xt[m * ds + l] = (center ? (double)center[m * ds + l] : 0.0) +
                                 (double)codebooks[((size_t)m * kc + code[m]) * ds + l];
        }
        if (!changed) break;
    }
}

/* codes[n][M] (one byte per subspace). eta per point from its own norm
 * (Theorem 3.2 weights depend on ||x_i||) unless eta_mode == 2. */
int orc_encode(const float *x, int64_t n, int d, int M, int kc, const float *codebooks,
               const float *leaf_centers, const int32_t *leaf_assign, int eta_mode, double T,
               double eta_explicit, int passes, uint8_t *codes)
{
    if (M < 1 || d % M != 0 || kc > 256) return ORC_EINVAL;
#pragma omp parallel
    {
        double *ws = (double *)malloc(sizeof(double) * 4 * (size_t)d);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            const float *xi = x + (size_t)i * d;
            double eta = orc_eta(eta_mode, d, T, norm_d(xi, d), eta_explicit);
            encode_point(xi, leaf_centers ? leaf_centers + (size_t)leaf_assign[i] * d : NULL,
                         codebooks, d, M, kc, eta, passes, codes + (size_t)i * M, ws);
        }
        free(ws);
    }
    return ORC_OK;
}

/* Exhaustive minimiser over all kc^M code vectors (Definition 4.3's inner
 * min written out); only for tiny M. First minimiser in lexicographic order
 * with code[0] the slowest digit. Returns the minimum loss. */
double orc_encode_exhaustive(const float *x, const float *center, int d, int M, int kc,
                             const float *codebooks, double eta, uint8_t *code_out)
{
    double *ws = (double *)malloc(sizeof(double) * 4 * (size_t)d);
    double *xd = ws, *xt = ws + d, *scr = ws + 2 * d;
    uint8_t *code = (uint8_t *)calloc((size_t)M, 1);
    for (int l = 0; l < d; ++l) xd[l] = (double)x[l];
    double bestv = INFINITY;
    for (;;) {
        reconstruct(code, codebooks, center, d, M, kc, xt);
        double v = aniso_loss_ws(xd, xt, d, eta, scr);
        if (v < bestv) { bestv = v; memcpy(code_out, code, (size_t)M); }
        int m = M - 1;
        while (m >= 0 && ++code[m] == kc) { code[m] = 0; --m; }
        if (m < 0) break;
    }
    free(ws); free(code);
    return bestv;
}

/* Logical packed layout handed to the library: bits = 8 -> byte m is code m;
 * bits = 4 -> byte m/2 holds code m, even m in the low nibble. */
void orc_pack_codes(const uint8_t *codes, int64_t n, int M, int bits, uint8_t *packed)
{
    int bpp = (M * bits + 7) / 8;
    memset(packed, 0, (size_t)n * bpp);
    for (int64_t i = 0; i < n; ++i)
        for (int m = 0; m < M; ++m) {
            uint8_t c = codes[(size_t)i * M + m];
            if (bits == 8) packed[(size_t)i * bpp + m] = c;
            else packed[(size_t)i * bpp + m / 2] |= (uint8_t)((c & 15) << (4 * (m & 1)));
        }
}

/* ------------------------------------------------------------------------ */
/* closed-form codeword update (Theorem 4.2)                                */
/* ------------------------------------------------------------------------ */

/* Solve A y = b for symmetric positive definite A (dim x dim, row-major,
 * overwritten) by Cholesky. Returns nonzero if not positive definite. */
static int spd_solve(double *A, double *b, int dim)
{
    for (int i = 0; i < dim; ++i) {
        for (int j = 0; j <= i; ++j) {
            double s = A[(size_t)i * dim + j];
            for (int t = 0; t < j; ++t) s -= A[(size_t)i * dim + t] * A[(size_t)j * dim + t];
            if (i == j) {
                if (s <= 0.0) return 1;
                A[(size_t)i * dim + i] = sqrt(s);
            } else {
                A[(size_t)i * dim + j] = s / A[(size_t)j * dim + j];
            }
        }
    }
    for (int i = 0; i < dim; ++i) {
        double s = b[i];
        for (int t = 0; t < i; ++t) s -= A[(size_t)i * dim + t] * b[t];
        b[i] = s / A[(size_t)i * dim + i];
    }
    for (int i = dim - 1; i >= 0; --i) {
        double s = b[i];
        for (int t = i + 1; t < dim; ++t) s -= A[(size_t)t * dim + i] * b[t];
        b[i] = s / A[(size_t)i * dim + i];
    }
    return 0;
}

/* Theorem 4.2: c* = (I sum h_perp + sum (h_par-h_perp)/||x||^2 x x^T)^-1
 * sum h_par x over the members of one partition. h_par[i], h_perp[i] are the
 * per-point weights (only their ratio eta matters for the loss's argmin, but
 * the update uses both). x: members[cnt][d] in fp64. */
int orc_vq_update(const double *x, int64_t cnt, int d, const double *h_par,
                  const double *h_perp, double *c_out)
{
    double *A = (double *)calloc((size_t)d * d, sizeof(double));
    if (!A) return ORC_ENOMEM;
    for (int l = 0; l < d; ++l) c_out[l] = 0.0;
    for (int64_t i = 0; i < cnt; ++i) {
        const double *xi = x + (size_t)i * d;
        double nx2 = 0.0;
        for (int l = 0; l < d; ++l) nx2 += xi[l] * xi[l];
        double w = nx2 > 0.0 ? (h_par[i] - h_perp[i]) / nx2 : 0.0;
        for (int a = 0; a < d; ++a) {
            A[(size_t)a * d + a] += h_perp[i];
            for (int b = 0; b < d; ++b) A[(size_t)a * d + b] += w * xi[a] * xi[b];
            c_out[a] += h_par[i] * xi[a];
        }
    }
    int rc = spd_solve(A, c_out, d);
    free(A);
    return rc ? ORC_EINVAL : ORC_OK;
}

/* Appendix 7.5: joint update of all PQ codewords with the partitions fixed.
 * c in R^{M kc ds} stacks the dictionaries; x~_i = B_i c where B_i selects
 * codeword code_i[m] of every dictionary m. Normal equations
 * (sum B_i^T A_i B_i) c = sum h_par B_i^T x_i with
 * A_i = (h_par-h_perp) x x^T/||x||^2 + h_perp I (the right-hand side is read
 * as B_i^T x_i, the only dimensionally consistent form). Codewords that no
 * point uses keep their old value (their rows are replaced by identity).
 * Dense solve: only for small M*kc*ds. Here h_perp = 1, h_par = eta_i. */
int orc_pq_joint_update(const float *x, int64_t n, int d, int M, int kc,
                        const uint8_t *codes, const double *eta, float *codebooks)
{
    int ds = d / M;
    int D = M * kc * ds;
    double *A = (double *)calloc((size_t)D * D, sizeof(double));
    double *b = (double *)calloc((size_t)D, sizeof(double));
    int *col = (int *)malloc(sizeof(int) * (size_t)d);
    char *used = (char *)calloc((size_t)M * kc, 1);
    if (!A || !b || !col || !used) { free(A); free(b); free(col); free(used); return ORC_ENOMEM; }
    for (int64_t i = 0; i < n; ++i) {
        const float *xi = x + (size_t)i * d;
        double nx2 = 0.0;
        for (int l = 0; l < d; ++l) nx2 += (double)xi[l] * (double)xi[l];
        double w = nx2 > 0.0 ? (eta[i] - 1.0) / nx2 : 0.0;
        for (int m = 0; m < M; ++m) {
            used[m * kc + codes[(size_t)i * M + m]] = 1;
            for (int l = 0; l < ds; ++l)
                col[m * ds + l] = (m * kc + codes[(size_t)i * M + m]) * ds + l;
        }
        for (int a = 0; a < d; ++a) {
            A[(size_t)col[a] * D + col[a]] += 1.0;
            for (int c = 0; c < d; ++c)
                A[(size_t)col[a] * D + col[c]] += w * (double)xi[a] * (double)xi[c];
            b[col[a]] += eta[i] * (double)xi[a];
        }
    }
    for (int mj = 0; mj < M * kc; ++mj)
        if (!used[mj])
            for (int l = 0; l < ds; ++l) {
                int r = mj * ds + l;
                A[(size_t)r * D + r] = 1.0;
                b[r] = (double)codebooks[r];
            }
    int rc = spd_solve(A, b, D);
    if (!rc)
        for (int r = 0; r < D; ++r) codebooks[r] = (float)b[r];
    free(A); free(b); free(col); free(used);
    return rc ? ORC_EINVAL : ORC_OK;
}

/* Appendix 7.5 for a partitioned index: x~_i = center(leaf(i)) + B_i c, the
 * loss still taken against the original x_i (its direction and norm define
 * A_i). Minimising sum_i (x_i - g_i - B_i c)^T A_i (x_i - g_i - B_i c) over c,
 * g_i the point's leaf center, gives the same matrix as the flat case and the
 * right-hand side sum_i B_i^T A_i (x_i - g_i) with
 * A_i v = v + w_i x_i (x_i^T v), w_i = (eta_i - 1)/||x_i||^2. centers == NULL:
 * g_i = 0, the flat case (A_i x_i = eta_i x_i). */
int orc_pq_joint_update_resid(const float *x, int64_t n, int d, int M, int kc,
                              const uint8_t *codes, const double *eta, const float *centers,
                              const int32_t *assign, float *codebooks)
{
    int ds = d / M;
    int D = M * kc * ds;
    double *A = (double *)calloc((size_t)D * D, sizeof(double));
    double *b = (double *)calloc((size_t)D, sizeof(double));
    double *r = (double *)malloc(sizeof(double) * (size_t)d);
    int *col = (int *)malloc(sizeof(int) * (size_t)d);
    char *used = (char *)calloc((size_t)M * kc, 1);
    if (!A || !b || !r || !col || !used) { free(A); free(b); free(r); free(col); free(used); return ORC_ENOMEM; }
    for (int64_t i = 0; i < n; ++i) {
        const float *xi = x + (size_t)i * d;
        double nx2 = 0.0, xr = 0.0;
        for (int l = 0; l < d; ++l) {
            double g = centers ? (double)centers[(size_t)assign[i] * d + l] : 0.0;
            r[l] = (double)xi[l] - g;
            nx2 += (double)xi[l] * (double)xi[l];
            xr += (double)xi[l] * r[l];
        }
        double w = nx2 > 0.0 ? (eta[i] - 1.0) / nx2 : 0.0;
        for (int m = 0; m < M; ++m) {
            used[m * kc + codes[(size_t)i * M + m]] = 1;
            for (int l = 0; l < ds; ++l)
                col[m * ds + l] = (m * kc + codes[(size_t)i * M + m]) * ds + l;
        }
        for (int a = 0; a < d; ++a) {
            A[(size_t)col[a] * D + col[a]] += 1.0;
            for (int c = 0; c < d; ++c)
                A[(size_t)col[a] * D + col[c]] += w * (double)xi[a] * (double)xi[c];
            b[col[a]] += r[a] + w * xr * (double)xi[a];
        }
    }
    for (int mj = 0; mj < M * kc; ++mj)
        if (!used[mj])
            for (int l = 0; l < ds; ++l) {
                int rr = mj * ds + l;
                A[(size_t)rr * D + rr] = 1.0;
                b[rr] = (double)codebooks[rr];
            }
    int rc = spd_solve(A, b, D);
    if (!rc)
        for (int rr = 0; rr < D; ++rr) codebooks[rr] = (float)b[rr];
    free(A); free(b); free(r); free(col); free(used);
    return rc ? ORC_EINVAL : ORC_OK;
}

/* Definition 4.1's partition-assignment step for a vector quantizer whose
 * codewords are the leaf centers: every row goes to the center with the
 * smallest anisotropic loss eta*||r_par||^2 + ||r_perp||^2, r = x - center
 * (Section 3.2), lowest index on equal loss; eta per point from its own norm. */
void orc_assign_aniso(const float *x, int64_t n, int d, const float *centers, int k,
                      int eta_mode, double T, double eta_explicit, int32_t *assign)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *xd = (double *)malloc(sizeof(double) * 4 * (size_t)d);
        double *cd = xd + d, *ws = cd + d;
        const float *xi = x + (size_t)i * d;
        for (int l = 0; l < d; ++l) xd[l] = (double)xi[l];
        double eta = orc_eta(eta_mode, d, T, norm_d(xi, d), eta_explicit);
        int best = 0;
        double best_loss = 0.0;
        for (int j = 0; j < k; ++j) {
            for (int l = 0; l < d; ++l) cd[l] = (double)centers[(size_t)j * d + l];
            double v = aniso_loss_ws(xd, cd, d, eta, ws);
            if (j == 0 || v < best_loss) { best_loss = v; best = j; }
        }
        assign[i] = best;
        free(xd);
    }
}

/* ------------------------------------------------------------------------ */
/* query path: tables, ADC, top-k, re-ranking (Section 4.1, Section 2.2.2)   */
/* ------------------------------------------------------------------------ */

/* fp32 inner product with a fixed order: s = 0; s = fma(a_l, b_l, s), l up. */
static float dot_chain(const float *a, const float *b, int len)
{
    float s = 0.0f;
    for (int l = 0; l < len; ++l) s = fmaf(a[l], b[l], s);
    return s;
}

/* Section 4.1: for every dictionary the partial dot product of the query's
 * subspace with every codeword. L[M][kc]. */
void orc_lut_f32(const float *q, const float *codebooks, int d, int M, int kc, float *L)
{
    int ds = d / M;
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < kc; ++j)
            L[(size_t)m * kc + j] = dot_chain(q + m * ds, codebooks + ((size_t)m * kc + j) * ds, ds);
}

/* 8-bit table (not in the paper; defined by this build): per subspace
 * lo_m = min_j L; one range for the whole query R = max_m (max_j L - lo_m);
 * R == 0 -> all codes 0 and scale 0; otherwise inv = 255/R,
 * code = clamp(round-half-even((L - lo_m) * inv), 0, 255), scale = R/255,
 * bias = sum_m lo_m in subspace order. All fp32, one rounding per operation. */
void orc_lut_u8(const float *L, int M, int kc, uint8_t *Q8, float *scale, float *bias)
{
    float R = 0.0f, b = 0.0f;
    for (int m = 0; m < M; ++m) {
        float lo = L[(size_t)m * kc], hi = lo;
        for (int j = 1; j < kc; ++j) {
            float v = L[(size_t)m * kc + j];
            if (v < lo) lo = v;
            if (v > hi) hi = v;
        }
        float w = hi - lo;
        if (w > R) R = w;
        b = b + lo;
    }
    *bias = b;
    if (R == 0.0f) {
        memset(Q8, 0, (size_t)M * kc);
        *scale = 0.0f;
        return;
    }
    float inv = 255.0f / R;
    *scale = R / 255.0f;
    for (int m = 0; m < M; ++m) {
        float lo = L[(size_t)m * kc];
        for (int j = 1; j < kc; ++j)
            if (L[(size_t)m * kc + j] < lo) lo = L[(size_t)m * kc + j];
        for (int j = 0; j < kc; ++j) {
            float t = L[(size_t)m * kc + j] - lo;
            t = t * inv;
            t = rintf(t);
            if (t < 0.0f) t = 0.0f;
            if (t > 255.0f) t = 255.0f;
            Q8[(size_t)m * kc + j] = (uint8_t)t;
        }
    }
}

/* Section 4.1: the score of a quantized point is the sum of its M table
 * entries. The paper fixes no summation order; the order taken here is:
 * 8-bit codes: s = 0; s += L[m][code_m] for m = 0..M-1.
 * 4-bit codes: the two entries of one packed byte are added first,
 * s = 0; s += (L[2p][c_2p] + L[2p+1][c_2p+1]) for p = 0..M/2-1, and for odd M
 * finally s += L[M-1][c_{M-1}]. code: one byte per subspace. */
float orc_adc_one_f32(const float *L, const uint8_t *code, int M, int kc, int bits)
{
    float s = 0.0f;
    if (bits == 8) {
        for (int m = 0; m < M; ++m) s = s + L[(size_t)m * kc + code[m]];
    } else {
        int p;
        for (p = 0; p + 1 < M; p += 2) {
            float t = L[(size_t)p * kc + code[p]] + L[(size_t)(p + 1) * kc + code[p + 1]];
            s = s + t;
        }
        if (p < M) s = s + L[(size_t)p * kc + code[p]];
    }
    return s;
}

uint32_t orc_adc_one_u8(const uint8_t *Q8, const uint8_t *code, int M, int kc)
{
    uint32_t acc = 0;
    for (int m = 0; m < M; ++m) acc += Q8[(size_t)m * kc + code[m]];
    return acc;
}

void orc_adc_f32(const float *L, const uint8_t *codes, int64_t n, int M, int kc, int bits,
                 float *scores)
{
    for (int64_t i = 0; i < n; ++i)
        scores[i] = orc_adc_one_f32(L, codes + (size_t)i * M, M, kc, bits);
}

void orc_adc_u8(const uint8_t *Q8, const uint8_t *codes, int64_t n, int M, int kc,
                uint32_t *acc)
{
    for (int64_t i = 0; i < n; ++i) acc[i] = orc_adc_one_u8(Q8, codes + (size_t)i * M, M, kc);
}

/* Total order used at every selection: higher score first, equal scores by
 * lower id (+0 and -0 compare equal). */
typedef struct { float s; int32_t id; } cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* Top-k by a full sort of all candidates. Missing entries: id -1, -inf. */
void orc_topk(const float *scores, const int32_t *ids, int64_t n, int k, int32_t *ids_out,
              float *scores_out)
{
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) {
        c[i].s = scores[i];
        c[i].id = ids ? ids[i] : (int32_t)i;
    }
    qsort(c, (size_t)n, sizeof(cand_t), cand_cmp);
    for (int j = 0; j < k; ++j) {
        ids_out[j] = j < n ? c[j].id : -1;
        scores_out[j] = j < n ? c[j].s : -INFINITY;
    }
    free(c);
}

/* Exact scores of the whole database, Section 1's definition of MIPS:
 * <q, x_i> in fp32 with the fixed fma order. */
void orc_exact_scores(const float *x, int64_t n, int d, const float *q, float *scores)
{
    for (int64_t i = 0; i < n; ++i) scores[i] = dot_chain(q, x + (size_t)i * d, d);
}

void orc_brute_force(const float *x, int64_t n, int d, const float *queries, int nq, int k,
                     int32_t *ids_out, float *scores_out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int qi = 0; qi < nq; ++qi) {
        float *s = (float *)malloc(sizeof(float) * (size_t)n);
        orc_exact_scores(x, n, d, queries + (size_t)qi * d, s);
        orc_topk(s, NULL, n, k, ids_out + (size_t)qi * k, scores_out + (size_t)qi * k);
        free(s);
    }
}

/* Leaf scores <q, center_l> (fixed fma order) and the top-L leaves by
 * (score desc, leaf id asc). */
void orc_leaf_select(const float *centers, int n_leaves, int d, const float *q, int L,
                     int32_t *leaf_ids, float *leaf_ip)
{
    float *s = (float *)malloc(sizeof(float) * (size_t)n_leaves);
    for (int l = 0; l < n_leaves; ++l) s[l] = dot_chain(q, centers + (size_t)l * d, d);
    orc_topk(s, NULL, n_leaves, L, leaf_ids, leaf_ip);
    free(s);
}

/* ADC ranking keys of one query over the points it scans, as (key, id) pairs.
 * lut_mode 0: fp32 tables; key = s (+ leaf_ip when partitioned, one fp32 add).
 * lut_mode 1: 8-bit tables; flat index: key = (float)acc, exact because
 * acc <= 255*M < 2^24, so ranking by key is ranking by the integer;
 * partitioned: key = fma((float)acc, scale, bias + leaf_ip).
 * Returns the number of candidates written. acc_out (optional) gets acc. */
static int64_t adc_candidates(const float *q, int d, int M, int bits, const float *codebooks,
                              const uint8_t *codes, int64_t n, int n_leaves,
                              const float *centers, const int32_t *assign, int lut_mode,
                              int L_probe, float *keys, int32_t *ids, float *scale_out,
                              float *bias_out)
{
    int kc = 1 << bits;
    float *L = (float *)malloc(sizeof(float) * (size_t)M * kc);
    uint8_t *Q8 = (uint8_t *)malloc((size_t)M * kc);
    float scale = 0.0f, bias = 0.0f;
    orc_lut_f32(q, codebooks, d, M, kc, L);
    if (lut_mode == 1) orc_lut_u8(L, M, kc, Q8, &scale, &bias);
    int64_t cnt = 0;
    if (n_leaves <= 0) {
        for (int64_t i = 0; i < n; ++i) {
            const uint8_t *c = codes + (size_t)i * M;
            keys[i] = lut_mode == 1 ? (float)orc_adc_one_u8(Q8, c, M, kc)
                                    : orc_adc_one_f32(L, c, M, kc, bits);
            ids[i] = (int32_t)i;
        }
        cnt = n;
    } else {
        int32_t *leaf_ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)L_probe);
        float *leaf_ip = (float *)malloc(sizeof(float) * (size_t)L_probe);
        float *ip_of_leaf = (float *)malloc(sizeof(float) * (size_t)n_leaves);
        char *probed = (char *)calloc((size_t)n_leaves, 1);
        orc_leaf_select(centers, n_leaves, d, q, L_probe, leaf_ids, leaf_ip);
        for (int j = 0; j < L_probe; ++j)
            if (leaf_ids[j] >= 0) { probed[leaf_ids[j]] = 1; ip_of_leaf[leaf_ids[j]] = leaf_ip[j]; }
        for (int64_t i = 0; i < n; ++i) {
            int lf = assign[i];
            if (!probed[lf]) continue;
            const uint8_t *c = codes + (size_t)i * M;
            float key;
            if (lut_mode == 1) {
                float off = bias + ip_of_leaf[lf];
                key = fmaf((float)orc_adc_one_u8(Q8, c, M, kc), scale, off);
            } else {
                key = orc_adc_one_f32(L, c, M, kc, bits) + ip_of_leaf[lf];
            }
            keys[cnt] = key;
            ids[cnt] = (int32_t)i;
            ++cnt;
        }
        free(leaf_ids); free(leaf_ip); free(ip_of_leaf); free(probed);
    }
    if (scale_out) *scale_out = scale;
    if (bias_out) *bias_out = bias;
    free(L); free(Q8);
    return cnt;
}

/* All ADC keys of one query (flat index only), for score-level parity. */
void orc_adc_keys_flat(const float *q, int d, int M, int bits, const float *codebooks,
                       const uint8_t *codes, int64_t n, int lut_mode, float *keys,
                       float *scale_out, float *bias_out)
{
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    adc_candidates(q, d, M, bits, codebooks, codes, n, 0, NULL, NULL, lut_mode, 0, keys, ids,
                   scale_out, bias_out);
    free(ids);
}

/* The whole query path for a batch: tables -> ADC over the scanned points ->
 * top-R by the total order -> exact fp32 re-scoring of those R -> top-k.
 * reorder_k == 0: no re-scoring, the ADC top-k is returned; its scores are
 * the ADC keys, except in flat 8-bit mode where the score reported is
 * fma((float)acc, scale, bias). x may be NULL when reorder_k == 0. */
int orc_search(const float *x, int64_t n, int d, int M, int bits, const float *codebooks,
               const uint8_t *codes, int n_leaves, const float *centers,
               const int32_t *assign, const float *queries, int nq, int k, int reorder_k,
               int lut_mode, int L_probe, int32_t *ids_out, float *scores_out)
{
    if (d % M != 0 || (bits != 4 && bits != 8) || k < 1 || (reorder_k != 0 && reorder_k < k))
        return ORC_EINVAL;
    if (n_leaves > 0 && (L_probe < 1 || L_probe > n_leaves)) return ORC_EINVAL;
    int R = reorder_k ? reorder_k : k;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int qi = 0; qi < nq; ++qi) {
        const float *q = queries + (size_t)qi * d;
        float *keys = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
        int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        int32_t *top_ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)R);
        float *top_s = (float *)malloc(sizeof(float) * (size_t)R);
        if (!keys || !ids || !top_ids || !top_s) {
            err = 1;
        } else {
            float scale, bias;
            int64_t cnt = adc_candidates(q, d, M, bits, codebooks, codes, n, n_leaves, centers,
                                         assign, lut_mode, L_probe, keys, ids, &scale, &bias);
            orc_topk(keys, ids, cnt, R, top_ids, top_s);
            if (reorder_k == 0) {
                for (int j = 0; j < k; ++j) {
                    ids_out[(size_t)qi * k + j] = top_ids[j];
                    float s = top_s[j];
                    if (lut_mode == 1 && n_leaves <= 0 && top_ids[j] >= 0)
                        s = fmaf(s, scale, bias);
                    scores_out[(size_t)qi * k + j] = s;
                }
            } else {
                int have = 0;
                for (int j = 0; j < R; ++j)
                    if (top_ids[j] >= 0) {
                        top_s[have] = dot_chain(q, x + (size_t)top_ids[j] * d, d);
                        top_ids[have] = top_ids[j];
                        ++have;
                    }
                orc_topk(top_s, top_ids, have, k, ids_out + (size_t)qi * k,
                         scores_out + (size_t)qi * k);
            }
        }
        free(keys); free(ids); free(top_ids); free(top_s);
    }
    return err ? ORC_ENOMEM : ORC_OK;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int t)
{
#ifdef _OPENMP
    omp_set_num_threads(t);
#else
    (void)t;
#endif
}
