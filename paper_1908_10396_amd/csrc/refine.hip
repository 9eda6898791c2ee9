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
// Let acc_(R) be the R-th largest integer sum of the index. The R points of largest acc all have
// fp32 score >= bound = sum lo + (acc_(R) - E)/c - rho, so the R-th best fp32 score of the
// index is >= bound; a point with acc < acc_(R) - margin, margin >= 2E + 2 rho c, has fp32 score
// <= sum lo + (acc + E)/c + rho < bound: it is not among the R best, ties included. So the R
// best by fp32 score are the R best of the candidate set {acc >= acc_(R) - margin}.
//
// The matrix-core scan in candidate mode keeps, per query and chunk, every point whose sum came
// within the margin of its running lower bound of acc_(R); the bound never exceeds acc_(R), so the
// candidate set is among the kept points. The margin is computed once per query, before the
// scan. Here the kept points at or above acc_(R) - margin are re-scored in fp32, in the scan's
// order of additions, and ranked. A query without a usable margin (tables with a tiny range) or
// with more kept points than the buffers hold is handed to the plain fp32 scan instead.
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

__global__ void __launch_bounds__(64)
prefilter_margin_kernel(const float *__restrict__ lut, const float *__restrict__ scale, int M, int NB, int nq,
                        int32_t *__restrict__ margin)
{
    const int q = blockIdx.x, lane = threadIdx.x;
    float a = 0.0f;
    if (lane < M) {
        const float *L = lut + ((size_t)q * M + lane) * 16;
        for (int j = 0; j < 16; ++j) a = fmaxf(a, fabsf(L[j]));
    }
    for (int m = 32; m > 0; m >>= 1) a += __shfl_xor(a, m, 64);
    if (lane == 0) {
        const float sc = scale[q];
        const float rho = (float)(NB + 2) * 5.9604645e-8f * a * 1.01f;
        const float marg_f = (float)M + 0.01f + (sc > 0.0f ? 2.02f * rho / sc : INFINITY);
        margin[q] = marg_f < 1.0e6f ? (int32_t)ceilf(marg_f) + 1 : -1; // -1: no usable bound, the query is scanned plainly
    }
}

int launch_prefilter_margin(const float *lut, const float *scale, int M, int NB, int nq, int32_t *margin, hipStream_t st)
{
    if (M > 64) { set_error("prefilter: M > 64"); return AVQ_EINVAL; }
    hipLaunchKernelGGL(prefilter_margin_kernel, dim3(nq), dim3(64), 0, st, lut, scale, M, NB, nq, margin);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

constexpr int kMaxChunks = 256;  // chunks of the scan (scan_mfma_plan never makes more)
constexpr int kKeysPerThread = 32; // kept keys of one query that the refinement can look at: 256 threads x 32; more: plain scan
constexpr int kFinalMax = 2048;  // of those, the ones within the margin of the R-th best sum; more: plain scan


// out[rank] = key for the R best of keys[0 .. n_cand) (distinct, in LDS, n_cand <= kFinalMax, keys[n_cand] = 0 when
// n_cand is odd), ranks by counting: a thread holds its own keys (PER of them) and reads all keys, two at a
// time, at addresses the whole wave shares. 256 threads.
template <int PER>
__device__ __forceinline__ void rank_and_store_per(const u64 *keys, int n_cand, int R, u64 *__restrict__ out, int tid)
{
    constexpr int nt = 256;
    u64 mine[PER];
    int rank[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int j = tid + k * nt;
        mine[k] = j < n_cand ? keys[j] : ~0ull;
        rank[k] = 0;
    }
    for (int t = 0; t < n_cand; t += 2) {
        const ulonglong2 two = *(const ulonglong2 *)(keys + t);
#pragma unroll
        for (int k = 0; k < PER; ++k) rank[k] += (int)(two.x > mine[k]) + (int)(two.y > mine[k]);
    }
#pragma unroll
    for (int k = 0; k < PER; ++k)
        if (tid + k * nt < n_cand && rank[k] < R) out[rank[k]] = mine[k];
}

__device__ __forceinline__ void rank_and_store(const u64 *keys, int n_cand, int R, u64 *__restrict__ out, int tid)
{
    if (n_cand <= 256) rank_and_store_per<1>(keys, n_cand, R, out, tid);
    else if (n_cand <= 512) rank_and_store_per<2>(keys, n_cand, R, out, tid);
    else if (n_cand <= 1024) rank_and_store_per<4>(keys, n_cand, R, out, tid);
    else rank_and_store_per<kFinalMax / 256>(keys, n_cand, R, out, tid);
}

template <int NBT>
__global__ void __launch_bounds__(256)
refine_cand_kernel(const RefineCandParams r)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    constexpr int nt = 256;
    const int q = blockIdx.x;
    const int C = 64 * r.ns;
    const int n_tab = 2 * r.NB;
    float *tbl = (float *)smem;                                               // [n_tab][16]
    u64 *keys = (u64 *)(smem + (((size_t)n_tab * 64 + 15) & ~(size_t)15));    // [kFinalMax] ids of the finalists, then their fp32 keys
    __shared__ int n_top_s, bad_s, n_fin_s, wave_cnt[2][4];
    __shared__ uint32_t first_of[kMaxChunks + 1]; // first_of[c] = kept keys in the chunks before c

    // lut == NULL: the integer sums themselves are what is ranked (8-bit-table search): no margin, no re-scoring
    const bool rescore = r.lut != nullptr;
    if (rescore) {
        const float *L = r.lut + (size_t)q * r.M * 16;
        for (int e = tid; e < n_tab * 16; e += nt) tbl[e] = e < r.M * 16 ? L[e] : 0.0f;
    }
    if (tid == 0) { n_top_s = 0; bad_s = 0; n_fin_s = 0; }
    // the chunks' fill counts (one load each, all in flight together) and their running sum
    uint32_t my_cnt = 0u;
    if (tid < r.n_chunks) my_cnt = r.cand_cnt[(size_t)q * r.n_chunks + tid];
    __syncthreads();
    if (tid < r.n_chunks && my_cnt > (uint32_t)r.cand_cap) bad_s = 1; // that chunk's buffer overflowed
    first_of[tid + 1 <= kMaxChunks ? tid + 1 : kMaxChunks] = my_cnt;  // tid 255 -> slot 256
    if (tid == 0) first_of[0] = 0u;
    __syncthreads();
    for (int d = 1; d < kMaxChunks; d *= 2) { // inclusive scan over slots 1 .. kMaxChunks
        const uint32_t add = tid + 1 > d ? first_of[tid + 1 - d] : 0u;
        __syncthreads();
        first_of[tid + 1] += add;
        __syncthreads();
    }
    const bool fixed = r.bound != nullptr;
    const int margin = rescore ? r.margin[q] : 0;
    const uint32_t um = (uint32_t)(margin > 0 ? margin : 0);
    uint32_t keep = 0u; // ordering value from which a kept key is a finalist
    if (!fixed) {
        const u64 *top = r.top + (size_t)q * C;
        int mine_top = 0;
        for (int i = tid; i < r.R; i += nt) mine_top += top[i] != 0ull;
        if (mine_top) atomicAdd(&n_top_s, mine_top);
        __syncthreads();
        // fewer than R points in the whole index: the bound never rose above zero and every point was kept
        const uint32_t ord_r = n_top_s == r.R ? key_ord(top[r.R - 1]) : 0u;
        keep = ord_r > um ? ord_r - um : 0u;
    }
    const uint32_t total = first_of[r.n_chunks];
    bool ok = margin >= 0 && bad_s == 0 && total <= (uint32_t)(nt * kKeysPerThread);
    int why = margin >= 0 ? 1 : 3;
    if (r.force_fail_odd && (q & 1)) { ok = false; why = 3; }
    // every thread takes the kept keys tid, tid + 256, ... of the chunks laid end to end, into registers
    uint32_t mine[kKeysPerThread];
    if (ok) {
        int c = 0;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k) {
            const uint32_t flat = (uint32_t)(tid + k * nt);
            mine[k] = 0u;
            if (flat < total) {
                while (flat >= first_of[c + 1]) ++c;
                mine[k] = r.cand_keys[((size_t)q * r.n_chunks + c) * r.cand_cap + (flat - first_of[c])];
            }
        }
    }
    if (ok && fixed) {
        // The scan kept every point at or above bound - margin. If R of them reach the bound itself, the
        // R-th best sum of the index does too, and nothing that matters was dropped. Then that R-th best
        // sum is found by bisection (every thread counts its own keys), and only keys within the margin of
        // it go on. (Unused slots hold 0: ordering value 0, below every bound.)
        const uint32_t T = r.bound[q];
        // keys with ordering value >= v (v >= 1), over the workgroup; one barrier per call, the waves' counts
        // in alternating rows
        int parity = 0;
        auto count_ge = [&](uint32_t v) -> int {
            int cn = 0;
#pragma unroll
            for (int k = 0; k < kKeysPerThread; ++k) cn += __popcll(__builtin_amdgcn_ballot_w64((mine[k] >> 18) >= v));
            if ((tid & 63) == 0) wave_cnt[parity][tid >> 6] = cn;
            __syncthreads();
            const int tot = wave_cnt[parity][0] + wave_cnt[parity][1] + wave_cnt[parity][2] + wave_cnt[parity][3];
            parity ^= 1;
            return tot;
        };
        if (T == 0u || count_ge(T) < r.R) {
            ok = false;
            why = 2;
        } else {
            uint32_t lo = T, hi = 1u << 14; // count_ge(lo) >= R > count_ge(hi): ordering values stay below 2^14
            while (hi - lo > 1u) {
                const uint32_t mid = (lo + hi) >> 1;
                if (count_ge(mid) >= r.R) lo = mid; else hi = mid;
            }
            keep = lo > um ? lo - um : 0u; // lo = the R-th best sum's ordering value
        }
    }
    if (ok) {
        int c = 0;
#pragma unroll
        for (int k = 0; k < kKeysPerThread; ++k) {
            const uint32_t flat = (uint32_t)(tid + k * nt);
            if (flat < total && (mine[k] >> 18) >= keep) {
                while (flat >= first_of[c + 1]) ++c;
                const int slot = atomicAdd(&n_fin_s, 1);
                if (slot < kFinalMax) {
                    const int32_t id = (int32_t)((int64_t)c * r.chunk_points) + (int32_t)(~mine[k] & 0x3ffffu);
                    keys[slot] = rescore ? (u64)(uint32_t)id : make_key(mine[k] >> 18, id);
                }
            }
        }
        __syncthreads();
        ok = n_fin_s <= kFinalMax;
    }
    if (!ok) {
        if (tid == 0) {
            r.fail_list[atomicAdd(r.fail_count, 1u)] = q;
            atomicAdd(r.fail_count + why, 1u); // statistics: 1 = too many kept points, 2 = bound guessed too high, 3 = other
        }
        return;
    }
    const int n_cand = n_fin_s;
    for (int i = tid; rescore && i < n_cand; i += nt) {
        const int32_t id = (int32_t)(uint32_t)keys[i]; // replaced by the key below, by this thread
        const uint8_t *row = r.codes + (size_t)id * r.NB;
        float s = 0.0f;
        if constexpr (NBT != 0) {
            uint32_t bytes[NBT];
#pragma unroll
            for (int b = 0; b < NBT; ++b) bytes[b] = row[b];
#pragma unroll
            for (int b = 0; b < NBT; ++b) {
                const float v = __fadd_rn(tbl[(2 * b) * 16 + (bytes[b] & 15u)], tbl[(2 * b + 1) * 16 + (bytes[b] >> 4)]);
                s = __fadd_rn(s, v);
            }
        } else {
            for (int b = 0; b < r.NB; ++b) {
                const uint32_t byte = row[b];
                const float v = __fadd_rn(tbl[(2 * b) * 16 + (byte & 15u)], tbl[(2 * b + 1) * 16 + (byte >> 4)]);
                s = __fadd_rn(s, v);
            }
        }
        keys[i] = make_key(ord_from_f32(s), id);
    }
    if (tid == 0 && (n_cand & 1)) keys[n_cand] = 0ull; // n_cand odd: below kFinalMax, which is even
    __syncthreads();
    u64 *out = r.out + (size_t)q * C;
    rank_and_store(keys, n_cand, r.R, out, tid);
    const int n_fin = n_cand < r.R ? n_cand : r.R;
    for (int i = n_fin + tid; i < C; i += nt) out[i] = 0ull;
}

// bound[q] = ordering value of the r-th key of query q's sorted list (0 if there are fewer)
__global__ void __launch_bounds__(256)
list_bound_kernel(const u64 *__restrict__ lists, int C, int r, int nq, uint32_t *__restrict__ bound)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nq) bound[q] = key_ord(lists[(size_t)q * C + (r - 1)]);
}

// bound[q] = the r-th largest of query q's S class maxima (ordering values below 2^14; 0 = no point), 0 if fewer
// than r are non-zero. Bisection over the ordering values with the maxima in registers, 32 per lane at most:
// one wave per query (S <= 2048), or the four waves of a workgroup together (WIDE, S <= 8192; one barrier per round).
template <bool WIDE>
__global__ void __launch_bounds__(256)
sample_bound_kernel(const uint32_t *__restrict__ smax, int S, int r, int nq, uint32_t *__restrict__ bound)
{
    __shared__ int wave_cnt[2][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = WIDE ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave;
    if (q >= nq) return; // WIDE: the whole workgroup leaves
    const uint32_t *v = smax + (size_t)q * S;
    const int first = WIDE ? threadIdx.x : lane, step = WIDE ? 256 : 64;
    uint32_t mine[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        const int i = first + k * step;
        mine[k] = i < S ? v[i] : 0u;
    }
    int parity = 0;
    auto count_ge = [&](uint32_t t) -> int { // t >= 1
        int cn = 0;
#pragma unroll
        for (int k = 0; k < 32; ++k) cn += __popcll(__builtin_amdgcn_ballot_w64(mine[k] >= t));
        if (WIDE) {
            if (lane == 0) wave_cnt[parity][wave] = cn;
            __syncthreads();
            cn = wave_cnt[parity][0] + wave_cnt[parity][1] + wave_cnt[parity][2] + wave_cnt[parity][3];
            parity ^= 1;
        }
        return cn;
    };
    uint32_t lo = 0u;
    if (count_ge(1u) >= r) {
        lo = 1u;
        uint32_t hi = 1u << 14; // count_ge(lo) >= r > count_ge(hi)
        while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (count_ge(mid) >= r) lo = mid; else hi = mid;
        }
    }
    if ((WIDE ? threadIdx.x : lane) == 0) bound[q] = lo;
}

int launch_sample_bound(const uint32_t *sample_max, int S, int r, int nq, uint32_t *bound, hipStream_t st)
{
    if (S < 1 || S > 8192 || r < 1) { set_error("sample bound: bad shape (%d maxima)", S); return AVQ_EINVAL; }
    if (S <= 2048) hipLaunchKernelGGL(sample_bound_kernel<false>, dim3((nq + 3) / 4), dim3(256), 0, st, sample_max, S, r, nq, bound);
    else hipLaunchKernelGGL(sample_bound_kernel<true>, dim3(nq), dim3(256), 0, st, sample_max, S, r, nq, bound);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_list_bound(const u64 *lists, int ns, int r, int nq, uint32_t *bound, hipStream_t st)
{
    hipLaunchKernelGGL(list_bound_kernel, dim3((nq + 255) / 256), dim3(256), 0, st, lists, 64 * ns, r, nq, bound);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_refine_cand(const RefineCandParams &r, hipStream_t st)
{
    if (r.M > 64 || r.R > 64 * r.ns || r.cand_cap < 1 || r.n_chunks > kMaxChunks || (r.lut != nullptr && r.margin == nullptr) || (r.top == nullptr) == (r.bound == nullptr)) { set_error("refine: bad shape (M %d, R %d)", r.M, r.R); return AVQ_EINVAL; }
    const size_t lds = (((size_t)2 * r.NB * 64 + 15) & ~(size_t)15) + sizeof(u64) * (size_t)kFinalMax;
    switch (r.NB) {
    case 8: hipLaunchKernelGGL(refine_cand_kernel<8>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 13: hipLaunchKernelGGL(refine_cand_kernel<13>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 25: hipLaunchKernelGGL(refine_cand_kernel<25>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 32: hipLaunchKernelGGL(refine_cand_kernel<32>, dim3(r.nq), dim3(256), lds, st, r); break;
    default: hipLaunchKernelGGL(refine_cand_kernel<0>, dim3(r.nq), dim3(256), lds, st, r); break;
    }
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// ---- partitioned index ------------------------------------------------------------------------
//
// With leaves (Section 5.3) a point's score is its table sum plus <q, center of its leaf>, so the
// integer sums of different leaves do not compare; the estimate a = fma(sum, scale, bias + leaf_ip)
// does. The scan kept every point whose estimate could reach a bound known to be at or below the
// R-th best score (the R-th best of the query's first few leaves, scanned with the tables the search
// asked for). Here: the estimates of the kept points, the R-th best of them by bisection over the
// ordering values, and then either the R best estimates themselves (8-bit tables: the estimate is the
// score) or, for fp32 tables, the fp32 scores of the points within margin * scale of it (the estimate
// is within half of that of the fp32 score, by the argument at the top of this file).

constexpr int kIvfKeysPerThread = 16; // 4096 kept keys per query at most

template <int NBT>
__global__ void __launch_bounds__(256)
ivf_refine_kernel(const IvfRefineParams r)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    constexpr int nt = 256;
    const int q = blockIdx.x;
    const int C = 64 * r.ns;
    const int n_tab = 2 * r.NB;
    const bool rescore = r.lut != nullptr;
    float *tbl = (float *)smem;                                               // [n_tab][16] (fp32 tables only)
    u64 *keys = (u64 *)(smem + (((size_t)n_tab * 64 + 15) & ~(size_t)15));    // [kFinalMax]
    int32_t *fin_ids = (int32_t *)(keys + kFinalMax);                         // [kFinalMax]
    float *fin_ip = (float *)(fin_ids + kFinalMax);                           // [kFinalMax]
    __shared__ int n_fin_s, wave_cnt[2][4];
    __shared__ uint32_t wave_ext[2][4];

    if (rescore) {
        const float *L = r.lut + (size_t)q * r.M * 16;
        for (int e = tid; e < n_tab * 16; e += nt) tbl[e] = e < r.M * 16 ? L[e] : 0.0f;
    }
    if (tid == 0) n_fin_s = 0;
    __syncthreads();
    const uint32_t total = r.kept_cnt[q];
    const int margin = rescore ? r.margin[q] : 0;
    bool ok = total <= (uint32_t)r.kept_cap && total <= (uint32_t)(nt * kIvfKeysPerThread) && margin >= 0;
    int why = margin >= 0 ? 1 : 3;
    if (r.force_fail_odd && (q & 1)) { ok = false; why = 3; }
    const float scale = r.scale[q], bias = r.bias[q];
    uint32_t est[kIvfKeysPerThread]; // ordering value of the estimate, 0: no point
    int32_t ids[kIvfKeysPerThread];
    float ips[kIvfKeysPerThread];
    if (ok) {
#pragma unroll
        for (int k = 0; k < kIvfKeysPerThread; ++k) {
            const uint32_t i = (uint32_t)(tid + k * nt);
            est[k] = 0u;
            ids[k] = -1;
            ips[k] = 0.0f;
            if (i < total) {
                const u64 e = r.kept[(size_t)q * r.kept_cap + i];
                const uint32_t hi = (uint32_t)(e >> 32), k32 = (uint32_t)e;
                const int leaf = (int)(hi & 0x1fffffu), slot = (int)(hi >> 21);
                const int32_t id = r.perm[(size_t)r.leaf_blk[leaf] * kBlockPoints + (~k32 & 0x3ffffu)];
                if (id >= 0) {
                    const float ip = r.leaf_ip[(size_t)q * r.leaf_stride + slot];
                    const int sum = (int)(k32 >> 18) - 1;
                    ids[k] = id;
                    ips[k] = ip;
                    est[k] = ord_from_f32(__fmaf_rn((float)sum, scale, __fadd_rn(bias, ip)));
                }
            }
        }
    }
    uint32_t keep = 0u;
    if (ok) {
        // estimates >= v over the workgroup, v >= 1; one barrier per call, the waves' counts in alternating rows
        int parity = 0;
        auto count_ge = [&](uint32_t v) -> int {
            int cn = 0;
#pragma unroll
            for (int k = 0; k < kIvfKeysPerThread; ++k) cn += __popcll(__builtin_amdgcn_ballot_w64(est[k] >= v));
            if ((tid & 63) == 0) wave_cnt[parity][tid >> 6] = cn;
            __syncthreads();
            const int tot = wave_cnt[parity][0] + wave_cnt[parity][1] + wave_cnt[parity][2] + wave_cnt[parity][3];
            parity ^= 1;
            return tot;
        };
        // smallest and largest estimate: the search runs between them
        uint32_t emin = 0xffffffffu, emax = 0u;
#pragma unroll
        for (int k = 0; k < kIvfKeysPerThread; ++k) {
            emax = est[k] > emax ? est[k] : emax;
            emin = est[k] != 0u && est[k] < emin ? est[k] : emin;
        }
        for (int m = 32; m > 0; m >>= 1) {
            const uint32_t a = (uint32_t)__shfl_xor((int)emax, m, 64), b2 = (uint32_t)__shfl_xor((int)emin, m, 64);
            emax = a > emax ? a : emax;
            emin = b2 < emin ? b2 : emin;
        }
        if ((tid & 63) == 0) { wave_ext[0][tid >> 6] = emin; wave_ext[1][tid >> 6] = emax; }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            emin = wave_ext[0][w] < emin ? wave_ext[0][w] : emin;
            emax = wave_ext[1][w] > emax ? wave_ext[1][w] : emax;
        }
        if (emax != 0u && count_ge(emin) >= r.R) {
            // ordering value of the R-th best estimate: the largest v with at least R estimates >= v
            uint32_t lo = emin, hi = emax == 0xffffffffu ? emax : emax + 1u; // count_ge(lo) >= R > count_ge(hi) (no finite score maps to 2^32 - 1)
            while (hi - lo > 1u) {
                const uint32_t mid = lo + ((hi - lo) >> 1);
                if (count_ge(mid) >= r.R) lo = mid; else hi = mid;
            }
            keep = lo;
            if (rescore) {
                // estimates within margin units of scale below it, with a little room for the rounding here
                const float a_r = f32_from_ord(lo);
                const float t = a_r - ((float)margin * scale + 4.0e-6f * fabsf(a_r));
                keep = ord_from_f32(t);
            }
        } // fewer than R points were kept: they are all there is (keep = 0)
#pragma unroll
        for (int k = 0; k < kIvfKeysPerThread; ++k) {
            if (est[k] != 0u && est[k] >= keep) {
                const int slot = atomicAdd(&n_fin_s, 1);
                if (slot < kFinalMax) {
                    fin_ids[slot] = ids[k];
                    fin_ip[slot] = ips[k];
                    if (!rescore) keys[slot] = make_key(est[k], ids[k]);
                }
            }
        }
        __syncthreads();
        ok = n_fin_s <= kFinalMax;
    }
    if (!ok) {
        if (tid == 0) {
            r.fail_list[atomicAdd(r.fail_count, 1u)] = q;
            atomicAdd(r.fail_count + why, 1u);
        }
        return;
    }
    const int n_cand = n_fin_s;
    for (int i = tid; rescore && i < n_cand; i += nt) {
        const int32_t id = fin_ids[i];
        const uint8_t *row = r.codes + (size_t)id * r.NB;
        float s = 0.0f;
        if constexpr (NBT != 0) {
            uint32_t bytes[NBT];
#pragma unroll
            for (int b = 0; b < NBT; ++b) bytes[b] = row[b];
#pragma unroll
            for (int b = 0; b < NBT; ++b) {
                const float v = __fadd_rn(tbl[(2 * b) * 16 + (bytes[b] & 15u)], tbl[(2 * b + 1) * 16 + (bytes[b] >> 4)]);
                s = __fadd_rn(s, v);
            }
        } else {
            for (int b = 0; b < r.NB; ++b) {
                const uint32_t byte = row[b];
                const float v = __fadd_rn(tbl[(2 * b) * 16 + (byte & 15u)], tbl[(2 * b + 1) * 16 + (byte >> 4)]);
                s = __fadd_rn(s, v);
            }
        }
        keys[i] = make_key(ord_from_f32(__fadd_rn(s, fin_ip[i])), id);
    }
    if (tid == 0 && (n_cand & 1)) keys[n_cand] = 0ull; // n_cand odd: below kFinalMax, which is even
    __syncthreads();
    u64 *out = r.out + (size_t)q * C;
    rank_and_store(keys, n_cand, r.R, out, tid);
    const int n_fin = n_cand < r.R ? n_cand : r.R;
    for (int i = n_fin + tid; i < C; i += nt) out[i] = 0ull;
}

int launch_ivf_refine(const IvfRefineParams &r, hipStream_t st)
{
    if (r.M > 64 || r.R > 64 * r.ns || r.kept_cap < 1 || r.kept_cap > 256 * kIvfKeysPerThread || (r.lut != nullptr && r.margin == nullptr)) {
        set_error("refine (leaves): bad shape (M %d, R %d, capacity %d)", r.M, r.R, r.kept_cap);
        return AVQ_EINVAL;
    }
    const size_t lds = (((size_t)2 * r.NB * 64 + 15) & ~(size_t)15) + (sizeof(u64) + sizeof(int32_t) + sizeof(float)) * (size_t)kFinalMax;
    switch (r.NB) {
    case 8: hipLaunchKernelGGL(ivf_refine_kernel<8>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 13: hipLaunchKernelGGL(ivf_refine_kernel<13>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 25: hipLaunchKernelGGL(ivf_refine_kernel<25>, dim3(r.nq), dim3(256), lds, st, r); break;
    case 32: hipLaunchKernelGGL(ivf_refine_kernel<32>, dim3(r.nq), dim3(256), lds, st, r); break;
    default: hipLaunchKernelGGL(ivf_refine_kernel<0>, dim3(r.nq), dim3(256), lds, st, r); break;
    }
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
