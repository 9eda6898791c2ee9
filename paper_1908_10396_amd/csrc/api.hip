// C ABI of libavq (declared in include/avq.h): argument checking, the index
// object, device buffers and the sequence of kernel launches of each call.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "avq_internal.h"
#include <cmath>

namespace avq {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int DevBuf::reserve(size_t bytes)
{
    if (bytes <= cap) return AVQ_OK;
    if (p) { (void)hipFree(p); p = nullptr; cap = 0; }
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        p = nullptr;
        set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
        return e == hipErrorOutOfMemory ? AVQ_ENOMEM : AVQ_EHIP;
    }
    cap = bytes;
    return AVQ_OK;
}

void DevBuf::release()
{
    if (p) (void)hipFree(p);
    p = nullptr;
    cap = 0;
}

} // namespace avq

using namespace avq;

struct avq_index {
    avq_config cfg;
    int kc = 0, ds = 0, NB = 0;
    bool have_codebooks = false, have_centers = false;
    DevBuf codebooks, centers, centers_t;
    // database
    int64_t n = 0, n_slots = 0, n_blocks = 0, max_leaf_blocks = 0;
    const float *x = nullptr;
    DevBuf x_own, codes_logical, codes_blocked, assign, perm, leaf_blk;
    // per-call scratch
    DevBuf lut, lut8, scale, bias, partial, cand, leaf_ids, leaf_ip, tmp, thr;
    int tune_target_wgs = 0, tune_waves = 0, tune_qt = 0, tune_small_batch = -1, tune_small_impl = 0, tune_select_split = 0, tune_rerank_split = 0, tune_bound_bits = 0;
    int tune_stream_loads = 0; // single-query scan of the code array: 0 = nontemporal loads when the array exceeds the Infinity Cache, 1 = never, 2 = always
    int tune_mfma = 0; // 0 = use the matrix-core scan where it applies, 1 = never
    int tune_prefilter = 0; // 0 = fp32-table batches go through the 8-bit-table scan where it applies, 1 = never,
                            // 2 = as 0 but odd queries always take the plain scan afterwards (exercises that branch)
    int tune_bound_leaves = 0; // leaves per query that supply the bound of the grouped scan over leaves, 0 = built-in
    int tune_group_min = 0; // (query, leaf) pairs from which a batch on a partitioned index is regrouped by leaf; 0 = built in
    int tune_sample = 0; // 0 = batches guess the candidate scan's bounds from a sample where possible, 1 = never, 2 = from a sample scanned with lists
    int tune_prefilter_cap = 0; // candidate keys per (query, chunk) of that scan, 0 = built-in
    DevBuf block_max, lists, refined, lut_fail, fail, cand_keys, groups, kept, fail_rows;
    // optional per-stage timing with HIP events recorded on the caller's stream
    bool prof_on = false;
    std::vector<hipEvent_t> prof_pool;
    size_t prof_used = 0;
    struct ProfRec { int stage; hipEvent_t a, b; };
    std::vector<ProfRec> prof_recs;
};

// Records an event pair around one stage's launches while profiling is on.
struct StageTimer {
    avq_index *idx;
    hipStream_t st;
    hipEvent_t a = nullptr, b = nullptr;
    int stage;
    StageTimer(avq_index *i, int stage_, hipStream_t s, bool enabled = true) : idx(i), st(s), stage(stage_)
    {
        if (!idx->prof_on || !enabled) return; // (creating an event allocates)
        while (idx->prof_pool.size() < idx->prof_used + 2) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            idx->prof_pool.push_back(e);
        }
        a = idx->prof_pool[idx->prof_used++];
        b = idx->prof_pool[idx->prof_used++];
        (void)hipEventRecord(a, st);
    }
    ~StageTimer()
    {
        if (!a) return;
        (void)hipEventRecord(b, st);
        idx->prof_recs.push_back({stage, a, b});
    }
};

static int check_index(const avq_index *idx)
{
    if (!idx) { set_error("index is NULL"); return AVQ_EINVAL; }
    return AVQ_OK;
}

extern "C" const char *avq_last_error(void) { return g_err; }
extern "C" const char *avq_version(void) { return "avq 0.1 (gfx950)"; }

extern "C" double avq_eta(int32_t d, double T, double norm, int32_t eta_mode)
{
    if (eta_mode != AVQ_ETA_LIMIT && eta_mode != AVQ_ETA_EXACT) return -1.0;
    return eta_host(d, T, norm, eta_mode);
}

extern "C" int avq_create(const avq_config *cfg, avq_index **out)
{
    if (!cfg || !out) { set_error("avq_create: NULL argument"); return AVQ_EINVAL; }
    *out = nullptr;
    if (cfg->d < 2 || cfg->M < 1 || cfg->d % cfg->M != 0) {
        set_error("avq_create: need d >= 2, M >= 1, d %% M == 0 (d=%d M=%d)", cfg->d, cfg->M);
        return AVQ_EINVAL;
    }
    if (cfg->bits != 4 && cfg->bits != 8) { set_error("avq_create: bits must be 4 or 8"); return AVQ_EINVAL; }
    if (!(cfg->T >= 0.0f)) { set_error("avq_create: T must be >= 0"); return AVQ_EINVAL; }
    if (cfg->eta_mode < 0 || cfg->eta_mode > 2) { set_error("avq_create: bad eta_mode"); return AVQ_EINVAL; }
    if (cfg->eta_mode == AVQ_ETA_EXPLICIT && !(cfg->eta_explicit >= 1.0f)) {
        set_error("avq_create: eta_explicit must be >= 1");
        return AVQ_EINVAL;
    }
    if (cfg->kmeans_iters < 0 || cfg->encode_passes < 0 || cfg->n_leaves < 0 || cfg->leaf_kmeans_iters < 0 ||
        cfg->leaf_aniso_iters < 0) {
        set_error("avq_create: negative count");
        return AVQ_EINVAL;
    }
    if (cfg->M > 256) { set_error("avq_create: M > 256 not supported"); return AVQ_EINVAL; }
    avq_index *idx = new (std::nothrow) avq_index();
    if (!idx) { set_error("avq_create: out of host memory"); return AVQ_ENOMEM; }
    idx->cfg = *cfg;
    idx->kc = 1 << cfg->bits;
    idx->ds = cfg->d / cfg->M;
    idx->NB = (cfg->M * cfg->bits + 7) / 8;
    int rc = idx->codebooks.reserve(sizeof(float) * (size_t)cfg->M * idx->kc * idx->ds);
    if (rc == AVQ_OK && cfg->n_leaves > 0) {
        rc = idx->centers.reserve(sizeof(float) * (size_t)cfg->n_leaves * cfg->d);
        if (rc == AVQ_OK) rc = idx->centers_t.reserve(sizeof(float) * (size_t)cfg->n_leaves * cfg->d);
    }
    if (rc != AVQ_OK) { avq_destroy(idx); return rc; }
    *out = idx;
    return AVQ_OK;
}

extern "C" void avq_destroy(avq_index *idx)
{
    if (!idx) return;
    DevBuf *all[] = {&idx->codebooks, &idx->centers, &idx->centers_t, &idx->x_own, &idx->codes_logical,
                     &idx->codes_blocked, &idx->assign, &idx->perm, &idx->leaf_blk, &idx->lut, &idx->lut8,
                     &idx->scale, &idx->bias, &idx->partial, &idx->cand, &idx->leaf_ids, &idx->leaf_ip,
                     &idx->tmp, &idx->block_max, &idx->lists, &idx->thr, &idx->refined, &idx->lut_fail,
                     &idx->fail, &idx->cand_keys, &idx->groups, &idx->kept, &idx->fail_rows};
    for (DevBuf *b : all) b->release();
    for (hipEvent_t e : idx->prof_pool) (void)hipEventDestroy(e);
    delete idx;
}

extern "C" int64_t avq_size(const avq_index *idx) { return idx ? idx->n : 0; }

extern "C" int avq_set_tuning(avq_index *idx, const char *name, int32_t value)
{
    AVQ_TRY(check_index(idx));
    if (!name || value < 0) { set_error("avq_set_tuning: bad argument"); return AVQ_EINVAL; }
    if (!strcmp(name, "scan_target_wgs")) idx->tune_target_wgs = value;
    else if (!strcmp(name, "scan_waves")) idx->tune_waves = value;
    else if (!strcmp(name, "scan_qt")) idx->tune_qt = value;
    else if (!strcmp(name, "small_batch_max")) idx->tune_small_batch = value - 1; // 0 = built-in
    else if (!strcmp(name, "small_batch_impl")) idx->tune_small_impl = value;
    else if (!strcmp(name, "scan_mfma")) idx->tune_mfma = value;
    else if (!strcmp(name, "scan_prefilter")) idx->tune_prefilter = value;
    else if (!strcmp(name, "prefilter_cap")) idx->tune_prefilter_cap = value;
    else if (!strcmp(name, "scan_sample")) idx->tune_sample = value;
    else if (!strcmp(name, "group_min_pairs")) idx->tune_group_min = value;
    else if (!strcmp(name, "bound_leaves")) idx->tune_bound_leaves = value;
    else if (!strcmp(name, "select_split")) idx->tune_select_split = value;
    else if (!strcmp(name, "rerank_split")) idx->tune_rerank_split = value;
    else if (!strcmp(name, "bound_bits")) idx->tune_bound_bits = value;
    else if (!strcmp(name, "stream_loads")) idx->tune_stream_loads = value;
    else { set_error("avq_set_tuning: unknown name '%s'", name); return AVQ_EINVAL; }
    return AVQ_OK;
}

extern "C" int avq_profile_enable(avq_index *idx, int32_t on)
{
    AVQ_TRY(check_index(idx));
    idx->prof_on = on != 0;
    return AVQ_OK;
}

extern "C" int avq_profile_read(avq_index *idx, double *ms_out, int64_t *launches_out, int32_t reset)
{
    AVQ_TRY(check_index(idx));
    if (!ms_out || !launches_out) { set_error("avq_profile_read: NULL output"); return AVQ_EINVAL; }
    for (int s = 0; s < AVQ_N_STAGES; ++s) { ms_out[s] = 0.0; launches_out[s] = 0; }
    for (const avq_index::ProfRec &r : idx->prof_recs) {
        AVQ_HIP(hipEventSynchronize(r.b));
        float ms = 0.0f;
        AVQ_HIP(hipEventElapsedTime(&ms, r.a, r.b));
        ms_out[r.stage] += (double)ms;
        launches_out[r.stage] += 1;
    }
    if (reset) { idx->prof_recs.clear(); idx->prof_used = 0; }
    return AVQ_OK;
}

// ---- dictionaries and leaf centers -------------------------------------------------

extern "C" int avq_set_codebooks(avq_index *idx, const float *codebooks)
{
    AVQ_TRY(check_index(idx));
    if (!codebooks) { set_error("avq_set_codebooks: NULL"); return AVQ_EINVAL; }
    AVQ_HIP(hipMemcpy(idx->codebooks.p, codebooks, sizeof(float) * (size_t)idx->cfg.M * idx->kc * idx->ds,
                      hipMemcpyDefault));
    idx->have_codebooks = true;
    return AVQ_OK;
}

extern "C" int avq_get_codebooks(avq_index *idx, float *out)
{
    AVQ_TRY(check_index(idx));
    if (!out) { set_error("avq_get_codebooks: NULL"); return AVQ_EINVAL; }
    if (!idx->have_codebooks) { set_error("avq_get_codebooks: no dictionaries yet"); return AVQ_ESTATE; }
    AVQ_HIP(hipMemcpy(out, idx->codebooks.p, sizeof(float) * (size_t)idx->cfg.M * idx->kc * idx->ds,
                      hipMemcpyDefault));
    return AVQ_OK;
}

static int refresh_centers_t(avq_index *idx, hipStream_t st)
{
    AVQ_TRY(launch_transpose(idx->centers.as<float>(), idx->cfg.n_leaves, idx->cfg.d,
                             idx->centers_t.as<float>(), st));
    AVQ_HIP(hipStreamSynchronize(st));
    return AVQ_OK;
}

extern "C" int avq_set_leaf_centers(avq_index *idx, const float *centers)
{
    AVQ_TRY(check_index(idx));
    if (idx->cfg.n_leaves <= 0) { set_error("avq_set_leaf_centers: flat index"); return AVQ_ESTATE; }
    if (!centers) { set_error("avq_set_leaf_centers: NULL"); return AVQ_EINVAL; }
    AVQ_HIP(hipMemcpy(idx->centers.p, centers, sizeof(float) * (size_t)idx->cfg.n_leaves * idx->cfg.d,
                      hipMemcpyDefault));
    AVQ_TRY(refresh_centers_t(idx, nullptr));
    idx->have_centers = true;
    return AVQ_OK;
}

extern "C" int avq_get_leaf_centers(avq_index *idx, float *out)
{
    AVQ_TRY(check_index(idx));
    if (idx->cfg.n_leaves <= 0 || !idx->have_centers) {
        set_error("avq_get_leaf_centers: no leaf centers");
        return AVQ_ESTATE;
    }
    if (!out) { set_error("avq_get_leaf_centers: NULL"); return AVQ_EINVAL; }
    AVQ_HIP(hipMemcpy(out, idx->centers.p, sizeof(float) * (size_t)idx->cfg.n_leaves * idx->cfg.d,
                      hipMemcpyDefault));
    return AVQ_OK;
}

// Assignment of rows to leaves: nearest center, or smallest anisotropic loss when the index learns its
// leaves as an anisotropic vector quantizer (cfg.leaf_aniso_iters > 0).
static int assign_to_leaves(avq_index *idx, const float *x, int64_t n, int32_t *assign, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    if (c.leaf_aniso_iters > 0)
        return launch_assign_aniso(x, n, c.d, idx->centers.as<float>(), c.n_leaves, c.eta_mode, (double)c.T,
                                   (double)c.eta_explicit, assign, st);
    return launch_assign_nearest(x, n, c.d, idx->centers.as<float>(), c.n_leaves, assign, st);
}

// Theorem 4.2 for every leaf at once: the leaf centers are the codewords of a one-dictionary quantizer whose
// codes are the leaf assignments, so the joint update of Appendix 7.5 with M = 1 is the theorem's closed form.
static int update_leaf_centers(avq_index *idx, const float *x, int64_t n, const int32_t *assign, int max_iters, double tol,
                               int *iters, double *rel, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    const int D = c.n_leaves * c.d;
    DevBuf scratch;
    int rc = scratch.reserve(pq_update_scratch_bytes(n, D, c.n_leaves));
    if (rc == AVQ_OK)
        rc = pq_joint_update_device(x, n, c.d, 1, c.n_leaves, 32, (const uint8_t *)assign, nullptr, nullptr, c.eta_mode,
                                    (double)c.T, (double)c.eta_explicit, idx->centers.as<float>(), scratch.p, max_iters, tol,
                                    iters, rel, st);
    if (rc == AVQ_OK && hipStreamSynchronize(st) != hipSuccess) { set_error("leaf center update: stream error"); rc = AVQ_EHIP; }
    scratch.release();
    if (rc == AVQ_OK) rc = refresh_centers_t(idx, st);
    return rc;
}

extern "C" int avq_train(avq_index *idx, const float *x, int64_t n_train, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (!x || n_train < idx->kc || n_train < c.n_leaves || n_train > 0x7fffffff) {
        set_error("avq_train: need a device pointer and max(k_c, n_leaves) <= n_train < 2^31");
        return AVQ_EINVAL;
    }
    const int32_t *assign = nullptr;
    if (c.n_leaves > 0) {
        // leaf centers from at most 256 rows per leaf, then every training row to its leaf
        const int64_t n_leaf_train = std::min<int64_t>(n_train, (int64_t)256 * c.n_leaves);
        AVQ_TRY(kmeans_device(x, n_leaf_train, c.d, 0, c.d, c.n_leaves, c.leaf_kmeans_iters, c.seed, 0u,
                              nullptr, nullptr, idx->centers.as<float>(), st));
        AVQ_TRY(refresh_centers_t(idx, st));
        idx->have_centers = true;
        AVQ_TRY(idx->tmp.reserve(sizeof(int32_t) * (size_t)n_train));
        // Section 4 with the leaf centers as codewords: alternate the assignment under the anisotropic loss
        // (Definition 4.1) and Theorem 4.2's update, starting from the l2 centers
        for (int it = 0; it < c.leaf_aniso_iters; ++it) {
            AVQ_TRY(launch_assign_aniso(x, n_leaf_train, c.d, idx->centers.as<float>(), c.n_leaves, c.eta_mode, (double)c.T,
                                        (double)c.eta_explicit, idx->tmp.as<int32_t>(), st));
            AVQ_TRY(update_leaf_centers(idx, x, n_leaf_train, idx->tmp.as<int32_t>(), 500, 1e-10, nullptr, nullptr, st));
        }
        AVQ_TRY(assign_to_leaves(idx, x, n_train, idx->tmp.as<int32_t>(), st));
        assign = idx->tmp.as<int32_t>();
    }
    for (int m = 0; m < c.M; ++m)
        AVQ_TRY(kmeans_device(x, n_train, c.d, m * idx->ds, idx->ds, idx->kc, c.kmeans_iters, c.seed,
                              (uint32_t)(1 + m), assign ? idx->centers.as<float>() : nullptr, assign,
                              idx->codebooks.as<float>() + (size_t)m * idx->kc * idx->ds, st));
    AVQ_HIP(hipStreamSynchronize(st));
    idx->have_codebooks = true;
    return AVQ_OK;
}

// ---- database ------------------------------------------------------------------------

// codes_logical (and assign, if partitioned) are on the device; builds the blocked layout.
static int install_database(avq_index *idx, const float *x, int64_t n, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    idx->n = 0;
    if (x && !c.borrow_x) {
        AVQ_TRY(idx->x_own.reserve(sizeof(float) * (size_t)n * c.d));
        AVQ_HIP(hipMemcpyAsync(idx->x_own.p, x, sizeof(float) * (size_t)n * c.d, hipMemcpyDeviceToDevice, st));
        idx->x = idx->x_own.as<float>();
    } else {
        idx->x = x;
    }
    if (c.n_leaves <= 0) {
        idx->n_blocks = (n + kBlockPoints - 1) / kBlockPoints;
        idx->n_slots = idx->n_blocks * kBlockPoints;
        AVQ_TRY(idx->codes_blocked.reserve((size_t)idx->n_slots * idx->NB));
        AVQ_TRY(launch_to_blocked(idx->codes_logical.as<uint8_t>(), n, idx->NB, nullptr,
                                  idx->codes_blocked.as<uint8_t>(), idx->n_slots, st));
    } else {
        // group the points by leaf (ascending id inside a leaf), each leaf padded to whole blocks
        std::vector<int32_t> assign(n);
        AVQ_HIP(hipMemcpyAsync(assign.data(), idx->assign.p, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
        AVQ_HIP(hipStreamSynchronize(st));
        std::vector<int64_t> count(c.n_leaves, 0);
        for (int64_t i = 0; i < n; ++i) {
            if (assign[i] < 0 || assign[i] >= c.n_leaves) {
                set_error("leaf assignment %d of point %lld out of range", assign[i], (long long)i);
                return AVQ_EINVAL;
            }
            count[assign[i]]++;
        }
        std::vector<int32_t> leaf_blk(c.n_leaves + 1);
        int64_t blk = 0;
        idx->max_leaf_blocks = 0;
        for (int l = 0; l < c.n_leaves; ++l) {
            leaf_blk[l] = (int32_t)blk;
            blk += (count[l] + kBlockPoints - 1) / kBlockPoints;
            idx->max_leaf_blocks = std::max<int64_t>(idx->max_leaf_blocks, (count[l] + kBlockPoints - 1) / kBlockPoints);
        }
        leaf_blk[c.n_leaves] = (int32_t)blk;
        if (blk * kBlockPoints > 0x7fffffff) { set_error("index too large"); return AVQ_EINVAL; }
        idx->n_blocks = blk;
        idx->n_slots = blk * kBlockPoints;
        std::vector<int32_t> slot_of(n), perm((size_t)idx->n_slots, -1);
        std::vector<int64_t> next(c.n_leaves);
        for (int l = 0; l < c.n_leaves; ++l) next[l] = (int64_t)leaf_blk[l] * kBlockPoints;
        for (int64_t i = 0; i < n; ++i) {
            const int64_t s = next[assign[i]]++;
            slot_of[i] = (int32_t)s;
            perm[s] = (int32_t)i;
        }
        AVQ_TRY(idx->tmp.reserve(sizeof(int32_t) * (size_t)n));
        AVQ_TRY(idx->perm.reserve(sizeof(int32_t) * (size_t)std::max<int64_t>(idx->n_slots, 1)));
        AVQ_TRY(idx->leaf_blk.reserve(sizeof(int32_t) * (size_t)(c.n_leaves + 1)));
        AVQ_TRY(idx->codes_blocked.reserve((size_t)std::max<int64_t>(idx->n_slots, 1) * idx->NB));
        AVQ_HIP(hipMemcpyAsync(idx->tmp.p, slot_of.data(), sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, st));
        AVQ_HIP(hipMemcpyAsync(idx->perm.p, perm.data(), sizeof(int32_t) * (size_t)idx->n_slots,
                               hipMemcpyHostToDevice, st));
        AVQ_HIP(hipMemcpyAsync(idx->leaf_blk.p, leaf_blk.data(), sizeof(int32_t) * (size_t)(c.n_leaves + 1),
                               hipMemcpyHostToDevice, st));
        AVQ_TRY(launch_to_blocked(idx->codes_logical.as<uint8_t>(), n, idx->NB, idx->tmp.as<int32_t>(),
                                  idx->codes_blocked.as<uint8_t>(), idx->n_slots, st));
        AVQ_HIP(hipStreamSynchronize(st)); // host vectors go out of scope
    }
    AVQ_HIP(hipStreamSynchronize(st));
    idx->n = n;
    return AVQ_OK;
}

static int check_n(int64_t n)
{
    if (n < 1 || n >= 0x7fffffffll - 512) { set_error("n = %lld out of range", (long long)n); return AVQ_EINVAL; }
    return AVQ_OK;
}

extern "C" int avq_set_database(avq_index *idx, const float *x, const uint8_t *packed,
                                const int32_t *leaf_assign, int64_t n, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    AVQ_TRY(check_n(n));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (!packed) { set_error("avq_set_database: packed is NULL"); return AVQ_EINVAL; }
    if ((c.n_leaves > 0) != (leaf_assign != nullptr)) {
        set_error("avq_set_database: leaf_assign must be given exactly for a partitioned index");
        return AVQ_EINVAL;
    }
    if (c.n_leaves > 0 && !idx->have_centers) { set_error("avq_set_database: no leaf centers yet"); return AVQ_ESTATE; }
    AVQ_TRY(idx->codes_logical.reserve((size_t)n * idx->NB));
    AVQ_HIP(hipMemcpyAsync(idx->codes_logical.p, packed, (size_t)n * idx->NB, hipMemcpyDefault, st));
    if (leaf_assign) {
        AVQ_TRY(idx->assign.reserve(sizeof(int32_t) * (size_t)n));
        AVQ_HIP(hipMemcpyAsync(idx->assign.p, leaf_assign, sizeof(int32_t) * (size_t)n, hipMemcpyDefault, st));
    }
    AVQ_HIP(hipStreamSynchronize(st));
    return install_database(idx, x, n, st);
}

extern "C" int avq_encode(avq_index *idx, const float *x, int64_t n, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    AVQ_TRY(check_n(n));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (!x) { set_error("avq_encode: x is NULL"); return AVQ_EINVAL; }
    if (!idx->have_codebooks) { set_error("avq_encode: no dictionaries yet (avq_train first)"); return AVQ_ESTATE; }
    if (c.n_leaves > 0 && !idx->have_centers) { set_error("avq_encode: no leaf centers yet"); return AVQ_ESTATE; }
    AVQ_TRY(idx->codes_logical.reserve((size_t)n * idx->NB));
    const int32_t *assign = nullptr;
    if (c.n_leaves > 0) {
        AVQ_TRY(idx->assign.reserve(sizeof(int32_t) * (size_t)n));
        AVQ_TRY(assign_to_leaves(idx, x, n, idx->assign.as<int32_t>(), st));
        assign = idx->assign.as<int32_t>();
    }
    AVQ_TRY(launch_encode(x, n, c.d, c.M, idx->kc, c.bits, idx->codebooks.as<float>(),
                          assign ? idx->centers.as<float>() : nullptr, assign, c.eta_mode, (double)c.T,
                          (double)c.eta_explicit, c.encode_passes, idx->codes_logical.as<uint8_t>(), st));
    return install_database(idx, x, n, st);
}

extern "C" int avq_update_codebooks(avq_index *idx, const float *x, int64_t n, int32_t max_iters, double tol,
                                    int32_t *iters_out, double *rel_residual_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (!x) { set_error("avq_update_codebooks: x is NULL"); return AVQ_EINVAL; }
    if (idx->n <= 0) { set_error("avq_update_codebooks: no codes yet (avq_encode first)"); return AVQ_ESTATE; }
    if (n != idx->n) {
        set_error("avq_update_codebooks: n = %lld but the codes are of %lld points", (long long)n, (long long)idx->n);
        return AVQ_EINVAL;
    }
    if (max_iters < 1 || !(tol >= 0.0)) { set_error("avq_update_codebooks: max_iters < 1 or tol < 0"); return AVQ_EINVAL; }
    const int ds = c.d / c.M, D = c.M * idx->kc * ds;
    DevBuf scratch;
    int iters = 0;
    double rel = 0.0;
    int rc = scratch.reserve(pq_update_scratch_bytes(n, D, c.M * idx->kc));
    if (rc == AVQ_OK)
        rc = pq_joint_update_device(x, n, c.d, c.M, idx->kc, c.bits, idx->codes_logical.as<uint8_t>(),
                                    c.n_leaves > 0 ? idx->centers.as<float>() : nullptr,
                                    c.n_leaves > 0 ? idx->assign.as<int32_t>() : nullptr, c.eta_mode,
                                    (double)c.T, (double)c.eta_explicit, idx->codebooks.as<float>(), scratch.p,
                                    max_iters, tol, &iters, &rel, st);
    if (rc == AVQ_OK && hipStreamSynchronize(st) != hipSuccess) { set_error("avq_update_codebooks: stream error"); rc = AVQ_EHIP; }
    scratch.release();
    if (rc != AVQ_OK) return rc;
    if (iters_out) *iters_out = iters;
    if (rel_residual_out) *rel_residual_out = rel;
    return AVQ_OK;
}

extern "C" int avq_update_leaf_centers(avq_index *idx, const float *x, int64_t n, int32_t max_iters, double tol,
                                       int32_t *iters_out, double *rel_residual_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (!x) { set_error("avq_update_leaf_centers: x is NULL"); return AVQ_EINVAL; }
    if (c.n_leaves <= 0) { set_error("avq_update_leaf_centers: flat index"); return AVQ_EINVAL; }
    if (idx->n <= 0) { set_error("avq_update_leaf_centers: no database yet (avq_encode first)"); return AVQ_ESTATE; }
    if (n != idx->n) {
        set_error("avq_update_leaf_centers: n = %lld but the stored assignment is of %lld points", (long long)n, (long long)idx->n);
        return AVQ_EINVAL;
    }
    if (max_iters < 1 || !(tol >= 0.0)) { set_error("avq_update_leaf_centers: max_iters < 1 or tol < 0"); return AVQ_EINVAL; }
    int iters = 0;
    double rel = 0.0;
    AVQ_TRY(update_leaf_centers(idx, x, n, idx->assign.as<int32_t>(), max_iters, tol, &iters, &rel, st));
    if (iters_out) *iters_out = iters;
    if (rel_residual_out) *rel_residual_out = rel;
    return AVQ_OK;
}

extern "C" int avq_get_codes(avq_index *idx, uint8_t *out)
{
    AVQ_TRY(check_index(idx));
    if (idx->n <= 0) { set_error("avq_get_codes: no database"); return AVQ_ESTATE; }
    if (!out) { set_error("avq_get_codes: NULL"); return AVQ_EINVAL; }
    AVQ_HIP(hipMemcpy(out, idx->codes_logical.p, (size_t)idx->n * idx->NB, hipMemcpyDefault));
    return AVQ_OK;
}

extern "C" int avq_get_leaf_assign(avq_index *idx, int32_t *out)
{
    AVQ_TRY(check_index(idx));
    if (idx->n <= 0 || idx->cfg.n_leaves <= 0) { set_error("avq_get_leaf_assign: no partitioned database"); return AVQ_ESTATE; }
    if (!out) { set_error("avq_get_leaf_assign: NULL"); return AVQ_EINVAL; }
    AVQ_HIP(hipMemcpy(out, idx->assign.p, sizeof(int32_t) * (size_t)idx->n, hipMemcpyDefault));
    return AVQ_OK;
}

// ---- query path ----------------------------------------------------------------------

static int build_tables(avq_index *idx, const float *queries, int nq, int lut_mode, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    const size_t entries = (size_t)nq * c.M * idx->kc;
    AVQ_TRY(idx->lut.reserve(entries * sizeof(float)));
    if (lut_mode == AVQ_LUT_U8) {
        AVQ_TRY(idx->lut8.reserve(entries));
        AVQ_TRY(idx->scale.reserve(sizeof(float) * (size_t)nq));
        AVQ_TRY(idx->bias.reserve(sizeof(float) * (size_t)nq));
    }
    return launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, idx->lut.as<float>(),
                      lut_mode == AVQ_LUT_U8 ? idx->lut8.as<uint8_t>() : nullptr, idx->scale.as<float>(),
                      idx->bias.as<float>(), st);
}

// The scan of the whole code array for one or a few queries reads an array that does not fit the 256 MB Infinity
// Cache once per query: nontemporal loads and a wave per block then (block_bound_stream_kernel). Measured per call,
// plain against streamed: 320 MB 80 / 73 us for one query, 127 / 118 for two, equal at four, 614 / 766 at sixteen
// (the queries of a call share what the caches hold when few workgroups per query walk the array together);
// 1.6 GB 326 / 262, 606 / 494, 1139 / 967, 2220 / 1899 (eight queries), 3291 / 3765 (sixteen). An array that fits
// the cache stays resident between calls and is loaded the plain way.
static bool stream_loads_nontemporal(const avq_index *idx, int nq)
{
    if (idx->tune_stream_loads == 1) return false;
    if (idx->tune_stream_loads == 2) return true;
    const size_t bytes = (size_t)idx->n_blocks * 256 * (size_t)idx->NB;
    return bytes > ((size_t)256 << 20) && (nq <= 2 || (nq <= 8 && bytes > ((size_t)1 << 30)));
}

static void fill_scan_params(const avq_index *idx, int nq, int R, int ns, ScanParams *p)
{
    memset(p, 0, sizeof(*p));
    p->codes = idx->codes_blocked.as<uint8_t>();
    p->n_blocks = idx->n_blocks;
    p->n_valid = (int32_t)idx->n;
    p->lut = idx->lut.as<float>();
    p->lut8 = idx->lut8.as<uint8_t>();
    p->scale = idx->scale.as<float>();
    p->bias = idx->bias.as<float>();
    p->B = nq;
    p->M = idx->cfg.M;
    p->bits = idx->cfg.bits;
    p->NB = idx->NB;
    p->R = R;
    p->ns = ns;
}

// Chooses the flat scan's grid: query tiles x chunks of the block range.
static void plan_flat(const avq_index *idx, const ScanShape &s, int nq, ScanParams *p)
{
    p->n_tiles = (nq + s.qt - 1) / s.qt;
    // one resident set of workgroups: the fp32 tile of 8 runs two workgroups per compute unit
    const int builtin = (s.qt == 8 && s.lists_global && idx->cfg.bits == 4) ? 512 : 1024;
    const int target = idx->tune_target_wgs > 0 ? idx->tune_target_wgs : builtin;
    int64_t chunks = (target + p->n_tiles - 1) / p->n_tiles;
    if (idx->tune_target_wgs <= 0 && p->n_tiles > target) {
        // more tiles than fit at once: a few chunks per tile so that the last round of workgroups
        // is nearly full (each extra chunk costs about 2 % in list handling)
        double best = 0.0;
        for (int c = 1; c <= 4; ++c) {
            const double rounds = (double)p->n_tiles * c / target;
            const double score = rounds / std::ceil(rounds) * (1.0 - 0.02 * (c - 1));
            if (score > best) { best = score; chunks = c; }
        }
    }
    const int64_t max_chunks = std::max<int64_t>(1, idx->n_blocks / s.waves);
    chunks = std::max<int64_t>(1, std::min(chunks, max_chunks));
    const int64_t bpc = (idx->n_blocks + chunks - 1) / chunks;
    p->blocks_per_chunk = (int32_t)bpc;
    p->n_chunks = (int32_t)((idx->n_blocks + bpc - 1) / bpc);
}

// The matrix-core scan serves batches of 8-bit-table queries on a flat index of 4-bit codes.
static bool use_mfma_scan(const avq_index *idx, int nq, int lut_mode)
{
    return idx->tune_mfma == 0 && lut_mode == AVQ_LUT_U8 && idx->cfg.n_leaves == 0 && nq >= 16 &&
           scan_mfma_supported(idx->NB, idx->cfg.bits);
}

// Batches with fp32 tables on a flat index of 4-bit codes: the matrix-core scan over the 8-bit
// tables collects every point that the rounding of the tables could still place among the R
// best, and those are re-scored and ranked in fp32.
static bool use_prefilter(const avq_index *idx, int nq, int lut_mode, int R)
{
    return idx->tune_prefilter != 1 && idx->tune_mfma == 0 && lut_mode == AVQ_LUT_F32 && idx->cfg.n_leaves == 0 &&
           nq >= 16 && scan_mfma_supported(idx->NB, idx->cfg.bits) && idx->cfg.M <= 64 && idx->n > R;
}

// Whether the matrix-core scan of this batch would be given bounds guessed from a sample.
static bool mfma_scan_samples(const avq_index *idx, int nq, int R, int ns)
{
    if (idx->tune_sample == 1) return false;
    ScanParams p, sample;
    memset(&p, 0, sizeof(p));
    p.R = R;
    p.ns = ns;
    scan_mfma_plan(nq, idx->n_blocks, idx->tune_target_wgs, &p);
    return scan_mfma_sample_plan(p, &sample);
}

// u8: the 8-bit-table search itself through the same machinery (fixed bounds from a sample, kept
// keys ranked by their integer sums: no margin, no fp32 tables); only called when the scan samples.
static int search_through_candidates(avq_index *idx, const float *queries, int nq, int k, int reorder_k, int R, int ns,
                              bool u8, int32_t *ids_out, float *scores_out, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    const int C = 64 * ns;
    // 1. matrix-core scan over the 8-bit tables in candidate mode
    ScanParams pm;
    fill_scan_params(idx, nq, R, ns, &pm);
    scan_mfma_plan(nq, idx->n_blocks, idx->tune_target_wgs, &pm);
    pm.cand_cap = idx->tune_prefilter_cap > 0 ? std::max(128, idx->tune_prefilter_cap) : std::max(2048, 16 * C);
    // 2. the plain fp32 scan for the queries whose candidates cannot be used (no margin, a buffer
    // that overflowed): its grid is cut on the device to the number of such queries
    ScanParams pf;
    fill_scan_params(idx, nq, R, ns, &pf);
    ScanShape shape;
    AVQ_TRY(scan_pick_shape(idx->NB, c.bits, u8, ns, nq, false, 8, idx->tune_waves, &shape));
    pf.n_tiles = (nq + shape.qt - 1) / shape.qt;
    pf.n_chunks = (int32_t)std::max<int64_t>(1, std::min<int64_t>(128, idx->n_blocks / shape.waves)); // at most
    pf.blocks_per_chunk = 0; // derived on the device

    const size_t partial_m = sizeof(u64) * (size_t)nq * pm.n_chunks * C;
    // the plain scan writes (live queries, rounded up to tiles) x chunks lists: at most max(kDynamicItems, tiles) tiles' worth
    const size_t partial_f = sizeof(u64) * (size_t)std::max(kDynamicItems, pf.n_tiles) * shape.qt * C;
    AVQ_TRY(idx->partial.reserve(std::max(partial_m, partial_f)));
    const size_t lists_f = shape.lists_global ? sizeof(u64) * (size_t)std::max(kDynamicItems, pf.n_tiles) * shape.waves * shape.qt * C : 0;
    AVQ_TRY(idx->lists.reserve(std::max(scan_mfma_lists_bytes(pm), lists_f)));
    const size_t thr_bytes = sizeof(uint32_t) * (size_t)nq * (1 + (size_t)pm.n_chunks);
    AVQ_TRY(idx->thr.reserve(thr_bytes));
    AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * C));
    AVQ_TRY(idx->refined.reserve(sizeof(u64) * (size_t)nq * C));
    const size_t row_floats = u8 ? (size_t)c.M * idx->kc / 4 : (size_t)c.M * idx->kc; // a query's tables, in 4-byte units
    AVQ_TRY(idx->lut_fail.reserve(sizeof(float) * (size_t)pf.n_tiles * shape.qt * row_floats));
    // fail: [4] count | [nq] list | [nq] margins | [nq][chunks] candidate counts
    AVQ_TRY(idx->fail.reserve(sizeof(int32_t) * (4 + (size_t)nq * (2 + (size_t)pm.n_chunks))));
    AVQ_TRY(idx->cand_keys.reserve(sizeof(uint32_t) * (size_t)nq * pm.n_chunks * pm.cand_cap));
    uint32_t *fail_count = idx->fail.as<uint32_t>();
    int32_t *fail_list = idx->fail.as<int32_t>() + 4;
    int32_t *margin = fail_list + nq;

    pm.partial = idx->partial.as<u64>();
    pm.lists_ws = idx->lists.as<u64>();
    pm.thr_shared = idx->thr.as<uint32_t>();
    pm.kth_shared = pm.thr_shared + nq;
    pm.cand_keys = idx->cand_keys.as<uint32_t>();
    pm.cand_cnt = (uint32_t *)(margin + nq);
    pm.cand_margin = u8 ? nullptr : margin;
    {
        StageTimer t(idx, AVQ_STAGE_SAMPLE, st);
        AVQ_HIP(hipMemsetAsync(fail_count, 0, 16, st));
        AVQ_HIP(hipMemsetAsync(pm.thr_shared, 0, thr_bytes, st));
        if (!u8) AVQ_TRY(launch_prefilter_margin(idx->lut.as<float>(), idx->scale.as<float>(), c.M, idx->NB, nq, margin, st));
        // guess the bounds from a sample of the index and scan against them, where the index is large
        // enough for that; otherwise the scan keeps lists and raises its bounds itself
        ScanParams sample;
        if (idx->tune_sample != 1 && scan_mfma_sample_plan(pm, &sample)) {
            // The r-th best sum of the sample. With enough waves per query it comes without lists: every wave
            // records the best sum of each of its 32 disjoint point classes, and the r-th largest of a query's
            // class maxima is the r-th best of the sample unless two of those fell into one class (then it is a
            // little lower, which only keeps more points). Otherwise, or when asked, from sorted lists.
            const int classes = sample.n_chunks * 32;
            if (idx->tune_sample != 2 && classes >= 8 * sample.R && classes <= 8192) {
                sample.sample_max = (uint32_t *)idx->lists.p; // the lists' scratch: no launch here keeps lists
                AVQ_TRY(launch_scan_mfma(sample, st));
                AVQ_TRY(launch_sample_bound(sample.sample_max, classes, sample.R, nq, pm.thr_shared, st));
            } else {
                AVQ_TRY(launch_scan_mfma(sample, st));
                const u64 *best = sample.partial;
                if (sample.n_chunks > 1) {
                    AVQ_TRY(launch_merge_partials(sample.partial, nq, sample.n_chunks, sample.ns, idx->cand.as<u64>(), st));
                    best = idx->cand.as<u64>();
                }
                AVQ_TRY(launch_list_bound(best, sample.ns, sample.R, nq, pm.thr_shared, st));
            }
            pm.fixed_bound = 1;
        }
    }
    {
        StageTimer t(idx, AVQ_STAGE_SCAN, st); // the launch over all blocks, nothing else
        AVQ_TRY(launch_scan_mfma(pm, st));
    }
    const u64 *top = pm.fixed_bound ? nullptr : pm.partial;
    if (!pm.fixed_bound && pm.n_chunks > 1) {
        StageTimer t(idx, AVQ_STAGE_MERGE, st);
        AVQ_TRY(launch_merge_partials(pm.partial, nq, pm.n_chunks, ns, idx->cand.as<u64>(), st));
        top = idx->cand.as<u64>();
    }
    {
        StageTimer t(idx, AVQ_STAGE_RESCAN, st);
        RefineCandParams r;
        r.top = top;
        r.bound = pm.fixed_bound ? pm.thr_shared : nullptr;
        r.R = R; r.ns = ns; r.nq = nq; r.M = c.M; r.NB = idx->NB;
        r.n_chunks = pm.n_chunks;
        r.cand_cap = pm.cand_cap;
        r.chunk_points = (int64_t)pm.blocks_per_chunk * kBlockPoints;
        r.cand_keys = pm.cand_keys;
        r.cand_cnt = pm.cand_cnt;
        r.margin = u8 ? nullptr : margin;
        r.lut = u8 ? nullptr : idx->lut.as<float>();
        r.codes = idx->codes_logical.as<uint8_t>();
        r.out = idx->refined.as<u64>();
        r.fail_list = fail_list;
        r.fail_count = fail_count;
        r.force_fail_odd = idx->tune_prefilter == 2;
        AVQ_TRY(launch_refine_cand(r, st));
        // the other queries: their tables side by side, the plain scan over them, and their lists
        // merged into their own rows of the refined candidates
        AVQ_TRY(launch_gather_rows(u8 ? (const float *)idx->lut8.p : idx->lut.as<float>(), idx->lut_fail.as<float>(), fail_list,
                                   fail_count, nq, (int)row_floats, st));
        pf.lut = idx->lut_fail.as<float>();
        pf.lut8 = idx->lut_fail.as<uint8_t>();
        pf.partial = idx->partial.as<u64>(); // the matrix-core scan's lists are merged by now
        if (shape.lists_global) pf.lists_ws = idx->lists.as<u64>();
        pf.active_queries = fail_count;
        AVQ_TRY(launch_scan(pf, u8, SCAN_CHUNK, shape, st));
        AVQ_TRY(launch_merge_partials(pf.partial, nq, pf.n_chunks, ns, idx->refined.as<u64>(), st, fail_list, fail_count,
                                      shape.qt));
    }
    StageTimer t(idx, AVQ_STAGE_FINAL, st);
    return launch_finalize(idx->refined.as<u64>(), ns, nq, R, k, reorder_k != 0, u8 ? 1 : 0, idx->x, c.d, queries,
                           idx->scale.as<float>(), idx->bias.as<float>(), ids_out, scores_out, st);
}

// Batches on a partitioned index of 4-bit codes: the (query, leaf) pairs are regrouped by leaf and
// every leaf is scanned once per 32 of its queries on the matrix cores, against a bound per query
// that the query's best few leaves supply; the kept points are scored and ranked per query.
static bool use_grouped_leaves(const avq_index *idx, int nq, int L, int R)
{
    // below about 1.3e5 pairs (1,300 queries x 100 leaves) one workgroup per query is faster: regrouping, bounds and
    // the hand-over of kept points cost a fixed 0.2 ms
    const int64_t min_pairs = idx->tune_group_min > 0 ? idx->tune_group_min : 100000;
    return idx->tune_prefilter != 1 && idx->tune_mfma == 0 && idx->cfg.n_leaves > 0 && nq >= 64 && nq <= (1 << 16) &&
           (int64_t)nq * L >= min_pairs &&
           scan_mfma_supported(idx->NB, idx->cfg.bits) && idx->cfg.M <= 64 && L >= 16 && L <= 512 &&
           idx->cfg.n_leaves <= (1 << 21) && idx->max_leaf_blocks <= 1024 && R <= 2048;
}

static int search_leaves_grouped(avq_index *idx, const float *queries, int nq, int k, int reorder_k, int R, int ns, int L,
                                 bool u8, int32_t *ids_out, float *scores_out, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    const int C = 64 * ns;
    AVQ_TRY(idx->leaf_ids.reserve(sizeof(int32_t) * (size_t)nq * L));
    AVQ_TRY(idx->leaf_ip.reserve(sizeof(float) * (size_t)nq * L));
    AVQ_TRY(idx->groups.reserve(sizeof(uint32_t) * group_by_leaf_words(nq, L, c.n_leaves)));
    LeafGroups g;
    {
        StageTimer t(idx, AVQ_STAGE_LEAF, st);
        AVQ_TRY(group_by_leaf_prepare(nq, L, c.n_leaves, idx->groups.as<uint32_t>(), &g, st));
        AVQ_TRY(launch_leaf_select(idx->centers_t.as<float>(), c.n_leaves, c.d, queries, nq, L,
                                   idx->leaf_ids.as<int32_t>(), idx->leaf_ip.as<float>(), st, g.cnt_wide, g.pos, g.cnt_stride));
    }
    // scratch: [4] counts | [nq] unverified queries | [nq] margins | [nq] bounds | [nq] kept counts
    AVQ_TRY(idx->fail.reserve(sizeof(int32_t) * (4 + (size_t)4 * nq)));
    uint32_t *fail_count = idx->fail.as<uint32_t>();
    int32_t *fail_list = idx->fail.as<int32_t>() + 4;
    int32_t *margin = fail_list + nq;
    uint32_t *bound = (uint32_t *)(margin + nq);
    uint32_t *kept_cnt = bound + nq;
    const int kept_cap = idx->tune_prefilter_cap > 0 ? std::min(4096, std::max(128, idx->tune_prefilter_cap)) : 2048;
    AVQ_TRY(idx->kept.reserve(sizeof(u64) * (size_t)nq * kept_cap));
    AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * C));
    AVQ_TRY(idx->refined.reserve(sizeof(u64) * (size_t)nq * C));

    // the plain scan over leaves, used twice: over the first leaves of every query for the bounds, and
    // over all leaves of the queries that are handed back
    ScanShape shape;
    const int waves_hint = idx->tune_waves > 0 ? idx->tune_waves : 0;
    AVQ_TRY(scan_pick_shape(idx->NB, c.bits, u8, ns, nq, true, idx->tune_qt, waves_hint, &shape));
    ScanParams pl;
    fill_scan_params(idx, nq, R, ns, &pl);
    pl.perm = idx->perm.as<int32_t>();
    pl.leaf_ids = idx->leaf_ids.as<int32_t>();
    pl.leaf_ip = idx->leaf_ip.as<float>();
    pl.leaf_blk = idx->leaf_blk.as<int32_t>();
    pl.n_tiles = nq;
    pl.n_chunks = 1;
    AVQ_TRY(idx->partial.reserve(sizeof(u64) * (size_t)nq * C));
    pl.partial = idx->partial.as<u64>();
    if (shape.lists_global) {
        AVQ_TRY(idx->lists.reserve(sizeof(u64) * (size_t)nq * shape.waves * shape.qt * C));
        pl.lists_ws = idx->lists.as<u64>();
    }
    const int bound_leaves = idx->tune_bound_leaves > 0 ? std::min(L, idx->tune_bound_leaves) : std::min(L, std::max(8, u8 ? (L + 11) / 12 : (2 * L + 24) / 25));
    ScanParams pi;
    {
        StageTimer t(idx, AVQ_STAGE_SAMPLE, st); // here: margins, bounds from the first leaves, regrouping
        AVQ_HIP(hipMemsetAsync(fail_count, 0, 16, st));
        AVQ_HIP(hipMemsetAsync(kept_cnt, 0, sizeof(uint32_t) * (size_t)nq, st));
        if (!u8) AVQ_TRY(launch_prefilter_margin(idx->lut.as<float>(), idx->scale.as<float>(), c.M, idx->NB, nq, margin, st));
        ScanParams pb = pl;
        pb.Lp = bound_leaves;
        pb.leaf_stride = L;
        if (idx->max_leaf_blocks <= kLeafBoundMaxBlocks) {
            AVQ_TRY(launch_leaf_bound(pb, u8, (int)idx->max_leaf_blocks, (int)((idx->n_blocks + c.n_leaves - 1) / c.n_leaves), bound, st));
        } else {
            AVQ_TRY(launch_scan(pb, u8, SCAN_LEAVES, shape, st));
            AVQ_TRY(launch_list_bound(pb.partial, ns, R, nq, bound, st));
        }
        AVQ_TRY(launch_group_by_leaf(idx->leaf_ids.as<int32_t>(), nq, L, c.n_leaves, g, st));
        fill_scan_params(idx, nq, R, ns, &pi);
        pi.n_valid = 0x7fffffff; // padding slots are told from points by perm, afterwards
        pi.leaf_blk = idx->leaf_blk.as<int32_t>();
        pi.leaf_ip = idx->leaf_ip.as<float>();
        pi.Lp = L;
        pi.leaf_stride = L;
        pi.item_list = g.item_list;
        pi.n_items = g.n_items;
        pi.qlist = g.qlist;
        pi.leaf_off = g.leaf_off;
        pi.leaf_cnt = g.leaf_cnt;
        pi.max_items = g.max_items;
        pi.item_bound = bound;
        pi.cand_margin = u8 ? nullptr : margin;
        pi.kept = idx->kept.as<u64>();
        pi.kept_cnt = kept_cnt;
        pi.kept_cap = kept_cap;
    }
    {
        StageTimer t(idx, AVQ_STAGE_SCAN, st); // the scan over all leaves, nothing else
        AVQ_TRY(launch_scan_mfma(pi, st));
    }
    {
        StageTimer t(idx, AVQ_STAGE_RESCAN, st);
        IvfRefineParams r;
        r.kept = idx->kept.as<u64>();
        r.kept_cnt = kept_cnt;
        r.kept_cap = kept_cap;
        r.R = R; r.ns = ns; r.nq = nq; r.M = c.M; r.NB = idx->NB; r.leaf_stride = L;
        r.lut = u8 ? nullptr : idx->lut.as<float>();
        r.scale = idx->scale.as<float>();
        r.bias = idx->bias.as<float>();
        r.leaf_ip = idx->leaf_ip.as<float>();
        r.margin = u8 ? nullptr : margin;
        r.leaf_blk = idx->leaf_blk.as<int32_t>();
        r.perm = idx->perm.as<int32_t>();
        r.codes = idx->codes_logical.as<uint8_t>();
        r.out = idx->refined.as<u64>();
        r.fail_list = fail_list;
        r.fail_count = fail_count;
        r.force_fail_odd = idx->tune_prefilter == 2;
        AVQ_TRY(launch_ivf_refine(r, st));
        // the queries handed back: their rows (tables, scale, bias, probed leaves) side by side, the plain
        // scan over all their leaves, and their lists into their own rows of the refined candidates
        const size_t lut_row = u8 ? (size_t)c.M * idx->kc / 4 : (size_t)c.M * idx->kc; // 4-byte units
        AVQ_TRY(idx->lut_fail.reserve(sizeof(float) * (size_t)nq * lut_row));
        AVQ_TRY(idx->fail_rows.reserve(sizeof(float) * (size_t)nq * (2 + (size_t)2 * L)));
        float *scale_c = idx->fail_rows.as<float>(), *bias_c = scale_c + nq;
        float *ip_c = bias_c + nq;
        int32_t *ids_c = (int32_t *)(ip_c + (size_t)nq * L);
        AVQ_TRY(launch_gather_rows(u8 ? (const float *)idx->lut8.p : idx->lut.as<float>(), idx->lut_fail.as<float>(), fail_list,
                                   fail_count, nq, (int)lut_row, st));
        AVQ_TRY(launch_gather_rows(idx->scale.as<float>(), scale_c, fail_list, fail_count, nq, 1, st));
        AVQ_TRY(launch_gather_rows(idx->bias.as<float>(), bias_c, fail_list, fail_count, nq, 1, st));
        AVQ_TRY(launch_gather_rows(idx->leaf_ip.as<float>(), ip_c, fail_list, fail_count, nq, L, st));
        AVQ_TRY(launch_gather_rows((const float *)idx->leaf_ids.p, (float *)ids_c, fail_list, fail_count, nq, L, st));
        // few queries, one workgroup each: as many waves per workgroup as the kernel takes
        ScanShape shape_f;
        AVQ_TRY(scan_pick_shape(idx->NB, c.bits, u8, ns, nq, true, idx->tune_qt, waves_hint ? waves_hint : 16, &shape_f));
        ScanParams pf = pl;
        pf.lut = idx->lut_fail.as<float>();
        pf.lut8 = idx->lut_fail.as<uint8_t>();
        pf.scale = scale_c;
        pf.bias = bias_c;
        pf.leaf_ip = ip_c;
        pf.leaf_ids = ids_c;
        pf.Lp = L;
        pf.active_queries = fail_count;
        AVQ_TRY(launch_scan(pf, u8, SCAN_LEAVES, shape_f, st));
        AVQ_TRY(launch_merge_partials(pf.partial, nq, 1, ns, idx->refined.as<u64>(), st, fail_list, fail_count, 0));
    }
    StageTimer t(idx, AVQ_STAGE_FINAL, st);
    return launch_finalize(idx->refined.as<u64>(), ns, nq, R, k, reorder_k != 0, 0, idx->x, c.d, queries,
                           idx->scale.as<float>(), idx->bias.as<float>(), ids_out, scores_out, st);
}

static int check_query_args(const avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode)
{
    if (idx->n <= 0) { set_error("no database yet (avq_encode or avq_set_database first)"); return AVQ_ESTATE; }
    if (!idx->have_codebooks) { set_error("no dictionaries yet"); return AVQ_ESTATE; }
    if (!queries || nq < 1) { set_error("queries NULL or nq < 1"); return AVQ_EINVAL; }
    if (lut_mode != AVQ_LUT_F32 && lut_mode != AVQ_LUT_U8) { set_error("bad lut_mode %d", lut_mode); return AVQ_EINVAL; }
    return AVQ_OK;
}

// ---- a handful of queries on a flat index ------------------------------------------------
// Full scan recording block maxima, selection of the R best blocks, scan of those, final
// selection with exact re-scoring. Its device scratch is described by SmallWs, so that the
// same launches can run from buffers the index owns (avq_search) or from the library's static
// scratch array (avq_search_noalloc).
struct SmallWs {
    float *lut;          // [nq][M][kc]      (unused when the scan computes its own tables)
    uint8_t *lut8;       // [nq][M][kc]      (8-bit tables only)
    float *scale, *bias; // [nq]             (8-bit tables only)
    u64 *block_max;      // [nq][n_blocks]
    u64 *cand;           // [nq][256 * R]
    int32_t *sel_blk;    // [nq][R], or [nq][n_blocks] on the block-bound path
    SmallMeta *meta;     // [nq]
    uint32_t *block_bound; // [nq][n_blocks]   (block-bound path)
    BoundMeta *bound_meta; // [nq]             (block-bound path)
    uint8_t *bound_tbl;    // [nq][NB][256]    (block-bound path)
    uint32_t *sel_hist;    // [nq][8192]       (block-bound path, selection over several workgroups per query)
    u64 *fin_out;          // [nq][R]          (exact re-scoring over several workgroups per query)
    uint32_t *fin_n;       // [nq][2]
};

// 0: the scan records block maxima of 8-bit sums (bounds of the scores) where the code size has its
// kernels; 2 (tuning "small_batch_impl"): always the exact block maxima.
static bool small_uses_bounds(const avq_index *idx)
{
    return idx->tune_small_impl == 0 && block_bound_supported(idx->NB, idx->cfg.bits);
}

// Blocks per workgroup when the selection of a query's blocks is spread over several workgroups; 0: one workgroup
// per query. Built in: a few queries on an index of 32,768 blocks or more, where one compute unit's two passes over
// the block maxima take longer than everything else after the scan. Tuning "select_split": 1 never, v >= 2: always,
// v blocks per workgroup.
static int small_select_split_per(const avq_index *idx, int nq)
{
    if (!small_uses_bounds(idx) || idx->tune_select_split == 1) return 0;
    if (idx->tune_select_split >= 2) return std::min(idx->tune_select_split, 8192);
    return nq <= 16 && idx->n_blocks >= 32768 ? 8192 : 0;
}

// Candidates per workgroup when the exact re-scoring of a query's candidates is spread over several workgroups; 0:
// the final kernel does it. Built in: up to 16 queries whose R rows of d values one workgroup would stage in more
// than one pass (its LDS holds `stage_rows` of them): 64 rows per workgroup. Tuning "rerank_split": 1 never,
// v >= 2: always, v rows per workgroup (as many as fit LDS at most).
static int small_rerank_rows(const avq_index *idx, int nq, int R, int stage_rows, bool reorder)
{
    if (!reorder || idx->tune_rerank_split == 1) return 0;
    const int fit = (int)std::min<size_t>(1024, ((size_t)128 * 1024) / ((size_t)(idx->cfg.d + 1) * 4));
    if (fit < 1) return 0;
    if (idx->tune_rerank_split >= 2) return std::min(idx->tune_rerank_split, fit);
    return nq <= 16 && R > stage_rows ? std::min(64, fit) : 0;
}

// Lays the scratch out from `base` (256-byte aligned pieces); returns the bytes needed.
// base == NULL: only the size.
static size_t small_ws_carve(const avq_index *idx, int nq, int R, unsigned char *base, SmallWs *w)
{
    const int nq_tiles = (nq + 15) / 16 * 16; // the batch form of the block-bound scan lays its tables out in tiles of 16
    size_t off = 0;
    auto take = [&](size_t bytes) -> void * {
        const size_t at = (off + 255) & ~(size_t)255;
        off = at + bytes;
        return base ? (void *)(base + at) : nullptr;
    };
    const size_t entries = (size_t)nq * idx->cfg.M * idx->kc;
    w->lut = (float *)take(entries * sizeof(float));
    w->lut8 = (uint8_t *)take(entries);
    w->scale = (float *)take(sizeof(float) * (size_t)nq);
    w->bias = (float *)take(sizeof(float) * (size_t)nq);
    w->block_max = (u64 *)take(sizeof(u64) * (size_t)nq * idx->n_blocks);
    w->cand = (u64 *)take(sizeof(u64) * (size_t)nq * 256 * R);
    const bool bounds = small_uses_bounds(idx);
    w->sel_blk = (int32_t *)take(sizeof(int32_t) * (size_t)nq * (bounds ? (size_t)idx->n_blocks : (size_t)R));
    w->meta = (SmallMeta *)take(sizeof(SmallMeta) * (size_t)nq);
    w->block_bound = (uint32_t *)take(bounds ? sizeof(uint32_t) * (size_t)nq * idx->n_blocks : 0);
    w->bound_meta = (BoundMeta *)take(bounds ? sizeof(BoundMeta) * (size_t)nq : 0);
    w->bound_tbl = (uint8_t *)take(bounds ? (size_t)nq_tiles * idx->NB * 256 : 0);
    const bool split = small_select_split_per(idx, nq) > 0;
    w->sel_hist = (uint32_t *)take(split ? sizeof(uint32_t) * (size_t)nq * 8192 : 0);
    w->fin_out = (u64 *)take(sizeof(u64) * (size_t)nq * R);
    w->fin_n = (uint32_t *)take(sizeof(uint32_t) * (size_t)nq * 2);
    return off;
}

static int small_ws_from_index(avq_index *idx, int nq, int R, SmallWs *w)
{
    const size_t bytes = small_ws_carve(idx, nq, R, nullptr, w);
    AVQ_TRY(idx->tmp.reserve(bytes));
    small_ws_carve(idx, nq, R, (unsigned char *)idx->tmp.p, w);
    return AVQ_OK;
}

// Launches only: no allocation, no synchronisation. timers: per-stage event pairs while profiling is on.
// tile: the batch form (8-bit codes): the full scan takes the queries sixteen at a time, with 6-bit byte tables.
static int search_small(avq_index *idx, const float *queries, int nq, int k, int reorder_k, bool u8, bool fuse_tables,
                        const SmallWs &w, bool timers, int32_t *ids_out, float *scores_out, hipStream_t st, bool tile = false)
{
    const avq_config &c = idx->cfg;
    const int R = reorder_k ? reorder_k : k;
    const int ns = (R + 63) / 64;
    const bool bounds = small_uses_bounds(idx);
    if (!fuse_tables) {
        StageTimer t(idx, AVQ_STAGE_LUT, st, timers);
        AVQ_TRY(launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, w.lut, u8 ? w.lut8 : nullptr, w.scale,
                           w.bias, st));
    }
    ScanParams p;
    fill_scan_params(idx, nq, R, ns, &p);
    p.lut = w.lut;
    p.lut8 = w.lut8;
    p.scale = w.scale;
    p.bias = w.bias;
    if (fuse_tables) {
        p.fuse_queries = queries;
        p.fuse_codebooks = idx->codebooks.as<float>();
        p.fuse_d = c.d;
    }
    p.block_max = w.block_max;
    p.n_tiles = nq;
    p.n_chunks = 1;
    p.max_wgs = idx->tune_target_wgs;
    p.nt_loads = stream_loads_nontemporal(idx, nq) ? 1 : 0;
    p.block_bound = w.block_bound;
    p.bound_meta = w.bound_meta;
    p.lut_out = fuse_tables ? w.lut : nullptr;
    p.bound_tbl = w.bound_tbl;
    p.sel_split_per = small_select_split_per(idx, nq);
    if (p.sel_split_per > 0) p.sel_hist = w.sel_hist;
    if (tile) {
        p.bound_tile = 16;
        // Entries of 6, 7 or 8 bits (tuning "bound_bits"): each bit more halves the width of the bounds, so fewer
        // blocks are scored exactly, and halves how many entries the full scan adds as packed bytes before it must
        // spread them into 16-bit sums. Seven is the best of the three at 1.2 and at 50 million points.
        const int bits_e = idx->tune_bound_bits >= 6 && idx->tune_bound_bits <= 8 ? idx->tune_bound_bits : 7;
        p.bound_levels = (1 << bits_e) - 1;
        p.bound_shift = 8 - bits_e;
        p.blocks_per_chunk = block_bound_tile_chunk(idx->n_blocks, nq);
    }
    if (bounds) {
        StageTimer t(idx, AVQ_STAGE_LUT, st, timers);
        AVQ_TRY(launch_bound_tables(p, u8, st));
    }
    {
        StageTimer t(idx, AVQ_STAGE_SCAN, st, timers);
        if (bounds && tile) AVQ_TRY(launch_block_bound_tile(p, st));
        else if (bounds) AVQ_TRY(launch_block_bound(p, idx->tune_waves, st));
        else AVQ_TRY(launch_block_max(p, u8, idx->tune_waves > 0 ? idx->tune_waves : 4, st));
    }
    FinishParams f;
    memset(&f, 0, sizeof(f));
    f.x = idx->x;
    f.queries = queries;
    f.d = c.d;
    f.k = k;
    f.reorder = reorder_k != 0;
    f.stage_rows = small_finish_stage_rows(p, c.d, u8);
    f.cand_stride = (int64_t)256 * R;
    f.cand = w.cand;
    f.sel_blk = w.sel_blk;
    f.meta = w.meta;
    f.ids_out = ids_out;
    f.scores_out = scores_out;
    f.rerank_rows = small_rerank_rows(idx, nq, R, f.stage_rows, f.reorder != 0);
    f.fin_out = w.fin_out;
    f.fin_n = w.fin_n;
    if (bounds) {
        f.block_max = w.block_max;
        f.n_blocks = idx->n_blocks;
        f.n_valid = (int32_t)idx->n;
        f.NB = idx->NB;
        f.M = c.M;
        f.bits = c.bits;
        f.u8 = u8 ? 1 : 0;
        f.codes_logical = idx->codes_logical.as<uint8_t>();
        f.lut = w.lut;
        f.lut8 = w.lut8;
    }
    {
        StageTimer t(idx, AVQ_STAGE_MERGE, st, timers);
        if (bounds) AVQ_TRY(launch_select_bound_blocks(p, f, u8, st));
        else AVQ_TRY(launch_small_select(p, f, st));
    }
    {
        StageTimer t(idx, AVQ_STAGE_RESCAN, st, timers);
        if (bounds) AVQ_TRY(launch_rescan_listed(p, f, u8, st));
        else AVQ_TRY(launch_small_rescan(p, f, u8, st));
    }
    StageTimer t(idx, AVQ_STAGE_FINAL, st, timers);
    return launch_small_final(p, f, u8, st);
}


static int check_search_args(const avq_index *idx, const float *queries, int32_t nq, int32_t k, int32_t reorder_k,
                             int32_t lut_mode, int32_t leaves_to_search, const int32_t *ids_out, const float *scores_out)
{
    AVQ_TRY(check_index(idx));
    AVQ_TRY(check_query_args(idx, queries, nq, lut_mode));
    const avq_config &c = idx->cfg;
    if (!ids_out || !scores_out) { set_error("avq_search: output pointer is NULL"); return AVQ_EINVAL; }
    if (k < 1 || k > AVQ_MAX_SELECT || k > idx->n || (reorder_k != 0 && (reorder_k < k || reorder_k > AVQ_MAX_SELECT))) {
        set_error("avq_search: need 1 <= k <= min(n, %d) and reorder_k == 0 or k <= reorder_k <= %d",
                  AVQ_MAX_SELECT, AVQ_MAX_SELECT);
        return AVQ_EINVAL;
    }
    if (reorder_k != 0 && !idx->x) { set_error("avq_search: re-scoring needs the datapoints"); return AVQ_ESTATE; }
    if (c.n_leaves > 0 && (leaves_to_search < 1 || leaves_to_search > c.n_leaves || leaves_to_search > AVQ_MAX_SELECT)) {
        set_error("avq_search: leaves_to_search must be in [1, min(n_leaves, %d)]", AVQ_MAX_SELECT);
        return AVQ_EINVAL;
    }
    return AVQ_OK;
}

// ---- a handful of queries on a partitioned index -------------------------------------------
// Leaf selection, exact block maxima over the blocks of the probed leaves, selection of the R best blocks, the
// points of those at or above the R-th best maximum, final selection with exact re-scoring: the first design of the
// flat small-batch path, run on the few hundred blocks a query probes. Up to this many queries (measured crossover
// with the one-query-per-workgroup scan over leaves, which keeps sorted lists per wave: between 64 and 96 queries at
// 100 of 2,000 leaves).
constexpr int kLeafSmallMaxQueries = 80;
static bool use_leaf_small(const avq_index *idx, int nq, int L)
{
    const int max_q = idx->tune_small_batch >= 0 ? std::min(idx->tune_small_batch, 4096) : kLeafSmallMaxQueries;
    return idx->cfg.n_leaves > 0 && idx->tune_small_impl != 1 && nq <= max_q && L <= 512 &&
           leaf_small_supported(idx->NB, idx->cfg.bits);
}

static int search_leaves_small(avq_index *idx, const float *queries, int nq, int k, int reorder_k, int R, int L, bool u8,
                               int32_t *ids_out, float *scores_out, hipStream_t st)
{
    const avq_config &c = idx->cfg;
    const int ns = (R + 63) / 64;
    // a few queries: every workgroup computes the short fp32 tables itself (one launch less); more: the table kernel
    const bool fuse_tables = nq <= 4 && small_batch_can_fuse_tables(c.bits, c.M, c.d, u8);
    const int64_t stride = std::min<int64_t>(idx->n_blocks, (int64_t)L * std::max<int64_t>(1, idx->max_leaf_blocks));
    // scratch, 256-byte aligned pieces of idx->tmp
    size_t off = 0;
    auto take = [&](size_t bytes) -> size_t { const size_t at = (off + 255) & ~(size_t)255; off = at + bytes; return at; };
    const size_t entries = (size_t)nq * c.M * idx->kc;
    const size_t o_lut = take(entries * sizeof(float)), o_lut8 = take(entries), o_scale = take(sizeof(float) * (size_t)nq),
                 o_bias = take(sizeof(float) * (size_t)nq), o_best = take(sizeof(u64) * (size_t)nq * stride),
                 o_blk = take(sizeof(int32_t) * (size_t)nq * stride), o_ip = take(sizeof(float) * (size_t)nq * stride),
                 o_n = take(sizeof(uint32_t) * (size_t)nq), o_sel = take(sizeof(int32_t) * (size_t)nq * R),
                 o_meta = take(sizeof(SmallMeta) * (size_t)nq), o_cand = take(sizeof(u64) * (size_t)nq * 256 * R),
                 o_keys = take(sizeof(u64) * (size_t)nq * c.n_leaves);
    AVQ_TRY(idx->tmp.reserve(off));
    unsigned char *base = (unsigned char *)idx->tmp.p;
    AVQ_TRY(idx->leaf_ids.reserve(sizeof(int32_t) * (size_t)nq * L));
    AVQ_TRY(idx->leaf_ip.reserve(sizeof(float) * (size_t)nq * L));
    {
        StageTimer t(idx, AVQ_STAGE_LEAF, st);
        AVQ_TRY(launch_leaf_select_few(idx->centers_t.as<float>(), c.n_leaves, c.d, queries, nq, L, (u64 *)(base + o_keys),
                                       idx->leaf_ids.as<int32_t>(), idx->leaf_ip.as<float>(), st));
    }
    ScanParams p;
    fill_scan_params(idx, nq, R, ns, &p);
    p.lut = (float *)(base + o_lut);
    p.lut8 = base + o_lut8;
    p.scale = (float *)(base + o_scale);
    p.bias = (float *)(base + o_bias);
    if (fuse_tables) {
        p.fuse_queries = queries;
        p.fuse_codebooks = idx->codebooks.as<float>();
        p.fuse_d = c.d;
    } else {
        StageTimer t(idx, AVQ_STAGE_LUT, st);
        AVQ_TRY(launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, (float *)(base + o_lut),
                           u8 ? base + o_lut8 : nullptr, (float *)(base + o_scale), (float *)(base + o_bias), st));
    }
    p.perm = idx->perm.as<int32_t>();
    p.leaf_ids = idx->leaf_ids.as<int32_t>();
    p.leaf_ip = idx->leaf_ip.as<float>();
    p.leaf_blk = idx->leaf_blk.as<int32_t>();
    p.Lp = L;
    LeafSmallBuffers b;
    b.best = (u64 *)(base + o_best);
    b.blk = (int32_t *)(base + o_blk);
    b.ip = (float *)(base + o_ip);
    b.n_listed = (uint32_t *)(base + o_n);
    b.stride = stride;
    FinishParams f;
    memset(&f, 0, sizeof(f));
    f.x = idx->x;
    f.queries = queries;
    f.d = c.d;
    f.k = k;
    f.reorder = reorder_k != 0;
    f.stage_rows = small_finish_stage_rows(p, c.d, u8);
    f.cand_stride = (int64_t)256 * R;
    f.cand = (u64 *)(base + o_cand);
    f.sel_blk = (int32_t *)(base + o_sel);
    f.meta = (SmallMeta *)(base + o_meta);
    f.ids_out = ids_out;
    f.scores_out = scores_out;
    {
        StageTimer t(idx, AVQ_STAGE_SCAN, st);
        AVQ_TRY(launch_leaf_block_max(p, u8, b, st));
    }
    {
        StageTimer t(idx, AVQ_STAGE_MERGE, st);
        AVQ_TRY(launch_select_listed_blocks(p, f, b, st));
    }
    {
        StageTimer t(idx, AVQ_STAGE_RESCAN, st);
        AVQ_TRY(launch_rescan_leaf_blocks(p, f, u8, b, st));
    }
    StageTimer t(idx, AVQ_STAGE_FINAL, st);
    return launch_small_final(p, f, false, st); // keys carry fp32 scores with either kind of table
}

extern "C" int avq_search(avq_index *idx, const float *queries, int32_t nq, int32_t k, int32_t reorder_k,
                          int32_t lut_mode, int32_t leaves_to_search, int32_t *ids_out, float *scores_out,
                          void *hip_stream)
{
    AVQ_TRY(check_search_args(idx, queries, nq, k, reorder_k, lut_mode, leaves_to_search, ids_out, scores_out));
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    const bool ivf = c.n_leaves > 0;
    const int R = reorder_k ? reorder_k : k;
    const int ns = (R + 63) / 64;
    const int C = 64 * ns;
    const bool u8 = lut_mode == AVQ_LUT_U8;

    // 4-bit codes: the block-maxima path costs about 4.5 us per query and million points, the batch scans a fixed
    // 0.2 ms per million points up to a few hundred queries: measured crossover near 36 queries
    // 8-bit codes: a query by itself costs a scan of its own, sixteen together about one scan and a half (byte
    // tables side by side): the tile of sixteen wins from about 120,000 query-blocks on (24 queries at 1.2 million
    // points, 4 at 8 million), where the code size has the kernels for it; else up to 8 queries
    // 4-bit codes: the per-query path costs about 40 us + (0.1 + 0.00093 x blocks) us per query, the batch path
    // 150 us + 0.017 us per block up to a few hundred queries -- or 600 us on an index so small that its bounds
    // cannot be guessed from the class maxima of a sample and sorted lists take nearly every point. Measured
    // crossovers: 36 to 44 queries at 1.2 million points, 20 at 10 million, about 200 at 100,000, thousands at
    // 10,000 points.
    int small_max = c.bits == 4 ? (idx->n_blocks < 12000 ? 35 : 20) : 8; // code sizes without kernels of their own: as measured at first
    if (c.bits == 4 && small_uses_bounds(idx)) {
        const double nb = (double)idx->n_blocks;
        double batch_us = 150.0 + 0.017 * nb;
        ScanParams plan, sample;
        fill_scan_params(idx, nq, R, ns, &plan);
        scan_mfma_plan(nq, idx->n_blocks, idx->tune_target_wgs, &plan);
        const bool guessed = scan_mfma_sample_plan(plan, &sample) && sample.n_chunks * 32 >= 8 * sample.R && sample.n_chunks * 32 <= 8192;
        if (!guessed) batch_us = 600.0;
        small_max = (int)std::min(4096.0, std::max(8.0, (batch_us - 40.0) / (0.1 + 0.00093 * nb)));
    }
    if (c.bits == 8 && block_bound_supported(idx->NB, c.bits) && idx->tune_small_impl == 0)
        // two queries at least: measured per call, per-query path / batch path, at 8, 20 and 50 million points:
        // 125 / 165, 229 / 399 and 500 / 716 us for two queries, equal for three
        small_max = (int)std::min<int64_t>(32, std::max<int64_t>(2, 120000 / std::max<int64_t>(1, idx->n_blocks)));
    if (idx->tune_small_batch >= 0) small_max = idx->tune_small_batch;
    const bool small = !ivf && nq <= small_max;
    // the single-query kernels compute short fp32 tables themselves (one launch less)
    const bool fuse_tables = small && idx->tune_small_impl != 1 && small_batch_can_fuse_tables(c.bits, c.M, c.d, u8);
    const bool prefilter = !small && use_prefilter(idx, nq, lut_mode, R);
    const bool grouped = ivf && use_grouped_leaves(idx, nq, leaves_to_search, R);
    if (ivf && use_leaf_small(idx, nq, leaves_to_search))
        return search_leaves_small(idx, queries, nq, k, reorder_k, R, leaves_to_search, u8, ids_out, scores_out, st);
    if (small && idx->tune_small_impl != 1) {
        SmallWs w;
        AVQ_TRY(small_ws_from_index(idx, nq, R, &w));
        return search_small(idx, queries, nq, k, reorder_k, u8, fuse_tables, w, true, ids_out, scores_out, st);
    }
    // Batches of 8-bit codes on a flat index: the same search through block bounds, the full scan taking the queries
    // sixteen at a time (byte tables of six bits); "scan_prefilter" = 1 scores every point instead
    if (!ivf && !small && c.bits == 8 && idx->tune_prefilter != 1 && small_uses_bounds(idx)) {
        SmallWs w;
        AVQ_TRY(small_ws_from_index(idx, nq, R, &w));
        return search_small(idx, queries, nq, k, reorder_k, u8, false, w, true, ids_out, scores_out, st, true);
    }
    if (!fuse_tables) {
        StageTimer t(idx, AVQ_STAGE_LUT, st);
        AVQ_TRY(build_tables(idx, queries, nq, (prefilter || grouped) ? AVQ_LUT_U8 : lut_mode, st));
    }
    if (grouped) return search_leaves_grouped(idx, queries, nq, k, reorder_k, R, ns, leaves_to_search, u8, ids_out, scores_out, st);
    if (prefilter) return search_through_candidates(idx, queries, nq, k, reorder_k, R, ns, false, ids_out, scores_out, st);
    ScanParams p;
    fill_scan_params(idx, nq, R, ns, &p);
    const int key_kind = (u8 && !ivf) ? 1 : 0;
    if (small) {
        // three-kernel variant of the same algorithm (kept as a cross-check)
        AVQ_TRY(idx->block_max.reserve(sizeof(u64) * (size_t)nq * idx->n_blocks));
        AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * C));
        AVQ_TRY(idx->partial.reserve(sizeof(u64) * (size_t)nq * C));
        p.block_max = idx->block_max.as<u64>();
        p.block_keys = idx->cand.as<u64>();
        p.partial = idx->partial.as<u64>();
        p.n_tiles = nq;
        p.n_chunks = 1;
        p.max_wgs = idx->tune_target_wgs;
        {
            StageTimer t(idx, AVQ_STAGE_SCAN, st);
            AVQ_TRY(launch_block_max(p, u8, idx->tune_waves > 0 ? idx->tune_waves : 4, st));
        }
        {
            StageTimer t(idx, AVQ_STAGE_MERGE, st);
            AVQ_TRY(launch_select_keys(p.block_max, nq, idx->n_blocks, ns, R, idx->cand.as<u64>(), st));
        }
        ScanShape shape;
        int rc = AVQ_EINVAL;
        for (int w16 = 16; w16 >= 1 && rc != AVQ_OK; w16 /= 2) rc = scan_pick_shape(idx->NB, idx->cfg.bits, u8, ns, nq, true, 1, w16, &shape);
        AVQ_TRY(rc);
        {
            StageTimer t(idx, AVQ_STAGE_RESCAN, st);
            AVQ_TRY(launch_scan(p, u8, SCAN_BLOCKLIST, shape, st));
        }
        StageTimer t(idx, AVQ_STAGE_FINAL, st);
        return launch_finalize(p.partial, ns, nq, R, k, reorder_k != 0, key_kind, idx->x, c.d, queries,
                               idx->scale.as<float>(), idx->bias.as<float>(), ids_out, scores_out, st);
    }
    if (use_mfma_scan(idx, nq, lut_mode) && idx->tune_prefilter != 1 && c.M <= 64 && idx->n > R && mfma_scan_samples(idx, nq, R, ns))
        return search_through_candidates(idx, queries, nq, k, reorder_k, R, ns, true, ids_out, scores_out, st);
    if (use_mfma_scan(idx, nq, lut_mode)) {
        // 4-bit codes, 8-bit tables, flat index: the table sums are a one-hot contraction on the matrix cores
        scan_mfma_plan(nq, idx->n_blocks, idx->tune_target_wgs, &p);
        AVQ_TRY(idx->partial.reserve(sizeof(u64) * (size_t)nq * p.n_chunks * C));
        AVQ_TRY(idx->lists.reserve(scan_mfma_lists_bytes(p)));
        const size_t thr_bytes = sizeof(uint32_t) * (size_t)nq * (1 + (size_t)p.n_chunks);
        AVQ_TRY(idx->thr.reserve(thr_bytes));
        p.partial = idx->partial.as<u64>();
        p.lists_ws = idx->lists.as<u64>();
        p.thr_shared = idx->thr.as<uint32_t>();
        p.kth_shared = p.thr_shared + nq;
        {
            StageTimer t(idx, AVQ_STAGE_SCAN, st);
            AVQ_HIP(hipMemsetAsync(p.thr_shared, 0, thr_bytes, st));
            AVQ_TRY(launch_scan_mfma(p, st));
        }
        const u64 *cand = p.partial;
        if (p.n_chunks > 1) {
            AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * C));
            StageTimer t(idx, AVQ_STAGE_MERGE, st);
            AVQ_TRY(launch_merge_partials(p.partial, nq, p.n_chunks, ns, idx->cand.as<u64>(), st));
            cand = idx->cand.as<u64>();
        }
        StageTimer t(idx, AVQ_STAGE_FINAL, st);
        return launch_finalize(cand, ns, nq, R, k, reorder_k != 0, key_kind, idx->x, c.d, queries,
                               idx->scale.as<float>(), idx->bias.as<float>(), ids_out, scores_out, st);
    }
    ScanShape shape;
    // few queries on a partitioned index: sixteen waves per workgroup and several workgroups per query
    const int waves_hint = idx->tune_waves > 0 ? idx->tune_waves : (ivf && nq <= 64 ? 16 : 0);
    if (scan_pick_shape(idx->NB, idx->cfg.bits, u8, ns, nq, ivf, idx->tune_qt, waves_hint, &shape) != AVQ_OK)
        AVQ_TRY(scan_pick_shape(idx->NB, idx->cfg.bits, u8, ns, nq, ivf, idx->tune_qt, idx->tune_waves, &shape));
    if (ivf) {
        const int L = leaves_to_search;
        AVQ_TRY(idx->leaf_ids.reserve(sizeof(int32_t) * (size_t)nq * L));
        AVQ_TRY(idx->leaf_ip.reserve(sizeof(float) * (size_t)nq * L));
        {
            StageTimer t(idx, AVQ_STAGE_LEAF, st);
            AVQ_TRY(launch_leaf_select(idx->centers_t.as<float>(), c.n_leaves, c.d, queries, nq, L,
                                       idx->leaf_ids.as<int32_t>(), idx->leaf_ip.as<float>(), st));
        }
        p.perm = idx->perm.as<int32_t>();
        p.leaf_ids = idx->leaf_ids.as<int32_t>();
        p.leaf_ip = idx->leaf_ip.as<float>();
        p.leaf_blk = idx->leaf_blk.as<int32_t>();
        p.Lp = L;
        p.n_tiles = nq;
        // about one leaf per wave when the batch alone cannot fill the chip
        const int target = idx->tune_target_wgs > 0 ? idx->tune_target_wgs : 512;
        int chunks = target / nq;
        const int max_chunks = (L + shape.waves - 1) / shape.waves;
        p.n_chunks = std::max(1, std::min(chunks, max_chunks));
    } else {
        plan_flat(idx, shape, nq, &p);
    }
    AVQ_TRY(idx->partial.reserve(sizeof(u64) * (size_t)p.n_tiles * shape.qt * p.n_chunks * C));
    p.partial = idx->partial.as<u64>();
    if (shape.lists_global) {
        AVQ_TRY(idx->lists.reserve(sizeof(u64) * (size_t)p.n_tiles * p.n_chunks * shape.waves * shape.qt * C));
        p.lists_ws = idx->lists.as<u64>();
    }
    {
        StageTimer t(idx, AVQ_STAGE_SCAN, st);
        AVQ_TRY(launch_scan(p, u8, ivf ? SCAN_LEAVES : SCAN_CHUNK, shape, st));
    }
    const u64 *cand = p.partial;
    if (p.n_chunks > 1) {
        AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * C));
        StageTimer t(idx, AVQ_STAGE_MERGE, st);
        AVQ_TRY(launch_merge_partials(p.partial, nq, p.n_chunks, ns, idx->cand.as<u64>(), st));
        cand = idx->cand.as<u64>();
    }
    StageTimer t(idx, AVQ_STAGE_FINAL, st);
    return launch_finalize(cand, ns, nq, R, k, reorder_k != 0, key_kind, idx->x, c.d, queries,
                           idx->scale.as<float>(), idx->bias.as<float>(), ids_out, scores_out, st);
}

// ---- the entry point that allocates nothing ---------------------------------------------
// Device scratch of avq_search_noalloc: one array per GPU, part of the library's code object,
// held from the moment the library is loaded on that GPU until the process ends. In host code
// the array's name only stands for the symbol; the address on the current device comes from
// hipGetSymbolAddress and is looked up once per device.
static __device__ __align__(256) unsigned char scratch[AVQ_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char *g_scratch_ptr[kMaxDevices] = {};

static int noalloc_scratch(unsigned char **out)
{
    int dev = -1;
    AVQ_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("avq_search_noalloc: device %d not supported", dev); return AVQ_EINVAL; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        unsigned char *ptr = nullptr;
        AVQ_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) { set_error("avq_search_noalloc: no address for the scratch array"); return AVQ_EHIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return AVQ_OK;
}

extern "C" int avq_search_noalloc(avq_index *idx, const float *queries, int32_t nq, int32_t k, int32_t reorder_k,
                                  int32_t lut_mode, int32_t *ids_out, float *scores_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    const avq_config &c = idx->cfg;
    if (c.n_leaves > 0) { set_error("avq_search_noalloc: flat index only"); return AVQ_EINVAL; }
    AVQ_TRY(check_search_args(idx, queries, nq, k, reorder_k, lut_mode, 0, ids_out, scores_out));
    if (nq > AVQ_NOALLOC_MAX_QUERIES) {
        set_error("avq_search_noalloc: at most %d queries per call (got %d)", AVQ_NOALLOC_MAX_QUERIES, nq);
        return AVQ_EINVAL;
    }
    const int R = reorder_k ? reorder_k : k;
    const bool u8 = lut_mode == AVQ_LUT_U8;
    SmallWs w;
    const size_t need = small_ws_carve(idx, nq, R, nullptr, &w);
    if (need > (size_t)AVQ_NOALLOC_SCRATCH_BYTES) {
        set_error("avq_search_noalloc: %d queries x %lld points with reorder_k %d need %zu bytes of scratch, the library holds %zu",
                  nq, (long long)idx->n, reorder_k, need, (size_t)AVQ_NOALLOC_SCRATCH_BYTES);
        return AVQ_EINVAL;
    }
    if ((size_t)idx->NB * 256 * 4 > kMaxDynLds && !(c.bits == 4 && (size_t)c.M * 64 <= 60 * 1024)) {
        set_error("avq_search_noalloc: the tables of this index do not fit the single-query kernels");
        return AVQ_EINVAL;
    }
    unsigned char *base = nullptr;
    AVQ_TRY(noalloc_scratch(&base));
    small_ws_carve(idx, nq, R, base, &w);
    const bool fuse_tables = small_batch_can_fuse_tables(c.bits, c.M, c.d, u8);
    return search_small(idx, queries, nq, k, reorder_k, u8, fuse_tables, w, false, ids_out, scores_out, (hipStream_t)hip_stream);
}

extern "C" int avq_brute_force(avq_index *idx, const float *queries, int32_t nq, int32_t k,
                               int32_t *ids_out, float *scores_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    if (idx->n <= 0 || !idx->x) { set_error("avq_brute_force: no datapoints stored"); return AVQ_ESTATE; }
    if (!queries || nq < 1 || !ids_out || !scores_out || k < 1 || k > AVQ_MAX_SELECT || k > idx->n) {
        set_error("avq_brute_force: bad argument");
        return AVQ_EINVAL;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const int ns = (k + 63) / 64;
    const int chunks = brute_force_chunks(idx->n, nq);
    AVQ_TRY(idx->partial.reserve(sizeof(u64) * (size_t)nq * chunks * 64 * ns));
    AVQ_TRY(idx->cand.reserve(sizeof(u64) * (size_t)nq * 64 * ns));
    return launch_brute_force(idx->x, idx->n, idx->cfg.d, queries, nq, k, idx->partial.as<u64>(), chunks,
                              idx->cand.as<u64>(), ids_out, scores_out, st);
}

// ---- stage-level inspection -------------------------------------------------------------

extern "C" int avq_debug_lut(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode,
                             void *lut_out, float *scale_out, float *bias_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    if (!idx->have_codebooks) { set_error("avq_debug_lut: no dictionaries yet"); return AVQ_ESTATE; }
    if (!queries || nq < 1 || !lut_out) { set_error("avq_debug_lut: bad argument"); return AVQ_EINVAL; }
    if (lut_mode != AVQ_LUT_F32 && lut_mode != AVQ_LUT_U8) { set_error("bad lut_mode"); return AVQ_EINVAL; }
    if (lut_mode == AVQ_LUT_U8 && (!scale_out || !bias_out)) { set_error("avq_debug_lut: scale/bias NULL"); return AVQ_EINVAL; }
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    if (lut_mode == AVQ_LUT_F32)
        return launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, (float *)lut_out, nullptr,
                          nullptr, nullptr, st);
    return launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, nullptr, (uint8_t *)lut_out,
                      scale_out, bias_out, st);
}

extern "C" int avq_debug_adc_scores(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode,
                                    void *scores_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    AVQ_TRY(check_query_args(idx, queries, nq, lut_mode));
    if (idx->cfg.n_leaves > 0) { set_error("avq_debug_adc_scores: flat index only"); return AVQ_ESTATE; }
    if (!scores_out) { set_error("avq_debug_adc_scores: NULL output"); return AVQ_EINVAL; }
    hipStream_t st = (hipStream_t)hip_stream;
    const bool u8 = lut_mode == AVQ_LUT_U8;
    AVQ_TRY(build_tables(idx, queries, nq, lut_mode, st));
    ScanParams p;
    fill_scan_params(idx, nq, 1, 2, &p);
    if (use_mfma_scan(idx, nq, lut_mode)) {
        scan_mfma_plan(nq, idx->n_blocks, idx->tune_target_wgs, &p);
        p.scores_out = scores_out;
        p.score_stride = idx->n;
        return launch_scan_mfma(p, st);
    }
    ScanShape shape;
    AVQ_TRY(scan_pick_shape(idx->NB, idx->cfg.bits, u8, 2, nq, false, idx->tune_qt, idx->tune_waves, &shape));
    plan_flat(idx, shape, nq, &p);
    p.scores_out = scores_out;
    p.score_stride = idx->n;
    AVQ_TRY(idx->partial.reserve(64));
    p.partial = idx->partial.as<u64>();
    if (shape.lists_global) {
        AVQ_TRY(idx->lists.reserve(sizeof(u64) * (size_t)p.n_tiles * p.n_chunks * shape.waves * shape.qt * 128));
        p.lists_ws = idx->lists.as<u64>();
    }
    return launch_scan(p, u8, SCAN_CHUNK, shape, st);
}

extern "C" int avq_debug_stream_codes(avq_index *idx, uint32_t *words_out, int64_t *n_blocks_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    if (idx->n <= 0) { set_error("avq_debug_stream_codes: no codes yet"); return AVQ_ESTATE; }
    if (n_blocks_out) *n_blocks_out = idx->n_blocks;
    if (!words_out) return AVQ_OK;
    return launch_stream_codes(idx->codes_blocked.as<uint8_t>(), idx->n_blocks, idx->NB, words_out, (hipStream_t)hip_stream,
                               stream_loads_nontemporal(idx, 1));
}

extern "C" int avq_debug_scan_parts(avq_index *idx, const float *queries, int32_t nq, int32_t lut_mode, int32_t part,
                                    int32_t reps, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    AVQ_TRY(check_query_args(idx, queries, nq, lut_mode));
    if (idx->cfg.n_leaves > 0) { set_error("avq_debug_scan_parts: flat index only"); return AVQ_ESTATE; }
    if (part < 0 || part > 2 || reps < 1 || nq > 64) { set_error("avq_debug_scan_parts: bad argument"); return AVQ_EINVAL; }
    hipStream_t st = (hipStream_t)hip_stream;
    const avq_config &c = idx->cfg;
    const bool u8 = lut_mode == AVQ_LUT_U8;
    const bool bounds = small_uses_bounds(idx);
    if (part == 2 && !bounds) { set_error("avq_debug_scan_parts: no lookup-only kernel for this code size"); return AVQ_EINVAL; }
    SmallWs w;
    AVQ_TRY(small_ws_from_index(idx, nq, 1, &w));
    const bool fuse_tables = small_batch_can_fuse_tables(c.bits, c.M, c.d, u8);
    if (!fuse_tables)
        AVQ_TRY(launch_lut(queries, nq, idx->codebooks.as<float>(), c.d, c.M, idx->kc, w.lut, u8 ? w.lut8 : nullptr, w.scale,
                           w.bias, st));
    ScanParams p;
    fill_scan_params(idx, nq, 1, 1, &p);
    p.lut = w.lut; p.lut8 = w.lut8; p.scale = w.scale; p.bias = w.bias;
    if (fuse_tables) { p.fuse_queries = queries; p.fuse_codebooks = idx->codebooks.as<float>(); p.fuse_d = c.d; }
    p.block_max = w.block_max;
    p.block_bound = w.block_bound;
    p.bound_meta = w.bound_meta;
    p.bound_tbl = w.bound_tbl;
    p.lut_out = fuse_tables ? w.lut : nullptr;
    p.n_tiles = nq;
    p.n_chunks = 1;
    p.max_wgs = idx->tune_target_wgs;
    p.nt_loads = stream_loads_nontemporal(idx, nq) ? 1 : 0;
    if (bounds) AVQ_TRY(launch_bound_tables(p, u8, st));
    for (int r = 0; r < reps; ++r) {
        if (part == 1) AVQ_TRY(launch_stream_codes(idx->codes_blocked.as<uint8_t>(), idx->n_blocks, idx->NB, (uint32_t *)w.block_max, st, stream_loads_nontemporal(idx, nq)));
        else if (bounds) AVQ_TRY(launch_block_bound(p, idx->tune_waves, st, part == 2));
        else AVQ_TRY(launch_block_max(p, u8, idx->tune_waves > 0 ? idx->tune_waves : 4, st));
    }
    return AVQ_OK;
}

extern "C" int avq_debug_unverified_queries(avq_index *idx, int32_t *counts_out)
{
    AVQ_TRY(check_index(idx));
    if (!counts_out) { set_error("avq_debug_unverified_queries: NULL"); return AVQ_EINVAL; }
    counts_out[0] = -1;
    counts_out[1] = counts_out[2] = counts_out[3] = 0;
    if (!idx->fail.p) return AVQ_OK;
    AVQ_HIP(hipDeviceSynchronize());
    uint32_t c[4] = {0, 0, 0, 0};
    AVQ_HIP(hipMemcpy(c, idx->fail.p, sizeof(c), hipMemcpyDeviceToHost));
    for (int i = 0; i < 4; ++i) counts_out[i] = (int32_t)c[i];
    return AVQ_OK;
}

extern "C" int avq_debug_leaf_select(avq_index *idx, const float *queries, int32_t nq, int32_t L,
                                     int32_t *leaf_ids_out, float *leaf_ip_out, void *hip_stream)
{
    AVQ_TRY(check_index(idx));
    const avq_config &c = idx->cfg;
    if (c.n_leaves <= 0 || !idx->have_centers) { set_error("avq_debug_leaf_select: no leaf centers"); return AVQ_ESTATE; }
    if (!queries || nq < 1 || !leaf_ids_out || !leaf_ip_out || L < 1 || L > c.n_leaves || L > AVQ_MAX_SELECT) {
        set_error("avq_debug_leaf_select: bad argument");
        return AVQ_EINVAL;
    }
    if (nq <= 32) { // the kernels the few-query search uses
        AVQ_TRY(idx->tmp.reserve(sizeof(u64) * (size_t)nq * c.n_leaves));
        return launch_leaf_select_few(idx->centers_t.as<float>(), c.n_leaves, c.d, queries, nq, L, (u64 *)idx->tmp.p,
                                      leaf_ids_out, leaf_ip_out, (hipStream_t)hip_stream);
    }
    return launch_leaf_select(idx->centers_t.as<float>(), c.n_leaves, c.d, queries, nq, L, leaf_ids_out,
                              leaf_ip_out, (hipStream_t)hip_stream);
}
