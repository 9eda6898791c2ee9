// Workgroup-level exact selection on 64-bit keys (see wave_topk.h for the key
// format): the R-th largest of N keys in global memory, found by narrowing a key
// range with LDS histograms -- a radix select whose digits adapt to the range
// that is still open, so keys that share their high bits (scores of one query
// do) cost no extra passes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace avq {

typedef unsigned long long u64;

constexpr int kSelBins = 2048;  // histogram bins per pass (a power of two: the bin index is packed into 11 bits)
constexpr int kSelList = 512;   // once this few keys remain in range they are ranked directly (by counting pairs:
                                // beyond a few hundred keys another pass over the histogram is cheaper)
static_assert((kSelBins & (kSelBins - 1)) == 0 && kSelBins <= 2048, "the bin index travels in 11 bits");
constexpr int kSelRegs = 8;     // keys a thread caches in registers (N <= kSelRegs * threads)

struct WgSelectScratch {
    uint32_t hist[kSelBins];
    u64 list[kSelList];
    u64 red_max[16], red_min[16];
    uint32_t red_cnt[16];
    uint32_t wave_sum[16];
    u64 found;       // published by the thread that owns the bin of the wanted key, in ONE word: population of the bin
                     // << 32 | keys above the bin << 11 | bin. As three adjacent 32-bit words (which the compiler stores
                     // and loads with one 96-bit LDS access) a 16-wave workgroup returned a wrong threshold about once
                     // in ten calls on MI355X; a second barrier before the loads, or words placed apart, removed that.
    uint32_t list_cnt;
    u64 result;
};

// All threads of the workgroup (a multiple of 64, at most 1024) must call this.
// Keys equal to 0 are empty slots and never selected. Returns the R-th largest
// non-empty key, or 1 when there are fewer than R of them (so "key >= result"
// selects min(R, count) keys; keys are distinct). The keys are read from global
// memory once when N <= kSelRegs * blockDim.x, else once per pass. R <= 2^21, N < 2^32.
__device__ inline u64 wg_select_threshold(const u64 *__restrict__ keys, int64_t N, int R, WgSelectScratch *s)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, n_waves = nt >> 6;
    const bool cached = N <= (int64_t)kSelRegs * nt;
    u64 kreg[kSelRegs];
    if (cached) {
#pragma unroll
        for (int r = 0; r < kSelRegs; ++r) {
            const int64_t i = (int64_t)r * nt + tid;
            kreg[r] = i < N ? keys[i] : 0ull;
        }
    }
    // visits every non-empty key once
    auto for_each_key = [&](auto &&fn) {
        if (cached) {
#pragma unroll
            for (int r = 0; r < kSelRegs; ++r)
                if (kreg[r]) fn(kreg[r]);
        } else {
            for (int64_t i = tid; i < N; i += nt) {
                const u64 kkey = keys[i];
                if (kkey) fn(kkey);
            }
        }
    };

    // pass 0: range and population
    u64 mx = 0ull, mn = ~0ull;
    uint32_t cnt = 0;
    for_each_key([&](u64 kkey) { mx = kkey > mx ? kkey : mx; mn = kkey < mn ? kkey : mn; ++cnt; });
    for (int m = 32; m > 0; m >>= 1) {
        const u64 omx = ((u64)(uint32_t)__shfl_xor((int)(mx >> 32), m, 64) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)mx, m, 64);
        const u64 omn = ((u64)(uint32_t)__shfl_xor((int)(mn >> 32), m, 64) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)mn, m, 64);
        mx = omx > mx ? omx : mx;
        mn = omn < mn ? omn : mn;
        cnt += (uint32_t)__shfl_xor((int)cnt, m, 64);
    }
    __syncthreads(); // scratch may still be in use by a previous call
    if (lane == 0) { s->red_max[wave] = mx; s->red_min[wave] = mn; s->red_cnt[wave] = cnt; }
    __syncthreads();
    u64 hi = 0ull, lo = ~0ull;
    uint32_t total = 0;
    for (int w = 0; w < n_waves; ++w) {
        hi = s->red_max[w] > hi ? s->red_max[w] : hi;
        lo = s->red_min[w] < lo ? s->red_min[w] : lo;
        total += s->red_cnt[w];
    }
    if (total < (uint32_t)R || total == 0) return 1ull;
    uint32_t need = (uint32_t)R; // rank, counted from the top, inside [lo, hi]
    uint32_t pop = total;

    for (;;) {
        if (pop <= (uint32_t)kSelList) {
            // few keys left in range: gather them and rank directly
            __syncthreads();
            if (tid == 0) s->list_cnt = 0;
            __syncthreads();
            for_each_key([&](u64 kkey) {
                if (kkey >= lo && kkey <= hi) s->list[atomicAdd(&s->list_cnt, 1u)] = kkey;
            });
            __syncthreads();
            const uint32_t c = s->list_cnt;
            for (uint32_t j = tid; j < c; j += nt) {
                const u64 mine = s->list[j];
                uint32_t rank = 0;
#pragma unroll 8
                for (uint32_t t = 0; t < c; ++t) rank += s->list[t] > mine;
                if (rank == need - 1) s->result = mine;
            }
            __syncthreads();
            return s->result;
        }
        const u64 width = hi - lo;
        const int shift = width < (u64)kSelBins ? 0 : (64 - __builtin_clzll(width)) - 11;
        __syncthreads();
        for (int b = tid; b < kSelBins; b += nt) s->hist[b] = 0u;
        __syncthreads();
        for_each_key([&](u64 kkey) {
            if (kkey >= lo && kkey <= hi) atomicAdd(&s->hist[(uint32_t)((kkey - lo) >> shift)], 1u);
        });
        __syncthreads();
        // find the bin holding the need-th key from the top: suffix counts over the bins
        const int per = (kSelBins + nt - 1) / nt;
        uint32_t mine_sum = 0;
        const int b0 = tid * per;
        for (int j = 0; j < per; ++j) { const int b = b0 + j; if (b < kSelBins) mine_sum += s->hist[b]; }
        // inclusive suffix sum across lanes (lane l gets the sum over lanes >= l)
        uint32_t suf = mine_sum;
        for (int m = 1; m < 64; m <<= 1) {
            const uint32_t o = (uint32_t)__shfl_down((int)suf, m, 64);
            if (lane + m < 64) suf += o;
        }
        if (lane == 0) s->wave_sum[wave] = suf;
        __syncthreads();
        uint32_t above_waves = 0;
        for (int w = wave + 1; w < n_waves; ++w) above_waves += s->wave_sum[w];
        // keys in bins above this thread's bins
        uint32_t above = above_waves + (suf - mine_sum);
        for (int j = per - 1; j >= 0; --j) {
            const int b = b0 + j;
            if (b >= kSelBins) continue;
            const uint32_t h = s->hist[b];
            if (above < need && need <= above + h) s->found = ((u64)h << 32) | (above << 11) | (uint32_t)b; // above < R <= 2^21
            above += h;
        }
        __syncthreads();
        const u64 found = s->found;
        const uint32_t fb = (uint32_t)found & (uint32_t)(kSelBins - 1);
        need -= ((uint32_t)found >> 11);
        pop = (uint32_t)(found >> 32);
        const u64 nlo = lo + ((u64)fb << shift);
        u64 nhi = nlo + (((u64)1 << shift) - 1ull);
        if (nhi > hi || nhi < nlo) nhi = hi;
        lo = nlo;
        hi = nhi;
    }
}

} // namespace avq
