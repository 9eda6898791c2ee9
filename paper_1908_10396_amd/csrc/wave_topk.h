// Wavefront-level top-k on 64-bit keys for gfx950 (wave64).
//
// A key packs (ordering value, id): high word = a 32-bit unsigned that grows
// with the score, low word = ~id, so "larger key" means "higher score, then
// lower id" -- the total order every selection stage uses. Key 0 is the empty
// slot (no real candidate maps to it).
//
// A candidate list of C = 64*ns keys lives in LDS (or global memory), sorted descending
// (list[0] is the best). A wave merges batches of 64 keys into it with bitonic
// networks whose compare-exchanges run across lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace avq {

typedef unsigned long long u64;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

__device__ __forceinline__ u64 shfl_u64(u64 v, int src)
{
    int lo = __shfl((int)(uint32_t)v, src, 64);
    int hi = __shfl((int)(uint32_t)(v >> 32), src, 64);
    return ((u64)(uint32_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int mask)
{
    int lo = __shfl_xor((int)(uint32_t)v, mask, 64);
    int hi = __shfl_xor((int)(uint32_t)(v >> 32), mask, 64);
    return ((u64)(uint32_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ u64 umax64(u64 a, u64 b) { return a > b ? a : b; }
__device__ __forceinline__ u64 umin64(u64 a, u64 b) { return a < b ? a : b; }

// Orders lanes of a bitonic sequence descending (lane 0 largest).
__device__ __forceinline__ u64 wave_bitonic_merge_desc(u64 v)
{
    const int lane = lane_id();
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
        u64 o = shfl_xor_u64(v, j);
        v = (lane & j) ? umin64(v, o) : umax64(v, o);
    }
    return v;
}

// Full bitonic sort of one key per lane, descending.
__device__ __forceinline__ u64 wave_sort_desc(u64 v)
{
    const int lane = lane_id();
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            u64 o = shfl_xor_u64(v, j);
            bool desc_block = (lane & k) == 0; // k == 64: always true
            bool lower = (lane & j) == 0;
            v = (lower == desc_block) ? umax64(v, o) : umin64(v, o);
        }
    }
    return v;
}

__device__ __forceinline__ void wave_lds_fence()
{
    // Lists and pending buffers are exchanged between lanes of one wave through memory
    // (LDS, or global memory for the lists of the batch kernels): make earlier stores
    // visible and later loads fresh. Workgroup scope is enough: the waves of a workgroup
    // share one L1, so this costs a wait and no cache action.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Merges a batch p (one key per lane, sorted descending, empty lanes 0) into
// the sorted list (ns slots of 64 keys, in LDS). Keeps the 64*ns largest.
__device__ __noinline__ void wave_list_insert_sorted(u64 *list, int ns, u64 p)
{
    const int lane = lane_id();
    if (shfl_u64(p, 0) <= list[ns * 64 - 1]) return; // best of p is below the whole list
    for (int s = 0; s < ns; ++s) {
        u64 v = list[s * 64 + lane];
        u64 pmax = shfl_u64(p, 0);
        u64 vmin = shfl_u64(v, 63);
        if (pmax == 0ull) break;      // nothing left to place
        if (pmax <= vmin) continue;   // slot s keeps all its keys; p may still beat later slots
        u64 pr = shfl_u64(p, 63 - lane);
        u64 hi = umax64(v, pr); // the 64 largest of slot + batch, bitonic
        u64 lo = umin64(v, pr); // the 64 smallest, bitonic
        list[s * 64 + lane] = wave_bitonic_merge_desc(hi);
        if (s + 1 < ns) p = wave_bitonic_merge_desc(lo);
    }
    wave_lds_fence();
}

// Sorts the cnt (<= 64) pending keys and merges them into the list.
__device__ __noinline__ void wave_list_flush(u64 *list, int ns, const u64 *pend, int cnt)
{
    wave_lds_fence();
    u64 p = lane_id() < cnt ? pend[lane_id()] : 0ull;
    p = wave_sort_desc(p);
    wave_list_insert_sorted(list, ns, p);
}

// Merges another sorted list (same shape, LDS or global) into `list`.
__device__ __forceinline__ void wave_list_merge_from(u64 *list, int ns, const u64 *other)
{
    const int lane = lane_id();
    for (int s = 0; s < ns; ++s) {
        u64 p = other[s * 64 + lane];
        if (shfl_u64(p, 0) == 0ull) break; // empty from here on
        u64 worst = list[ns * 64 - 1];
        if (shfl_u64(p, 0) <= worst) break; // sorted: later slots are smaller still
        wave_list_insert_sorted(list, ns, p);
    }
}

// Appends the keys of the lanes with `hit` to the pending buffer (flushing it
// into the list first if they would not fit). Must be called by the whole
// wave. Returns true when a flush happened (the caller's threshold is stale).
__device__ __forceinline__ bool wave_push(u64 *list, int ns, u64 *pend, int &cnt, bool hit, u64 key)
{
    const u64 mask = __builtin_amdgcn_ballot_w64(hit);
    if (mask == 0ull) return false;
    const int c = __builtin_popcountll(mask);
    bool flushed = false;
    if (cnt + c > 64) {
        wave_list_flush(list, ns, pend, cnt);
        cnt = 0;
        flushed = true;
    }
    if (hit) pend[cnt + __builtin_popcountll(mask & ((1ull << lane_id()) - 1ull))] = key;
    cnt += c;
    return flushed;
}

__device__ __forceinline__ void wave_list_clear(u64 *list, int ns)
{
    for (int s = 0; s < ns; ++s) list[s * 64 + lane_id()] = 0ull;
    wave_lds_fence();
}

// ---- ordering values -----------------------------------------------------

// fp32 -> unsigned that orders like the float; -0 and +0 map to the same value.
__device__ __forceinline__ uint32_t ord_from_f32(float s)
{
    uint32_t b = __float_as_uint(s + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float f32_from_ord(uint32_t o)
{
    uint32_t b = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(b);
}

__device__ __forceinline__ u64 make_key(uint32_t ord, int32_t id)
{
    return ((u64)ord << 32) | (uint32_t)(~(uint32_t)id);
}

__device__ __forceinline__ int32_t key_id(u64 key) { return (int32_t)(~(uint32_t)key); }
__device__ __forceinline__ uint32_t key_ord(u64 key) { return (uint32_t)(key >> 32); }

} // namespace avq
