// ADC scan of 4-bit codes against 8-bit tables on the matrix cores of gfx950.
//
// With 16 codewords per subspace the table sum  sum_m Q[q][m][code[n][m]]  is a dense
// contraction of a one-hot matrix with the tables: row n of A has, for every subspace,
// sixteen 0/1 bytes with the 1 at the point's code; column q of B holds the sixteen
// table bytes of every subspace. A one-hot row has one non-zero in sixteen positions, so
// it fits the 2:4 structured sparsity of v_smfmac_i32_32x32x64_i8: that instruction
// multiplies 32 points by 32 queries over 64 positions (four subspaces, two code bytes)
// in the time the dense instruction takes for 32, from a compressed A operand (for every
// group of four positions two values, and two bits each that say where in the group they
// sit) and accumulates exact 32-bit integers, so the result is the integer sum the 8-bit
// path is defined by, bit for bit. Tables are biased by -128 to fit the signed operand;
// the bias, 128 per subspace, is added back when a key is made.
//
// Operand layout of the instruction (one lane: row or column lane % 32, half lane / 32):
// A, 16 compressed bytes per lane, bytes 0-7 pair with the B lanes of half 0, bytes 8-15 with
// those of half 1, in both cases with B bytes 16 * (A's half) .. + 15: compressed bytes 2g and
// 2g + 1 are the two values of the group of B bytes 4g .. 4g + 3, and bits 2i, 2i + 1 of the
// lane's index operand give the position of compressed byte i inside its group. Nothing
// requires the two positions of a group to differ or to be ordered; a value of 0 contributes
// nothing wherever its position points.
//
// One wave owns 32 queries and a chunk of the blocks. Its B operands (13 register groups
// of 32 bytes for 50 subspaces) stay in registers for the whole scan. Lanes 0-31 take the
// even code bytes of their four points, lanes 32-63 the odd ones; the A operand of a
// (point, code byte) is one 16-byte read from a 256-byte LDS table of the sixteen value
// patterns (which groups hold the 1 of the low and of the high nibble; no bank conflicts,
// the patterns cover every bank once), and its index operand is the code byte itself copied
// to all four bytes (one permute). The order of the sum does not matter (integers), so any
// pairing of operand positions with table entries is valid as long as A and B agree.
//
// A lane ends up with the scores of 16 points for one query (lanes l and l + 32 share
// query l % 32). Scores above the query's threshold go to a lane-private pending
// buffer in LDS; when a lane's buffer is three quarters full the two buffers of the query are
// sorted and merged into the query's candidate list (global scratch), which tightens
// the threshold.
//
// Thresholds are shared between the waves that scan different chunks for the same
// queries, through global arrays and relaxed atomics; a stale value only lets more
// points through. thr_shared[q] (atomic max) collects lower bounds of the final R-th
// best score of query q, of two kinds:
//  * any wave's own R-th best score;
//  * for a group of g waves that run side by side, the smallest of their ceil(R/g)-th
//    best scores (published in kth_shared[q][chunk]): that many points at or above it
//    exist in every one of the g chunks, R in all. This one is close to the R-th best
//    of the group's union, which no wave could compute alone, and cuts the keys that
//    reach the lists roughly by the size of the group.
// A wave reads its queries' bounds once per block, one block ahead of their use.
//
// Guess and check (the FIXED instantiation). While a list is young its bound is weak and nearly
// every point passes; sorting those keys into lists is a fifth of the scan's time. Batches, which
// only need a superset of the R best (candidate mode), scan against a guessed bound instead: a first
// launch (the STORE instantiation with sample_max set) scores a sample of the points, every
// block_stride-th block of every chunk, and keeps no lists either: a lane's 16 accumulators see 16
// disjoint classes of points, so the wave records the best sum of each of its 32 classes per query,
// and the r-th largest of a query's class maxima (r chosen so that a few times R points of the whole
// index lie above it) becomes the query's bound in thr_shared. The second launch scans everything
// against that fixed bound, appends what reaches it (less the margin) to the candidate buffers and
// keeps no lists. Afterwards the guess is checked per query: if at least R kept points reach the
// bound, the R-th best sum of the index is at or above it and nothing was missed; otherwise the
// query is scanned again. (A sample scanned with lists, block_stride > 1 in the list instantiation,
// remains for queries with too few classes.)
//
// Template parameters: STORE (scores or class maxima are written, nothing is selected), ITEMS (work
// items of a partitioned index, one leaf and 32 of its queries per wave, instead of query tile x
// chunk), FIXED (bounds are given and never raised, no lists).
#include <cmath>
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) v16i lds_v16i;

constexpr int kMfmaQueries = 32; // queries per wave
constexpr int kMfmaPend = 64;    // pending keys per lane
constexpr int kMfmaWaves = 4;    // waves per workgroup

// Inside the scan a key is 32 bits: (ordering value << 18) | (~id & 0x3ffff), with ids
// counted from the chunk's first point. It orders like the 64-bit key (score, then lower
// id) as long as a chunk has at most 2^18 points and ordering values stay below 2^14
// (255 * 64 + 1 does); sorting and merging 32-bit keys costs half the shuffles.
constexpr int kIdBits = 18;
constexpr uint32_t kIdMask = (1u << kIdBits) - 1u;
constexpr int kMfmaMaxChunkBlocks = (1 << kIdBits) / kBlockPoints;

__device__ __forceinline__ uint32_t merge32_desc(uint32_t v) // lanes of a bitonic sequence -> descending
{
    const int lane = lane_id();
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, j, 64);
        v = (lane & j) ? (o < v ? o : v) : (o > v ? o : v);
    }
    return v;
}

__device__ __forceinline__ uint32_t sort32_desc(uint32_t v) // one key per lane -> descending
{
    const int lane = lane_id();
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)v, j, 64);
            const bool desc_block = (lane & k) == 0; // k == 64: always true
            const bool lower = (lane & j) == 0;
            v = (lower == desc_block) ? (o > v ? o : v) : (o < v ? o : v);
        }
    }
    return v;
}

constexpr int kMfmaMaxNs = 8; // list slots of 64 keys (R <= 512)

__device__ __forceinline__ uint32_t uniform_lane(uint32_t v, int src) // lane src's value, as a scalar
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src);
}

// Merges a batch (one key per lane, sorted descending, empty lanes 0) into a sorted list of ns
// slots of 64 keys held in registers (v[s] = key s*64 + lane); keeps the 64*ns largest.
__device__ __forceinline__ void list32_insert_sorted(uint32_t (&v)[kMfmaMaxNs], int ns, uint32_t b)
{
    const int lane = lane_id();
#pragma unroll
    for (int s = 0; s < kMfmaMaxNs; ++s) {
        if (s >= ns) break;
        const uint32_t bmax = uniform_lane(b, 0), vmin = uniform_lane(v[s], 63);
        if (bmax == 0u) break;      // nothing left to place
        if (bmax <= vmin) continue; // slot s keeps all its keys; the batch may still beat later slots
        const uint32_t br = (uint32_t)__shfl((int)b, 63 - lane, 64);
        const uint32_t hi = v[s] > br ? v[s] : br; // the 64 largest of slot + batch, bitonic
        const uint32_t lo = v[s] > br ? br : v[s]; // the 64 smallest, bitonic
        v[s] = merge32_desc(hi);
        b = merge32_desc(lo);
    }
}

// Rare path of the scan below, kept out of line so that it costs the scan no registers:
// merges the pending keys of one query (cnt_a keys at pend_a, the buffer of lane jq, and
// cnt_b keys at pend_b, that of lane jq + 32) into the query's list, publishes the wave's
// kw-th best in kth_row[self], reads the group's (gsz entries of kth_row) and returns the
// query's new lower bound of the final R-th best ordering value, which it also publishes
// in *bound_q. Called by the whole wave with uniform arguments. The list (global scratch)
// is read once at the start, so that its latency passes while the keys are sorted, and
// written back once.
// With cand_dst set, the pending keys are first appended, unsorted, at cand_dst[cand_pos]: the
// scan then lets through every point within a margin below the bound, and all of them are
// wanted later, not only those that make the list. The new fill count comes back in the
// upper half of the result (cand_cap + 1 once the buffer has overflowed; nothing is written
// past cand_cap).
__device__ __noinline__ u64 mfma_flush_query(const lds_u32 *pend_a, const lds_u32 *pend_b, int cnt_a, int cnt_b,
                                             uint32_t *list, int ns, int R, int kw, uint32_t *kth_row, int gsz,
                                             int self, uint32_t *bound_q, uint32_t *cand_dst, int cand_pos, int cand_cap)
{
    const int lane = lane_id();
    if (cand_dst != nullptr) {
        if (cand_pos + cnt_a + cnt_b <= cand_cap) {
            if (lane < cnt_a) cand_dst[cand_pos + lane] = pend_a[lane];
            if (lane < cnt_b) cand_dst[cand_pos + cnt_a + lane] = pend_b[lane];
            cand_pos += cnt_a + cnt_b;
        } else {
            cand_pos = cand_cap + 1;
        }
    }
    uint32_t member = 0xffffffffu; // lane c < gsz: the kw-th best of the group's chunk c
    if (lane < gsz && lane != self)
        member = __hip_atomic_load(kth_row + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t v[kMfmaMaxNs];
#pragma unroll
    for (int s = 0; s < kMfmaMaxNs; ++s) v[s] = s < ns ? list[s * 64 + lane] : 0u;
    wave_lds_fence();
    if (cnt_a > 0) list32_insert_sorted(v, ns, sort32_desc(lane < cnt_a ? pend_a[lane] : 0u));
    if (cnt_b > 0) list32_insert_sorted(v, ns, sort32_desc(lane < cnt_b ? pend_b[lane] : 0u));
    uint32_t ord = 0u, ord_kw = 0u;
#pragma unroll
    for (int s = 0; s < kMfmaMaxNs; ++s) {
        if (s >= ns) break;
        list[s * 64 + lane] = v[s];
        if ((R - 1) >> 6 == s) ord = uniform_lane(v[s], (R - 1) & 63) >> kIdBits;
        if ((kw - 1) >> 6 == s) ord_kw = uniform_lane(v[s], (kw - 1) & 63) >> kIdBits;
    }
    if (lane == self) member = ord_kw;
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)member, m, 64);
        member = o < member ? o : member;
    }
    const uint32_t best = ord > member ? ord : member; // member: 0 while a chunk of the group has fewer than kw keys
    if (lane == 0) {
        if (ord_kw > 0u) __hip_atomic_store(kth_row + self, ord_kw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (best > 0u) __hip_atomic_fetch_max(bound_q, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wave_lds_fence();
    return ((u64)(uint32_t)cand_pos << 32) | best;
}

// The flush of the fixed-bound scan: the pending keys are appended to the candidate buffer and
// that is all (no list, no bound to raise). Returns the new fill count (cand_cap + 1: overflowed).
__device__ __noinline__ int mfma_dump_query(const lds_u32 *pend_a, const lds_u32 *pend_b, int cnt_a, int cnt_b,
                                            uint32_t *cand_dst, int cand_pos, int cand_cap)
{
    const int lane = lane_id();
    if (cand_pos + cnt_a + cnt_b > cand_cap) return cand_cap + 1;
    if (lane < cnt_a) cand_dst[cand_pos + lane] = pend_a[lane];
    if (lane < cnt_b) cand_dst[cand_pos + cnt_a + lane] = pend_b[lane];
    wave_lds_fence();
    return cand_pos + cnt_a + cnt_b;
}

// The same for a partitioned index, where many waves (one per leaf) keep points of the same query:
// all 32 queries of the wave are flushed together. Lane j takes room for its own and lane j + 32's
// pending keys in query q's buffer with one atomic add (32 of them in flight at once, not one
// round trip per query), then every lane copies its keys; `hi` (leaf and its slot in the query's
// probe list) goes into the upper half of every entry. A count beyond the capacity tells the
// reader that keys were dropped. cnt: this lane's pending keys, at pend0.
__device__ __noinline__ void mfma_dump_items(const lds_u32 *pend0, int cnt, int q, uint32_t hi, u64 *kept, uint32_t *kept_cnt, int cap)
{
    const int lane = lane_id();
    const int other = __shfl_xor(cnt, 32, 64);
    const int total = cnt + other;
    uint32_t base = 0u;
    if (lane < 32 && total > 0) base = atomicAdd(kept_cnt + q, (uint32_t)total);
    base = (uint32_t)__shfl((int)base, lane & 31, 64);
    if (base + (uint32_t)total <= (uint32_t)cap) {
        u64 *dst = kept + (size_t)q * cap + base + (lane >= 32 ? (uint32_t)other : 0u);
        for (int i = 0; i < cnt; ++i) dst[i] = ((u64)hi << 32) | pend0[i];
    }
    wave_lds_fence();
}

// STORE: inspection mode, every score is written to scores_out and nothing is selected.
template <int NBT, bool STORE, bool ITEMS, bool FIXED>
__global__ void __launch_bounds__(kMfmaWaves * 64, 2)
adc_mfma_scan_kernel(const ScanParams p)
{
    // A lane's operand is 16 compressed bytes: two halves of four groups, two slots per group; a slot holds a
    // value and, in the index operand, which of its group's four positions the value sits at. The sixteen codes
    // of a code byte's low nibble take the first slots of groups 0 and 2 of both halves (code 4 g + p: half g / 2,
    // group 2 (g % 2), position p), those of its high nibble the first slots of groups 1 and 3. The index operand
    // has one nibble per group (first slot's position in its low two bits): even nibbles belong to the low code
    // nibble, odd ones to the high one, so the code byte itself, copied to all four bytes, is the index operand.
    // Entry t = g0 + 4 * g1 of this table is the pattern of values for a byte with groups g0 and g1.
    __shared__ __align__(16) uint32_t pat_tab[64];
    __shared__ __align__(16) uint32_t zeros16[16]; // accumulators start from here: four LDS reads instead of eight register moves
    extern __shared__ __align__(16) unsigned char dyn_smem[]; // [waves][64 lanes][kMfmaPend] 32-bit keys
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // uniform: block and chunk arithmetic stays scalar
    if (threadIdx.x < 16) {
        zeros16[threadIdx.x] = 0u;
        const int t = threadIdx.x, g0 = t & 3, g1 = t >> 2;
        const int b0 = 8 * (g0 >> 1) + 4 * (g0 & 1), b1 = 8 * (g1 >> 1) + 4 * (g1 & 1) + 2; // compressed bytes that hold a 1
        for (int wd = 0; wd < 4; ++wd)
            pat_tab[4 * t + wd] = (b0 / 4 == wd ? 1u << (8 * (b0 % 4)) : 0u) | (b1 / 4 == wd ? 1u << (8 * (b1 % 4)) : 0u);
    }
    __syncthreads();
    constexpr int NS = (NBT + 1) / 2; // matrix instructions per chain: two code bytes (four subspaces) each
    const int64_t gw = (int64_t)blockIdx.x * kMfmaWaves + wave; // wave index over (chunk, tile), or over the items
    const int j = lane & 31, h = lane >> 5;
    constexpr bool items = ITEMS; // work items (leaf, 32 of its queries) instead of (query tile, chunk)
    int tile = 0, chunk = 0, q = 0;
    bool live = false;
    int64_t first = 0, end = 0;
    uint32_t item_hi = 0u; // items: leaf slot << 21 | leaf of this lane's query
    if (items) {
        if (gw >= (int64_t)*p.n_items) return;
        const uint32_t it = p.item_list[gw];
        const int leaf = (int)(it >> 11), t = (int)(it & 2047u);
        const int at = t * kMfmaQueries + j;
        live = (uint32_t)at < p.leaf_cnt[leaf];
        const uint32_t entry = live ? p.qlist[p.leaf_off[leaf] + at] : 0u;
        q = (int)(entry >> 9);
        item_hi = ((entry & 511u) << 21) | (uint32_t)leaf;
        first = p.leaf_blk[leaf];
        end = p.leaf_blk[leaf + 1];
    } else {
        if (gw >= (int64_t)p.n_tiles * p.n_chunks) return;
        tile = (int)(gw % p.n_tiles);
        chunk = (int)(gw / p.n_tiles);
        q = tile * kMfmaQueries + j;
        live = q < p.B;
        // the chunk's blocks
        first = (int64_t)chunk * p.blocks_per_chunk;
        end = first + p.blocks_per_chunk;
        if (end > p.n_blocks) end = p.n_blocks;
    }
    const int C = 64 * p.ns;
    const int off = 128 * p.M;
    constexpr bool store = STORE;

    // table operands: step s covers subspaces 4s .. 4s + 3. This lane's first sixteen bytes meet the patterns
    // of lanes 0-31 (code byte 2s), its last sixteen those of lanes 32-63 (code byte 2s + 1); of each, bytes
    // 0-3 and 8-11 are the entries 8h .. 8h + 7 of the low nibble's table, bytes 4-7 and 12-15 those of the high
    // nibble's (the layout of the patterns above)
    v8i bq[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        uint2 r[4]; // [code byte][nibble]
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int row = 4 * s + c;
            r[c] = make_uint2(0x80808080u, 0x80808080u); // -> 0
            if (live && row < p.M) r[c] = *(const uint2 *)(p.lut8 + ((size_t)q * p.M + row) * 16 + 8 * h);
            r[c].x ^= 0x80808080u;
            r[c].y ^= 0x80808080u;
        }
        bq[s] = v8i{(int)r[0].x, (int)r[1].x, (int)r[0].y, (int)r[1].y, (int)r[2].x, (int)r[3].x, (int)r[2].y, (int)r[3].y};
    }

    uint32_t *my_lists = nullptr; // [32 queries][C] 32-bit keys
    lds_u32 *const pend0 = (lds_u32 *)dyn_smem + (wave * 64 + lane) * kMfmaPend;
    lds_u32 *const pend_end = pend0 + kMfmaPend;
    lds_u32 *pend = pend0; // next free slot of this lane's pending buffer
    // fixed_bound: the bounds in thr_shared are taken as they are and never raised: every point at
    // or above them (less the margin) goes to the candidate buffer, and no lists are kept
    constexpr bool fixed = !store && (FIXED || items); // FIXED: what the host found in p.fixed_bound
    if (!store && !fixed) {
        my_lists = (uint32_t *)p.lists_ws + (size_t)gw * kMfmaQueries * C;
        for (int i = lane; i < kMfmaQueries * C; i += 64) my_lists[i] = 0u;
        wave_lds_fence();
    }
    // the group of chunks whose waves share ceil(R / size)-th best scores
    const int g0 = (chunk / p.group) * p.group;
    const int gsz = p.n_chunks - g0 < p.group ? p.n_chunks - g0 : p.group;
    const int kw = (p.R + gsz - 1) / gsz;
    uint32_t bound_ord = 0u; // best known lower bound of the final R-th best ordering value of this lane's query
    // A score enters when its ordering value (sum + 1) is >= the bound's: later points of a
    // wave can have lower ids than earlier ones, so equal scores must pass.
    // Candidate mode (cand_keys set): everything within the query's margin below the bound passes
    // too and is kept (see mfma_flush_query); the lists and bounds work as usual.
    const bool cand_mode = p.cand_keys != nullptr;
    int marg = 0;
    if ((cand_mode || items) && live && p.cand_margin != nullptr) { marg = p.cand_margin[q]; marg = marg > 0 ? marg : 0; }
    int cpos = 0; // lanes 0-31: keys of this lane's query in its candidate buffer so far
    auto thr_of = [&]() -> int { return live ? (int)bound_ord - off - 2 - marg : 0x7fffffff; };
    // a bound may already be there: that of an earlier launch over a sample of the same points (bounds_only)
    if (!store && !items && live) bound_ord = __hip_atomic_load(p.thr_shared + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int thr = thr_of();
    if (items && live) {
        // fma(sum, scale, off_q) >= bound can only hold from sum = floor((bound - off_q) / scale) - 2 on (two
        // units for the rounding of this estimate) less what the roundings at the magnitude of the scores can
        // move: the difference bound - off_q and the score itself (the fma, or the fp32 addition of <q, center>)
        // are each within half an ulp of |bound| + |off_q|, which is many units when the table range is small
        // against the leaf scores (tight leaves far from the origin); no bound, or tables without a range:
        // everything is kept
        const uint32_t bound_o = p.item_bound[q]; // ordering value of the fp32 bound, 0: none
        const float sc = p.scale[q], bound = bound_o ? f32_from_ord(bound_o) : -INFINITY;
        const float off_q = __fadd_rn(p.bias[q], p.leaf_ip[(size_t)q * (p.leaf_stride ? p.leaf_stride : p.Lp) + (item_hi >> 21)]);
        thr = -0x7fffffff;
        if (sc > 0.0f && bound > -INFINITY) {
            float a_f = floorf((bound - off_q) / sc);
            a_f = fminf(fmaxf(a_f, -1.0e9f), 1.0e9f);
            const float ulp = (fabsf(bound) + fabsf(off_q)) * 1.1920929e-7f;
            const float extra = fminf(ceilf(2.0f * ulp / sc), 1.0e9f);
            a_f = fmaxf(a_f - extra, -1.0e9f);
            thr = (int)a_f - marg - 3 - off;
        }
    }

    // flushes query jq (lanes jq and jq + 32 hold its pending keys)
    auto flush_query = [&](int jq) {
        const int qq = tile * kMfmaQueries + jq; // < B: only live lanes collect keys (not used with items)
        const int cnt = (int)(pend - pend0);
        const int cnt_a = __builtin_amdgcn_readlane(cnt, jq), cnt_b = __builtin_amdgcn_readlane(cnt, jq + 32);
        const lds_u32 *pa = (const lds_u32 *)dyn_smem + (wave * 64 + jq) * kMfmaPend;
        uint32_t *cand_dst = cand_mode ? p.cand_keys + ((size_t)qq * p.n_chunks + chunk) * p.cand_cap : nullptr;
        if (fixed) {
            const int np = mfma_dump_query(pa, pa + 32 * kMfmaPend, cnt_a, cnt_b, cand_dst, __builtin_amdgcn_readlane(cpos, jq),
                                           p.cand_cap);
            if (j == jq) { pend = pend0; cpos = np; }
            return;
        }
        const u64 res = mfma_flush_query(pa, pa + 32 * kMfmaPend, cnt_a, cnt_b, my_lists + (size_t)jq * C, p.ns, p.R,
                                         kw, p.kth_shared + (size_t)qq * p.n_chunks + g0, gsz, chunk - g0,
                                         p.thr_shared + qq, cand_dst, __builtin_amdgcn_readlane(cpos, jq), p.cand_cap);
        const uint32_t best = (uint32_t)res;
        if (j == jq) {
            pend = pend0;
            cpos = (int)(res >> 32);
            bound_ord = best > bound_ord ? best : bound_ord;
            thr = thr_of();
        }
    };

    // a sampling launch takes only every block_stride-th of its blocks
    const int64_t stride = p.block_stride > 1 ? p.block_stride : 1;
    const int64_t n_half = end > first ? 2 * ((end - first + stride - 1) / stride) : 0; // half blocks to visit
    const int32_t id_base = (int32_t)(first * kBlockPoints); // ids inside keys count from here
    // lane (j, h) takes code bytes h, h + 2, ... of the four points of lane slot H*32 + j of a block's rows:
    // a uniform base per half block, this lane's offsets (rows of four byte planes, 16 bytes per slot; then
    // single planes, 4 bytes per slot), and a constant per byte
    const uint32_t lane_row = 16u * (uint32_t)j + 4u * (uint32_t)h, lane_tail = 4u * (uint32_t)j + 256u * (uint32_t)h;
    auto load_half = [&](uint32_t (&w)[NS], int64_t hb) {
        const uint8_t *base = p.codes + (size_t)(hb >> 1) * 256 * NBT;
        const uint8_t *base_row = base + (hb & 1) * 512, *base_tail = base + (NBT / 4) * 1024 + (hb & 1) * 128;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int b0 = 2 * s; // the byte of lanes 0-31; lanes 32-63 take b0 + 1, in the same row or the next plane
            if (b0 < 4 * (NBT / 4)) w[s] = *(const uint32_t *)(base_row + ((b0 / 4) * 1024 + (b0 % 4) * 4) + lane_row);
            else if (b0 + 1 < NBT) w[s] = *(const uint32_t *)(base_tail + (b0 - 4 * (NBT / 4)) * 256 + lane_tail);
            else w[s] = h ? 0u : *(const uint32_t *)(base_tail + (b0 - 4 * (NBT / 4)) * 256 + lane_tail); // no such byte: code 0 against a zero table
        }
    };

    // sampling launch without lists (store variant only): the best sum of each of this lane's 16 point classes
    constexpr int32_t kNone = -0x7fffffff;
    int32_t smax[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) smax[v] = kNone;
    uint32_t nxt_bound = bound_ord; // the shared bound, read one block ahead of its use
    uint32_t w_cur[NS], w_nxt[NS];
    auto half_of = [&](int64_t i) -> int64_t { return 2 * (first + (i >> 1) * stride) + (i & 1); };
    if (n_half > 0) load_half(w_cur, half_of(0));
    for (int64_t i = 0; i < n_half; ++i) {
        const int64_t hb = half_of(i);
        const int64_t blk = hb >> 1;
        const int H = (int)(hb & 1);
        if (i + 1 < n_half) load_half(w_nxt, half_of(i + 1));
        if (!store && !fixed && H == 0 && live) {
            bound_ord = nxt_bound > bound_ord ? nxt_bound : bound_ord;
            thr = thr_of();
            nxt_bound = __hip_atomic_load(p.thr_shared + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // per code byte (low nibble 4 g0 + p0, high nibble 4 g1 + p1): the offset 16 (g0 + 4 g1) of its pattern entry
        uint32_t grp16[NS];
#pragma unroll
        for (int b = 0; b < NS; ++b) {
            grp16[b] = ((w_cur[b] << 2) & 0x30303030u) | (w_cur[b] & 0xc0c0c0c0u);
            asm volatile("" : "+v"(grp16[b])); // keeps the mask here: one extract per step below
        }
        // Chains of NS matrix instructions, one per u (points 4i + u of the 32 lane slots), two
        // at a time: a chain's next instruction needs the previous one's result, so two chains
        // take turns (and the SIMD's other wave fills what is left). The pattern operands of a
        // step are read from LDS two steps ahead; scheduling barriers keep that order.
        struct Pattern { v4i a; int idx; };
        auto read_a = [&](int u, int s) -> Pattern {
            const uint32_t o = (grp16[s] >> (8 * u)) & 0xffu;
            return Pattern{*(const v4i *)((const unsigned char *)pat_tab + o),
                           (int)__builtin_amdgcn_perm(w_cur[s], w_cur[s], 0x01010101u * (uint32_t)u)};
        };
#pragma unroll
        for (int u0 = 0; u0 < 4; u0 += 2) {
            constexpr int kAhead = 2; // steps between an operand's LDS read and its use
            Pattern abuf[kAhead + 1][2];
            v16i acc[2], zero_acc[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                // the address passes through an empty asm statement so that the read stays here, one per chain
                uint32_t za = (uint32_t)(uintptr_t)(const lds_u32 *)zeros16;
                asm volatile("" : "+v"(za));
                zero_acc[a] = *(const lds_v16i *)(uintptr_t)za;
            }
#pragma unroll
            for (int t = 0; t < kAhead; ++t) {
#pragma unroll
                for (int a = 0; a < 2; ++a) abuf[t][a] = read_a(u0 + a, t);
            }
            // a wave inside its chains goes before one that is comparing or storing candidates (2.5 % per launch, measured)
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const Pattern &pa = abuf[s % (kAhead + 1)][a];
                    if (s == 0)
                        acc[a] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(pa.a, bq[0], zero_acc[a], pa.idx, 0, 0);
                    else
                        acc[a] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(pa.a, bq[s], acc[a], pa.idx, 0, 0);
                    if (s + kAhead < NS) abuf[(s + kAhead) % (kAhead + 1)][a] = read_a(u0 + a, s + kAhead);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                // accumulator v of lane (j, h): point row 8*(v/4) + 4*h + v%4 of the 32, query j
                const int32_t id0 = (int32_t)(blk * 256) + H * 128 + 16 * h + u0 + a;
                if constexpr (store) {
                    if (p.sample_max != nullptr) {
                        const bool whole = (blk + 1) * 256 <= (int64_t)p.n_valid; // no padding slots in this block
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            int32_t sum = acc[a][v];
                            if (!whole && id0 + 32 * (v / 4) + 4 * (v % 4) >= p.n_valid) sum = kNone;
                            smax[v] = sum > smax[v] ? sum : smax[v];
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int32_t id = id0 + 32 * (v / 4) + 4 * (v % 4);
                            if (live && id < p.n_valid)
                                ((int32_t *)p.scores_out)[(size_t)q * p.score_stride + id] = acc[a][v] + off;
                        }
                    }
                } else {
                    // A compare whose result decides a branch costs a wave far more than the compare itself (the
                    // branch waits for it), so the sixteen accumulators are first folded by maxima: one compare and
                    // one branch when no lane has a candidate in the whole chain, else one per group of four
                    // accumulators, and one per accumulator only inside a group that has one. The lanes that have a
                    // candidate append it to their pending buffers, which always have room for a whole chain (ids
                    // past the end are padding).
                    auto max4 = [](int32_t x, int32_t y, int32_t z, int32_t w) -> int32_t {
                        const int32_t m = x > y ? x : y, n = z > w ? z : w;
                        return m > n ? m : n;
                    };
                    if (items) {
                        // over leaves the bound comes from a query's first few leaves only and most accumulators
                        // hold a candidate in some lane: no tests that skip, one predicated append per accumulator
                        // (padding slots are told from points afterwards)
                        // The key is (sum + off + 1) << kIdBits | ~(id - id_base) & kIdMask with id = id0 + c(v); ids of a
                        // leaf's blocks stay below id_base + 2^kIdBits, so the id part is that of id0 less c(v) and the
                        // whole key one shift-and-add per accumulator; the store is the only predicated instruction.
                        const uint32_t kb = ((uint32_t)(off + 1) << kIdBits) + (~(uint32_t)(id0 - id_base) & kIdMask);
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const uint32_t key = ((uint32_t)acc[a][v] << kIdBits) + (kb - (uint32_t)(32 * (v / 4) + 4 * (v % 4)));
                            const bool hit = acc[a][v] > thr;
                            if (hit) *pend = key;
                            pend += hit ? 1 : 0;
                        }
                    }
                    int32_t gmax[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) gmax[g] = max4(acc[a][4 * g], acc[a][4 * g + 1], acc[a][4 * g + 2], acc[a][4 * g + 3]);
                    if (!items && __builtin_expect(__builtin_amdgcn_ballot_w64(max4(gmax[0], gmax[1], gmax[2], gmax[3]) > thr) != 0ull, 0)) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            if (__builtin_amdgcn_ballot_w64(gmax[g] > thr) == 0ull) continue;
#pragma unroll
                            for (int v = 4 * g; v < 4 * g + 4; ++v) {
                                const bool hit = acc[a][v] > thr;
                                if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
                                const int32_t id = id0 + 32 * (v / 4) + 4 * (v % 4);
                                if (hit && id < p.n_valid) {
                                    *pend = ((uint32_t)(acc[a][v] + off + 1) << kIdBits) | (~(uint32_t)(id - id_base) & kIdMask);
                                    ++pend;
                                }
                            }
                        }
                    }
                    // a chain adds at most 16 keys to a lane: flush the queries with less room than that
                    u64 need = __builtin_amdgcn_ballot_w64(pend_end - pend < 16);
                    if (items && __builtin_expect(need != 0ull, 0)) { // every query of the wave at once
                        mfma_dump_items(pend0, (int)(pend - pend0), q, item_hi, p.kept, p.kept_cnt, p.kept_cap);
                        pend = pend0;
                        need = 0ull;
                    }
                    while (__builtin_expect(need != 0ull, 0)) {
                        const int jq = (int)(__builtin_ctzll(need) & 31);
                        flush_query(jq);
                        need &= ~((1ull << jq) | (1ull << (jq + 32)));
                    }
                }
            }
        }
#pragma unroll
        for (int b = 0; b < NS; ++b) w_cur[b] = w_nxt[b];
    }
    if (store) {
        if (p.sample_max != nullptr && live) {
            uint32_t *dst = p.sample_max + ((size_t)q * p.n_chunks + chunk) * 32 + 16 * h;
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[v] = smax[v] == kNone ? 0u : (uint32_t)(smax[v] + off + 1);
        }
        return;
    }

    // drain, then hand the lists over: partial[q][chunk][C]
    {
        u64 rest = __builtin_amdgcn_ballot_w64(pend != pend0);
        if (items && rest) {
            mfma_dump_items(pend0, (int)(pend - pend0), q, item_hi, p.kept, p.kept_cnt, p.kept_cap);
            pend = pend0;
            rest = 0ull;
        }
        while (rest) {
            const int jq = (int)(__builtin_ctzll(rest) & 31);
            flush_query(jq);
            rest &= ~((1ull << jq) | (1ull << (jq + 32)));
        }
    }
    wave_lds_fence();
    if (p.bounds_only) return; // the flushes above have published this wave's bounds; its lists are not wanted
    if (cand_mode && !items && live && h == 0) p.cand_cnt[(size_t)q * p.n_chunks + chunk] = (uint32_t)cpos;
    if (fixed) return;
    for (int jq = 0; jq < kMfmaQueries; ++jq) {
        const int qq = tile * kMfmaQueries + jq;
        if (qq >= p.B) break;
        const uint32_t *list = my_lists + (size_t)jq * C;
        u64 *out = p.partial + ((size_t)qq * p.n_chunks + chunk) * C;
        for (int i = lane; i < C; i += 64) {
            const uint32_t k32 = list[i];
            out[i] = k32 ? make_key(k32 >> kIdBits, id_base + (int32_t)(~k32 & kIdMask)) : 0ull;
        }
    }
}

// ---- host side -----------------------------------------------------------------

bool scan_mfma_supported(int NB, int bits)
{
    return bits == 4 && (NB == 8 || NB == 13 || NB == 25 || NB == 32);
}

void scan_mfma_plan(int B, int64_t n_blocks, int target_waves, ScanParams *p)
{
    p->n_tiles = (B + kMfmaQueries - 1) / kMfmaQueries;
    // Two waves per SIMD on 256 compute units are resident at once: 2048. All waves of a launch do the same
    // work, so a launch takes whole rounds of 2048 waves; unless told otherwise, the number of rounds (1 to 4)
    // is the smallest that leaves less than 3 % of the last round empty, else the one that leaves least
    // (313 tiles: 6 chunks fill 92 % of one round, 13 chunks 99 % of two).
    int64_t target = target_waves > 0 ? target_waves : 2048;
    if (target_waves <= 0) {
        double best = 0.0;
        for (int r = 1; r <= 4; ++r) {
            const int64_t c = (int64_t)r * 2048 / p->n_tiles;
            if (c < 1) continue;
            const double fill = (double)(c * p->n_tiles) / (double)(r * 2048);
            if (fill > best + 1e-9) { best = fill; target = (int64_t)r * 2048; }
            if (fill >= 0.97) break;
        }
    }
    int64_t chunks = target / p->n_tiles;
    const int64_t max_chunks = std::max<int64_t>(1, std::min<int64_t>(256, n_blocks / 4));
    const int64_t min_chunks = (n_blocks + kMfmaMaxChunkBlocks - 1) / kMfmaMaxChunkBlocks; // ids in 32-bit keys
    chunks = std::max<int64_t>(std::max<int64_t>(1, min_chunks), std::min(chunks, max_chunks));
    const int64_t bpc = (n_blocks + chunks - 1) / chunks;
    p->blocks_per_chunk = (int32_t)bpc;
    p->n_chunks = (int32_t)((n_blocks + bpc - 1) / bpc);
    // chunks whose waves are resident together form a threshold group
    const int64_t resident = std::max<int64_t>(1, 2048 / p->n_tiles);
    p->group = (int32_t)std::max<int64_t>(1, std::min<int64_t>(16, std::min<int64_t>(resident, p->n_chunks)));
}

// The sampling launch for a fixed-bound scan planned in `full`: the same queries and chunks, a few
// blocks of every chunk at equal distances (about one in 32, at most 16 per chunk); sample->R is the rank r
// whose sum becomes the bound (see below), sample->ns the list slots for it should the caller scan the
// sample with lists (it sets sample_max to take class maxima instead). Returns false when the chunks are too
// short for a sample (then the caller scans with lists).
bool scan_mfma_sample_plan(const ScanParams &full, ScanParams *sample)
{
    const int64_t bpc = full.blocks_per_chunk;
    if (full.scores_out != nullptr || bpc < 4) return false;
    const int64_t per_chunk = std::max<int64_t>(2, std::min<int64_t>(16, (bpc + 31) / 32));
    const int64_t stride = bpc / per_chunk; // >= 2
    const int64_t visited = (bpc + stride - 1) / stride;
    *sample = full;
    sample->block_stride = (int32_t)stride;
    sample->bounds_only = 0;
    sample->fixed_bound = 0;
    sample->cand_keys = nullptr;
    sample->cand_cnt = nullptr;
    sample->cand_margin = nullptr;
    sample->sample_max = nullptr;
    // mu of the R best of the index fall into the sample on average (Poisson); the r-th best of the
    // sample is below the R-th best of the index unless r or more of them do: r = mu + 5 sigma + 1
    // (a query for which that still happens costs a second scan, a few hundred microseconds per batch)
    const double mu = (double)full.R * (double)visited / (double)bpc;
    int r = std::max(8, (int)std::ceil(mu + 5.0 * std::sqrt(mu) + 1.0));
    if (r > 64 * kMfmaMaxNs) return false;
    sample->R = r;
    sample->ns = (r + 63) / 64;
    return true;
}

size_t scan_mfma_lists_bytes(const ScanParams &p)
{
    return sizeof(u64) * (size_t)p.n_tiles * p.n_chunks * kMfmaQueries * 64 * p.ns;
}

template <int NBT, bool STORE, bool ITEMS, bool FIXED>
static int launch_mfma_one(const ScanParams &p, hipStream_t st)
{
    auto kern = adc_mfma_scan_kernel<NBT, STORE, ITEMS, FIXED>;
    static LdsLimitOnce attr_done; // per instantiation
    AVQ_TRY(set_lds_limit((const void *)kern, kMaxDynLds, &attr_done));
    const int64_t waves = p.item_list ? (int64_t)p.max_items : (int64_t)p.n_tiles * p.n_chunks;
    const int64_t grid = (waves + kMfmaWaves - 1) / kMfmaWaves;
    if (grid > 0x7fffffff) { set_error("scan: grid too large"); return AVQ_EINVAL; }
    const size_t lds = (size_t)kMfmaWaves * 64 * kMfmaPend * sizeof(uint32_t);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kMfmaWaves * 64), lds, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

// flat index: the store variant (scores or class maxima), the scan against fixed bounds, or the scan with lists
template <int NBT>
static int launch_mfma_mode(const ScanParams &p, bool store, hipStream_t st)
{
    if (store) return launch_mfma_one<NBT, true, false, false>(p, st);
    return p.fixed_bound ? launch_mfma_one<NBT, false, false, true>(p, st) : launch_mfma_one<NBT, false, false, false>(p, st);
}

int launch_scan_mfma(const ScanParams &p, hipStream_t st)
{
    if (!scan_mfma_supported(p.NB, p.bits)) { set_error("scan: no matrix-core kernel for this code size"); return AVQ_EINVAL; }
    if (p.item_list != nullptr) {
        if (!p.n_items || !p.qlist || !p.leaf_off || !p.leaf_cnt || !p.leaf_blk || !p.leaf_ip || !p.item_bound || !p.kept ||
            !p.kept_cnt || p.kept_cap < 128 || p.max_items < 1 || !p.scale || !p.bias || p.scores_out || p.M > 64) {
            set_error("scan: the matrix-core kernel over leaves needs its lists, bounds and buffers");
            return AVQ_EINVAL;
        }
        switch (p.NB) {
        case 8: return launch_mfma_one<8, false, true, true>(p, st);
        case 13: return launch_mfma_one<13, false, true, true>(p, st);
        case 25: return launch_mfma_one<25, false, true, true>(p, st);
        default: return launch_mfma_one<32, false, true, true>(p, st);
        }
    }
    if (p.fixed_bound && (p.cand_keys == nullptr || p.thr_shared == nullptr)) {
        set_error("scan: a fixed-bound scan needs bounds and candidate buffers");
        return AVQ_EINVAL;
    }
    if (p.scores_out == nullptr && p.sample_max == nullptr && !p.fixed_bound &&
        (p.lists_ws == nullptr || p.thr_shared == nullptr || p.kth_shared == nullptr || (p.partial == nullptr && !p.bounds_only) ||
         p.group < 1)) {
        set_error("scan: matrix-core kernel needs its scratch buffers");
        return AVQ_EINVAL;
    }
    if (p.sample_max == nullptr && (p.R < 1 || p.R > 64 * p.ns)) { set_error("scan: R does not fit the lists"); return AVQ_EINVAL; }
    if (p.cand_keys != nullptr && (p.cand_cnt == nullptr || p.cand_cap < 128)) {
        set_error("scan: candidate mode needs counts and room for one flush");
        return AVQ_EINVAL;
    }
    if (p.blocks_per_chunk > kMfmaMaxChunkBlocks || p.M > 64) { set_error("scan: chunk or code too large for 32-bit keys"); return AVQ_EINVAL; }
    const bool store = p.scores_out != nullptr || p.sample_max != nullptr;
    switch (p.NB) {
    case 8: return launch_mfma_mode<8>(p, store, st);
    case 13: return launch_mfma_mode<13>(p, store, st);
    case 25: return launch_mfma_mode<25>(p, store, st);
    default: return launch_mfma_mode<32>(p, store, st);
    }
}

} // namespace avq
