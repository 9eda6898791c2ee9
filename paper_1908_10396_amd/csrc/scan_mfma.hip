// ADC scan of 4-bit codes against 8-bit tables on the matrix cores of gfx950.
//
// With 16 codewords per subspace the table sum  sum_m Q[q][m][code[n][m]]  is a dense
// contraction of a one-hot matrix with the tables: row n of A has, for every subspace,
// sixteen 0/1 bytes with the 1 at the point's code; column q of B holds the sixteen
// table bytes of every subspace. v_mfma_i32_32x32x32_i8 multiplies 32 points by 32
// queries over 32 such positions (two subspaces: lanes 0-31 carry one, lanes 32-63 the
// other) and accumulates exact 32-bit integers, so the result is the integer sum the
// 8-bit path is defined by, bit for bit. Tables are biased by -128 to fit the signed
// operand; the bias, 128 per subspace, is added back when a key is made.
//
// One wave owns 32 queries and a chunk of the blocks. Its B operands (25 registers
// of 16 bytes for 50 subspaces) stay in registers for the whole scan; the A operand
// of a (point, subspace) is one 16-byte read from a 256-byte LDS table of the sixteen
// one-hot patterns, addressed by the code -- no bank conflicts, since the patterns
// cover every bank once. The order of the sum does not matter (integers), so any
// pairing of operand positions with subspaces is valid as long as A and B agree.
//
// A lane ends up with the scores of 16 points for one query (lanes l and l + 32 share
// query l % 32). Scores above the query's threshold go to a lane-private pending
// buffer in LDS; when a lane's buffer is half full the two buffers of the query are
// sorted and merged into the query's candidate list (global scratch), which tightens
// the threshold. The waves that scan different chunks for the same queries share
// their thresholds through a global array (atomic max): any wave's R-th best score
// is a lower bound of the final R-th best score, so points below it can be dropped
// by every wave, whatever the timing.
#include "avq_internal.h"
#include "wave_topk.h"

namespace avq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMfmaQueries = 32; // queries per wave
constexpr int kMfmaPend = 32;    // pending keys per lane
constexpr int kMfmaWaves = 4;    // waves per workgroup

template <int NBT>
__global__ void __launch_bounds__(kMfmaWaves * 64)
adc_mfma_scan_kernel(const ScanParams p)
{
    __shared__ __align__(16) uint32_t onehot[64];
    extern __shared__ __align__(16) unsigned char dyn_smem[]; // [waves][64 lanes][kMfmaPend] keys
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x < 64) {
        const int c = threadIdx.x >> 2, dw = threadIdx.x & 3; // pattern c, dword dw
        onehot[threadIdx.x] = (dw == (c >> 2)) ? (1u << (8 * (c & 3))) : 0u;
    }
    __syncthreads();
    const int64_t gw = (int64_t)blockIdx.x * kMfmaWaves + wave; // wave index over (chunk, tile)
    if (gw >= (int64_t)p.n_tiles * p.n_chunks) return;
    const int tile = (int)(gw % p.n_tiles), chunk = (int)(gw / p.n_tiles);
    const int j = lane & 31, h = lane >> 5;
    const int q = tile * kMfmaQueries + j;
    const bool live = q < p.B;
    const int C = 64 * p.ns;
    const int off = 128 * p.M;
    const bool store = p.scores_out != nullptr;

    // table operands: position s takes subspaces 2s (lanes 0-31) and 2s + 1 (lanes 32-63)
    v4i bq[NBT];
#pragma unroll
    for (int s = 0; s < NBT; ++s) {
        const int row = 2 * s + h;
        uint4 r = make_uint4(0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u); // -> 0
        if (live && row < p.M) r = *(const uint4 *)(p.lut8 + ((size_t)q * p.M + row) * 16);
        bq[s] = v4i{(int)(r.x ^ 0x80808080u), (int)(r.y ^ 0x80808080u), (int)(r.z ^ 0x80808080u),
                    (int)(r.w ^ 0x80808080u)};
    }

    u64 *my_lists = nullptr;
    u64 *my_pend = (u64 *)dyn_smem + ((size_t)wave * 64 + lane) * kMfmaPend;
    if (!store) {
        my_lists = p.lists_ws + (size_t)gw * kMfmaQueries * C;
        for (int i = lane; i < kMfmaQueries * C; i += 64) my_lists[i] = 0ull;
        wave_lds_fence();
    }
    int cnt = 0;                 // keys in this lane's pending buffer
    uint32_t local_ord = 0u;     // ordering value of the R-th best key of this lane's query in this wave
    uint32_t shared_ord = 0u;    // the same, best over all waves (as last read)
    // A score enters when its ordering value (sum + 1) is >= the threshold's: later points
    // of a wave can have lower ids than earlier ones, so equal scores must pass.
    auto thr_of = [&]() -> int {
        if (!live) return 0x7fffffff;
        const uint32_t o = local_ord > shared_ord ? local_ord : shared_ord;
        return (int)o - off - 2;
    };
    int thr = thr_of();

    // merges the pending keys of query jq (lanes jq and jq + 32) into its list
    auto flush_query = [&](int jq) {
        const int src = jq + 32 * h;
        const int cnt_src = __shfl(cnt, src, 64);
        wave_lds_fence();
        u64 key = j < cnt_src ? ((const u64 *)dyn_smem)[((size_t)wave * 64 + src) * kMfmaPend + j] : 0ull;
        key = wave_sort_desc(key);
        u64 *list = my_lists + (size_t)jq * C;
        wave_list_insert_sorted(list, p.ns, key);
        const u64 kth = list[p.R - 1];
        const uint32_t ord = key_ord(kth);
        if (j == jq) {
            cnt = 0;
            local_ord = ord;
            thr = thr_of();
            if (h == 0 && ord > 0u && live)
                __hip_atomic_fetch_max(p.thr_shared + q, ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    const int64_t first = (int64_t)chunk * p.blocks_per_chunk;
    int64_t end = first + p.blocks_per_chunk;
    if (end > p.n_blocks) end = p.n_blocks;
    const uint32_t nib_shift = 4u * (uint32_t)(1 - h); // brings this half-wave's nibble to bits 4..7 of each byte

    for (int64_t blk = first; blk < end; ++blk) {
        const uint8_t *base = p.codes + (size_t)blk * 256 * NBT;
        if (!store && live) {
            shared_ord = __hip_atomic_load(p.thr_shared + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            thr = thr_of();
        }
#pragma unroll 1
        for (int H = 0; H < 2; ++H) {
            // lane (j, h) takes the four points of lane slot H*32 + j of the block's rows
            const int slot = H * 32 + j;
            uint32_t w[NBT];
#pragma unroll
            for (int r = 0; r < NBT / 4; ++r) {
                const uint4 t = ((const uint4 *)(base + (size_t)r * 1024))[slot];
                w[4 * r] = t.x; w[4 * r + 1] = t.y; w[4 * r + 2] = t.z; w[4 * r + 3] = t.w;
            }
#pragma unroll
            for (int t = 0; t < NBT % 4; ++t)
                w[(NBT / 4) * 4 + t] = ((const uint32_t *)(base + (size_t)(NBT / 4) * 1024 + (size_t)t * 256))[slot];
#pragma unroll
            for (int b = 0; b < NBT; ++b) w[b] <<= nib_shift;
#pragma unroll
            for (int u0 = 0; u0 < 4; u0 += 2) {
                // two independent accumulation chains: points 4i + u0 and 4i + u0 + 1
                v16i acc[2];
#pragma unroll
                for (int a = 0; a < 2; ++a) acc[a] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int s = 0; s < NBT; ++s) {
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        const uint32_t o = (w[s] >> (8 * (u0 + a))) & 0xf0u;
                        const v4i av = *(const v4i *)((const unsigned char *)onehot + o);
                        acc[a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bq[s], acc[a], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    // accumulator v of lane (j, h): point row 8*(v/4) + 4*h + v%4 of the 32, query j
                    const int32_t id0 = (int32_t)(blk * 256) + H * 128 + 16 * h + (u0 + a);
                    if (store) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int32_t id = id0 + 32 * (v / 4) + 4 * (v % 4);
                            if (live && id < p.n_valid)
                                ((int32_t *)p.scores_out)[(size_t)q * p.score_stride + id] = acc[a][v] + off;
                        }
                        continue;
                    }
                    bool pushed = false;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int32_t id = id0 + 32 * (v / 4) + 4 * (v % 4);
                        const bool hit = acc[a][v] > thr && id < p.n_valid;
                        if (__builtin_amdgcn_ballot_w64(hit) == 0ull) continue;
                        if (hit) {
                            my_pend[cnt] = make_key((uint32_t)(acc[a][v] + off + 1), id);
                            ++cnt;
                        }
                        pushed = true;
                    }
                    if (pushed) {
                        // a chain adds at most 16 keys to a lane: keep every buffer at most half full
                        u64 full = __builtin_amdgcn_ballot_w64(cnt > kMfmaPend - 16);
                        while (full) {
                            const int jq = (int)(__builtin_ctzll(full) & 31);
                            flush_query(jq);
                            full &= ~((1ull << jq) | (1ull << (jq + 32)));
                        }
                    }
                }
            }
        }
    }
    if (store) return;

    // drain, then hand the lists over: partial[q][chunk][C]
    {
        u64 rest = __builtin_amdgcn_ballot_w64(cnt > 0);
        while (rest) {
            const int jq = (int)(__builtin_ctzll(rest) & 31);
            flush_query(jq);
            rest &= ~((1ull << jq) | (1ull << (jq + 32)));
        }
    }
    wave_lds_fence();
    for (int jq = 0; jq < kMfmaQueries; ++jq) {
        const int qq = tile * kMfmaQueries + jq;
        if (qq >= p.B) break;
        const u64 *list = my_lists + (size_t)jq * C;
        u64 *out = p.partial + ((size_t)qq * p.n_chunks + chunk) * C;
        for (int i = lane; i < C; i += 64) out[i] = list[i];
    }
}

// ---- host side -----------------------------------------------------------------

bool scan_mfma_supported(int NB, int bits)
{
    return bits == 4 && (NB == 8 || NB == 25 || NB == 32);
}

void scan_mfma_plan(int B, int64_t n_blocks, int target_waves, ScanParams *p)
{
    p->n_tiles = (B + kMfmaQueries - 1) / kMfmaQueries;
    // two rounds of two waves per SIMD over 256 compute units, unless told otherwise
    const int64_t target = target_waves > 0 ? target_waves : 4096;
    int64_t chunks = (target + p->n_tiles / 2) / p->n_tiles;
    const int64_t max_chunks = std::max<int64_t>(1, std::min<int64_t>(256, n_blocks / 4));
    chunks = std::max<int64_t>(1, std::min(chunks, max_chunks));
    const int64_t bpc = (n_blocks + chunks - 1) / chunks;
    p->blocks_per_chunk = (int32_t)bpc;
    p->n_chunks = (int32_t)((n_blocks + bpc - 1) / bpc);
}

size_t scan_mfma_lists_bytes(const ScanParams &p)
{
    return sizeof(u64) * (size_t)p.n_tiles * p.n_chunks * kMfmaQueries * 64 * p.ns;
}

template <int NBT>
static int launch_mfma_one(const ScanParams &p, hipStream_t st)
{
    auto kern = adc_mfma_scan_kernel<NBT>;
    static bool attr_done = false;
    if (!attr_done) {
        AVQ_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds));
        attr_done = true;
    }
    const int64_t waves = (int64_t)p.n_tiles * p.n_chunks;
    const int64_t grid = (waves + kMfmaWaves - 1) / kMfmaWaves;
    if (grid > 0x7fffffff) { set_error("scan: grid too large"); return AVQ_EINVAL; }
    const size_t lds = (size_t)kMfmaWaves * 64 * kMfmaPend * sizeof(u64);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kMfmaWaves * 64), lds, st, p);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

int launch_scan_mfma(const ScanParams &p, hipStream_t st)
{
    if (!scan_mfma_supported(p.NB, p.bits)) { set_error("scan: no matrix-core kernel for this code size"); return AVQ_EINVAL; }
    if (p.scores_out == nullptr && (p.lists_ws == nullptr || p.thr_shared == nullptr || p.partial == nullptr)) {
        set_error("scan: matrix-core kernel needs its scratch buffers");
        return AVQ_EINVAL;
    }
    if (p.R < 1 || p.R > 64 * p.ns) { set_error("scan: R does not fit the lists"); return AVQ_EINVAL; }
    switch (p.NB) {
    case 8: return launch_mfma_one<8>(p, st);
    case 25: return launch_mfma_one<25>(p, st);
    default: return launch_mfma_one<32>(p, st);
    }
}

} // namespace avq
