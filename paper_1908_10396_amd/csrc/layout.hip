// Logical code layout ([n][NB] bytes, what the C ABI exchanges) -> the blocked
// layout the scan streams: blocks of 256 points, byte position b of a block is
// a 256-byte plane (lane l = points 4l..4l+3), planes grouped by four into
// 1 KiB rows of 16 bytes per lane, left-over planes stored as dword rows.
#include "avq_internal.h"

namespace avq {

__global__ void to_blocked_kernel(const uint8_t *__restrict__ logical, int64_t n, int NB,
                                  const int32_t *__restrict__ slot_of, uint8_t *__restrict__ blocked)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * NB) return;
    const int64_t i = t / NB;
    const int b = (int)(t % NB);
    const int64_t slot = slot_of ? (int64_t)slot_of[i] : i;
    const int64_t blk = slot >> 8;
    const int within = (int)(slot & 255);
    const int lane = within >> 2, pt = within & 3;
    const int nfull = NB / 4;
    size_t off = (size_t)blk * 256 * NB;
    if (b < nfull * 4) off += (size_t)(b / 4) * 1024 + (size_t)lane * 16 + (size_t)(b % 4) * 4 + pt;
    else off += (size_t)nfull * 1024 + (size_t)(b - nfull * 4) * 256 + (size_t)lane * 4 + pt;
    blocked[off] = logical[t];
}

int launch_to_blocked(const uint8_t *logical, int64_t n, int NB, const int32_t *slot_of,
                      uint8_t *blocked, int64_t n_slots, hipStream_t st)
{
    AVQ_HIP(hipMemsetAsync(blocked, 0, (size_t)n_slots * NB, st));
    const int64_t total = n * NB;
    const int64_t grid = (total + 255) / 256;
    if (grid > 0x7fffffff) { set_error("layout: too many code bytes for one launch"); return AVQ_EINVAL; }
    hipLaunchKernelGGL(to_blocked_kernel, dim3((unsigned)grid), dim3(256), 0, st, logical, n, NB,
                       slot_of, blocked);
    AVQ_HIP(hipGetLastError());
    return AVQ_OK;
}

} // namespace avq
