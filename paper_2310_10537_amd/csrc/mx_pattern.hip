// Measurement aid, not part of the MX path: kernels that move bytes in the access pattern of the
// row cast and the dequantize (a wave takes consecutive 16-byte pieces, several loads in flight per
// lane, 16-byte stores) with no arithmetic beyond an XOR, so that a benchmark can measure, on the
// same box and in the same run, what such a pattern can reach: pure read, pure write, copy, and R
// bytes read per byte written (R = 2: an 8-bit cast of bf16; R = 4: a 4-bit cast).
#include "../../include/mx.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mx_device.hpp"

namespace {

constexpr int LANES = 256;

constexpr int UNROLL = 2;   // groups per thread: R * UNROLL loads in flight per lane, as in the cast kernels

// R 16-byte loads per 16-byte store, UNROLL such groups per thread; a work-group covers consecutive
// memory.  R = 0: stores only.  W = false: loads only (a store guarded by a test that never holds
// keeps the loads alive).
template <int R, bool W>
__global__ __launch_bounds__(LANES) void pattern_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, uint32_t never)
{
    constexpr int NL = R > 0 ? R * UNROLL : 1;
    uint4 v[NL];
    if (R > 0) {
        // the work-group reads R * UNROLL * LANES consecutive pieces; piece j goes to lane j % LANES
        const uint4 *p = src + (int64_t)blockIdx.x * (LANES * NL) + threadIdx.x;
#pragma unroll
        for (int i = 0; i < NL; i++) v[i] = mx::ld16_nt(p + (int64_t)i * LANES);   // streaming loads, as in the casts
    }
    uint4 *q = dst + (int64_t)blockIdx.x * (LANES * UNROLL) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < UNROLL; u++) {
        uint4 acc = make_uint4(threadIdx.x, 1, 2, (uint32_t)u);
#pragma unroll
        for (int i = 0; i < R; i++) { const uint4 w = v[u * R + i]; acc.x ^= w.x; acc.y ^= w.y; acc.z ^= w.z; acc.w ^= w.w; }
        if (W) q[(int64_t)u * LANES] = acc;
        else if (acc.x == never && acc.y == never + 1 && acc.z == never + 2) dst[0] = acc;
    }
}

}  // namespace

extern "C" int mx_stream_pattern(const void *src, void *dst, int64_t dst_bytes, int read_per_write, int write, void *hip_stream)
{
    if (dst_bytes < 0 || dst_bytes % 16 || read_per_write < 0 || (read_per_write != 0 && read_per_write != 1 && read_per_write != 2 && read_per_write != 4) ||
        (read_per_write == 0 && !write))
        return MX_ERR_SHAPE;
    if (dst_bytes == 0) return MX_OK;
    if (!dst || (read_per_write > 0 && !src)) return MX_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return MX_ERR_ALIGN;
    const int64_t groups = dst_bytes / 16;
    if (groups % (LANES * UNROLL)) return MX_ERR_SHAPE;     // whole work-groups only: every load stays inside src
    const unsigned grid = (unsigned)(groups / (LANES * UNROLL));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint4 *s = static_cast<const uint4 *>(src);
    uint4 *d = static_cast<uint4 *>(dst);
    const uint32_t never = 0x9E3779B9u;
#define MX_GO(R, W) hipLaunchKernelGGL((pattern_kernel<R, W>), dim3(grid), dim3(LANES), 0, st, s, d, never)
    switch (read_per_write * 2 + (write ? 1 : 0)) {
        case 1: MX_GO(0, true); break;
        case 2: MX_GO(1, false); break;
        case 3: MX_GO(1, true); break;
        case 4: MX_GO(2, false); break;
        case 5: MX_GO(2, true); break;
        case 8: MX_GO(4, false); break;
        default: MX_GO(4, true); break;
    }
#undef MX_GO
    return hipGetLastError() == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}
