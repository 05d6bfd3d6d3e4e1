// Measurement aid (no part of the MX path): the LDS-tiled GEMM kernels of three format pairs, built
// so that every work-group also reports how long its K loop took in shader clocks and in ticks of
// the constant 100 MHz counter.  A benchmark derives from that the shader clock under the GEMM's
// load (which drops with the switching activity of the operands: the power limit) and the clocks
// one K step takes (against 2048 / 1024 clocks of matrix instructions for 8-bit / narrower pairs).
#include "mx_gemm_tile8.hpp"
#include "mx_gemm_tile16.hpp"

#include "../../include/mx.h"

namespace mx {
namespace {

template <int FA, int FB>
hipError_t probe4(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be, const uint8_t *Bs,
                  void *C, int64_t ldc, unsigned long long *probe, hipStream_t st)
{
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
    const Raster rast = choose_raster(tiles_m, tiles_n, Fmt<FA>::bits, Fmt<FB>::bits);
    if (K >= 1024)      // as mx_gemm picks them
        hipLaunchKernelGGL((gemm_tile16_kernel<FA, FB, DT_BF16, true>), dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(256), 0, st, M, N, K,
                           Ae, As, Be, Bs, C, ldc, tiles_m, tiles_n, rast, probe);
    else
        hipLaunchKernelGGL((gemm_tile_kernel<FA, FB, DT_BF16, false, ROUND_RNE, true>), dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(256),
                           0, st, M, N, K, Ae, As, static_cast<const uint16_t *>(nullptr), (int64_t)0, Be, Bs, C, ldc, tiles_m, tiles_n,
                           static_cast<uint8_t *>(nullptr), 0, rast, probe);
    return hipGetLastError();
}

template <int FA, int FB>
hipError_t probe8(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be, const uint8_t *Bs,
                  void *C, int64_t ldc, unsigned long long *probe, hipStream_t st)
{
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
    const Raster rast = choose_raster(tiles_m, tiles_n, Fmt<FA>::bits, Fmt<FB>::bits);
    hipLaunchKernelGGL((gemm_tile8_kernel<FA, FB, DT_BF16, true>), dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(512), 0, st, M, N, K, Ae,
                       As, Be, Bs, C, ldc, tiles_m, tiles_n, rast, probe);
    return hipGetLastError();
}

// The matrix instruction alone: four waves per compute unit, each issuing 16 * iters instructions on
// operand registers loaded once (eight 32-byte fragments per lane from `codes`), 256 accumulator
// registers as in the GEMM kernels, no memory access inside the loop.
template <int HF>
__global__ __launch_bounds__(256, 1) void mfma_stream_kernel(const v8i_t *__restrict__ codes, int iters, float *__restrict__ sink,
                                                             unsigned long long *__restrict__ probe)
{
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    const int tid = threadIdx.x;
    v8i_t a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; i++) { a[i] = codes[i * 256 + tid]; b[i] = codes[(4 + i) * 256 + tid]; }
    v16f_t acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][y][t] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int x = 0; x < 4; x++)
                acc[x][y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[x], b[y], acc[x][y], HF, HF, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
    float sum = 0.f;
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) sum += acc[x][y][t];
    sink[blockIdx.x * 256 + tid] = sum;
    if (tid == 0) {
        probe[2 * blockIdx.x] = __builtin_readcyclecounter() - c0;
        probe[2 * blockIdx.x + 1] = __builtin_amdgcn_s_memrealtime() - r0;
    }
}

}  // namespace
}  // namespace mx

extern "C" int mx_mfma_stream_probe(mx_format_t fmt, const void *codes, int iters, float *sink, uint64_t *probe, void *hip_stream)
{
    using namespace mx;
    if (iters <= 0 || iters > (1 << 20)) return MX_ERR_SHAPE;
    if (!codes || !sink || !probe) return MX_ERR_NULL;
    if (((uintptr_t)codes & 31) || ((uintptr_t)sink & 15) || ((uintptr_t)probe & 15)) return MX_ERR_ALIGN;
    const auto *src = static_cast<const v8i_t *>(codes);
    auto *pr = reinterpret_cast<unsigned long long *>(probe);
    auto st = static_cast<hipStream_t>(hip_stream);
    constexpr int WGS = MX_MFMA_STREAM_WGS;
    switch (fmt) {
        case MX_FP8_E4M3: hipLaunchKernelGGL((mfma_stream_kernel<hw_fmt(FP8_E4M3)>), dim3(WGS), dim3(256), 0, st, src, iters, sink, pr); break;
        case MX_FP8_E5M2: hipLaunchKernelGGL((mfma_stream_kernel<hw_fmt(FP8_E5M2)>), dim3(WGS), dim3(256), 0, st, src, iters, sink, pr); break;
        case MX_FP6_E3M2: hipLaunchKernelGGL((mfma_stream_kernel<hw_fmt(FP6_E3M2)>), dim3(WGS), dim3(256), 0, st, src, iters, sink, pr); break;
        case MX_FP6_E2M3: hipLaunchKernelGGL((mfma_stream_kernel<hw_fmt(FP6_E2M3)>), dim3(WGS), dim3(256), 0, st, src, iters, sink, pr); break;
        case MX_FP4_E2M1: hipLaunchKernelGGL((mfma_stream_kernel<hw_fmt(FP4_E2M1)>), dim3(WGS), dim3(256), 0, st, src, iters, sink, pr); break;
        default: return MX_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

extern "C" int mx_gemm_probe(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
                             const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C_bf16, int64_t ldc,
                             uint64_t *probe, int64_t probe_len, void *hip_stream)
{
    using namespace mx;
    if (M <= 0 || N <= 0 || K < 512 || M % TM || N % TN || K % TK || ldc < N) return MX_ERR_SHAPE;
    if (!A_elems || !A_scales || !B_elems || !B_scales || !C_bf16 || !probe) return MX_ERR_NULL;
    // the linear tile walk pads the grid to a multiple of 8 work-groups
    const int64_t wgs = ((M / TM) * (N / TN) + 7) / 8 * 8;
    if (probe_len < 2 * wgs) return MX_ERR_SHAPE;
    if (((uintptr_t)A_elems | (uintptr_t)B_elems | (uintptr_t)C_bf16 | (uintptr_t)A_scales | (uintptr_t)B_scales | (uintptr_t)probe) & 15)
        return MX_ERR_ALIGN;
    const auto *Ae = static_cast<const uint8_t *>(A_elems), *Be = static_cast<const uint8_t *>(B_elems);
    auto *pr = reinterpret_cast<unsigned long long *>(probe);
    auto st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (fmtA == MX_FP8_E4M3 && fmtB == MX_FP8_E4M3) e = probe4<FP8_E4M3, FP8_E4M3>(M, N, K, Ae, A_scales, Be, B_scales, C_bf16, ldc, pr, st);
    else if (fmtA == MX_FP6_E3M2 && fmtB == MX_FP6_E3M2) e = probe8<FP6_E3M2, FP6_E3M2>(M, N, K, Ae, A_scales, Be, B_scales, C_bf16, ldc, pr, st);
    else if (fmtA == MX_FP6_E3M2 && fmtB == MX_FP4_E2M1) e = probe8<FP6_E3M2, FP4_E2M1>(M, N, K, Ae, A_scales, Be, B_scales, C_bf16, ldc, pr, st);
    else return MX_ERR_UNSUPPORTED;
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}
