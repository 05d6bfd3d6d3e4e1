// Inverse of the 3-D cast: v = X * P (Section 2 of arXiv 2310.10537) for an MX tensor whose blocks
// run along any axis of a [d0][d1][d2] tensor (Section 3: the principal axis of a multi-dimensional
// tensor), in either layout that launch_cast_3d writes.  The result is written with element strides
// (stride0, stride1, 1).
//
// Block-major layout: every choice of axis is a batch of the 2-D dequantize kernels on slices (the
// same decomposition as the cast).  Source-order layout: codes sit where the elements sat, the
// scale of element (i0, i1, i2) is the scale array's entry with the block axis index divided by 32;
// one lane decodes 8 consecutive codes of a row, each with its own scale byte when the blocks run
// along d0 or d1 (the scale bytes of 8 neighbours are then 8 consecutive bytes).
#include "mx_device.hpp"
#include "mx_launch.hpp"

namespace mx {
namespace {

// codes i .. i+7 of a row whose packed bytes start at p (w-bit codes, little-endian dense packing);
// reads only the bytes those n <= 8 codes occupy
template <int W>
__device__ __forceinline__ uint64_t load_code_bits(const uint8_t *p, int64_t i, int n)
{
    const int64_t first = i * W / 8;                      // i is a multiple of 8: first bit is byte-aligned
    const int nbytes = (n * W + 7) / 8;
    uint64_t bits = 0;
#pragma unroll
    for (int b = 0; b < W; b++)
        if (b < nbytes) bits |= (uint64_t)p[first + b] << (8 * b);
    return bits;
}

template <int FMT, int DST>
__global__ __launch_bounds__(256) void dequant_keep_kernel(const uint8_t *__restrict__ elems, const uint8_t *__restrict__ scales,
                                                           void *__restrict__ dst, int64_t d0, int64_t d1, int64_t d2, int axis,
                                                           int64_t nblk, int64_t stride0, int64_t stride1)
{
    constexpr int w = Fmt<FMT>::bits;
    const int64_t units_per_row = (d2 + 7) / 8, n_units = d0 * d1 * units_per_row, row_bytes = d2 * w / 8;
    const int64_t step = (int64_t)gridDim.x * 256;
    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < n_units; u += step) {
        const int64_t row = u / units_per_row, k = (u - row * units_per_row) * 8;
        const int64_t i0 = row / d1, i1 = row - i0 * d1;
        const int n = d2 - k < 8 ? (int)(d2 - k) : 8;
        const uint64_t bits = load_code_bits<w>(elems + row * row_bytes, k, n);
        // scale of element k + j: the block axis index divided by 32 in the scale array's shape
        const uint8_t *sp;
        int64_t sstep;                                    // distance between the scales of neighbours along d2
        if (axis == 2)      { sp = scales + row * nblk + k / BLOCK; sstep = 0; }          // 8 | 32: one block per unit
        else if (axis == 1) { sp = scales + (i0 * nblk + i1 / BLOCK) * d2 + k; sstep = 1; }
        else                { sp = scales + ((i0 / BLOCK) * d1 + i1) * d2 + k; sstep = 1; }
        const int64_t o = i0 * stride0 + i1 * stride1 + k;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (j >= n) break;
            const float v = decode_scaled<FMT>((uint32_t)(bits >> (w * j)) & ((1u << w) - 1u), sp[j * sstep]);
            if (DST == DT_F32) reinterpret_cast<float *>(dst)[o + j] = v;
            else reinterpret_cast<uint16_t *>(dst)[o + j] = (uint16_t)f32_to_bf16_bits(v);
        }
    }
}

template <int FMT>
hipError_t launch_keep_t(const uint8_t *elems, const uint8_t *scales, void *dst, int dst_dt, int64_t d0, int64_t d1, int64_t d2,
                         int axis, int64_t nblk, int64_t stride0, int64_t stride1, hipStream_t st)
{
    int64_t nb = (d0 * d1 * ((d2 + 7) / 8) + 255) / 256;
    if (nb > 0x7FFFFFFF) nb = 0x7FFFFFFF;
    if (dst_dt == DT_F32)
        hipLaunchKernelGGL((dequant_keep_kernel<FMT, DT_F32>), dim3((unsigned)nb), dim3(256), 0, st, elems, scales, dst, d0, d1, d2, axis,
                           nblk, stride0, stride1);
    else
        hipLaunchKernelGGL((dequant_keep_kernel<FMT, DT_BF16>), dim3((unsigned)nb), dim3(256), 0, st, elems, scales, dst, d0, d1, d2, axis,
                           nblk, stride0, stride1);
    return hipGetLastError();
}

hipError_t launch_keep(int fmt, const uint8_t *elems, const uint8_t *scales, void *dst, int dst_dt, int64_t d0, int64_t d1, int64_t d2,
                       int axis, int64_t nblk, int64_t stride0, int64_t stride1, hipStream_t st)
{
    switch (fmt) {
        case FP8_E4M3: return launch_keep_t<FP8_E4M3>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
        case FP8_E5M2: return launch_keep_t<FP8_E5M2>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
        case FP6_E3M2: return launch_keep_t<FP6_E3M2>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
        case FP6_E2M3: return launch_keep_t<FP6_E2M3>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
        case FP4_E2M1: return launch_keep_t<FP4_E2M1>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
        default:       return launch_keep_t<INT8>(elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
    }
}

}  // namespace

hipError_t launch_dequant_3d(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t d0, int64_t d1, int64_t d2, int axis,
                             bool keep_order, void *dst, int dst_dt, int64_t stride0, int64_t stride1, hipStream_t st)
{
    const int64_t dim[3] = {d0, d1, d2};
    const int64_t L = dim[axis], nblk = (L + BLOCK - 1) / BLOCK;
    const int w = fmt_bits(fmt);
    const int64_t line_bytes = nblk * BLOCK * w / 8, esz = dst_dt == DT_F32 ? 4 : 2;
    uint8_t *d8 = static_cast<uint8_t *>(dst);
    if (keep_order && !(axis == 2 && d2 % BLOCK == 0))    // (whole blocks along the last axis: both layouts coincide)
        return launch_keep(fmt, elems, scales, dst, dst_dt, d0, d1, d2, axis, nblk, stride0, stride1, st);
    if (axis == 2) {
        if (stride0 == d1 * stride1) return launch_dequant(elems, scales, fmt, d0 * d1, d2, 1, dst, dst_dt, stride1, st);
        for (int64_t i = 0; i < d0; i++) {
            const hipError_t e = launch_dequant(elems + i * d1 * line_bytes, scales + i * d1 * nblk, fmt, d1, d2, 1,
                                                d8 + i * stride0 * esz, dst_dt, stride1, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (axis == 1) {        // per i0 the transposed-axis dequantize of [d2] lines of length d1 into the [d1][d2] slice
        for (int64_t i = 0; i < d0; i++) {
            const hipError_t e = launch_dequant(elems + i * d2 * line_bytes, scales + i * d2 * nblk, fmt, d1, d2, 0,
                                                d8 + i * stride0 * esz, dst_dt, stride1, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    // axis 0: [d1 * d2] lines of length d0; one launch when the rows of the result are dense
    if (stride1 == d2) return launch_dequant(elems, scales, fmt, d0, d1 * d2, 0, dst, dst_dt, stride0, st);
    for (int64_t i = 0; i < d1; i++) {
        const hipError_t e = launch_dequant(elems + i * d2 * line_bytes, scales + i * d2 * nblk, fmt, d0, d2, 0,
                                            d8 + i * stride1 * esz, dst_dt, stride0, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace mx
