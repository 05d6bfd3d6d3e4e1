// MX dequantize kernels: v = X * P (Section 2 of arXiv 2310.10537) for gfx950.
// One lane turns 8 consecutive element codes of a block (w bytes) into 8 values.
#include "mx_device.hpp"
#include "mx_launch.hpp"

namespace mx {

// 8 codes = w bytes starting at a w-byte-aligned address
template <int FMT>
__device__ __forceinline__ void load_codes8(const uint8_t *p, uint32_t (&c)[8])
{
    constexpr int w = Fmt<FMT>::bits;
    uint64_t bits;
    if (w == 8) {
        uint2 d = *reinterpret_cast<const uint2 *>(p);
        bits = (uint64_t)d.x | ((uint64_t)d.y << 32);
    } else if (w == 4) {
        bits = *reinterpret_cast<const uint32_t *>(p);
    } else {
        const uint16_t *h = reinterpret_cast<const uint16_t *>(p);
        bits = (uint64_t)h[0] | ((uint64_t)h[1] << 16) | ((uint64_t)h[2] << 32);
    }
#pragma unroll
    for (int i = 0; i < 8; i++) c[i] = (uint32_t)(bits >> (w * i)) & ((1u << w) - 1u);
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x32_t __attribute__((ext_vector_type(32)));
typedef uint32_t u32x6_t_ __attribute__((ext_vector_type(6)));
typedef __bf16 bf16x2_t_ __attribute__((ext_vector_type(2)));

// 8 consecutive codes (w bytes at p) times X = 2^(s-127) as Float32, with gfx950's scaled
// up-converts (V_CVT_SCALEF32_PK_F32_FP8 / _BF8 / _FP4, _PK32_F32_FP6 / _BF6): checked against the
// CPU reference for every code at every scale byte 0 .. 254 -- subnormal codes, NaN and Inf
// codes, products that overflow Float32 and X = 2^-127 included -- they return exactly X * P.
// (The integer decode costs about 20 vector instructions per element, which made the kernel
// compute-bound.)  The NaN scale 0xFF is the caller's business.
template <int FMT>
__device__ __forceinline__ void decode8_hw(const uint8_t *p, uint32_t s, float (&f)[8])
{
    const float sf = __uint_as_float(s << 23);
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) {
        const uint2 d = *reinterpret_cast<const uint2 *>(p);
        const uint32_t dw[2] = {d.x, d.y};
#pragma unroll
        for (int j = 0; j < 2; j++) {
            f32x2_t lo, hi;
            if (FMT == FP8_E4M3) {
                lo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(dw[j], sf, false);
                hi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(dw[j], sf, true);
            } else {
                lo = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(dw[j], sf, false);
                hi = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(dw[j], sf, true);
            }
            f[4 * j] = lo[0]; f[4 * j + 1] = lo[1]; f[4 * j + 2] = hi[0]; f[4 * j + 3] = hi[1];
        }
    } else if constexpr (FMT == FP4_E2M1) {
        const uint32_t d = *reinterpret_cast<const uint32_t *>(p);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            f32x2_t v;
            if (j == 0) v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(d, sf, 0);
            if (j == 1) v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(d, sf, 1);
            if (j == 2) v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(d, sf, 2);
            if (j == 3) v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(d, sf, 3);
            f[2 * j] = v[0]; f[2 * j + 1] = v[1];
        }
    } else if constexpr (FMT == FP6_E3M2 || FMT == FP6_E2M3) {
        // 8 codes = 48 bits; the 32-element convert takes them in the low bits of its six dwords
        const uint16_t *h = reinterpret_cast<const uint16_t *>(p);
        const u32x6_t_ d = {(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2], 0u, 0u, 0u, 0u};
        const f32x32_t v = FMT == FP6_E2M3 ? __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(d, sf)
                                           : __builtin_amdgcn_cvt_scalef32_pk32_f32_bf6(d, sf);
#pragma unroll
        for (int i = 0; i < 8; i++) f[i] = v[i];
    }
}

// TR = false: dst[o][l .. l+7] contiguous (blocks along the last axis).
// TR = true : the MX tensor is the cast of the transpose; value (o, l) goes to dst[l][o].
// len is the block-axis length of the result; the MX tensor stores whole blocks (plen = len
// rounded up to 32 positions per line) and the positions at or beyond len are not written.
template <int FMT, int DST, bool TR>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t *__restrict__ elems,
                                                      const uint8_t *__restrict__ scales, void *__restrict__ dst,
                                                      int64_t n_out, int64_t len, int64_t plen, int64_t ld)
{
    constexpr int w = Fmt<FMT>::bits;
    const int64_t units_per_row = plen / 8;
    const int64_t n_units = n_out * units_per_row;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < n_units; u += stride) {
        int64_t o, l;
        if (TR) {   // adjacent lanes take adjacent o so that the strided stores coalesce across the wave
            l = (u / n_out) * 8;
            o = u % n_out;
        } else {
            o = u / units_per_row;
            l = (u % units_per_row) * 8;
        }
        if (l >= len) continue;   // fill positions of a partial last block
        const int64_t unit_in_tensor = o * units_per_row + l / 8;
        const uint32_t s = scales[unit_in_tensor / 4];
        float f[8];
        constexpr bool HW = FMT != INT8;
        if (HW && s != SCALE_NAN) {
            decode8_hw<FMT>(elems + unit_in_tensor * w, s, f);
        } else {
            uint32_t c[8];
            load_codes8<FMT>(elems + unit_in_tensor * w, c);
#pragma unroll
            for (int i = 0; i < 8; i++) f[i] = decode_scaled<FMT>(c[i], s);
        }
        if (!TR && l + 8 > len) {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                if (l + i >= len) break;
                if (DST == DT_F32) reinterpret_cast<float *>(dst)[o * ld + l + i] = f[i];
                else reinterpret_cast<uint16_t *>(dst)[o * ld + l + i] = (uint16_t)f32_to_bf16_bits(f[i]);
            }
        } else if (!TR) {
            if (DST == DT_F32) {
                float *d = reinterpret_cast<float *>(dst) + o * ld + l;
                *reinterpret_cast<float4 *>(d) = make_float4(f[0], f[1], f[2], f[3]);
                *reinterpret_cast<float4 *>(d + 4) = make_float4(f[4], f[5], f[6], f[7]);
            } else {
                uint32_t h[4];   // hardware packed convert: round to nearest even, NaN stays NaN
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const f32x2_t pr = {f[2 * i], f[2 * i + 1]};
                    h[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2_t_));
                }
                st16(reinterpret_cast<uint16_t *>(dst) + o * ld + l, make_uint4(h[0], h[1], h[2], h[3]));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                if (l + i >= len) break;
                if (DST == DT_F32) reinterpret_cast<float *>(dst)[(l + i) * ld + o] = f[i];
                else reinterpret_cast<uint16_t *>(dst)[(l + i) * ld + o] = (uint16_t)f32_to_bf16_bits(f[i]);
            }
        }
    }
}

template <int FMT, int DST>
static hipError_t launch_t(const uint8_t *elems, const uint8_t *scales, int64_t rows, int64_t cols, int axis, void *dst,
                           int64_t ld, hipStream_t st)
{
    const int64_t n_out = axis == 1 ? rows : cols;
    const int64_t len = axis == 1 ? cols : rows;
    const int64_t plen = (len + BLOCK - 1) / BLOCK * BLOCK;
    int64_t nb = (n_out * (plen / 8) + 255) / 256;
    if (nb > 0x7FFFFFFF) nb = 0x7FFFFFFF;   // one unit per thread (a capped grid with a stride loop: Float32 output 20 % slower, bf16 3 % faster)
    if (axis == 1)
        hipLaunchKernelGGL((dequant_kernel<FMT, DST, false>), dim3((unsigned)nb), dim3(256), 0, st, elems, scales, dst,
                           n_out, len, plen, ld);
    else
        hipLaunchKernelGGL((dequant_kernel<FMT, DST, true>), dim3((unsigned)nb), dim3(256), 0, st, elems, scales, dst,
                           n_out, len, plen, ld);
    return hipGetLastError();
}

template <int DST>
static hipError_t launch_f(int fmt, const uint8_t *elems, const uint8_t *scales, int64_t rows, int64_t cols, int axis,
                           void *dst, int64_t ld, hipStream_t st)
{
    switch (fmt) {
        case FP8_E4M3: return launch_t<FP8_E4M3, DST>(elems, scales, rows, cols, axis, dst, ld, st);
        case FP8_E5M2: return launch_t<FP8_E5M2, DST>(elems, scales, rows, cols, axis, dst, ld, st);
        case FP6_E3M2: return launch_t<FP6_E3M2, DST>(elems, scales, rows, cols, axis, dst, ld, st);
        case FP6_E2M3: return launch_t<FP6_E2M3, DST>(elems, scales, rows, cols, axis, dst, ld, st);
        case FP4_E2M1: return launch_t<FP4_E2M1, DST>(elems, scales, rows, cols, axis, dst, ld, st);
        default:       return launch_t<INT8, DST>(elems, scales, rows, cols, axis, dst, ld, st);
    }
}

hipError_t launch_dequant(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t rows, int64_t cols, int axis,
                          void *dst, int dst_dt, int64_t ld, hipStream_t st)
{
    return dst_dt == DT_F32 ? launch_f<DT_F32>(fmt, elems, scales, rows, cols, axis, dst, ld, st)
                            : launch_f<DT_BF16>(fmt, elems, scales, rows, cols, axis, dst, ld, st);
}

}  // namespace mx
