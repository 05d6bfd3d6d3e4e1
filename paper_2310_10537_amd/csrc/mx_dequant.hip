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
    // (Float32 rows leave as two 16-byte stores per lane.  Letting two lanes share a unit, so that
    // each store instruction writes 1 KB without gaps, measured slower -- 107 against 94 us on 8192 x
    // 8192: a result that is four times the input runs at about 3.6 TB/s either way.)
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

// 8 codes already in registers (lo: the first 32 bits of the w-byte unit, hi: the rest) times X
template <int FMT>
__device__ __forceinline__ void decode8_regs(uint32_t lo, uint32_t hi, uint32_t s, float (&f)[8])
{
    constexpr int w = Fmt<FMT>::bits;
    if (FMT == INT8 || s == SCALE_NAN) {
        const uint64_t bits = (uint64_t)lo | ((uint64_t)hi << 32);
#pragma unroll
        for (int i = 0; i < 8; i++) f[i] = decode_scaled<FMT>((uint32_t)(bits >> (w * i)) & ((1u << w) - 1u), s);
        return;
    }
    const float sf = __uint_as_float(s << 23);
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) {
        const uint32_t dw[2] = {lo, hi};
#pragma unroll
        for (int j = 0; j < 2; j++) {
            f32x2_t a, b;
            if (FMT == FP8_E4M3) {
                a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(dw[j], sf, false);
                b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(dw[j], sf, true);
            } else {
                a = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(dw[j], sf, false);
                b = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(dw[j], sf, true);
            }
            f[4 * j] = a[0]; f[4 * j + 1] = a[1]; f[4 * j + 2] = b[0]; f[4 * j + 3] = b[1];
        }
    } else if constexpr (FMT == FP4_E2M1) {
        f32x2_t v;
        v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, sf, 0); f[0] = v[0]; f[1] = v[1];
        v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, sf, 1); f[2] = v[0]; f[3] = v[1];
        v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, sf, 2); f[4] = v[0]; f[5] = v[1];
        v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, sf, 3); f[6] = v[0]; f[7] = v[1];
    } else if constexpr (FMT == FP6_E3M2 || FMT == FP6_E2M3) {
        const u32x6_t_ d = {lo, hi, 0u, 0u, 0u, 0u};
        const f32x32_t v = FMT == FP6_E2M3 ? __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(d, sf)
                                           : __builtin_amdgcn_cvt_scalef32_pk32_f32_bf6(d, sf);
#pragma unroll
        for (int i = 0; i < 8; i++) f[i] = v[i];
    }
}

// Blocks along the last axis of a dense result (ld == len, whole blocks): the tensor is one run of
// 8-code units, unit u -> dst[8u .. 8u+7], no row arithmetic.  A thread takes U units 256 apart and
// requests all of them (streaming loads) before it converts the first, so that a wave has U loads in
// flight; adjacent lanes write adjacent 16 (bf16) or 32 (Float32) bytes.
constexpr int DQ_U = 4;
template <int FMT, int DST>
__global__ __launch_bounds__(256) void dequant_flat_kernel(const uint8_t *__restrict__ elems, const uint8_t *__restrict__ scales,
                                                           void *__restrict__ dst, int64_t n_units)
{
    constexpr int w = Fmt<FMT>::bits;
    const int64_t base = (int64_t)blockIdx.x * (256 * DQ_U) + threadIdx.x;
    uint32_t lo[DQ_U], hi[DQ_U], s[DQ_U];
#pragma unroll
    for (int i = 0; i < DQ_U; i++) {
        const int64_t u = base + i * 256;
        lo[i] = hi[i] = 0; s[i] = 127;
        if (u < n_units) {
            const uint8_t *p = elems + u * w;
            if (w == 8) { const uint2 d = ld8_nt(p); lo[i] = d.x; hi[i] = d.y; }
            else if (w == 4) lo[i] = ld4_nt(p);
            else { lo[i] = ld2_nt(p) | (ld2_nt(p + 2) << 16); hi[i] = ld2_nt(p + 4); }
            s[i] = scales[u >> 2];
        }
    }
#pragma unroll
    for (int i = 0; i < DQ_U; i++) {
        const int64_t u = base + i * 256;
        if (u >= n_units) continue;
        float f[8];
        decode8_regs<FMT>(lo[i], hi[i], s[i], f);
        if (DST == DT_F32) {
            float *d = reinterpret_cast<float *>(dst) + u * 8;
            *reinterpret_cast<float4 *>(d) = make_float4(f[0], f[1], f[2], f[3]);
            *reinterpret_cast<float4 *>(d + 4) = make_float4(f[4], f[5], f[6], f[7]);
        } else {
            uint32_t h[4];   // hardware packed convert: round to nearest even, NaN stays NaN
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const f32x2_t pr = {f[2 * k], f[2 * k + 1]};
                h[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2_t_));
            }
            st16(reinterpret_cast<uint16_t *>(dst) + u * 8, make_uint4(h[0], h[1], h[2], h[3]));
        }
    }
}

// The same for 8-bit codes and Float32 output with 4 codes per lane, so that every store instruction
// of a wave writes one gap-free kilobyte (with 8 codes per lane a lane's 32 bytes leave as two stores
// that each cover every other 16 bytes).
template <int FMT>
__global__ __launch_bounds__(256) void dequant_flat4_kernel(const uint8_t *__restrict__ elems, const uint8_t *__restrict__ scales,
                                                            float *__restrict__ dst, int64_t n_quads)
{
    static_assert(Fmt<FMT>::bits == 8, "one dword = four codes");
    const int64_t base = (int64_t)blockIdx.x * (256 * DQ_U) + threadIdx.x;
    uint32_t c[DQ_U], s[DQ_U];
#pragma unroll
    for (int i = 0; i < DQ_U; i++) {
        const int64_t u = base + i * 256;
        c[i] = 0; s[i] = 127;
        if (u < n_quads) { c[i] = ld4_nt(elems + u * 4); s[i] = scales[u >> 3]; }
    }
#pragma unroll
    for (int i = 0; i < DQ_U; i++) {
        const int64_t u = base + i * 256;
        if (u >= n_quads) continue;
        float4 v;
        if (FMT == INT8 || s[i] == SCALE_NAN) {
            v = make_float4(decode_scaled<FMT>(c[i] & 0xFFu, s[i]), decode_scaled<FMT>((c[i] >> 8) & 0xFFu, s[i]),
                            decode_scaled<FMT>((c[i] >> 16) & 0xFFu, s[i]), decode_scaled<FMT>(c[i] >> 24, s[i]));
        } else {
            const float sf = __uint_as_float(s[i] << 23);
            f32x2_t a, b;
            if (FMT == FP8_E4M3) {
                a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c[i], sf, false);
                b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c[i], sf, true);
            } else {
                a = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(c[i], sf, false);
                b = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(c[i], sf, true);
            }
            v = make_float4(a[0], a[1], b[0], b[1]);
        }
        *reinterpret_cast<float4 *>(dst + u * 4) = v;
    }
}

// Axis 0 through LDS: the MX tensor is the cast of the transpose ([n_out][len] with the block axis
// contiguous), the result is row-major [len][n_out].  A work-group takes 64 lines x 128 positions:
// 16 lanes read one line's 128 codes side by side (coalesced), every lane decodes 8 of them, the
// values go transposed into a [128][64] Float32 tile (pitch 65: reads below are conflict-free,
// writes two-way), and the tile leaves row by row with 16-byte stores, adjacent lanes writing
// adjacent 16 bytes, so that every store instruction fills whole 128-byte lines (a lane that owns
// a longer run and stores it 16 bytes at a time leaves every line to several instructions, which
// measured 60 instead of 40 us).  (One lane per 8 codes with strided 2-byte stores, the generic
// kernel above, reads 8 bytes per lane from 64 different lines.)
constexpr int DQT_O = 64, DQT_L = 128, DQT_PITCH = 65;
template <int FMT, int DST>
__global__ __launch_bounds__(256) void dequant_tr_tile_kernel(const uint8_t *__restrict__ elems,
                                                              const uint8_t *__restrict__ scales, void *__restrict__ dst,
                                                              int64_t n_out, int64_t len, int64_t ld)
{
    constexpr int w = Fmt<FMT>::bits;
    __shared__ float tile[DQT_L * DQT_PITCH];
    const int t = threadIdx.x;
    const int64_t tiles_o = n_out / DQT_O;
    const int64_t O0 = (int64_t)(blockIdx.x % tiles_o) * DQT_O, L0 = (int64_t)(blockIdx.x / tiles_o) * DQT_L;
    const int64_t units_per_row = len / 8;
#pragma unroll
    for (int p = 0; p < 4; p++) {
        const int o = 16 * p + (t >> 4), u = t & 15;
        const int64_t unit = (O0 + o) * units_per_row + L0 / 8 + u;
        const uint32_t s = scales[unit / 4];
        float f[8];
        if (FMT != INT8 && s != SCALE_NAN) {
            decode8_hw<FMT>(elems + unit * w, s, f);
        } else {
            uint32_t c[8];
            load_codes8<FMT>(elems + unit * w, c);
#pragma unroll
            for (int i = 0; i < 8; i++) f[i] = decode_scaled<FMT>(c[i], s);
        }
#pragma unroll
        for (int i = 0; i < 8; i++) tile[(8 * u + i) * DQT_PITCH + o] = f[i];
    }
    __syncthreads();
    if (DST == DT_F32) {
        // a result row of the tile is 256 bytes = 16 lanes x 16 bytes; 16 rows per pass
#pragma unroll
        for (int p = 0; p < DQT_L / 16; p++) {
            const int row = 16 * p + (t >> 4), q = t & 15;
            const float *src = tile + row * DQT_PITCH + 4 * q;
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(dst) + (L0 + row) * ld + O0 + 4 * q) =
                make_float4(src[0], src[1], src[2], src[3]);
        }
    } else {
        // 128 bytes = 8 lanes x 16 bytes; 32 rows per pass
#pragma unroll
        for (int p = 0; p < DQT_L / 32; p++) {
            const int row = 32 * p + (t >> 3), q = t & 7;
            const float *src = tile + row * DQT_PITCH + 8 * q;
            uint32_t h[4];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const f32x2_t pr = {src[2 * j], src[2 * j + 1]};
                h[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2_t_));
            }
            st16(reinterpret_cast<uint16_t *>(dst) + (L0 + row) * ld + O0 + 8 * q, make_uint4(h[0], h[1], h[2], h[3]));
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
    if (axis == 0 && n_out % DQT_O == 0 && len % DQT_L == 0 && (n_out / DQT_O) * (len / DQT_L) <= 0x7FFFFFFF) {
        hipLaunchKernelGGL((dequant_tr_tile_kernel<FMT, DST>), dim3((unsigned)((n_out / DQT_O) * (len / DQT_L))), dim3(256), 0,
                           st, elems, scales, dst, n_out, len, ld);
        return hipGetLastError();
    }
    if (axis == 1 && ld == len && plen == len) {
        // dense rows of whole blocks: one flat run of units
        const int64_t n_units = n_out * (len / 8);
        if (DST == DT_F32 && Fmt<FMT>::bits == 8) {
            if constexpr (Fmt<FMT>::bits == 8) {
                const int64_t nq = n_units * 2, nbq = (nq + 256 * DQ_U - 1) / (256 * DQ_U);
                if (nbq <= 0x7FFFFFFF) {
                    hipLaunchKernelGGL((dequant_flat4_kernel<FMT>), dim3((unsigned)nbq), dim3(256), 0, st, elems, scales,
                                       static_cast<float *>(dst), nq);
                    return hipGetLastError();
                }
            }
        }
        const int64_t nbf = (n_units + 256 * DQ_U - 1) / (256 * DQ_U);
        if (nbf <= 0x7FFFFFFF) {
            hipLaunchKernelGGL((dequant_flat_kernel<FMT, DST>), dim3((unsigned)nbf), dim3(256), 0, st, elems, scales, dst, n_units);
            return hipGetLastError();
        }
    }
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
