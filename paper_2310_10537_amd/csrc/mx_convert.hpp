// Fast element conversion for bf16 sources with gfx950's scaled converts
// (V_CVT_SCALEF32_*), used by the cast kernels and the quantize-on-load GEMM.
//
// What the hardware converts do, as established by dumping them over every bf16
// bit pattern (and Float32 patterns with sticky low bits) at a sweep of scales
// and comparing with the CPU reference of Algorithm 1 (arXiv 2310.10537, Sec. 3):
//   * result = round-to-nearest-even of src / 2^(E-127), E = exponent field of
//     the Float32 scale operand (mantissa ignored, E = 0 means 2^-127);
//     subnormal results and all 24 source bits are honoured;
//   * FP6 / FP4 saturate to the largest normal -- what Algorithm 1 asks for;
//   * FP8 does not saturate by default: anything above the largest normal becomes
//     NaN (E4M3, code 0x7F) or Inf (E5M2, code 0x7C).  With the wave's
//     MODE.FP16_OVFL bit set the same converts clamp a finite overflow to the
//     largest normal (0x7E / 0x7B) -- what Algorithm 1 asks for -- so every
//     kernel that converts to FP8 sets that bit first (fp8_saturate_mode);
//   * NaN / Inf inputs and Float32-subnormal inputs are not treated the way
//     Algorithm 1 needs.  Blocks that contain a non-finite value, or whose scale
//     byte is below 18 (only then can a Float32 subnormal reach half of the
//     smallest element subnormal), take the exact integer path instead.
// Round-half-away is obtained from the round-to-nearest-even hardware by
// widening to Float32 and setting the lowest significand bit: an exact tie
// becomes "just above the tie", and nothing else changes side, because every
// rounding boundary has that bit clear and at least 16 zero bits below a bf16.
#pragma once

#include "mx_device.hpp"

namespace mx {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x32_t __attribute__((ext_vector_type(32)));
typedef short i16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x6_t __attribute__((ext_vector_type(6)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr uint32_t FAST_MIN_SCALE = 18;

// max of the magnitudes of packed bf16 pairs, kept packed (two u16 lanes)
__device__ __forceinline__ uint32_t pk_absmax(uint32_t m, uint32_t d)
{
    u16x2_t a = __builtin_bit_cast(u16x2_t, d & 0x7FFF7FFFu);
    u16x2_t b = __builtin_bit_cast(u16x2_t, m);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
}
// packed maximum -> single bf16 magnitude (15 bits)
__device__ __forceinline__ uint32_t pk_hmax(uint32_t m)
{
    uint32_t lo = m & 0xFFFFu, hi = m >> 16;
    return lo > hi ? lo : hi;
}

// scale byte from the largest bf16 magnitude of a block with only finite values
template <int FMT>
__device__ __forceinline__ uint32_t scale_from_bf16_max(uint32_t amax16)
{
    int s = (int)(amax16 >> 7) - Fmt<FMT>::emax;
    return (uint32_t)(s < 0 ? 0 : s);
}

// true when the block can use the hardware converts
__device__ __forceinline__ bool fast_ok(uint32_t amax16, uint32_t s) { return amax16 < 0x7F80u && s >= FAST_MIN_SCALE; }

// FP8 codes converted with MODE.FP16_OVFL clear: NaN / Inf codes produced by finite
// overflow -> largest normal, sign kept
template <int FMT>
__device__ __forceinline__ uint32_t fp8_unoverflow(uint32_t codes)
{
    // E4M3: low 7 bits 0x7F; E5M2: low 7 bits 0x7C (the only code above 0x7B a finite input can produce)
    constexpr uint32_t add = FMT == FP8_E4M3 ? 0x01010101u : 0x04040404u;
    uint32_t ov = ((codes & 0x7F7F7F7Fu) + add) & 0x80808080u;
    return codes - (ov >> 7);
}

// Make the FP8 converts of this wave clamp instead of overflowing (on = true) or restore the
// default: MODE (hardware register 1) bit 23, FP16_OVFL.  Per-wave state.  The bit also makes
// the matrix instructions clamp NaN / Inf operands and results, so it must be clear whenever a
// matrix instruction whose result is kept can issue.
__device__ __forceinline__ void fp8_saturate_mode(bool on = true) { __builtin_amdgcn_s_setreg(1 | (23 << 6) | (0 << 11), on ? 1 : 0); }

// The 32-element FP6 converts, as inline assembly with an early-clobber result.  They read 16 or
// 32 source registers and write 6, over several passes; the compiler's builtins let the register
// allocator overlap the result with the sources at any offset, and when the result starts part
// way into a source the first result dword lands on a source element that has not been read yet
// (seen on the hardware: element 4 of every block wrong, nothing else).  A result that shares no
// register with the sources is always safe.  The trailing s_nop stands in for whatever wait
// states the compiler would place after the instruction: it does not look inside assembly text.
template <bool E2M3>
__device__ __forceinline__ u32x6_t cvt_pk32_fp6_from_bf16(bf16x32_t v, float sf)
{
    u32x6_t r;
    if (E2M3) asm("v_cvt_scalef32_pk32_fp6_bf16 %0, %1, %2\n\ts_nop 1" : "=&v"(r) : "v"(v), "v"(sf));
    else asm("v_cvt_scalef32_pk32_bf6_bf16 %0, %1, %2\n\ts_nop 1" : "=&v"(r) : "v"(v), "v"(sf));
    return r;
}
template <bool E2M3>
__device__ __forceinline__ u32x6_t cvt_2xpk16_fp6_from_f32(f32x16_t a, f32x16_t b, float sf)
{
    u32x6_t r;
    if (E2M3) asm("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, %3\n\ts_nop 1" : "=&v"(r) : "v"(a), "v"(b), "v"(sf));
    else asm("v_cvt_scalef32_2xpk16_bf6_f32 %0, %1, %2, %3\n\ts_nop 1" : "=&v"(r) : "v"(a), "v"(b), "v"(sf));
    return r;
}

// Convert ND packed bf16 dwords (2*ND consecutive elements of one block) with
// scale byte s (>= FAST_MIN_SCALE, finite inputs only) into packed codes.
// out receives 2*ND*bits/32 dwords.  FP6 needs the whole block (ND = 16).
// FP8 formats: with PATCH = false the caller has set fp8_saturate_mode(); with PATCH = true
// the wave runs in the default mode and overflowed codes are patched afterwards.
template <int FMT, int RND, int ND, bool PATCH = false>
__device__ __forceinline__ void convert_bf16_fast(const uint32_t (&d)[ND], uint32_t s, uint32_t *out)
{
    const float sf = __uint_as_float(s << 23);
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) {
#pragma unroll
        for (int j = 0; j < ND / 2; j++) {
            i16x2_t r = {0, 0};
            if (RND == ROUND_RNE) {
                bf16x2_t p0 = __builtin_bit_cast(bf16x2_t, d[2 * j]), p1 = __builtin_bit_cast(bf16x2_t, d[2 * j + 1]);
                if (FMT == FP8_E4M3) {
                    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(r, p0, sf, false);
                    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(r, p1, sf, true);
                } else {
                    r = __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(r, p0, sf, false);
                    r = __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(r, p1, sf, true);
                }
            } else {
                float a0 = __uint_as_float((d[2 * j] << 16) | 1u), a1 = __uint_as_float((d[2 * j] & 0xFFFF0000u) | 1u);
                float b0 = __uint_as_float((d[2 * j + 1] << 16) | 1u), b1 = __uint_as_float((d[2 * j + 1] & 0xFFFF0000u) | 1u);
                if (FMT == FP8_E4M3) {
                    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, a0, a1, sf, false);
                    r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, b0, b1, sf, true);
                } else {
                    r = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(r, a0, a1, sf, false);
                    r = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(r, b0, b1, sf, true);
                }
            }
            out[j] = PATCH ? fp8_unoverflow<FMT>(__builtin_bit_cast(uint32_t, r)) : __builtin_bit_cast(uint32_t, r);
        }
    } else if constexpr (FMT == FP4_E2M1) {
#pragma unroll
        for (int j = 0; j < ND / 4; j++) {
            uint32_t q = 0;
            if (RND == ROUND_RNE) {
                q = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(q, __builtin_bit_cast(bf16x2_t, d[4 * j + 0]), sf, 0);
                q = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(q, __builtin_bit_cast(bf16x2_t, d[4 * j + 1]), sf, 1);
                q = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(q, __builtin_bit_cast(bf16x2_t, d[4 * j + 2]), sf, 2);
                q = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(q, __builtin_bit_cast(bf16x2_t, d[4 * j + 3]), sf, 3);
            } else {
#define MX_FP4_AWAY(B)                                                                                         \
    q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, __uint_as_float((d[4 * j + B] << 16) | 1u),                 \
                                                 __uint_as_float((d[4 * j + B] & 0xFFFF0000u) | 1u), sf, B)
                MX_FP4_AWAY(0);
                MX_FP4_AWAY(1);
                MX_FP4_AWAY(2);
                MX_FP4_AWAY(3);
#undef MX_FP4_AWAY
            }
            out[j] = q;
        }
    } else if constexpr (FMT == FP6_E3M2 || FMT == FP6_E2M3) {
        static_assert(ND == 16, "FP6 converts a whole block at once");
        u32x6_t r;
        if (RND == ROUND_RNE) {
            uint32_t tmp[16];
#pragma unroll
            for (int i = 0; i < 16; i++) tmp[i] = d[i];
            bf16x32_t v;
            __builtin_memcpy(&v, tmp, 64);
            r = cvt_pk32_fp6_from_bf16<FMT == FP6_E2M3>(v, sf);
        } else {
            // the Float32 form interleaves its two sources: out[2i] = a[i], out[2i+1] = b[i],
            // which is exactly the low / high halves of the packed bf16 dwords
            f32x16_t a, b;
#pragma unroll
            for (int i = 0; i < 16; i++) {
                a[i] = __uint_as_float((d[i] << 16) | 1u);
                b[i] = __uint_as_float((d[i] & 0xFFFF0000u) | 1u);
            }
            r = cvt_2xpk16_fp6_from_f32<FMT == FP6_E2M3>(a, b, sf);
        }
#pragma unroll
        for (int i = 0; i < 6; i++) out[i] = r[i];
    } else {
        // INT8: q = round(V / X * 64), clamped to +-127, two's complement byte.
        // V * 2^(133 - s) is exact; the magic-number add leaves round-to-nearest-even
        // of the clamped value in the low byte of the sum.
        const float c = __uint_as_float((260u - s) << 23);
#pragma unroll
        for (int j = 0; j < ND / 2; j++) {
            uint32_t z[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const uint32_t dw = d[2 * j + (e >> 1)];
                float y = __uint_as_float((e & 1) ? (dw & 0xFFFF0000u) : (dw << 16)) * c;
                if (RND == ROUND_HALF_AWAY) y = truncf(y + copysignf(0.5f, y));   // exact for 8-bit significands below 128
                y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
                z[e] = __float_as_uint(y + 12582912.0f);
            }
            out[j] = (z[0] & 0xFFu) | ((z[1] & 0xFFu) << 8) | ((z[2] & 0xFFu) << 16) | (z[3] << 24);
        }
    }
}

// Exact integer path for any block: N Float32 bit patterns -> packed codes.
template <int FMT, int RND, int N>
__device__ __forceinline__ void encode_exact(const uint32_t (&v)[N], uint32_t s, uint32_t *packed)
{
    uint32_t c[N];
    if (!Fmt<FMT>::elem_nan && s == SCALE_NAN) {
#pragma unroll
        for (int i = 0; i < N; i++) c[i] = 0;
    } else {
#pragma unroll
        for (int i = 0; i < N; i++) c[i] = encode_elem<FMT, RND>(v[i], s);
    }
    pack_codes<FMT, N>(c, packed);
}

// packed bf16 dwords -> Float32 bit patterns
template <int ND>
__device__ __forceinline__ void widen_bf16(const uint32_t (&d)[ND], uint32_t (&v)[2 * ND])
{
#pragma unroll
    for (int i = 0; i < ND; i++) {
        v[2 * i] = d[i] << 16;
        v[2 * i + 1] = d[i] & 0xFFFF0000u;
    }
}

// Exact integer path for a whole block held by one lane as 16 packed bf16 dwords, written to
// need few registers (it sits in kernels whose occupancy matters and runs for rare blocks only):
// the encode loop is rolled, always works on dword 0 and rotates the 16 source registers by one
// place per trip, and shifts each pair of codes into the top of a w-dword shift register, so no
// register is ever indexed by the loop counter.
template <int FMT, int RND>
__device__ __forceinline__ uint32_t quantize_block_bf16_exact(const uint32_t (&d)[16], uint32_t *packed)
{
    constexpr int w = Fmt<FMT>::bits;
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const uint32_t k0 = amax_key<FMT>(d[i] << 16), k1 = amax_key<FMT>(d[i] & 0xFFFF0000u);
        amax = amax > k0 ? amax : k0;
        amax = amax > k1 ? amax : k1;
    }
    const uint32_t s = scale_byte<FMT>(amax);
    const bool nan_block = !Fmt<FMT>::elem_nan && s == SCALE_NAN;
    uint32_t r[16], o[w];
#pragma unroll
    for (int i = 0; i < 16; i++) r[i] = d[i];
#pragma unroll
    for (int i = 0; i < w; i++) o[i] = 0;
#pragma unroll 1
    for (int it = 0; it < 16; it++) {
        const uint32_t c0 = nan_block ? 0u : encode_elem<FMT, RND>(r[0] << 16, s);
        const uint32_t c1 = nan_block ? 0u : encode_elem<FMT, RND>(r[0] & 0xFFFF0000u, s);
        const uint32_t pair = c0 | (c1 << w);                       // 2w bits
#pragma unroll
        for (int j = 0; j < w - 1; j++) o[j] = (o[j] >> (2 * w)) | (o[j + 1] << (32 - 2 * w));
        o[w - 1] = (o[w - 1] >> (2 * w)) | (pair << (32 - 2 * w));
        const uint32_t first = r[0];
#pragma unroll
        for (int j = 0; j < 15; j++) r[j] = r[j + 1];
        r[15] = first;
    }
#pragma unroll
    for (int i = 0; i < w; i++) packed[i] = o[i];
    return s;
}

// A whole block held by one lane: 16 packed bf16 dwords -> scale byte + packed codes.
template <int FMT, int RND>
__device__ __forceinline__ uint32_t quantize_block_bf16(const uint32_t (&d)[16], uint32_t *packed)
{
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) m = pk_absmax(m, d[i]);
    const uint32_t amax16 = pk_hmax(m);
    uint32_t s = scale_from_bf16_max<FMT>(amax16);
    if (fast_ok(amax16, s)) {
        convert_bf16_fast<FMT, RND, 16>(d, s, packed);
    } else {
        s = quantize_block_bf16_exact<FMT, RND>(d, packed);
    }
    return s;
}

// ---------------------------------------------------------------------------------------------
// Float32 sources (the GEMM's accumulators, Float32 tensors staged in LDS)
// ---------------------------------------------------------------------------------------------
// Hardware converts on a whole block of Float32 values (finite, scale byte >= FAST_MIN_SCALE; FP8
// with the saturate mode set).  Ties away from zero: the lowest significand bit is set first -- a
// rounding boundary of these grids has that bit (and many above it) clear, so exactly the ties move.
template <int FMT, int RND>
__device__ __forceinline__ void convert_f32_fast(const uint32_t (&v)[32], uint32_t s, uint32_t *out)
{
    const float sf = __uint_as_float(s << 23);
    auto f = [](uint32_t b) { return __uint_as_float(RND == ROUND_HALF_AWAY ? (b | 1u) : b); };
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            i16x2_t r = {0, 0};
            if (FMT == FP8_E4M3) {
                r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, f(v[4 * j]), f(v[4 * j + 1]), sf, false);
                r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(r, f(v[4 * j + 2]), f(v[4 * j + 3]), sf, true);
            } else {
                r = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(r, f(v[4 * j]), f(v[4 * j + 1]), sf, false);
                r = __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(r, f(v[4 * j + 2]), f(v[4 * j + 3]), sf, true);
            }
            out[j] = __builtin_bit_cast(uint32_t, r);
        }
    } else if constexpr (FMT == FP4_E2M1) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint32_t q = 0;
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, f(v[8 * j + 0]), f(v[8 * j + 1]), sf, 0);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, f(v[8 * j + 2]), f(v[8 * j + 3]), sf, 1);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, f(v[8 * j + 4]), f(v[8 * j + 5]), sf, 2);
            q = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(q, f(v[8 * j + 6]), f(v[8 * j + 7]), sf, 3);
            out[j] = q;
        }
    } else if constexpr (FMT == INT8) {
        // q = round(V / X * 64) clamped to +-127, two's complement.  V * 2^(133 - s) is exact.  Ties
        // away: the integer part and the fraction are split first (both exact), and the fraction
        // alone decides -- adding a half to the whole value would round 0.5 - 2^-25 up to 1.
        // Ties to even: the magic-number add.
        const float c = __uint_as_float((260u - s) << 23);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            uint32_t z[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float y = __uint_as_float(v[4 * j + e]) * c;
                if (RND == ROUND_HALF_AWAY) {
                    const float t = truncf(y);
                    y = t + copysignf(fabsf(y - t) >= 0.5f ? 1.0f : 0.0f, y);
                }
                y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
                z[e] = __float_as_uint(y + 12582912.0f);
            }
            out[j] = (z[0] & 0xFFu) | ((z[1] & 0xFFu) << 8) | ((z[2] & 0xFFu) << 16) | (z[3] << 24);
        }
    } else {
        f32x16_t a, b;   // the instruction interleaves its two sources: element 2i from a, 2i+1 from b
#pragma unroll
        for (int i = 0; i < 16; i++) { a[i] = f(v[2 * i]); b[i] = f(v[2 * i + 1]); }
        const u32x6_t r = cvt_2xpk16_fp6_from_f32<FMT == FP6_E2M3>(a, b, sf);
#pragma unroll
        for (int i = 0; i < 6; i++) out[i] = r[i];
    }
}

// One block of 32 Float32 values in LDS, element i at src[i * stride] (stride 1: 16-byte aligned)
// -> scale byte and packed codes.
template <int FMT, int RND>
__device__ __forceinline__ uint32_t quantize_block_lds(const uint32_t *src, int stride, uint32_t *packed)
{
    constexpr int w = Fmt<FMT>::bits;
    uint32_t v[32];
    if (stride == 1) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const uint4 d = *reinterpret_cast<const uint4 *>(src + 4 * i);
            v[4 * i] = d.x; v[4 * i + 1] = d.y; v[4 * i + 2] = d.z; v[4 * i + 3] = d.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; i++) v[i] = src[i * stride];
    }
    uint32_t amax = 0, raw = 0;
#pragma unroll
    for (int i = 0; i < 32; i++) {
        const uint32_t a = v[i] & 0x7FFFFFFFu, k = amax_key<FMT>(v[i]);
        raw = raw > a ? raw : a;
        amax = amax > k ? amax : k;
    }
    const uint32_t s = scale_byte<FMT>(amax);
    if (raw < 0x7F800000u && s >= FAST_MIN_SCALE) {
        convert_f32_fast<FMT, RND>(v, s, packed);
        return s;
    }
    // rare: a non-finite value, or a scale so small that Float32 subnormals matter.  Exact integer
    // encoder, one element per trip from LDS, codes shifted into the top of a w-dword register.
    uint32_t o[w];
#pragma unroll
    for (int i = 0; i < w; i++) o[i] = 0;
    if (Fmt<FMT>::elem_nan || s != SCALE_NAN) {
#pragma unroll 1
        for (int it = 0; it < 32; it++) {
            const uint32_t code = encode_elem<FMT, RND>(src[it * stride], s);
#pragma unroll
            for (int j = 0; j < w - 1; j++) o[j] = (o[j] >> w) | (o[j + 1] << (32 - w));
            o[w - 1] = (o[w - 1] >> w) | (code << (32 - w));
        }
    }
#pragma unroll
    for (int i = 0; i < w; i++) packed[i] = o[i];
    return s;
}

}  // namespace mx
