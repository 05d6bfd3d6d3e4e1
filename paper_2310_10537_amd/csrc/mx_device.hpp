// Device-side primitives of the MX cast for gfx950: element-format traits,
// the shared-scale closed form, the per-element encoder working on Float32
// bit patterns, decoders, bit packers and small cross-lane helpers.
//
// Everything here follows Algorithm 1 of arXiv 2310.10537 (Section 3) and the
// element formats named in its Table 1.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mx {

enum : int { FP8_E4M3 = 0, FP8_E5M2 = 1, FP6_E3M2 = 2, FP6_E2M3 = 3, FP4_E2M1 = 4, INT8 = 5, NUM_FORMATS = 6 };
// ties to even (Section 4.3), ties away from zero (Section 4.5); the paper studies only those.  The
// other two extend quantize_to_element_format: the magnitude truncated, and the magnitude rounded
// up with probability equal to the discarded fraction.
enum : int { ROUND_RNE = 0, ROUND_HALF_AWAY = 1, ROUND_TOWARD_ZERO = 2, ROUND_STOCHASTIC = 3 };
enum : int { DT_F32 = 0, DT_BF16 = 1 };

constexpr int BLOCK = 32;          // elements per shared scale (Table 1)
constexpr uint32_t SCALE_NAN = 0xFF;

// bits: storage width.  mbits / bias: the sign-exponent-mantissa layout.
// emax: exponent of the largest normal (Algorithm 1).  maxcode: magnitude code
// of the largest normal.  INT8 is handled as a format whose grid is always the
// fixed step 2^-6: "mbits 6, bias 1" makes every value take the subnormal-style
// branch of the encoder, and the sign is applied as two's complement.
template <int FMT> struct Fmt;
template <> struct Fmt<FP8_E4M3> { static constexpr int bits = 8, mbits = 3, bias = 7,  emax = 8,  maxcode = 0x7E; static constexpr bool elem_nan = true;  };
template <> struct Fmt<FP8_E5M2> { static constexpr int bits = 8, mbits = 2, bias = 15, emax = 15, maxcode = 0x7B; static constexpr bool elem_nan = true;  };
template <> struct Fmt<FP6_E3M2> { static constexpr int bits = 6, mbits = 2, bias = 3,  emax = 4,  maxcode = 0x1F; static constexpr bool elem_nan = false; };
template <> struct Fmt<FP6_E2M3> { static constexpr int bits = 6, mbits = 3, bias = 1,  emax = 2,  maxcode = 0x1F; static constexpr bool elem_nan = false; };
template <> struct Fmt<FP4_E2M1> { static constexpr int bits = 4, mbits = 1, bias = 1,  emax = 2,  maxcode = 0x07; static constexpr bool elem_nan = false; };
template <> struct Fmt<INT8>     { static constexpr int bits = 8, mbits = 6, bias = 1,  emax = 0,  maxcode = 0x7F; static constexpr bool elem_nan = false; };

__host__ __device__ constexpr int fmt_bits(int fmt) { return fmt == FP4_E2M1 ? 4 : (fmt == FP6_E3M2 || fmt == FP6_E2M3) ? 6 : 8; }

// ---------------------------------------------------------------------------
// Block maximum.  For non-negative floats the integer order of the bit
// patterns is the numeric order, so max |V| is an unsigned max of (bits & 0x7FFFFFFF).
// Formats with element NaN codes take the maximum over finite inputs only;
// the others keep Inf/NaN in the maximum so that the block can be flagged.
// ---------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ uint32_t amax_key(uint32_t fbits)
{
    uint32_t a = fbits & 0x7FFFFFFFu;
    if (Fmt<FMT>::elem_nan) a = (a >= 0x7F800000u) ? 0u : a;
    return a;
}

// Algorithm 1 line 1 in closed form: floor(log2 m) is the Float32 exponent field
// minus 127, so the E8M0 byte is max(E - emax, 0).  A maximum that is zero or a
// Float32 subnormal (E = 0) gives byte 0; Inf/NaN in a format without element
// NaN gives the NaN scale.
template <int FMT>
__device__ __forceinline__ uint32_t scale_byte(uint32_t amax)
{
    if (!Fmt<FMT>::elem_nan && amax >= 0x7F800000u) return SCALE_NAN;
    int s = (int)(amax >> 23) - Fmt<FMT>::emax;
    return (uint32_t)(s < 0 ? 0 : s);
}

// ---------------------------------------------------------------------------
// quantize_to_element_format(V / X) on the bit pattern of V (Algorithm 1 line 4).
//   x = V / 2^(s-127) = 1.m * 2^(E - s); its biased element exponent is
//   be = E - s + bias.  The 24-bit significand is shifted right so that one unit
//   is one grid step (23 - mbits places for normals, more below the smallest
//   normal), rounded, and added onto the exponent field, so a rounding carry
//   moves into the next binade by itself.  Magnitudes beyond the largest normal
//   clamp to it; Float32 subnormals and zero give (signed) zero.
//   Stochastic mode: r25, a uniform 25-bit integer, is added as r25 * 2^-25 grid steps before the
//   magnitude is truncated.  The significand has 24 bits, so for shifts up to 25 only the top
//   `shift` bits of r25 can produce a carry, and beyond 25 only the bits of the significand at
//   or above 2^-25 of a step can: both truncations leave the floor unchanged.
// ---------------------------------------------------------------------------
template <int FMT, int RND>
__device__ __forceinline__ uint32_t encode_elem(uint32_t fbits, uint32_t s, uint32_t r25 = 0)
{
    using F = Fmt<FMT>;
    const uint32_t sign = fbits >> 31;
    const uint32_t a = fbits & 0x7FFFFFFFu;
    const int E = (int)(a >> 23);
    const uint32_t sig = (a & 0x7FFFFFu) | 0x800000u;
    const int be = E - (int)s + F::bias;
    int shift = (23 - F::mbits) + (be < 1 ? 1 - be : 0);
    const int shift_true = shift;
    shift = shift > 25 ? 25 : shift;
    uint32_t q;
    if (RND == ROUND_TOWARD_ZERO)
        q = sig >> shift;                       // shift 25 already empties the 24-bit significand
    else if (RND == ROUND_STOCHASTIC)
        q = shift_true <= 25 ? (sig + (r25 >> (25 - shift))) >> shift
                             : ((sig >> (shift_true - 25 > 31 ? 31 : shift_true - 25)) + r25) >> 25;
    else if (RND == ROUND_HALF_AWAY)
        q = (sig + (1u << (shift - 1))) >> shift;
    else
        q = (sig + ((1u << (shift - 1)) - 1u) + ((sig >> shift) & 1u)) >> shift;
    uint32_t code = ((uint32_t)(be > 1 ? be - 1 : 0) << F::mbits) + q;
    code = code > (uint32_t)F::maxcode ? (uint32_t)F::maxcode : code;
    if (E == 0) code = 0;   // Float32 subnormal or zero -> P = 0
    if (FMT == INT8) {
        return (sign ? (0u - code) : code) & 0xFFu;   // two's complement; -0 -> 0
    }
    if (F::elem_nan && E == 255) {
        if (FMT == FP8_E4M3) code = 0x7F;                         // NaN; no Inf code exists
        else code = (a & 0x7FFFFFu) ? 0x7E : 0x7C;                // E5M2 NaN / Inf
    }
    return code | (sign << (F::bits - 1));
}

// ---------------------------------------------------------------------------
// Element code -> Float32 value of X * P (Section 2), X = 2^(s-127).
// ---------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ float decode_scaled(uint32_t code, uint32_t s)
{
    using F = Fmt<FMT>;
    if (s == SCALE_NAN) return __uint_as_float(0x7FC00000u);
    float p;
    if (FMT == INT8) {
        p = (float)(int)(int8_t)code * 0.015625f;
    } else {
        constexpr int ebits = F::bits - 1 - F::mbits;
        const uint32_t sign = (code >> (F::bits - 1)) & 1u;
        const uint32_t Ef = (code >> F::mbits) & ((1u << ebits) - 1u);
        const uint32_t M = code & ((1u << F::mbits) - 1u);
        if (FMT == FP8_E4M3 && (code & 0x7Fu) == 0x7Fu) return __uint_as_float(0x7FC00000u);
        if (FMT == FP8_E5M2 && Ef == 31u) {
            if (M) return __uint_as_float(0x7FC00000u);
            return __uint_as_float(0x7F800000u | (sign << 31));
        }
        uint32_t bits;
        if (Ef == 0) {
            // subnormal: M * 2^(1 - bias - mbits), exact in Float32
            float sub = (float)M * __uint_as_float((uint32_t)(127 + 1 - F::bias - F::mbits) << 23);
            bits = __float_as_uint(sub);
        } else {
            bits = ((Ef + 127u - F::bias) << 23) | (M << (23 - F::mbits));
        }
        p = __uint_as_float(bits | (sign << 31));
    }
    return ldexpf(p, (int)s - 127);   // exact power-of-two scaling; overflow -> Inf
}

// Float32 -> bf16 bits, round to nearest even (also right for subnormals, whose
// bit patterns are linear in the value).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---------------------------------------------------------------------------
// Packing of N element codes (N a multiple of 8) into little-endian dense bits:
// element j at bits [j*w, (j+1)*w).  out receives N*w/32 dwords.
// ---------------------------------------------------------------------------
template <int FMT, int N>
__device__ __forceinline__ void pack_codes(const uint32_t (&c)[N], uint32_t *out)
{
    constexpr int w = Fmt<FMT>::bits;
    if (w == 8) {
#pragma unroll
        for (int i = 0; i < N / 4; i++)
            out[i] = c[4 * i] | (c[4 * i + 1] << 8) | (c[4 * i + 2] << 16) | (c[4 * i + 3] << 24);
    } else if (w == 4) {
#pragma unroll
        for (int i = 0; i < N / 8; i++) {
            uint32_t d = 0;
#pragma unroll
            for (int j = 0; j < 8; j++) d |= c[8 * i + j] << (4 * j);
            out[i] = d;
        }
    } else {
        // 16 codes -> 96 bits -> 3 dwords
        static_assert(w != 6 || N % 16 == 0, "FP6 packs in groups of 16");
#pragma unroll
        for (int i = 0; i < N / 16; i++) {
            const uint32_t *p = &c[16 * i];
            uint32_t g0 = p[0] | (p[1] << 6) | (p[2] << 12) | (p[3] << 18);      // 24 bits each
            uint32_t g1 = p[4] | (p[5] << 6) | (p[6] << 12) | (p[7] << 18);
            uint32_t g2 = p[8] | (p[9] << 6) | (p[10] << 12) | (p[11] << 18);
            uint32_t g3 = p[12] | (p[13] << 6) | (p[14] << 12) | (p[15] << 18);
            out[3 * i + 0] = g0 | (g1 << 24);
            out[3 * i + 1] = (g1 >> 8) | (g2 << 16);
            out[3 * i + 2] = (g2 >> 16) | (g3 << 8);
        }
    }
}

// element j (0 <= j < 32) of one packed block held in dwords
template <int FMT>
__device__ __forceinline__ uint32_t unpack_code(const uint32_t *blk, int j)
{
    constexpr int w = Fmt<FMT>::bits;
    int bit = j * w;
    uint64_t two = (uint64_t)blk[bit >> 5];
    if (w == 6 && (bit >> 5) + 1 < 6) two |= (uint64_t)blk[(bit >> 5) + 1] << 32;
    return (uint32_t)(two >> (bit & 31)) & ((1u << w) - 1u);
}

// ---------------------------------------------------------------------------
// Cross-lane maximum over groups of G adjacent lanes (G = 1, 2, 4) with DPP
// quad permutes: every lane of the group ends up with the group maximum.
// ---------------------------------------------------------------------------
template <int G>
__device__ __forceinline__ uint32_t group_max(uint32_t v)
{
    if (G >= 2) {
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false);
        v = v > o ? v : o;
    }
    if (G >= 4) {
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, false);
        v = v > o ? v : o;
    }
    return v;
}

// 16-byte global load / store helpers
__device__ __forceinline__ uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ void st16(void *p, uint4 v) { *reinterpret_cast<uint4 *>(p) = v; }

// Streaming (non-temporal) forms for data that is touched once: a tensor being cast or dequantized
// passes through the caches without any reuse, and marking its loads as such is worth 10-13 % of
// bandwidth in the 2 : 1 read : write pattern of a cast (measured with loads and stores only:
// 35.6 -> 31.5 us for 128 MiB in, 64 MiB out).
typedef uint32_t u32x4_ext_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_ext_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ld16_nt(const void *p)
{
    const u32x4_ext_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_ext_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ld8_nt(const void *p)
{
    const u32x2_ext_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_ext_t *>(p));
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t ld4_nt(const void *p) { return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p)); }
__device__ __forceinline__ uint32_t ld2_nt(const void *p) { return __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(p)); }
__device__ __forceinline__ void st16_nt(void *p, uint4 v)
{
    const u32x4_ext_t e = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(e, reinterpret_cast<u32x4_ext_t *>(p));
}

}  // namespace mx
