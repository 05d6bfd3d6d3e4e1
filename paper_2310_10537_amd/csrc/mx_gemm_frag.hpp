// Operand fragments of the block-scaled 32x32x64 f8f6f4 matrix instruction,
// straight from global memory, and the 32 x 32 tile product built on them
// (Section 4.1 of arXiv 2310.10537).  Shared by the direct GEMM kernel and the
// exact fallback of the LDS-tiled kernel.
#pragma once

#include "mx_device.hpp"

namespace mx {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// hardware format selectors of the f8f6f4 instruction (cbsz for A, blgp for B)
__host__ __device__ constexpr int hw_fmt(int fmt)
{
    return fmt == FP8_E4M3 ? 0 : fmt == FP8_E5M2 ? 1 : fmt == FP6_E2M3 ? 2 : fmt == FP6_E3M2 ? 3 : 4;
}

// Operand registers of one lane for one 64-wide K step, straight from global
// memory.  row points at the packed elements of this lane's row at the K step's
// first element; g is the lane's K group (0 or 1).
template <int FMT>
__device__ __forceinline__ v8i load_operand(const uint8_t *row, int g, bool valid0, bool valid1)
{
    constexpr int w = Fmt<FMT>::bits;
    v8i r = {0, 0, 0, 0, 0, 0, 0, 0};
    if (w == 8) {
        uint4 a = make_uint4(0, 0, 0, 0), b = a;
        if (valid0) a = ld16(row + 16 * g);
        if (valid1) b = ld16(row + 32 + 16 * g);
        r = v8i{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
    } else if (w == 6) {
        if (g ? valid1 : valid0) {
            const uint2 *q = reinterpret_cast<const uint2 *>(row + 24 * g);
            uint2 a = q[0], b = q[1], c = q[2];
            r = v8i{(int)a.x, (int)a.y, (int)b.x, (int)b.y, (int)c.x, (int)c.y, 0, 0};
        }
    } else {
        if (g ? valid1 : valid0) {
            uint4 a = ld16(row + 16 * g);
            r = v8i{(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
        }
    }
    return r;
}

// 16 consecutive bf16 values as Float32 bit patterns
__device__ __forceinline__ void load16_bf16(const uint16_t *p, uint32_t *v)
{
#pragma unroll
    for (int i = 0; i < 2; i++) {
        uint4 d = ld16(p + 8 * i);
        const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int j = 0; j < 4; j++) {
            v[8 * i + 2 * j] = dw[j] << 16;
            v[8 * i + 2 * j + 1] = dw[j] & 0xFFFF0000u;
        }
    }
}

template <int FMT, int N>
__device__ __forceinline__ uint32_t amax_of(const uint32_t *v)
{
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < N; i++) {
        uint32_t k = amax_key<FMT>(v[i]);
        m = m > k ? m : k;
    }
    return m;
}

// Quantize-on-load of the A operand: the lane's share of a raw bf16 row for one
// 64-wide K step, cast exactly as the row cast kernel does (same encoder, same
// scale rule), returned in operand-register layout together with the scale byte
// this lane must supply (block g).  For 8-bit formats a lane owns half of each
// block, so the two block maxima are completed with the partner lane l ^ 32.
template <int FMT, int RND>
__device__ __forceinline__ v8i quantize_operand_bf16(const uint16_t *row, int g, bool valid0, bool valid1, uint32_t &s_out)
{
    constexpr int w = Fmt<FMT>::bits;
    uint32_t packed[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (w == 8) {
        uint32_t v0[16], v1[16];
#pragma unroll
        for (int i = 0; i < 16; i++) v0[i] = v1[i] = 0;
        if (valid0) load16_bf16(row + 16 * g, v0);
        if (valid1) load16_bf16(row + 32 + 16 * g, v1);
        uint32_t m0 = amax_of<FMT, 16>(v0), m1 = amax_of<FMT, 16>(v1);
        uint32_t o0 = (uint32_t)__shfl_xor((int)m0, 32), o1 = (uint32_t)__shfl_xor((int)m1, 32);
        m0 = m0 > o0 ? m0 : o0;
        m1 = m1 > o1 ? m1 : o1;
        const uint32_t s0 = valid0 ? scale_byte<FMT>(m0) : 127u, s1 = valid1 ? scale_byte<FMT>(m1) : 127u;
        uint32_t c0[16], c1[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            c0[i] = valid0 ? encode_elem<FMT, RND>(v0[i], s0) : 0u;
            c1[i] = valid1 ? encode_elem<FMT, RND>(v1[i], s1) : 0u;
        }
        pack_codes<FMT, 16>(c0, packed);
        pack_codes<FMT, 16>(c1, packed + 4);
        s_out = g ? s1 : s0;
    } else {
        const bool valid = g ? valid1 : valid0;
        uint32_t v[BLOCK];
#pragma unroll
        for (int i = 0; i < BLOCK; i++) v[i] = 0;
        if (valid) {
            load16_bf16(row + 32 * g, v);
            load16_bf16(row + 32 * g + 16, v + 16);
        }
        const uint32_t s = valid ? scale_byte<FMT>(amax_of<FMT, BLOCK>(v)) : 127u;
        uint32_t c[BLOCK];
#pragma unroll
        for (int i = 0; i < BLOCK; i++) c[i] = (!valid || s == SCALE_NAN) ? 0u : encode_elem<FMT, RND>(v[i], s);
        pack_codes<FMT, BLOCK>(c, packed);
        s_out = s;
    }
    return v8i{(int)packed[0], (int)packed[1], (int)packed[2], (int)packed[3],
               (int)packed[4], (int)packed[5], (int)packed[6], (int)packed[7]};
}

// One 32 x 32 output tile of C = A * B^T over the whole K range, computed by one
// wave with operands taken straight from global memory in K steps of 64, in
// increasing K order.  (m0, n0) is the tile origin; rows >= M / columns >= N are masked.
template <int FA, int FB, bool QA, int RND, int CDT>
__device__ __forceinline__ void direct_tile(int64_t M, int64_t N, int64_t K, const uint8_t *__restrict__ Ae,
                                            const uint8_t *__restrict__ As, const uint16_t *__restrict__ Abf, int64_t lda,
                                            const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                            void *__restrict__ C, int64_t ldc, int64_t m0, int64_t n0, int lane)
{
    const int i = lane & 31, g = lane >> 5;
    const int64_t nkb = K / BLOCK;
    constexpr int wA = Fmt<FA>::bits, wB = Fmt<FB>::bits;
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);   // must reach the builtin as literal constants

    const int64_t row = m0 + i, col = n0 + i;
    const bool rv = row < M, cv = col < N;
    const int64_t rowc = rv ? row : 0, colc = cv ? col : 0;   // keep addresses in range for masked lanes

    v16f acc;
#pragma unroll
    for (int t = 0; t < 16; t++) acc[t] = 0.f;

    for (int64_t kb0 = 0; kb0 < nkb; kb0 += 2) {
        const bool v0 = true, v1 = kb0 + 1 < nkb;   // second block of the step may lie beyond K
        const bool mine = g ? v1 : v0;
        v8i a, b;
        int sa, sb;
        if (QA) {
            uint32_t s;
            a = quantize_operand_bf16<FA, RND>(Abf + rowc * lda + kb0 * BLOCK, g, rv && v0, rv && v1, s);
            sa = (int)s;
        } else {
            a = load_operand<FA>(Ae + rowc * (K * wA / 8) + kb0 * (BLOCK * wA / 8), g, rv && v0, rv && v1);
            sa = (rv && mine) ? (int)As[rowc * nkb + kb0 + g] : 127;
        }
        b = load_operand<FB>(Be + colc * (K * wB / 8) + kb0 * (BLOCK * wB / 8), g, cv && v0, cv && v1);
        sb = (cv && mine) ? (int)Bs[colc * nkb + kb0 + g] : 127;
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, HA, HB, 0, sa, 0, sb);
    }

#pragma unroll
    for (int t = 0; t < 16; t++) {
        const int64_t r = m0 + 8 * (t / 4) + 4 * g + (t % 4);
        if (r < M && cv) {
            if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = acc[t];
            else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(acc[t]);
        }
    }
}

}  // namespace mx
