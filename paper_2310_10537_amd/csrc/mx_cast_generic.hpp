// Loaders, stores and the per-lane encoder shared by the generic (integer-encoder) cast kernels.
#pragma once

#include "mx_device.hpp"
#include "mx_philox.hpp"

namespace mx {

// ---------------------------------------------------------------------------
// Source loaders: N consecutive elements as Float32 bit patterns.
// ---------------------------------------------------------------------------
template <int SRC, int N>
__device__ __forceinline__ void load_as_f32_bits(const void *p, uint32_t (&v)[N])
{
    if (SRC == DT_BF16) {
        static_assert(N % 8 == 0, "");
#pragma unroll
        for (int i = 0; i < N / 8; i++) {
            uint4 d = ld16_nt(reinterpret_cast<const char *>(p) + 16 * i);
            const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[8 * i + 2 * j] = dw[j] << 16;
                v[8 * i + 2 * j + 1] = dw[j] & 0xFFFF0000u;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < N / 4; i++) {
            uint4 d = ld16_nt(reinterpret_cast<const char *>(p) + 16 * i);
            v[4 * i] = d.x; v[4 * i + 1] = d.y; v[4 * i + 2] = d.z; v[4 * i + 3] = d.w;
        }
    }
}

// The first n (< N) of N consecutive elements, one by one; the rest read as zero (the fill of a
// partial last block).
template <int SRC, int N>
__device__ __forceinline__ void load_head_as_f32_bits(const void *p, int n, uint32_t (&v)[N])
{
#pragma unroll
    for (int i = 0; i < N; i++) {
        uint32_t x = 0;
        if (i < n) x = SRC == DT_BF16 ? (uint32_t)reinterpret_cast<const uint16_t *>(p)[i] << 16 : reinterpret_cast<const uint32_t *>(p)[i];
        v[i] = x;
    }
}

struct __attribute__((packed, aligned(4))) dword3 { uint32_t a, b, c; };

// store ND dwords to a pointer aligned to min(16, largest power of two dividing 4*ND)
template <int ND>
__device__ __forceinline__ void store_dwords(void *p, const uint32_t *d)
{
    char *c = reinterpret_cast<char *>(p);
    if (ND % 4 == 0) {
#pragma unroll
        for (int i = 0; i < ND / 4; i++) st16(c + 16 * i, make_uint4(d[4 * i], d[4 * i + 1], d[4 * i + 2], d[4 * i + 3]));
    } else if (ND % 2 == 0) {
#pragma unroll
        for (int i = 0; i < ND / 2; i++) *reinterpret_cast<uint2 *>(c + 8 * i) = make_uint2(d[2 * i], d[2 * i + 1]);
    } else if (ND == 3) {
        dword3 t{d[0], d[1], d[2]};
        *reinterpret_cast<dword3 *>(c) = t;
    } else {
#pragma unroll
        for (int i = 0; i < ND; i++) *reinterpret_cast<uint32_t *>(c + 4 * i) = d[i];
    }
}

// Quantize the N elements a lane holds, given the block's scale byte (r: their 25-bit random
// offsets, read by the stochastic mode only).
template <int FMT, int RND, int N>
__device__ __forceinline__ void encode_lane(const uint32_t (&v)[N], uint32_t s, const uint32_t (&r)[N], uint32_t *packed)
{
    uint32_t c[N];
    if (!Fmt<FMT>::elem_nan && s == SCALE_NAN) {
#pragma unroll
        for (int i = 0; i < N; i++) c[i] = 0;
    } else {
#pragma unroll
        for (int i = 0; i < N; i++) c[i] = encode_elem<FMT, RND>(v[i], s, r[i]);
    }
    pack_codes<FMT, N>(c, packed);
}

// ND dwords to a 16-byte aligned address
template <int ND>
__device__ __forceinline__ void store_dwords_any(void *p, const uint32_t *d)
{
    char *c = reinterpret_cast<char *>(p);
    if (ND == 3) {
        dword3 t{d[0], d[1], d[2]};
        *reinterpret_cast<dword3 *>(c) = t;
    } else {
        store_dwords<ND>(p, d);
    }
}

}  // namespace mx
