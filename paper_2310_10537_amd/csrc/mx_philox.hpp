// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC 2011): the counter-based generator behind the stochastic rounding mode.  The number that
// belongs to tensor element e = row * cols + col is word e % 4 of the output for counter e / 4
// (upper two counter words zero) under the 64-bit seed as key, top 25 bits -- a function of
// (seed, e) only, so every kernel, whatever its walk over the tensor, draws the same number.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mx {

struct Philox4 { uint32_t w[4]; };

__device__ __forceinline__ Philox4 philox4x32_10(uint64_t key, uint64_t counter)
{
    uint32_t c0 = (uint32_t)counter, c1 = (uint32_t)(counter >> 32), c2 = 0, c3 = 0;
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
#pragma unroll
    for (int round = 0; round < 10; round++) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0;
        c2 = h0 ^ c3 ^ k1;
        c1 = l1;
        c3 = l0;
        k0 += 0x9E3779B9u;      // the key schedule: one Weyl step per round
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// 25-bit offsets of the N consecutive elements e0 .. e0 + N - 1 (e0 and N multiples of 4)
template <int N>
__device__ __forceinline__ void sr_offsets_run(uint64_t seed, int64_t e0, uint32_t (&r)[N])
{
    static_assert(N % 4 == 0, "");
#pragma unroll
    for (int i = 0; i < N / 4; i++) {
        const Philox4 p = philox4x32_10(seed, (uint64_t)(e0 >> 2) + i);
#pragma unroll
        for (int j = 0; j < 4; j++) r[4 * i + j] = p.w[j] >> 7;
    }
}

// 25-bit offset of one element
__device__ __forceinline__ uint32_t sr_offset(uint64_t seed, int64_t e)
{
    const Philox4 p = philox4x32_10(seed, (uint64_t)e >> 2);
    const int j = (int)(e & 3);
    return (j == 0 ? p.w[0] : j == 1 ? p.w[1] : j == 2 ? p.w[2] : p.w[3]) >> 7;
}

}  // namespace mx
