// MXINT8 x MXINT8 GEMM (Section 4.1 of arXiv 2310.10537; MXINT8 is the format of Table 1
// with two's-complement elements and an implied scale of 2^-6).  The block-scaled matrix
// instruction has no integer form, so each 32-element block is one plain
// V_MFMA_I32_32X32X32_I8 -- its 32 products and their sum are exact integers -- and
// the block's contribution X_A * X_B * sum is added in Float32 with an exact
// power-of-two scaling (ldexp):
//   C[m][n] += float(sum_j qa[m][32b+j] * qb[n][32b+j]) * 2^(sA[m][b] + sB[n][b] - 254 - 12).
// Operand layout of the instruction (the same as each 32-wide half of the 8-bit f8f6f4 form):
// lane l holds, for row / column l % 32, the 16 consecutive K bytes [16 * (l / 32), + 16);
// result register t of lane l is C[8*(t/4) + 4*(l/32) + t%4][l % 32].
// One wave per 32 x 32 output tile, operands straight from global memory, any shape.  The
// A scale of a block is needed per output row, i.e. per result register: the 32 row bytes
// go through a wave-private LDS line and come back as the four dwords a lane needs.
#include "mx_device.hpp"
#include "mx_launch.hpp"

namespace mx {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void wave_lds_sync8()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
}

template <int CDT>
__global__ __launch_bounds__(256) void gemm_int8_kernel(int64_t M, int64_t N, int64_t K, const uint8_t *__restrict__ Ae,
                                                        const uint8_t *__restrict__ As, const uint8_t *__restrict__ Be,
                                                        const uint8_t *__restrict__ Bs, void *__restrict__ C, int64_t ldc)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint8_t *lds = lds_all + wave * 32;
    const int64_t m0 = (int64_t)blockIdx.y * 64 + (wave >> 1) * 32;
    const int64_t n0 = (int64_t)blockIdx.x * 64 + (wave & 1) * 32;
    const int i = lane & 31, g = lane >> 5;
    const int64_t nkb = K / BLOCK;
    const int64_t row = m0 + i, col = n0 + i;
    const bool rv = row < M, cv = col < N;
    const int64_t rowc = rv ? row : 0, colc = cv ? col : 0;   // keep addresses in range for masked lanes

    float acc[16];
#pragma unroll
    for (int t = 0; t < 16; t++) acc[t] = 0.f;

    for (int64_t kb = 0; kb < nkb; kb++) {
        const uint4 qa = ld16(Ae + rowc * K + kb * BLOCK + 16 * g);
        const uint4 qb = ld16(Be + colc * K + kb * BLOCK + 16 * g);
        const uint32_t sa = As[rowc * nkb + kb], sb = Bs[colc * nkb + kb];
        if (g == 0) lds[i] = (uint8_t)sa;
        wave_lds_sync8();
        uint32_t sa4[4];
#pragma unroll
        for (int q = 0; q < 4; q++) sa4[q] = *reinterpret_cast<const uint32_t *>(lds + 8 * q + 4 * g);
        const v4i_t a = rv ? v4i_t{(int)qa.x, (int)qa.y, (int)qa.z, (int)qa.w} : v4i_t{0, 0, 0, 0};
        const v4i_t b = cv ? v4i_t{(int)qb.x, (int)qb.y, (int)qb.z, (int)qb.w} : v4i_t{0, 0, 0, 0};
        v16i_t z;
#pragma unroll
        for (int t = 0; t < 16; t++) z[t] = 0;
        const v16i_t p = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, z, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 16; t++) {
            const uint32_t sat = (sa4[t >> 2] >> (8 * (t & 3))) & 0xFFu;
            const int e = (int)sat + (int)sb - 254 - 12;
            float term = ldexpf((float)p[t], e);
            if (sat == SCALE_NAN || sb == SCALE_NAN) term = __uint_as_float(0x7FC00000u);
            acc[t] += term;
        }
        wave_lds_sync8();   // the line is rewritten in the next trip
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

hipError_t launch_gemm_int8(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                            const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    if (c_dt == DT_F32) hipLaunchKernelGGL((gemm_int8_kernel<DT_F32>), grid, dim3(256), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    else hipLaunchKernelGGL((gemm_int8_kernel<DT_BF16>), grid, dim3(256), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    return hipGetLastError();
}

}  // namespace mx
