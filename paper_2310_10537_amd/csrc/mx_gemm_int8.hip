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
//
// Whole 256 x 256 tiles take a faster, equally exact route through the block-scaled
// instruction.  An MXINT8 element q / 64 (q the two's-complement code) is split as
//   q / 64 = sign(q) (H + L * 2^-3),   H = (|q| >> 3) / 8  in {0, ..., 2},   L = (|q| & 7) / 8  in {0, ..., 0.875},
// and both halves, each with the sign of q so that nothing cancels, are FP6 E2M3 numbers
// (code = sign bit and the integer |q| >> 3, resp. |q| & 7), with the factor 2^-3 moved into
// the block scale (byte s - 3).  Then
//   a b = Ha Hb + Ha Lb' + La' Hb + La' Lb'        (primed = with the lowered scale),
// which is ONE E2M3 x E2M3 product of depth 4K: every source block b becomes the four blocks
// [Ha, Ha, La, La] of A' and [Hb, Lb, Hb, Lb] of B'.  E2M3 products are exact in the
// instruction and the LDS-tiled kernel does the rest.  A scale byte below 3 cannot be lowered:
// the split kernel then raises a flag, and the direct kernel -- launched after the tiled one,
// leaving at once when the flag is clear -- recomputes the whole product.
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

// MXINT8 [R][K] -> FP6 E2M3 [R][4K]: one lane per source block.  B_SIDE picks the block order.
template <bool B_SIDE>
__global__ __launch_bounds__(256) void int8_split_kernel(const uint8_t *__restrict__ elems, const uint8_t *__restrict__ scales,
                                                         int64_t n_blocks, uint8_t *__restrict__ e6, uint8_t *__restrict__ s6,
                                                         uint32_t *__restrict__ flag)
{
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= n_blocks) return;
    const uint4 q0 = ld16(elems + b * 32), q1 = ld16(elems + b * 32 + 16);
    const uint32_t dw[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
    uint32_t hi[32], lo[32];
#pragma unroll
    for (int i = 0; i < 32; i++) {
        const int q = (int)(int8_t)(dw[i >> 2] >> (8 * (i & 3)));
        const uint32_t m = (uint32_t)(q < 0 ? -q : q), sg = q < 0 ? 32u : 0u;   // m <= 128
        const uint32_t h = m >> 3, l = m & 7;       // E2M3 codes of h / 8 (<= 2.0) and l / 8: the magnitude bits ARE the code
        hi[i] = h ? (sg | h) : 0u;
        lo[i] = l ? (sg | l) : 0u;
    }
    uint32_t ph[6], pl[6];
    pack_codes<FP6_E2M3, 32>(hi, ph);
    pack_codes<FP6_E2M3, 32>(lo, pl);
    const uint32_t s = scales[b];
    uint32_t sl = s == SCALE_NAN ? SCALE_NAN : s - 3;
    if (s < 3) { sl = 0; *flag = 1u; }              // cannot lower the scale: the caller's exact pass takes over
    uint4 *o = reinterpret_cast<uint4 *>(e6 + b * 96);
    const uint4 H0 = make_uint4(ph[0], ph[1], ph[2], ph[3]), H1 = make_uint4(ph[4], ph[5], 0, 0);
    const uint4 L0 = make_uint4(pl[0], pl[1], pl[2], pl[3]), L1 = make_uint4(pl[4], pl[5], 0, 0);
    // four blocks of 24 bytes: A side H H L L, B side H L H L
    const uint4 b0a = H0, b0b = H1;
    const uint4 b1a = B_SIDE ? L0 : H0, b1b = B_SIDE ? L1 : H1;
    const uint4 b2a = B_SIDE ? H0 : L0, b2b = B_SIDE ? H1 : L1;
    const uint4 b3a = L0, b3b = L1;
    o[0] = b0a;                                                         // bytes  0..15
    o[1] = make_uint4(b0b.x, b0b.y, b1a.x, b1a.y);                      //       16..31
    o[2] = make_uint4(b1a.z, b1a.w, b1b.x, b1b.y);                      //       32..47
    o[3] = b2a;                                                         //       48..63
    o[4] = make_uint4(b2b.x, b2b.y, b3a.x, b3a.y);                      //       64..79
    o[5] = make_uint4(b3a.z, b3a.w, b3b.x, b3b.y);                      //       80..95
    const uint32_t s1 = B_SIDE ? sl : s, s2 = B_SIDE ? s : sl;
    *reinterpret_cast<uint32_t *>(s6 + b * 4) = s | (s1 << 8) | (s2 << 16) | (sl << 24);
}

template <int CDT>
__global__ __launch_bounds__(256) void gemm_int8_kernel(int64_t M, int64_t N, int64_t K, const uint8_t *__restrict__ Ae,
                                                        const uint8_t *__restrict__ As, const uint8_t *__restrict__ Be,
                                                        const uint8_t *__restrict__ Bs, void *__restrict__ C, int64_t ldc,
                                                        const uint32_t *__restrict__ run_if)
{
    if (run_if && *run_if == 0) return;   // exact pass behind the split route: nothing to repair
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

// Few rows of A (a decoding step): the kernel above gives such a problem N / 32 waves that each walk
// the whole K range alone, one load-then-multiply after the other.  Here eight waves share 32 rows
// x 32 columns of C, each a contiguous eighth of the blocks, with the operands of four blocks
// requested before the first is multiplied; the eight partial sums meet in LDS and are added in
// the order w0 + w1 + ... + w7.
constexpr int I8_WAVES = 8, I8_U = 4;
template <int CDT>
__global__ __launch_bounds__(64 * I8_WAVES) void gemm_int8_shared_k_kernel(int64_t M, int64_t N, int64_t K,
                                                                            const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                                            const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                                            void *__restrict__ C, int64_t ldc)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[I8_WAVES * 32];
    __shared__ float red[I8_WAVES - 1][16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint8_t *lds = lds_all + wave * 32;
    const int64_t m0 = (int64_t)blockIdx.y * 32, n0 = (int64_t)blockIdx.x * 32;
    const int i = lane & 31, g = lane >> 5;
    const int64_t nkb = K / BLOCK;
    const int64_t chunk = (nkb + I8_WAVES - 1) / I8_WAVES;
    const int64_t kb_begin = wave * chunk, kb_end = kb_begin + chunk < nkb ? kb_begin + chunk : nkb;
    const int64_t row = m0 + i, col = n0 + i;
    const bool rv = row < M, cv = col < N;
    const int64_t rowc = rv ? row : 0, colc = cv ? col : 0;   // keep addresses in range for masked lanes

    float acc[16];
#pragma unroll
    for (int t = 0; t < 16; t++) acc[t] = 0.f;

    for (int64_t kb0 = kb_begin; kb0 < kb_end; kb0 += I8_U) {
        uint4 qa[I8_U], qb[I8_U];
        uint32_t sa[I8_U], sb[I8_U];
#pragma unroll
        for (int u = 0; u < I8_U; u++) {
            const int64_t kb = kb0 + u < kb_end ? kb0 + u : kb_end - 1;   // past the slice: a valid block, result unused
            qa[u] = ld16(Ae + rowc * K + kb * BLOCK + 16 * g);
            qb[u] = ld16(Be + colc * K + kb * BLOCK + 16 * g);
            sa[u] = As[rowc * nkb + kb];
            sb[u] = Bs[colc * nkb + kb];
        }
#pragma unroll
        for (int u = 0; u < I8_U; u++) {
            if (kb0 + u >= kb_end) break;                                 // wave-uniform
            if (g == 0) lds[i] = (uint8_t)sa[u];
            wave_lds_sync8();
            uint32_t sa4[4];
#pragma unroll
            for (int q = 0; q < 4; q++) sa4[q] = *reinterpret_cast<const uint32_t *>(lds + 8 * q + 4 * g);
            const v4i_t a = rv ? v4i_t{(int)qa[u].x, (int)qa[u].y, (int)qa[u].z, (int)qa[u].w} : v4i_t{0, 0, 0, 0};
            const v4i_t b = cv ? v4i_t{(int)qb[u].x, (int)qb[u].y, (int)qb[u].z, (int)qb[u].w} : v4i_t{0, 0, 0, 0};
            v16i_t z;
#pragma unroll
            for (int t = 0; t < 16; t++) z[t] = 0;
            const v16i_t p = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, z, 0, 0, 0);
#pragma unroll
            for (int t = 0; t < 16; t++) {
                const uint32_t sat = (sa4[t >> 2] >> (8 * (t & 3))) & 0xFFu;
                const int e = (int)sat + (int)sb[u] - 254 - 12;
                float term = ldexpf((float)p[t], e);
                if (sat == SCALE_NAN || sb[u] == SCALE_NAN) term = __uint_as_float(0x7FC00000u);
                acc[t] += term;
            }
            wave_lds_sync8();   // the line is rewritten for the next block
        }
    }

    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < 16; t++) red[wave - 1][t][lane] = acc[t];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int t = 0; t < 16; t++) {
        float v = acc[t];
#pragma unroll
        for (int w = 0; w < I8_WAVES - 1; w++) v += red[w][t][lane];
        const int64_t r = m0 + 8 * (t / 4) + 4 * g + (t % 4);
        if (r < M && cv) {
            if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = v;
            else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
        }
    }
}

static hipError_t launch_int8_direct(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                                     const uint8_t *Bs, void *C, int c_dt, int64_t ldc, const uint32_t *run_if, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    if (c_dt == DT_F32) hipLaunchKernelGGL((gemm_int8_kernel<DT_F32>), grid, dim3(256), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc, run_if);
    else hipLaunchKernelGGL((gemm_int8_kernel<DT_BF16>), grid, dim3(256), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc, run_if);
    return hipGetLastError();
}

hipError_t launch_gemm_int8(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                            const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    // the split route: whole tiles, a depth the tiled kernel takes (4K a multiple of 128, >= 512), and at
    // least 64 tiles -- below that the chip is so empty that the direct kernel's many small tiles finish
    // sooner (measured: 2048 x 2048 x 2048 level, 1024 x 4096 x 4096 14% ahead, 4096^3 three times faster)
    if (M > 0 && N > 0 && K >= 128 && (M / 256) * (N / 256) >= 64 && gemm_tiled_applies(M, N, 4 * K, FP6_E2M3, FP6_E2M3)) {
        const size_t nba = (size_t)M * (size_t)(K / BLOCK), nbb = (size_t)N * (size_t)(K / BLOCK);
        const size_t off_ea = 256, off_eb = off_ea + nba * 96, off_sa = off_eb + nbb * 96, off_sb = off_sa + nba * 4;
        uint8_t *ws = nullptr;
        hipError_t e = hipMallocAsync(reinterpret_cast<void **>(&ws), off_sb + nbb * 4, st);
        if (e == hipSuccess) {
            uint32_t *flag = reinterpret_cast<uint32_t *>(ws);
            e = hipMemsetAsync(flag, 0, 4, st);
            if (e == hipSuccess) {
                hipLaunchKernelGGL((int8_split_kernel<false>), dim3((unsigned)((nba + 255) / 256)), dim3(256), 0, st, Ae, As,
                                   (int64_t)nba, ws + off_ea, ws + off_sa, flag);
                hipLaunchKernelGGL((int8_split_kernel<true>), dim3((unsigned)((nbb + 255) / 256)), dim3(256), 0, st, Be, Bs,
                                   (int64_t)nbb, ws + off_eb, ws + off_sb, flag);
                e = hipGetLastError();
            }
            if (e == hipSuccess)
                e = launch_gemm_tiled(M, N, 4 * K, ws + off_ea, ws + off_sa, nullptr, 0, ROUND_RNE, FP6_E2M3, ws + off_eb,
                                      ws + off_sb, FP6_E2M3, C, c_dt, ldc, st);
            if (e == hipSuccess) e = launch_int8_direct(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, flag, st);
            const hipError_t f = hipFreeAsync(ws, st);
            return e != hipSuccess ? e : f;
        }
        (void)hipGetLastError();   // no workspace: the direct kernel needs none
    }
    // few rows: eight waves share the blocks of a tile.  Also where the direct kernel would put at most one
    // wave on a SIMD and K is long (measured: 256 x 4096 x 4096 81 -> 66 us, 1024 x 1024 x 4096 84 -> 64 us;
    // with 2048 tiles of 32 x 32 the direct kernel is ahead again, 114 vs 124 us)
    const int64_t tiles32 = ((M + 31) / 32) * ((N + 31) / 32);
    if (M > 0 && N > 0 && ((M <= 128 && K >= 8 * BLOCK) || (tiles32 <= 1024 && K >= 4096))) {
        const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 31) / 32));
        if (c_dt == DT_F32)
            hipLaunchKernelGGL((gemm_int8_shared_k_kernel<DT_F32>), grid, dim3(64 * I8_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
        else
            hipLaunchKernelGGL((gemm_int8_shared_k_kernel<DT_BF16>), grid, dim3(64 * I8_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
        return hipGetLastError();
    }
    return launch_int8_direct(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, nullptr, st);
}

}  // namespace mx
