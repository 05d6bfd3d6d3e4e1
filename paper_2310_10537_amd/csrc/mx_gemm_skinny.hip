// MX GEMM (Section 4.1 of arXiv 2310.10537) for few rows of A -- the shape of a decoding step,
// where the time goes into streaming the weight operand B once.
//
// The direct kernel gives such a problem one wave per 32 x 32 output tile and lets it walk the
// whole K range alone, one load-then-multiply after the other: with N / 32 waves on the chip and
// every step paying a full memory latency, 4096 x 4096 weights take 25-45 us (0.4-0.7 TB/s).  Here a
// work-group of eight waves owns 32 columns of C and all (up to 128) rows: the K range is cut into
// eight contiguous slices, one per wave, each wave requests the operands of several K steps before
// it multiplies the first, and the eight partial sums meet in LDS in a fixed order (so the result
// does not depend on timing).  B is read exactly once; A, a few KB per K step, comes from L2.
#include "mx_gemm_frag.hpp"
#include "mx_launch.hpp"

namespace mx {

constexpr int SK_WAVES = 8;

// MT: 32-row tiles of A per work-group (1, 2 or 4)
template <int FA, int FB, int MT, int CDT>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_kernel(int64_t M, int64_t N, int64_t K,
                                                                     const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                                     const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                                     void *__restrict__ C, int64_t ldc)
{
    constexpr int wA = Fmt<FA>::bits, wB = Fmt<FB>::bits;
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);   // must reach the builtin as literal constants
    constexpr int U = MT == 4 ? 2 : MT == 2 ? 4 : 8;  // K steps whose operands are requested together
    // partial sums: of seven waves at once (one barrier) while that fits in 64 KB, else of four at a time
    constexpr bool FLAT = MT <= 2;
    __shared__ float red[FLAT ? SK_WAVES - 1 : SK_WAVES / 2][MT][16][64];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 31, g = lane >> 5;
    const int64_t n0 = (int64_t)blockIdx.x * 32, m0 = (int64_t)blockIdx.y * (32 * MT);
    const int64_t nkb = K / BLOCK, steps = (nkb + 1) / 2;           // a K step = 64 elements = two blocks
    const int64_t chunk = (steps + SK_WAVES - 1) / SK_WAVES;
    const int64_t s_begin = wave * chunk, s_end = s_begin + chunk < steps ? s_begin + chunk : steps;

    const int64_t col = n0 + i;
    const bool cv = col < N;
    const uint8_t *brow = Be + (cv ? col : 0) * (K * wB / 8);       // masked lanes keep their addresses in range
    const uint8_t *bsc = Bs + (cv ? col : 0) * nkb;
    const uint8_t *arow[MT], *asc[MT];
    bool rv[MT];
#pragma unroll
    for (int x = 0; x < MT; x++) {
        const int64_t row = m0 + 32 * x + i;
        rv[x] = row < M;
        arow[x] = Ae + (rv[x] ? row : 0) * (K * wA / 8);
        asc[x] = As + (rv[x] ? row : 0) * nkb;
    }

    v16f acc[MT];
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 16; t++) acc[x][t] = 0.f;

    for (int64_t st = s_begin; st < s_end; st += U) {
        v8i a[U][MT], b[U];
        int sa[U][MT], sb[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int64_t kb0 = 2 * (st + u);
            const bool v0 = st + u < s_end, v1 = v0 && kb0 + 1 < nkb;   // steps beyond the slice, second block beyond K
            const bool mine = g ? v1 : v0;
            b[u] = load_operand<FB>(brow + kb0 * (BLOCK * wB / 8), g, cv && v0, cv && v1);
            sb[u] = (cv && mine) ? (int)bsc[kb0 + g] : 127;
#pragma unroll
            for (int x = 0; x < MT; x++) {
                a[u][x] = load_operand<FA>(arow[x] + kb0 * (BLOCK * wA / 8), g, rv[x] && v0, rv[x] && v1);
                sa[u][x] = (rv[x] && mine) ? (int)asc[x][kb0 + g] : 127;
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int x = 0; x < MT; x++)
                acc[x] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[u][x], b[u], acc[x], HA, HB, 0, sa[u][x], 0, sb[u]);
    }

    // ---- the eight partial sums, always in the same order: w0 + w1 + ... + w7 (one or two row tiles) ...
    if constexpr (FLAT) {
        if (wave > 0) {
#pragma unroll
            for (int x = 0; x < MT; x++)
#pragma unroll
                for (int t = 0; t < 16; t++) red[wave - 1][x][t][lane] = acc[x][t];
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) {
                float v = acc[x][t];
#pragma unroll
                for (int w = 0; w < SK_WAVES - 1; w++) v += red[w][x][t][lane];
                const int64_t r = m0 + 32 * x + 8 * (t / 4) + 4 * g + (t % 4);
                if (r < M && cv) {
                    if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = v;
                    else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
                }
            }
        return;
    }
    // ... or ((w0 + w4) + (w1 + w5)) + ((w2 + w6) + (w3 + w7)) (four row tiles)
    if (wave >= 4) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) red[wave - 4][x][t][lane] = acc[x][t];
    }
    __syncthreads();
    if (wave < 4) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][t] += red[wave][x][t][lane];
    }
    __syncthreads();
    if (wave == 1 || wave == 3) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) red[wave][x][t][lane] = acc[x][t];
    }
    __syncthreads();
    if (wave == 0 || wave == 2) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][t] += red[wave + 1][x][t][lane];
    }
    __syncthreads();
    if (wave == 2) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) red[0][x][t][lane] = acc[x][t];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 16; t++) {
            const float v = acc[x][t] + red[0][x][t][lane];
            const int64_t r = m0 + 32 * x + 8 * (t / 4) + 4 * g + (t % 4);   // result register t: row 8 (t/4) + 4g + t%4, column i
            if (r < M && cv) {
                if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = v;
                else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
            }
        }
}

template <int FA, int FB, int MT>
static hipError_t launch_mt(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                            const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 32 * MT - 1) / (32 * MT)));
    if (c_dt == DT_F32)
        hipLaunchKernelGGL((gemm_skinny_kernel<FA, FB, MT, DT_F32>), grid, dim3(64 * SK_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<FA, FB, MT, DT_BF16>), grid, dim3(64 * SK_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    return hipGetLastError();
}

template <int FA, int FB>
static hipError_t launch_pair(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                              const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    if (M <= 32) return launch_mt<FA, FB, 1>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    if (M <= 64) return launch_mt<FA, FB, 2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    return launch_mt<FA, FB, 4>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
}

template <int FA>
static hipError_t launch_b(int fmtB, int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                           const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    switch (fmtB) {
        case FP8_E4M3: return launch_pair<FA, FP8_E4M3>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP8_E5M2: return launch_pair<FA, FP8_E5M2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP6_E3M2: return launch_pair<FA, FP6_E3M2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP6_E2M3: return launch_pair<FA, FP6_E2M3>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        default:       return launch_pair<FA, FP4_E2M1>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    }
}

// at most 128 rows of A (any N, any K multiple of 32), FP8 / FP6 / FP4 operands
bool gemm_skinny_applies(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    return M > 0 && M <= 128 && N > 0 && K > 0 && fmtA >= FP8_E4M3 && fmtA <= FP4_E2M1 && fmtB >= FP8_E4M3 && fmtB <= FP4_E2M1 &&
           (N + 31) / 32 <= 0x7FFFFFFF;
}

hipError_t launch_gemm_skinny(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA, const uint8_t *Be,
                              const uint8_t *Bs, int fmtB, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    if (!gemm_skinny_applies(M, N, K, fmtA, fmtB)) return hipErrorNotSupported;
    switch (fmtA) {
        case FP8_E4M3: return launch_b<FP8_E4M3>(fmtB, M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP8_E5M2: return launch_b<FP8_E5M2>(fmtB, M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP6_E3M2: return launch_b<FP6_E3M2>(fmtB, M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        case FP6_E2M3: return launch_b<FP6_E2M3>(fmtB, M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
        default:       return launch_b<FP4_E2M1>(fmtB, M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    }
}

}  // namespace mx
