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
#include "mx_gemm_tile.hpp"

namespace mx {

constexpr int SK_WAVES = 8;

// ---------------------------------------------------------------------------------------------
// K a multiple of 128: operands staged through LDS.
// In the kernel further down every lane of an operand load addresses a different matrix row, so
// a load instruction touches 32 cache lines and a compute unit makes eight line accesses for every
// line it needs: that, not bandwidth or latency, bounds it (9.4 us for 4096 x 4096 weights at
// M = 1).  Here each wave fetches its slice 128 elements at a time with loads whose adjacent lanes
// read adjacent 16 bytes of a row (every line touched once), parks the 16-byte pieces in a private
// LDS tile laid out exactly as the large tiled kernel lays out its stages (same swizzles, same
// operand reads), and multiplies from there; the next chunk's loads are in flight meanwhile.
// Rows beyond M and columns beyond N read a valid row instead (clamped): rows and columns of the
// product are independent, and such results are never stored.
// ---------------------------------------------------------------------------------------------
template <int W> struct SkStage {                    // one 32-row block of a 128-element chunk
    static constexpr int NJ = W == 4 ? 2 : 4;        // loads per lane: 16 (4-bit) or 8 rows per wave-wide load
    static constexpr int BYTES = 32 * TileFmt<W>::ROW;
};

template <int FA, int FB, int MT, int CDT>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_lds_kernel(int64_t M, int64_t N, int64_t K,
                                                                         const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                                         const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                                         void *__restrict__ C, int64_t ldc)
{
    constexpr int WA = Fmt<FA>::bits, WB = Fmt<FB>::bits;
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);   // must reach the builtin as literal constants
    constexpr int A_BYTES = MT * SkStage<WA>::BYTES, B_BYTES = SkStage<WB>::BYTES, W_BYTES = A_BYTES + B_BYTES;
    constexpr int RED_BYTES = (SK_WAVES - 1) * MT * 16 * 64 * 4;
    constexpr int LDS_BYTES = SK_WAVES * W_BYTES > RED_BYTES ? SK_WAVES * W_BYTES : RED_BYTES;
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 31, g = lane >> 5;
    const int64_t n0 = (int64_t)blockIdx.x * 32, m0 = (int64_t)blockIdx.y * (32 * MT);
    const int64_t nkb = K / BLOCK, chunks = K / 128;
    const int64_t per_wave = (chunks + SK_WAVES - 1) / SK_WAVES;
    const int64_t c_begin = wave * per_wave, c_end = c_begin + per_wave < chunks ? c_begin + per_wave : chunks;
    uint8_t *tA = lds + wave * W_BYTES, *tB = tA + A_BYTES;

    // ---- staging: lane -> (row l / P, 16-byte piece l % P) of a wave-wide load; P pieces per row chunk
    constexpr int PA = WA == 4 ? 4 : 8, PB = WB == 4 ? 4 : 8;            // (6-bit: pieces 6 and 7 stay idle)
    const int ar = lane / PA, ap = lane % PA, br = lane / PB, bp = lane % PB;
    const bool a_on = WA != 6 || ap < 6, b_on = WB != 6 || bp < 6;
    const int64_t a_rb = K * WA / 8, b_rb = K * WB / 8;                   // bytes per matrix row
    auto lds_slot = [](int w, int r, int c) {
        return w == 8 ? r * 128 + ((c ^ ((r >> 1) & 7)) << 4) : w == 6 ? r * 96 + ((c ^ ((r >> 3) & 1)) << 4)
                                                                       : r * 64 + ((c ^ ((r >> 2) & 3)) << 4);
    };
    auto clampi = [](int64_t v, int64_t hi) { return v < hi ? v : hi; };
    uint4 ra[MT][SkStage<WA>::NJ], rb[SkStage<WB>::NJ];
    uint32_t sa_d[MT], sb_d;
    auto request = [&](int64_t c) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int j = 0; j < SkStage<WA>::NJ; j++) {
                const int64_t row = clampi(m0 + 32 * x + j * (64 / PA) + ar, M - 1);
                if (a_on) ra[x][j] = ld16(Ae + row * a_rb + c * (128 * WA / 8) + ap * 16);
            }
#pragma unroll
        for (int j = 0; j < SkStage<WB>::NJ; j++) {
            const int64_t row = clampi(n0 + j * (64 / PB) + br, N - 1);
            if (b_on) rb[j] = ld16(Be + row * b_rb + c * (128 * WB / 8) + bp * 16);
        }
#pragma unroll
        for (int x = 0; x < MT; x++) sa_d[x] = *reinterpret_cast<const uint32_t *>(As + clampi(m0 + 32 * x + i, M - 1) * nkb + c * 4);
        sb_d = *reinterpret_cast<const uint32_t *>(Bs + clampi(n0 + i, N - 1) * nkb + c * 4);
    };
    auto park = [&]() {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int j = 0; j < SkStage<WA>::NJ; j++)
                if (a_on) *reinterpret_cast<uint4 *>(tA + x * SkStage<WA>::BYTES + lds_slot(WA, j * (64 / PA) + ar, ap)) = ra[x][j];
#pragma unroll
        for (int j = 0; j < SkStage<WB>::NJ; j++)
            if (b_on) *reinterpret_cast<uint4 *>(tB + lds_slot(WB, j * (64 / PB) + br, bp)) = rb[j];
    };
    const FragOfs<WA> fa = frag_ofs<WA>(i, g);
    const FragOfs<WB> fb = frag_ofs<WB>(i, g);

    v16f_t acc[MT];
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 16; t++) acc[x][t] = 0.f;

    if (c_begin < c_end) request(c_begin);
    for (int64_t c = c_begin; c < c_end; c++) {
        park();
        // lanes 32 .. 63 shift their scale dword by a byte: one selector then addresses block 2 sub + g
        uint32_t sa[MT];
#pragma unroll
        for (int x = 0; x < MT; x++) sa[x] = g ? sa_d[x] >> 8 : sa_d[x];
        const uint32_t sb = g ? sb_d >> 8 : sb_d;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        if (c + 1 < c_end) request(c + 1);
        const v8i_t b0 = read_frag<WB>(tB, fb, 0, 0), b1 = read_frag<WB>(tB, fb, 1, 0);
#pragma unroll
        for (int x = 0; x < MT; x++) {
            const v8i_t a0 = read_frag<WA>(tA + x * SkStage<WA>::BYTES, fa, 0, 0), a1 = read_frag<WA>(tA + x * SkStage<WA>::BYTES, fa, 1, 0);
            acc[x] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, b0, acc[x], HA, HB, 0, (int)sa[x], 0, (int)sb);
            acc[x] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, b1, acc[x], HA, HB, 2, (int)sa[x], 2, (int)sb);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the tile is read before the next chunk is parked in it
        __builtin_amdgcn_wave_barrier();
    }

    // ---- the eight partial sums, always w0 + w1 + ... + w7; the staging tiles are done with
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
    if (wave > 0) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 16; t++) red[(((wave - 1) * MT + x) * 16 + t) * 64 + lane] = acc[x][t];
    }
    __syncthreads();
    if (wave != 0) return;
    const int64_t col = n0 + i;
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 16; t++) {
            float v = acc[x][t];
#pragma unroll
            for (int w = 0; w < SK_WAVES - 1; w++) v += red[((w * MT + x) * 16 + t) * 64 + lane];
            const int64_t r = m0 + 32 * x + 8 * (t / 4) + 4 * g + (t % 4);   // result register t: row 8 (t/4) + 4g + t%4, column i
            if (r < M && col < N) {
                if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = v;
                else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
            }
        }
}

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

template <int FA, int FB, int MT>
static hipError_t launch_lds(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                             const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 32 * MT - 1) / (32 * MT)));
    if (c_dt == DT_F32)
        hipLaunchKernelGGL((gemm_skinny_lds_kernel<FA, FB, MT, DT_F32>), grid, dim3(64 * SK_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    else
        hipLaunchKernelGGL((gemm_skinny_lds_kernel<FA, FB, MT, DT_BF16>), grid, dim3(64 * SK_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    return hipGetLastError();
}

template <int FA, int FB>
static hipError_t launch_pair(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                              const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    const bool staged = K % 128 == 0;   // whole 128-element chunks, 16-byte aligned rows
    if (M <= 32) return staged ? launch_lds<FA, FB, 1>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
                               : launch_mt<FA, FB, 1>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    if (M <= 64) return staged ? launch_lds<FA, FB, 2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
                               : launch_mt<FA, FB, 2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    return staged ? launch_lds<FA, FB, 4>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
                  : launch_mt<FA, FB, 4>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
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

// FP8 / FP6 / FP4 operands; at most 128 rows of A (any N, any K multiple of 32), or any number of rows
// in groups of 128 when K is a multiple of 128 (the LDS-staged kernel) and at least 512: with a
// shorter K most of the eight waves have no slice (256 x 256 x 256: 12 us against the direct kernel's 9)
bool gemm_skinny_applies(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    return M > 0 && (M <= 128 || (K % 128 == 0 && K >= 512 && (M + 127) / 128 <= 65535)) && N > 0 && K > 0 &&
           fmtA >= FP8_E4M3 && fmtA <= FP4_E2M1 && fmtB >= FP8_E4M3 && fmtB <= FP4_E2M1 && (N + 31) / 32 <= 0x7FFFFFFF;
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
