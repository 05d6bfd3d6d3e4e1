// LDS-tiled MX GEMM for 8-bit operands (Section 4.1 of arXiv 2310.10537) on
// gfx950's block-scaled 32x32x64 f8f6f4 matrix instruction.
//
// Work-group: 256 threads = 4 waves in a 2 x 2 arrangement, output tile
// 256 x 256, K step 128 (four MX blocks).  Each wave owns a 128 x 128 sub-tile:
// 4 x 4 matrix-instruction tiles of 32 x 32, i.e. 256 accumulator registers.
// Per K step the work-group stages 256 x 128 bytes of A and of B in LDS (double
// buffered, 128 KB in all); every 16-byte chunk c of row r sits at chunk
// position c ^ (r & 7) of the row, so both the 16-byte stores of the staging
// pass and the operand reads (32 rows, same chunk) are free of bank conflicts.
// Scale bytes go from global memory straight to registers: one dword holds the
// four scale bytes of a row for the K step; lanes 32..63 shift it by one byte so
// that a single op_sel value addresses block 2*sub + g for every lane.
#include "mx_device.hpp"
#include "mx_launch.hpp"

namespace mx {

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

constexpr int TM = 256, TN = 256, TK = 128;      // work-group tile (TK in elements = bytes for 8-bit formats)
constexpr int TILE_BYTES = TM * TK;              // 32 KB per operand per stage
constexpr int GEMM_LDS_BYTES = 4 * TILE_BYTES;   // A,B x 2 stages

__host__ __device__ constexpr int hw_fmt8(int fmt) { return fmt == FP8_E4M3 ? 0 : 1; }

// LDS byte offset of 16-byte chunk c (0..7) of tile row r
__device__ __forceinline__ int swz(int r, int c) { return r * TK + ((c ^ (r & 7)) << 4); }

template <int FA, int FB, int CDT>
__global__ __launch_bounds__(256, 1) void gemm8_tile_kernel(int64_t M, int64_t N, int64_t K,
                                                            const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                            const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                            void *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int HA = hw_fmt8(FA), HB = hw_fmt8(FB);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, g = lane >> 5;

    // XCD-aware rasterisation: work-groups are dealt round-robin to 8 XCDs; give each XCD
    // a contiguous band of M tiles so that its L2 sees few distinct A panels.
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + 7) >> 3;
    const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || tile_id >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile_id / tiles_n) * TM;
    const int64_t n0 = (int64_t)(tile_id % tiles_n) * TN;
    const int64_t nkb = K / BLOCK;
    const int T = (int)(K / TK);

    // ---- staging map: thread handles chunks q = tid + 256*j, j < 8: row q/8 = tid/8 + 32*j, chunk tid%8.
    // Rows 32 apart share (row & 7), so the LDS offset of chunk j is that of chunk 0 plus j * 4096.
    const int st_r = tid >> 3, st_c = tid & 7;
    const uint8_t *gA = Ae + (m0 + st_r) * K + st_c * 16;
    const uint8_t *gB = Be + (n0 + st_r) * K + st_c * 16;
    const int64_t g_step = 32 * K;                 // 32 rows further down
    const int st_l = swz(st_r, st_c);
    // ---- scale pointers: one dword per row per K step; row tiles are 32 rows apart
    const uint8_t *sA = As + (m0 + wm * 128 + li) * nkb;
    const uint8_t *sB = Bs + (n0 + wn * 128 + li) * nkb;
    const int64_t s_step = 32 * nkb;
    // ---- operand read offsets inside a stage's tile: row tile x adds x * 4096, the second 16-byte
    // chunk of a sub-step (chunk + 2) flips bit 5, sub-step 1 (chunk + 4) flips bit 6
    const int ra0 = swz(wm * 128 + li, g), rb0 = swz(wn * 128 + li, g);

    v16f_t acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][y][t] = 0.f;

    // Software pipeline (one work-group barrier per K step).
    //   global -> registers -> LDS runs two stages ahead of the multiply: during step t the
    //   registers holding stage t+1 are written to the other LDS buffer and immediately reloaded
    //   with stage t+2, so a global load has a whole step to arrive;
    //   LDS -> operand registers runs a few matrix instructions ahead, in program order
    //   interleaved with them (the compiler is fenced group by group), so that the LDS pipe and
    //   the matrix pipe work at the same time instead of taking turns.
    // Step t, buffer cur = t & 1 holds stage t:
    //   X  : 16 MFMA of sub-step 0 | read a1[0..3], b1[0..1] (sub-step 1) and b0[1..3] just in time
    //   Y1 :  8 MFMA of sub-step 1 | write stage t+1 to the other buffer, reload registers with
    //                                stage t+2, read b1[2..3]
    //   barrier: every read of stage t has been issued before it, every write of stage t+1 too
    //   Y2 :  8 MFMA of sub-step 1 | read a0[0..3], b0[0] of stage t+1
    // Stages beyond the last are clamped to the last one: the extra loads are harmless and the
    // loop body needs no branches.
    uint4 rA[8], rB[8];
    uint32_t scA[4], scB[4], scA1[4], scB1[4];
    v8i_t a0[4], a1[4], b0[2], b1[4];

    auto rd = [&](const uint8_t *buf, int ofs0, int sub, int x) -> v8i_t {
        const uint4 lo = *reinterpret_cast<const uint4 *>(buf + (ofs0 ^ (sub << 6)) + x * 4096);
        const uint4 hi = *reinterpret_cast<const uint4 *>(buf + (ofs0 ^ (sub << 6) ^ 32) + x * 4096);
        return v8i_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };
#define MX_FENCE() __builtin_amdgcn_sched_barrier(0)
#define MX_MFMA4(AF, BF, Y, OPS)                                                                                      \
    _Pragma("unroll") for (int x = 0; x < 4; x++)                                                                     \
        acc[x][Y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(AF[x], BF, acc[x][Y], HA, HB, OPS, (int)sa[x], OPS, (int)sb[Y])

    // ---- prologue: stage 0 to LDS, stage 1 to registers, first fragments
#pragma unroll
    for (int j = 0; j < 8; j++) { rA[j] = ld16(gA + j * g_step); rB[j] = ld16(gB + j * g_step); }
#pragma unroll
    for (int x = 0; x < 4; x++) {
        scA[x] = *reinterpret_cast<const uint32_t *>(sA + x * s_step);
        scB[x] = *reinterpret_cast<const uint32_t *>(sB + x * s_step);
    }
#pragma unroll
    for (int j = 0; j < 8; j++) {
        *reinterpret_cast<uint4 *>(lds + st_l + j * 4096) = rA[j];
        *reinterpret_cast<uint4 *>(lds + TILE_BYTES + st_l + j * 4096) = rB[j];
    }
    {
        const int64_t k1 = (T > 1 ? 1 : 0) * (int64_t)TK;
        const int s1 = (T > 1 ? 1 : 0) * 4;
#pragma unroll
        for (int j = 0; j < 8; j++) { rA[j] = ld16(gA + k1 + j * g_step); rB[j] = ld16(gB + k1 + j * g_step); }
#pragma unroll
        for (int x = 0; x < 4; x++) {
            scA1[x] = *reinterpret_cast<const uint32_t *>(sA + x * s_step + s1);
            scB1[x] = *reinterpret_cast<const uint32_t *>(sB + x * s_step + s1);
        }
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; x++) a0[x] = rd(lds, ra0, 0, x);
    b0[0] = rd(lds + TILE_BYTES, rb0, 0, 0);

    for (int t = 0; t < T; t++) {
        const int cur = t & 1;
        const uint8_t *bufA = lds + cur * 2 * TILE_BYTES;
        const uint8_t *bufB = bufA + TILE_BYTES;
        uint8_t *nxt = lds + (cur ^ 1) * 2 * TILE_BYTES;
        const int t2 = t + 2 < T ? t + 2 : T - 1;
        const int64_t kofs = (int64_t)t2 * TK;
        uint32_t sa[4], sb[4];
#pragma unroll
        for (int x = 0; x < 4; x++) { sa[x] = g ? scA[x] >> 8 : scA[x]; sb[x] = g ? scB[x] >> 8 : scB[x]; }
        MX_FENCE();

        // ---- X: sub-step 0 (the scale dwords of stage t+2 are requested first: they are the
        // oldest loads in flight when they are rotated in at the end of the step)
        uint32_t scA2[4], scB2[4];
#pragma unroll
        for (int x = 0; x < 4; x++) {
            scA2[x] = *reinterpret_cast<const uint32_t *>(sA + x * s_step + t2 * 4);
            scB2[x] = *reinterpret_cast<const uint32_t *>(sB + x * s_step + t2 * 4);
        }
        b0[1] = rd(bufB, rb0, 0, 1); a1[0] = rd(bufA, ra0, 1, 0); b1[0] = rd(bufB, rb0, 1, 0);
        MX_MFMA4(a0, b0[0], 0, 0);
        MX_FENCE();
        b0[0] = rd(bufB, rb0, 0, 2); a1[1] = rd(bufA, ra0, 1, 1); b1[1] = rd(bufB, rb0, 1, 1);
        MX_MFMA4(a0, b0[1], 1, 0);
        MX_FENCE();
        b0[1] = rd(bufB, rb0, 0, 3); a1[2] = rd(bufA, ra0, 1, 2);
        MX_MFMA4(a0, b0[0], 2, 0);
        MX_FENCE();
        a1[3] = rd(bufA, ra0, 1, 3);
        MX_MFMA4(a0, b0[1], 3, 0);
        MX_FENCE();

        // ---- Y1: sub-step 1, first half; stage t+1 registers -> LDS, reload with stage t+2
        b1[2] = rd(bufB, rb0, 1, 2);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            *reinterpret_cast<uint4 *>(nxt + st_l + j * 4096) = rA[j];
            rA[j] = ld16(gA + kofs + j * g_step);
        }
        MX_MFMA4(a1, b1[0], 0, 2);
        MX_FENCE();
        b1[3] = rd(bufB, rb0, 1, 3);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            *reinterpret_cast<uint4 *>(nxt + TILE_BYTES + st_l + j * 4096) = rB[j];
            rB[j] = ld16(gB + kofs + j * g_step);
        }
        MX_MFMA4(a1, b1[1], 1, 2);
        MX_FENCE();
        __syncthreads();
        MX_FENCE();

        // ---- Y2: sub-step 1, second half; first fragments of stage t+1
        a0[0] = rd(nxt, ra0, 0, 0); a0[1] = rd(nxt, ra0, 0, 1);
        MX_MFMA4(a1, b1[2], 2, 2);
        MX_FENCE();
        a0[2] = rd(nxt, ra0, 0, 2); a0[3] = rd(nxt, ra0, 0, 3); b0[0] = rd(nxt + TILE_BYTES, rb0, 0, 0);
        MX_MFMA4(a1, b1[3], 3, 2);
#pragma unroll
        for (int x = 0; x < 4; x++) { scA[x] = scA1[x]; scB[x] = scB1[x]; scA1[x] = scA2[x]; scB1[x] = scB2[x]; }
        MX_FENCE();
    }
#undef MX_MFMA4
#undef MX_FENCE

    // ---- epilogue: lane (li, g), register t of tile (x, y) -> C[8*(t/4) + 4g + t%4][li]
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) {
                const int64_t r = m0 + wm * 128 + x * 32 + 8 * (t / 4) + 4 * g + (t % 4);
                const int64_t c = n0 + wn * 128 + y * 32 + li;
                if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + c] = acc[x][y][t];
                else reinterpret_cast<uint16_t *>(C)[r * ldc + c] = (uint16_t)f32_to_bf16_bits(acc[x][y][t]);
            }
}

template <int FA, int FB, int CDT>
static hipError_t launch_t(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                           const uint8_t *Bs, void *C, int64_t ldc, hipStream_t st)
{
    static bool attr_set = false;   // raising the dynamic LDS limit is a per-function, per-process setting
    auto kern = gemm8_tile_kernel<FA, FB, CDT>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           GEMM_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
    const int per_xcd = (tiles_m * tiles_n + 7) / 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(256), GEMM_LDS_BYTES, st, M, N, K, Ae, As, Be, Bs, C, ldc,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

// Tiled path for 8-bit x 8-bit operands on full tiles; hipErrorNotSupported otherwise.
hipError_t launch_gemm_tiled(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA,
                             const uint8_t *Be, const uint8_t *Bs, int fmtB, void *C, int c_dt, int64_t ldc,
                             hipStream_t st)
{
    const bool a8 = fmtA == FP8_E4M3 || fmtA == FP8_E5M2, b8 = fmtB == FP8_E4M3 || fmtB == FP8_E5M2;
    if (!a8 || !b8 || M % TM || N % TN || K % TK || K == 0 || (M / TM) * (N / TN) > (1 << 24)) return hipErrorNotSupported;
#define MX_CASE(FA_, FB_)                                                                                          \
    if (fmtA == FA_ && fmtB == FB_)                                                                                \
        return c_dt == DT_F32 ? launch_t<FA_, FB_, DT_F32>(M, N, K, Ae, As, Be, Bs, C, ldc, st)                    \
                              : launch_t<FA_, FB_, DT_BF16>(M, N, K, Ae, As, Be, Bs, C, ldc, st);
    MX_CASE(FP8_E4M3, FP8_E4M3)
    MX_CASE(FP8_E4M3, FP8_E5M2)
    MX_CASE(FP8_E5M2, FP8_E4M3)
    MX_CASE(FP8_E5M2, FP8_E5M2)
#undef MX_CASE
    return hipErrorNotSupported;
}

}  // namespace mx
