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

    // Software pipeline, prefetch distance two: while stage t is multiplied out of LDS, stage t+1
    // (fetched during the previous iteration) moves from registers to the other LDS buffer and
    // stage t+2 is requested from global memory, so a load has a whole iteration to arrive.
    uint4 rA[8], rB[8];
    uint32_t scA[4], scB[4], scA1[4], scB1[4];

    // ---- prologue: stage 0 to LDS, stage 1 to registers
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
    if (T > 1) {
#pragma unroll
        for (int j = 0; j < 8; j++) { rA[j] = ld16(gA + TK + j * g_step); rB[j] = ld16(gB + TK + j * g_step); }
#pragma unroll
        for (int x = 0; x < 4; x++) {
            scA1[x] = *reinterpret_cast<const uint32_t *>(sA + x * s_step + 4);
            scB1[x] = *reinterpret_cast<const uint32_t *>(sB + x * s_step + 4);
        }
    }
    __syncthreads();

    for (int t = 0; t < T; t++) {
        const int cur = t & 1;
        const uint8_t *bufA = lds + cur * 2 * TILE_BYTES;
        const uint8_t *bufB = bufA + TILE_BYTES;
        uint8_t *nxt = lds + (cur ^ 1) * 2 * TILE_BYTES + st_l;
        uint32_t sa[4], sb[4];
#pragma unroll
        for (int x = 0; x < 4; x++) { sa[x] = g ? scA[x] >> 8 : scA[x]; sb[x] = g ? scB[x] >> 8 : scB[x]; }

        if (t + 1 < T) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                *reinterpret_cast<uint4 *>(nxt + j * 4096) = rA[j];
                *reinterpret_cast<uint4 *>(nxt + TILE_BYTES + j * 4096) = rB[j];
            }
#pragma unroll
            for (int x = 0; x < 4; x++) { scA[x] = scA1[x]; scB[x] = scB1[x]; }
        }
        if (t + 2 < T) {
            const int64_t kofs = (int64_t)(t + 2) * TK;
#pragma unroll
            for (int j = 0; j < 8; j++) { rA[j] = ld16(gA + kofs + j * g_step); rB[j] = ld16(gB + kofs + j * g_step); }
#pragma unroll
            for (int x = 0; x < 4; x++) {
                scA1[x] = *reinterpret_cast<const uint32_t *>(sA + x * s_step + (t + 2) * 4);
                scB1[x] = *reinterpret_cast<const uint32_t *>(sB + x * s_step + (t + 2) * 4);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

#pragma unroll
        for (int sub = 0; sub < 2; sub++) {
            v8i_t a[4];
#pragma unroll
            for (int x = 0; x < 4; x++) {
                const uint4 a0 = *reinterpret_cast<const uint4 *>(bufA + (ra0 ^ (sub << 6)) + x * 4096);
                const uint4 a1 = *reinterpret_cast<const uint4 *>(bufA + (ra0 ^ (sub << 6) ^ 32) + x * 4096);
                a[x] = v8i_t{(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
            }
#pragma unroll
            for (int y = 0; y < 4; y++) {
                const uint4 b0 = *reinterpret_cast<const uint4 *>(bufB + (rb0 ^ (sub << 6)) + y * 4096);
                const uint4 b1 = *reinterpret_cast<const uint4 *>(bufB + (rb0 ^ (sub << 6) ^ 32) + y * 4096);
                const v8i_t b = v8i_t{(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
#pragma unroll
                for (int x = 0; x < 4; x++) {
                    if (sub == 0)
                        acc[x][y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[x], b, acc[x][y], HA, HB, 0, (int)sa[x], 0, (int)sb[y]);
                    else
                        acc[x][y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[x], b, acc[x][y], HA, HB, 2, (int)sa[x], 2, (int)sb[y]);
                }
            }
        }
        __syncthreads();
    }

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
