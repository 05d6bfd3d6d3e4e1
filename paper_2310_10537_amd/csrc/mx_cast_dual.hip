// Dual-axis MX cast (Algorithm 1, Section 3 of arXiv 2310.10537, applied along both
// axes of one tensor): training needs every tensor cast with its blocks along the
// reduction axis of each GEMM that uses it -- X and X^T, W and W^T, dY and dY^T
// (Section 4.1: the two casts differ) -- so one pass over the bf16 source emits
// both MX tensors.  Source bytes are read once instead of twice.
//
// A work-group stages a 128-row x 64-column tile in LDS with coalesced 16-byte
// row loads.  Chunk c (16 bytes) of row r sits at chunk position
// (c + r + 2 * (r / 32)) % 8 of its 128-byte LDS row, which keeps all three
// access patterns free of bank conflicts: the staging stores (8 lanes cover a
// row), the row reads (a lane takes four consecutive chunks of its row; eight
// lanes = four rows x two halves hit eight different positions) and the column
// reads (sixteen adjacent columns of one row for each of four row blocks, the
// row blocks 32 bytes apart).
//   row part    thread t: row t / 2, columns 32 * (t % 2) .. + 31      -> axis-1 output
//   column part thread t: column t / 4, rows 32 * (t % 4) .. + 31      -> axis-0 output
// Both use the block cast of the stand-alone kernels, so each output is
// bit-identical to what mx_quantize writes for that axis.
#include "mx_convert.hpp"
#include "mx_launch.hpp"

namespace mx {

constexpr int DUAL_R = 128, DUAL_C = 64;

template <int w>
__device__ __forceinline__ void store_block(uint8_t *o, const uint32_t *out)
{
    if constexpr (w == 8) {
        st16(o, make_uint4(out[0], out[1], out[2], out[3]));
        st16(o + 16, make_uint4(out[4], out[5], out[6], out[7]));
    } else if constexpr (w == 6) {
        *reinterpret_cast<uint2 *>(o) = make_uint2(out[0], out[1]);
        *reinterpret_cast<uint2 *>(o + 8) = make_uint2(out[2], out[3]);
        *reinterpret_cast<uint2 *>(o + 16) = make_uint2(out[4], out[5]);
    } else {
        st16(o, make_uint4(out[0], out[1], out[2], out[3]));
    }
}

// rows a multiple of 128, cols a multiple of 64 (whole tiles only)
template <int FMT, int RND>
__global__ __launch_bounds__(256) void cast_dual_bf16_kernel(const uint16_t *__restrict__ src, int64_t rows, int64_t cols,
                                                             int64_t ld, uint8_t *__restrict__ e1, uint8_t *__restrict__ s1,
                                                             uint8_t *__restrict__ e0, uint8_t *__restrict__ s0,
                                                             int64_t row_tiles, int64_t n_tiles, int64_t per_xcd)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    __shared__ __attribute__((aligned(16))) uint8_t tile[DUAL_R * DUAL_C * 2];   // 16 KB, 128-byte rows
    const int t = threadIdx.x;
    // XCD-first tile order: each XCD owns a contiguous run of tiles
    const int64_t tile_id = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || tile_id >= n_tiles) return;   // uniform over the work-group
    int64_t ct = tile_id / row_tiles, rt = tile_id % row_tiles;
    {
        // Groups of up to 16 adjacent column strips are walked strips-fastest: the row-part pieces
        // a tile writes (64 / 48 / 32 bytes per row) are then completed to whole lines by the
        // neighbouring strips while they are still in L2 (measured: 188 -> 146 us on a
        // 16384 x 8192 FP6 cast), and the column-part pieces still follow each other closely.
        const int64_t col_tiles = n_tiles / row_tiles;
        const int64_t sg = (col_tiles & 15) == 0 ? 16 : (col_tiles & 7) == 0 ? 8 : (col_tiles & 3) == 0 ? 4 : (col_tiles & 1) == 0 ? 2 : 1;
        const int64_t grp = tile_id / (sg * row_tiles), in = tile_id % (sg * row_tiles);
        ct = grp * sg + in % sg;
        rt = in / sg;
    }
    const int64_t c0 = ct * DUAL_C;
    const int64_t r0 = rt * DUAL_R;

    // ---- coalesced loads: 8 lanes per 128-byte row segment, 32 rows per pass
    {
        const int lr = t >> 3, lc = t & 7;
        uint4 v[4];
#pragma unroll
        for (int p = 0; p < 4; p++) v[p] = ld16_nt(src + (r0 + p * 32 + lr) * ld + c0 + lc * 8);
#pragma unroll
        for (int p = 0; p < 4; p++) {
            const int r = p * 32 + lr;
            *reinterpret_cast<uint4 *>(tile + r * 128 + (((lc + r + 2 * p) & 7) << 4)) = v[p];
        }
    }
    __syncthreads();

    const int64_t n_cb = cols / BLOCK, n_rb = rows / BLOCK;
    // ---- row part
    {
        const int r = t >> 1, b = t & 1;
        const uint8_t *rowp = tile + r * 128;
        const int rot = r + 2 * (r >> 5);
        uint32_t d[16];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint4 q = *reinterpret_cast<const uint4 *>(rowp + (((4 * b + i + rot) & 7) << 4));
            d[4 * i] = q.x; d[4 * i + 1] = q.y; d[4 * i + 2] = q.z; d[4 * i + 3] = q.w;
        }
        uint32_t out[w];
        const uint32_t s = quantize_block_bf16<FMT, RND>(d, out);
        const int64_t blk = (r0 + r) * n_cb + c0 / BLOCK + b;
        store_block<w>(e1 + blk * (BLOCK * w / 8), out);
        // the two blocks of a row sit in adjacent lanes: one 16-bit store
        const uint32_t s2 = s | ((uint32_t)__shfl_down((int)s, 1) << 8);
        if (b == 0) *reinterpret_cast<uint16_t *>(s1 + blk) = (uint16_t)s2;
    }
    // ---- column part
    {
        const int c = t >> 2, rb = t & 3;
        uint32_t d[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            // rows rb*32 + 2i and + 2i + 1: chunk c / 8 of the row, rotated like the stores
            const int ra = 2 * i, rbw = 2 * i + 1;
            const uint32_t lo = *reinterpret_cast<const uint16_t *>(tile + (rb * 32 + ra) * 128 + ((((c >> 3) + ra + 2 * rb) & 7) << 4) + (c & 7) * 2);
            const uint32_t hi = *reinterpret_cast<const uint16_t *>(tile + (rb * 32 + rbw) * 128 + ((((c >> 3) + rbw + 2 * rb) & 7) << 4) + (c & 7) * 2);
            d[i] = lo | (hi << 16);
        }
        uint32_t out[w];
        const uint32_t s = quantize_block_bf16<FMT, RND>(d, out);
        const int64_t blk = (c0 + c) * n_rb + r0 / BLOCK + rb;
        store_block<w>(e0 + blk * (BLOCK * w / 8), out);
        const uint32_t s4 = s | ((uint32_t)__shfl_down((int)s, 1) << 8) | ((uint32_t)__shfl_down((int)s, 2) << 16) |
                            ((uint32_t)__shfl_down((int)s, 3) << 24);
        if (rb == 0) *reinterpret_cast<uint32_t *>(s0 + blk) = s4;
    }
}

template <int FMT>
static hipError_t launch_dual_r(int rnd, const uint16_t *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *e1, uint8_t *s1,
                                uint8_t *e0, uint8_t *s0, hipStream_t st)
{
    const int64_t row_tiles = rows / DUAL_R, n_tiles = row_tiles * (cols / DUAL_C), per_xcd = (n_tiles + 7) / 8;
    if (per_xcd * 8 > 0x7FFFFFFF) return hipErrorNotSupported;
    const dim3 grid((unsigned)(per_xcd * 8));
    if (rnd == ROUND_RNE)
        hipLaunchKernelGGL((cast_dual_bf16_kernel<FMT, ROUND_RNE>), grid, dim3(256), 0, st, src, rows, cols, ld, e1, s1, e0, s0,
                           row_tiles, n_tiles, per_xcd);
    else
        hipLaunchKernelGGL((cast_dual_bf16_kernel<FMT, ROUND_HALF_AWAY>), grid, dim3(256), 0, st, src, rows, cols, ld, e1, s1, e0,
                           s0, row_tiles, n_tiles, per_xcd);
    return hipGetLastError();
}

// One pass for both axes when the source is bf16 and made of whole 128 x 64 tiles; two ordinary
// casts otherwise (same bytes either way).
hipError_t launch_cast_dual(const void *src, int src_dt, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd,
                            uint8_t *e1, uint8_t *s1, uint8_t *e0, uint8_t *s0, hipStream_t st)
{
    if (src_dt == DT_BF16 && (rnd == ROUND_RNE || rnd == ROUND_HALF_AWAY) && rows % DUAL_R == 0 && cols % DUAL_C == 0) {
        const uint16_t *p = static_cast<const uint16_t *>(src);
        hipError_t e;
        switch (fmt) {
            case FP8_E4M3: e = launch_dual_r<FP8_E4M3>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
            case FP8_E5M2: e = launch_dual_r<FP8_E5M2>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
            case FP6_E3M2: e = launch_dual_r<FP6_E3M2>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
            case FP6_E2M3: e = launch_dual_r<FP6_E2M3>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
            case FP4_E2M1: e = launch_dual_r<FP4_E2M1>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
            default:       e = launch_dual_r<INT8>(rnd, p, rows, cols, ld, e1, s1, e0, s0, st); break;
        }
        if (e != hipErrorNotSupported) return e;
    }
    hipError_t e = launch_cast(src, src_dt, rows, cols, ld, 1, fmt, rnd, e1, s1, st);
    if (e != hipSuccess) return e;
    return launch_cast(src, src_dt, rows, cols, ld, 0, fmt, rnd, e0, s0, st);
}

}  // namespace mx
