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
#ifndef DUAL_SG128
#define DUAL_SG128 8
#endif

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

// rows a multiple of 128, cols a multiple of TC = 64 or 128 (whole tiles only).  With 128-column tiles a
// row holds 16 chunks and the same rotation works modulo 16; the row part then writes whole lines (four
// blocks per row, two per thread), the column part two columns per thread.
template <int FMT, int RND, int TC>
__global__ __launch_bounds__(256) void cast_dual_bf16_kernel(const uint16_t *__restrict__ src, int64_t rows, int64_t cols,
                                                             int64_t ld, uint8_t *__restrict__ e1, uint8_t *__restrict__ s1,
                                                             uint8_t *__restrict__ e0, uint8_t *__restrict__ s0,
                                                             int64_t row_tiles, int64_t n_tiles, int64_t per_xcd, int64_t sg)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    constexpr int PITCH = TC * 2, NCH = TC / 8;          // bytes and 16-byte chunks per tile row
    __shared__ __attribute__((aligned(16))) uint8_t tile[DUAL_R * PITCH];
    __shared__ __attribute__((aligned(16))) uint32_t xch[w == 6 ? 256 * 6 : 4];   // FP6 column codes on their way out
    const int t = threadIdx.x;
    // XCD-first tile order: each XCD owns a contiguous run of tiles
    const int64_t tile_id = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || tile_id >= n_tiles) return;   // uniform over the work-group
    // Groups of sg adjacent column strips are walked strips-fastest: the row-part pieces a 64-column
    // tile writes (64 / 48 / 32 bytes per row) are then completed to whole lines by the
    // neighbouring strips while they are still in L2 (measured: 188 -> 146 us on a
    // 16384 x 8192 FP6 cast), and the column-part pieces still follow each other closely.
    const int64_t grp = tile_id / (sg * row_tiles), in = tile_id % (sg * row_tiles);
    const int64_t ct = grp * sg + in % sg, rt = in / sg;
    const int64_t c0 = ct * TC;
    const int64_t r0 = rt * DUAL_R;

    // ---- coalesced loads: NCH lanes per row segment, all in flight before the first LDS write
    {
        constexpr int RPP = 256 / NCH, NP = DUAL_R / RPP;
        const int lr = t / NCH, lc = t % NCH;
        uint4 v[NP];
#pragma unroll
        for (int p = 0; p < NP; p++) v[p] = ld16_nt(src + (r0 + p * RPP + lr) * ld + c0 + lc * 8);
#pragma unroll
        for (int p = 0; p < NP; p++) {
            const int r = p * RPP + lr;
            *reinterpret_cast<uint4 *>(tile + r * PITCH + (((lc + r + 2 * (r >> 5)) & (NCH - 1)) << 4)) = v[p];
        }
    }
    __syncthreads();

    const int64_t n_cb = cols / BLOCK, n_rb = rows / BLOCK;
    // ---- row part: thread t takes row t / 2 and half t % 2 of its columns (one or two blocks)
    {
        constexpr int NBR = TC / 64;
        const int r = t >> 1, b = t & 1;
        const uint8_t *rowp = tile + r * PITCH;
        const int rot = r + 2 * (r >> 5);
        uint32_t sc = 0;
        uint32_t o6[12];
#pragma unroll
        for (int j = 0; j < NBR; j++) {
            const int bb = b * NBR + j;
            uint32_t d[16];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint4 q = *reinterpret_cast<const uint4 *>(rowp + (((4 * bb + i + rot) & (NCH - 1)) << 4));
                d[4 * i] = q.x; d[4 * i + 1] = q.y; d[4 * i + 2] = q.z; d[4 * i + 3] = q.w;
            }
            uint32_t out[w];
            const uint32_t s = quantize_block_bf16<FMT, RND>(d, out);
            const int64_t blk = (r0 + r) * n_cb + c0 / BLOCK + bb;
            if constexpr (w == 6 && NBR == 2) {
                // a thread's two FP6 blocks are 48 consecutive, 16-byte aligned bytes: three 16-byte stores
#pragma unroll
                for (int i = 0; i < 6; i++) o6[6 * j + i] = out[i];
                if (j == 1) {
                    uint8_t *o = e1 + (blk - 1) * 24;
                    st16(o, make_uint4(o6[0], o6[1], o6[2], o6[3]));
                    st16(o + 16, make_uint4(o6[4], o6[5], o6[6], o6[7]));
                    st16(o + 32, make_uint4(o6[8], o6[9], o6[10], o6[11]));
                }
            } else {
                store_block<w>(e1 + blk * (BLOCK * w / 8), out);
            }
            sc |= s << (8 * j);
        }
        // the blocks of a row sit in two adjacent lanes: one 16- or 32-bit store
        const int64_t blk0 = (r0 + r) * n_cb + c0 / BLOCK;
        const uint32_t sall = sc | ((uint32_t)__shfl_down((int)sc, 1) << (8 * NBR));
        if (b == 0) {
            if constexpr (NBR == 1) *reinterpret_cast<uint16_t *>(s1 + blk0) = (uint16_t)sall;
            else *reinterpret_cast<uint32_t *>(s1 + blk0) = sall;
        }
    }
    // ---- column part: thread t takes row block t % 4 of column t / 4 (and of column t / 4 + 64)
#pragma unroll
    for (int q = 0; q < TC / 64; q++) {
        const int c = (t >> 2) + 64 * q, rb = t & 3;
        uint32_t d[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            // rows rb*32 + 2i and + 2i + 1: chunk c / 8 of the row, rotated like the stores
            const int ra = 2 * i, rbw = 2 * i + 1;
            const uint32_t lo = *reinterpret_cast<const uint16_t *>(tile + (rb * 32 + ra) * PITCH + ((((c >> 3) + ra + 2 * rb) & (NCH - 1)) << 4) + (c & 7) * 2);
            const uint32_t hi = *reinterpret_cast<const uint16_t *>(tile + (rb * 32 + rbw) * PITCH + ((((c >> 3) + rbw + 2 * rb) & (NCH - 1)) << 4) + (c & 7) * 2);
            d[i] = lo | (hi << 16);
        }
        uint32_t out[w];
        const uint32_t s = quantize_block_bf16<FMT, RND>(d, out);
        const int64_t blk = (c0 + c) * n_rb + r0 / BLOCK + rb;
        if constexpr (w == 6) {
            // the four lanes of a column hold 96 consecutive, 16-byte aligned output bytes; through LDS
            // (a wave-private exchange: lanes of a quad are in one wave) they leave as six 16-byte stores
            uint32_t *x = xch + (t & ~3) * 6;
#pragma unroll
            for (int i = 0; i < 6; i += 2) *reinterpret_cast<uint2 *>(x + rb * 6 + i) = make_uint2(out[i], out[i + 1]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            uint8_t *oq = e0 + (blk - rb) * 24;
            st16(oq + rb * 16, *reinterpret_cast<const uint4 *>(x + rb * 4));
            if (rb < 2) st16(oq + 64 + rb * 16, *reinterpret_cast<const uint4 *>(x + 16 + rb * 4));
            if (q + 1 < TC / 64) {
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        } else {
            store_block<w>(e0 + blk * (BLOCK * w / 8), out);
        }
        const uint32_t s4 = s | ((uint32_t)__shfl_down((int)s, 1) << 8) | ((uint32_t)__shfl_down((int)s, 2) << 16) |
                            ((uint32_t)__shfl_down((int)s, 3) << 24);
        if (rb == 0) *reinterpret_cast<uint32_t *>(s0 + blk) = s4;
    }
}

template <int FMT, int RND, int TC>
static hipError_t launch_dual_t(const uint16_t *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *e1, uint8_t *s1,
                                uint8_t *e0, uint8_t *s0, hipStream_t st, int64_t sg_max)
{
    const int64_t row_tiles = rows / DUAL_R, col_tiles = cols / TC, n_tiles = row_tiles * col_tiles, per_xcd = (n_tiles + 7) / 8;
    if (per_xcd * 8 > 0x7FFFFFFF) return hipErrorNotSupported;
    int64_t sg = sg_max;                                   // the largest power of two up to sg_max that divides the strips
    while (sg > 1 && col_tiles % sg) sg >>= 1;
    hipLaunchKernelGGL((cast_dual_bf16_kernel<FMT, RND, TC>), dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, src, rows, cols, ld, e1,
                       s1, e0, s0, row_tiles, n_tiles, per_xcd, sg);
    return hipGetLastError();
}

template <int FMT>
static hipError_t launch_dual_r(int rnd, const uint16_t *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *e1, uint8_t *s1,
                                uint8_t *e0, uint8_t *s0, hipStream_t st)
{
    // 128-column tiles once they still give every compute unit several work-groups
    const bool wide = cols % 128 == 0 && (rows / DUAL_R) * (cols / 128) >= 1024;
    if (wide)
        return rnd == ROUND_RNE ? launch_dual_t<FMT, ROUND_RNE, 128>(src, rows, cols, ld, e1, s1, e0, s0, st, DUAL_SG128)
                                : launch_dual_t<FMT, ROUND_HALF_AWAY, 128>(src, rows, cols, ld, e1, s1, e0, s0, st, DUAL_SG128);
    return rnd == ROUND_RNE ? launch_dual_t<FMT, ROUND_RNE, 64>(src, rows, cols, ld, e1, s1, e0, s0, st, 16)
                            : launch_dual_t<FMT, ROUND_HALF_AWAY, 64>(src, rows, cols, ld, e1, s1, e0, s0, st, 16);
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
