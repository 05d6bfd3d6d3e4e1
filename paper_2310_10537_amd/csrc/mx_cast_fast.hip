// Bandwidth-oriented MX cast kernels for bf16 sources (Algorithm 1, Section 3 of
// arXiv 2310.10537) on gfx950.  Both are pure streaming kernels bound by HBM:
// per element they read 2 bytes and write bits/8 + 1/32 bytes.
//
//   cast_row_bf16_kernel   blocks along the contiguous axis.  A wave takes 2048
//       consecutive elements as four fully coalesced 16-byte-per-lane loads
//       (1 KB per instruction).  8-bit and 4-bit formats convert in place: four
//       adjacent lanes share a block, the block maximum is a packed-u16 max
//       finished with two DPP quad permutes.  FP6 converts 32 elements per
//       instruction, so the wave transposes its 64 blocks through a private LDS
//       region until each lane owns one block.  Scale bytes (and FP6 codes) are
//       staged in LDS so that they leave as 16-byte stores.
//   cast_col_bf16_kernel   blocks along dimension 0, output written as the cast of
//       the transpose.  A work-group stages a [128 rows x 128 (or 64) columns] tile in LDS
//       with coalesced row loads (rows rotated by 32 bytes per 32-row block so
//       that column reads are bank-conflict free); each lane then reads one
//       column of one 32-row block -- the block maximum is in-lane -- and the four
//       lanes of a column write one contiguous 128 / 96 / 64-byte output line.
#include "mx_convert.hpp"
#include "mx_launch.hpp"

namespace mx {

// Lanes of one wave exchange data through LDS without a work-group barrier: LDS
// operations of a wave execute in order, so it is enough to keep the compiler
// from moving accesses across this point and to wait for the wave's own writes.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
}

// ---------------------------------------------------------------------------
// Row cast
// ---------------------------------------------------------------------------
constexpr int ROW_CHUNKS = 4;                 // 16-byte loads in flight per lane (8 measured the same, 16 slower)
constexpr int ROW_WAVE_ELEMS = 64 * 8 * ROW_CHUNKS;   // 2048 elements = 64 blocks per wave

// element offset of linear element index e in a [rows][cols] tensor with pitch ld
template <bool FLAT>
__device__ __forceinline__ int64_t src_offset(int64_t e, int64_t cols, int64_t ld)
{
    if (FLAT) return e;
    int64_t r = e / cols;
    return r * ld + (e - r * cols);
}

template <int FMT, int RND, bool FLAT, bool WHOLE = false, int CH = ROW_CHUNKS>   // WHOLE: every wave's elements lie inside the tensor
__global__ __launch_bounds__(256) void cast_row_bf16_kernel(const uint16_t *__restrict__ src, int64_t cols, int64_t ld,
                                                            uint8_t *__restrict__ elems, uint8_t *__restrict__ scales,
                                                            int64_t n_elems)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    constexpr bool SIX = (w == 6);
    // per wave: FP6 needs 64 blocks x 80 bytes (padded) for the transpose; everyone needs 64 scale bytes
    static_assert(!SIX || CH == 4, "the FP6 transpose gives lane L block L of 64");
    constexpr int LDS_PER_WAVE = SIX ? 64 * 80 : 16 * CH;
    constexpr int WAVE_ELEMS = 512 * CH;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * LDS_PER_WAVE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint8_t *lds = lds_all + wave * LDS_PER_WAVE;

    const int64_t wave_id = (int64_t)blockIdx.x * 4 + wave;
    const int64_t e0 = wave_id * WAVE_ELEMS;          // first element of this wave
    if (!WHOLE && e0 >= n_elems) return;                  // whole wave out of range
    const int64_t blk0 = e0 / BLOCK;                      // first block of this wave

    // ---- coalesced loads: chunk u, lane l -> elements e0 + u*512 + l*8 .. +7
    uint32_t d[CH][4];
    bool valid[CH];
#pragma unroll
    for (int u = 0; u < CH; u++) {
        const int64_t e = e0 + u * 512 + lane * 8;
        valid[u] = WHOLE || e < n_elems;
        uint4 t = make_uint4(0, 0, 0, 0);
        if (valid[u]) t = ld16_nt(src + src_offset<FLAT>(e, cols, ld));
        d[u][0] = t.x; d[u][1] = t.y; d[u][2] = t.z; d[u][3] = t.w;
    }

    if constexpr (!SIX) {
        constexpr int OD = 8 * w / 32;   // output dwords per lane per chunk (2 or 1)
#pragma unroll
        for (int u = 0; u < CH; u++) {
            uint32_t m = 0;
#pragma unroll
            for (int i = 0; i < 4; i++) m = pk_absmax(m, d[u][i]);
            uint32_t amax16 = group_max<4>(pk_hmax(m));
            uint32_t s = scale_from_bf16_max<FMT>(amax16);
            uint32_t out[OD];
            if (fast_ok(amax16, s)) {
                convert_bf16_fast<FMT, RND, 4>(d[u], s, out);
            } else {
                // exact path; the condition is uniform over the four lanes of the block
                uint32_t v[8];
                widen_bf16<4>(d[u], v);
                uint32_t amax = 0;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    uint32_t k = amax_key<FMT>(v[i]);
                    amax = amax > k ? amax : k;
                }
                amax = group_max<4>(amax);
                s = scale_byte<FMT>(amax);
                encode_exact<FMT, RND, 8>(v, s, out);
            }
            if (valid[u]) {
                uint8_t *o = elems + (e0 + u * 512 + lane * 8) * w / 8;
                if constexpr (OD == 2) *reinterpret_cast<uint2 *>(o) = make_uint2(out[0], out[1]);
                else *reinterpret_cast<uint32_t *>(o) = out[0];
            }
            if ((lane & 3) == 0) lds[u * 16 + (lane >> 2)] = (uint8_t)s;   // block u*16 + lane/4 of this wave
        }
    } else {
        // ---- FP6: transpose so that lane L owns block L of the wave (chunk L/16, quad L%16)
#pragma unroll
        for (int u = 0; u < CH; u++) {
            const int b = u * 16 + (lane >> 2);
            *reinterpret_cast<uint4 *>(lds + b * 80 + (lane & 3) * 16) = make_uint4(d[u][0], d[u][1], d[u][2], d[u][3]);
        }
        wave_lds_sync();
        uint32_t blk[16];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint4 t = *reinterpret_cast<const uint4 *>(lds + lane * 80 + j * 16);
            blk[4 * j] = t.x; blk[4 * j + 1] = t.y; blk[4 * j + 2] = t.z; blk[4 * j + 3] = t.w;
        }
        uint32_t out[6];
        const uint32_t s = quantize_block_bf16<FMT, RND>(blk, out);
        wave_lds_sync();
        // codes back through LDS: 64 blocks x 24 bytes = 1536 contiguous bytes, then the scale bytes
        uint32_t *l32 = reinterpret_cast<uint32_t *>(lds);
#pragma unroll
        for (int i = 0; i < 6; i++) l32[lane * 6 + i] = out[i];
        lds[1536 + lane] = (uint8_t)s;
        wave_lds_sync();
        const int64_t n_blk_valid = WHOLE ? 64 : (n_elems - e0) / BLOCK;   // blocks of this wave inside the tensor (>= 1)
        uint8_t *o = elems + blk0 * 24;
        const uint4 a = *reinterpret_cast<const uint4 *>(lds + lane * 16);
        const uint2 c = *reinterpret_cast<const uint2 *>(lds + 1024 + lane * 8);
        if (n_blk_valid >= 64) {
            st16(o + lane * 16, a);
            *reinterpret_cast<uint2 *>(o + 1024 + lane * 8) = c;
        } else {
            const int64_t nbytes = n_blk_valid * 24;           // a multiple of 8
            if (lane * 16 + 16 <= nbytes) st16(o + lane * 16, a);
            else if (lane * 16 + 8 <= nbytes) *reinterpret_cast<uint2 *>(o + lane * 16) = make_uint2(a.x, a.y);
            if (1024 + lane * 8 + 8 <= nbytes) *reinterpret_cast<uint2 *>(o + 1024 + lane * 8) = c;
        }
    }

    // ---- scale bytes: 64 per wave, stored 16 at a time
    wave_lds_sync();
    {
        const uint8_t *sl = SIX ? lds + 1536 : lds;
        const int64_t n_blk_valid = WHOLE ? 16 * CH : (n_elems - e0) / BLOCK;
        if (lane < CH) {
            if ((lane + 1) * 16 <= n_blk_valid) {
                st16(scales + blk0 + lane * 16, *reinterpret_cast<const uint4 *>(sl + lane * 16));
            } else {
                for (int i = lane * 16; i < n_blk_valid && i < lane * 16 + 16; i++) scales[blk0 + i] = sl[i];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Column cast
// ---------------------------------------------------------------------------
constexpr int COL_TILE_R = 128;   // rows of a tile (256 measured slower)
constexpr int COL_TILE_C = 64;    // columns of a tile of the Float32 kernel

// A tile is 128 rows x TC columns, TC = 128 (256-byte row segments, two lines) or 64 for narrow
// tensors.  Work-groups are dealt round-robin to the 8 XCDs, each with its own L2.  Tile
// t = xcd * per_xcd + i, each XCD owning a contiguous run of column strips which it walks down
// the rows: what its work-groups write (128 bytes of codes and 4 scale bytes per column each) is
// consecutive in memory and merges into full lines in that XCD's L2.
// (Measured on the bare access pattern -- loads, LDS tile, stores, no arithmetic -- of an
// 8192 x 8192 tensor: 128 x 64 tiles 38.6 us, 256 x 64 37.2, 128 x 128 35.9, 256 x 128 40.5,
// 64 x 256 37.8; walking several adjacent strips abreast, which paid before the loads became
// non-temporal, now costs 1-2 us.  The kernel runs within 5 % of its pattern.)
template <int FMT, int RND, int TC, bool WHOLE>   // WHOLE: every tile lies inside the tensor (no bounds checks)
__global__ __launch_bounds__(256) void cast_col_bf16_kernel(const uint16_t *__restrict__ src, int64_t rows, int64_t cols,
                                                            int64_t ld, uint8_t *__restrict__ elems,
                                                            uint8_t *__restrict__ scales, int64_t row_tiles,
                                                            int64_t n_tiles, int64_t per_xcd)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    constexpr int PITCH = TC * 2;                        // bytes per tile row in LDS
    __shared__ __attribute__((aligned(16))) uint8_t tile[COL_TILE_R * PITCH];
    __shared__ __attribute__((aligned(16))) uint32_t xch[(w == 6 && WHOLE) ? 256 * 6 : 4];   // FP6 codes on their way out
    const int t = threadIdx.x;
    const int64_t tile_id = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || tile_id >= n_tiles) return;   // uniform over the work-group
    const int64_t ct = tile_id / row_tiles, rt = tile_id % row_tiles;
    const int64_t c0 = ct * TC;
    const int64_t r0 = rt * COL_TILE_R;

    // ---- coalesced loads: TC / 8 lanes per row segment, all in flight before the first LDS write
    constexpr int LPR = TC / 8, RPP = 256 / LPR, NP = COL_TILE_R / RPP;
    const int lr = t / LPR, lc = t % LPR;
    const bool full_cols = WHOLE || c0 + TC <= cols;
    uint4 v[NP];
#pragma unroll
    for (int p = 0; p < NP; p++) {
        const int r = p * RPP + lr;                      // row inside the tile
        v[p] = make_uint4(0, 0, 0, 0);
        if (WHOLE || r0 + r < rows) {
            const uint16_t *g = src + (r0 + r) * ld + c0 + lc * 8;
            if (full_cols || c0 + lc * 8 + 8 <= cols) {
                v[p] = ld16_nt(g);
            } else {
                uint16_t h[8];
#pragma unroll
                for (int i = 0; i < 8; i++) h[i] = (c0 + lc * 8 + i < cols) ? g[i] : (uint16_t)0;
                v[p] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NP; p++) {
        const int r = p * RPP + lr;
        // rotate the row by 32 bytes per row block: column reads of four adjacent blocks then hit different banks
        *reinterpret_cast<uint4 *>(tile + r * PITCH + ((lc * 16 + (r >> 5) * 32) & (PITCH - 1))) = v[p];
    }
    __syncthreads();

    // ---- lane (column c, row block rb): 32 values down the column, packed in pairs
    const int64_t n_rb = rows / BLOCK;
    const bool quad = WHOLE || (n_rb & 3) == 0;          // scale dwords are aligned
#pragma unroll
    for (int q = 0; q < TC / 64; q++) {
        const int c = (t >> 2) + 64 * q;
        const int64_t col = c0 + c;
        const int rb = t & 3;
        const int64_t row_blk = r0 / BLOCK + rb;
        const bool valid = WHOLE || (col < cols && row_blk < n_rb);
        const uint8_t *colp = tile + rb * 32 * PITCH + ((c * 2 + rb * 32) & (PITCH - 1));
        uint32_t d[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            uint32_t lo = *reinterpret_cast<const uint16_t *>(colp + (2 * i) * PITCH);
            uint32_t hi = *reinterpret_cast<const uint16_t *>(colp + (2 * i + 1) * PITCH);
            d[i] = lo | (hi << 16);
        }
        uint32_t out[w];
        const uint32_t s = quantize_block_bf16<FMT, RND>(d, out);
        // the four lanes of a column hold four consecutive scale bytes: one dword store when the
        // whole quad is valid and the address is aligned, else byte stores
        const uint32_t s4 = s | ((uint32_t)__shfl_down((int)s, 1) << 8) | ((uint32_t)__shfl_down((int)s, 2) << 16) |
                            ((uint32_t)__shfl_down((int)s, 3) << 24);
        if (valid) {
            uint8_t *o = elems + (col * n_rb + row_blk) * (BLOCK * w / 8);
            if constexpr (w == 8) {
                // (a transpose inside the quad, so that each of the two stores writes 64 consecutive
                // bytes of the column's 128-byte line instead of every second 16, changed nothing
                // measurable: 44.6 against 45.3 us)
                st16(o, make_uint4(out[0], out[1], out[2], out[3]));
                st16(o + 16, make_uint4(out[4], out[5], out[6], out[7]));
            } else if constexpr (w == 6) {
                if constexpr (WHOLE) {
                    // the four lanes of a column hold 96 consecutive output bytes (16-byte aligned: whole
                    // tiles are four blocks deep); through LDS they leave as six 16-byte stores
                    uint32_t *x = xch + (t & ~3) * 6;
#pragma unroll
                    for (int i = 0; i < 6; i += 2) *reinterpret_cast<uint2 *>(x + (t & 3) * 6 + i) = make_uint2(out[i], out[i + 1]);
                    wave_lds_sync();
                    uint8_t *oq = o - (t & 3) * 24;
                    st16(oq + (t & 3) * 16, *reinterpret_cast<const uint4 *>(x + (t & 3) * 4));
                    if ((t & 3) < 2) st16(oq + 64 + (t & 3) * 16, *reinterpret_cast<const uint4 *>(x + 16 + (t & 3) * 4));
                    if (q + 1 < TC / 64) wave_lds_sync();   // the exchange area is written again
                } else {
                    *reinterpret_cast<uint2 *>(o) = make_uint2(out[0], out[1]);
                    *reinterpret_cast<uint2 *>(o + 8) = make_uint2(out[2], out[3]);
                    *reinterpret_cast<uint2 *>(o + 16) = make_uint2(out[4], out[5]);
                }
            } else {
                st16(o, make_uint4(out[0], out[1], out[2], out[3]));
            }
            if (WHOLE || (quad && r0 / BLOCK + 4 <= n_rb)) {   // uniform over the work-group
                if ((t & 3) == 0) *reinterpret_cast<uint32_t *>(scales + col * n_rb + row_blk) = s4;
            } else {
                scales[col * n_rb + row_blk] = (uint8_t)s;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Column cast of a Float32 source made of whole 128 x 64 tiles (weights are cast from Float32,
// along the reduction axis of their GEMM, i.e. along dimension 0 of a [K][N] tensor).  Same plan
// as the bf16 kernel: coalesced row loads into an LDS tile (here 16 lanes x 16 bytes per 256-byte
// row segment), then lane (column c, row block rb) walks 32 values down its column, and the four
// lanes of a column write its four consecutive blocks.  Row block rb keeps its rows rotated by
// 16 rb columns, so the 64 lanes of a wave (16 columns x 4 row blocks) read 64 different banks.
// The one-lane-per-(block, column) kernel without LDS leaves every output line to eight
// work-groups that run far apart in time: 3.3 TB/s on 8192 x 28672 -> E2M1.
// ---------------------------------------------------------------------------
template <int FMT, int RND>
__global__ __launch_bounds__(256) void cast_col_f32_kernel(const float *__restrict__ src, int64_t rows, int64_t cols, int64_t ld,
                                                           uint8_t *__restrict__ elems, uint8_t *__restrict__ scales,
                                                           int64_t row_tiles, int64_t n_tiles, int64_t per_xcd)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    __shared__ __attribute__((aligned(16))) uint32_t tile[COL_TILE_R * COL_TILE_C];   // 32 KB, rows of 64 floats
    const int t = threadIdx.x;
    const int64_t tile_id = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || tile_id >= n_tiles) return;   // uniform over the work-group
    // strips one at a time, as in the bf16 kernel (several abreast cost 3 % with non-temporal loads)
    const int64_t ct = tile_id / row_tiles, rt = tile_id % row_tiles;
    const int64_t c0 = ct * COL_TILE_C, r0 = rt * COL_TILE_R;
    const int lr = t >> 4, lc = t & 15;
    uint4 v[COL_TILE_R / 16];
#pragma unroll
    for (int p = 0; p < COL_TILE_R / 16; p++) v[p] = ld16_nt(src + (r0 + p * 16 + lr) * ld + c0 + lc * 4);
#pragma unroll
    for (int p = 0; p < COL_TILE_R / 16; p++) {
        const int r = p * 16 + lr;                    // row inside the tile; its 32-row block is r / 32
        *reinterpret_cast<uint4 *>(tile + r * COL_TILE_C + ((lc * 4 + (r >> 5) * 16) & 63)) = v[p];
    }
    __syncthreads();
    const int c = t >> 2, rb = t & 3;
    const int64_t col = c0 + c, n_rb = rows / BLOCK, row_blk = r0 / BLOCK + rb;
    uint32_t out[w];
    const uint32_t s = quantize_block_lds<FMT, RND>(tile + rb * 32 * COL_TILE_C + ((c + rb * 16) & 63), COL_TILE_C, out);
    const uint32_t s4 = s | ((uint32_t)__shfl_down((int)s, 1) << 8) | ((uint32_t)__shfl_down((int)s, 2) << 16) |
                        ((uint32_t)__shfl_down((int)s, 3) << 24);
    uint8_t *o = elems + (col * n_rb + row_blk) * (BLOCK * w / 8);
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
    if (rb == 0) *reinterpret_cast<uint32_t *>(scales + col * n_rb + row_blk) = s4;   // n_rb is a multiple of 4: aligned
}

// ---------------------------------------------------------------------------
// Launchers.  Return hipErrorNotSupported when the fast path does not apply.
// ---------------------------------------------------------------------------
template <int FMT>
static hipError_t launch_col_f32_r(int rnd, const float *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *elems,
                                   uint8_t *scales, hipStream_t st)
{
    const int64_t row_tiles = rows / COL_TILE_R, n_tiles = row_tiles * (cols / COL_TILE_C), per_xcd = (n_tiles + 7) / 8;
    if (per_xcd * 8 > 0x7FFFFFFF) return hipErrorNotSupported;
    if (rnd == ROUND_RNE)
        hipLaunchKernelGGL((cast_col_f32_kernel<FMT, ROUND_RNE>), dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, src, rows, cols,
                           ld, elems, scales, row_tiles, n_tiles, per_xcd);
    else
        hipLaunchKernelGGL((cast_col_f32_kernel<FMT, ROUND_HALF_AWAY>), dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, src, rows,
                           cols, ld, elems, scales, row_tiles, n_tiles, per_xcd);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Row cast of a dense Float32 tensor (blocks along the contiguous axis; configs that cast Float32
// sources along rows: the round trip of a Float32 tensor, weights kept in Float32).  A wave takes
// 2048 consecutive elements = 64 blocks as eight fully coalesced 16-byte-per-lane loads (all in flight
// at once), parks them in a wave-private LDS region with a pitch of 36 dwords per block -- lane l then
// owns block l and reads it back with 16-byte reads that are free of bank conflicts (36 l mod 64 takes
// 16 different multiples of 4 over any 16 consecutive lanes) -- and quantizes it with the Float32
// block quantizer of the column kernel and the GEMM epilogue (hardware converts; the exact encoder
// for the rare blocks they cannot take).  No work-group barrier: waves are independent.
// ---------------------------------------------------------------------------
constexpr int RF_CHUNKS = 8;                       // 16-byte loads in flight per lane
constexpr int RF_WAVE_ELEMS = 64 * 4 * RF_CHUNKS;  // 2048 elements = 64 blocks per wave
constexpr int RF_PITCH = 36;                       // dwords per block in LDS

template <int FMT, int RND>
__global__ __launch_bounds__(256) void cast_row_f32_kernel(const float *__restrict__ src, uint8_t *__restrict__ elems,
                                                           uint8_t *__restrict__ scales, int64_t n_waves)
{
    if constexpr (FMT == FP8_E4M3 || FMT == FP8_E5M2) fp8_saturate_mode();
    constexpr int w = Fmt<FMT>::bits;
    __shared__ __attribute__((aligned(16))) uint32_t lds_all[4 * 64 * RF_PITCH];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t *lds = lds_all + wave * 64 * RF_PITCH;
    const int64_t wave_id = (int64_t)blockIdx.x * 4 + wave;
    if (wave_id >= n_waves) return;
    const int64_t e0 = wave_id * RF_WAVE_ELEMS, blk0 = e0 / BLOCK;

    uint4 v[RF_CHUNKS];
#pragma unroll
    for (int u = 0; u < RF_CHUNKS; u++) v[u] = ld16_nt(src + e0 + u * 256 + lane * 4);
#pragma unroll
    for (int u = 0; u < RF_CHUNKS; u++) {
        const int f = u * 256 + lane * 4;              // element of the wave's run: block f / 32, position f % 32
        *reinterpret_cast<uint4 *>(lds + (f >> 5) * RF_PITCH + (f & 31)) = v[u];
    }
    wave_lds_sync();
    uint32_t out[w];
    const uint32_t s = quantize_block_lds<FMT, RND>(lds + lane * RF_PITCH, 1, out);
    uint8_t *o = elems + (blk0 + lane) * (BLOCK * w / 8);
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
    scales[blk0 + lane] = (uint8_t)s;                  // 64 consecutive bytes per wave
}

template <int FMT>
static hipError_t launch_row_f32_r(int rnd, const float *src, int64_t n, uint8_t *elems, uint8_t *scales, hipStream_t st)
{
    const int64_t n_waves = n / RF_WAVE_ELEMS, nb = (n_waves + 3) / 4;
    if (nb > 0x7FFFFFFF) return hipErrorNotSupported;
    if (rnd == ROUND_RNE)
        hipLaunchKernelGGL((cast_row_f32_kernel<FMT, ROUND_RNE>), dim3((unsigned)nb), dim3(256), 0, st, src, elems, scales, n_waves);
    else
        hipLaunchKernelGGL((cast_row_f32_kernel<FMT, ROUND_HALF_AWAY>), dim3((unsigned)nb), dim3(256), 0, st, src, elems, scales, n_waves);
    return hipGetLastError();
}

// Float32 source, blocks along the last axis, dense rows of whole blocks and a whole number of
// 2048-element runs, round to nearest; hipErrorNotSupported otherwise
hipError_t launch_cast_row_f32_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd, uint8_t *elems,
                                    uint8_t *scales, hipStream_t st)
{
    const int64_t n = rows * cols;
    if (ld != cols || cols % BLOCK || n == 0 || n % RF_WAVE_ELEMS || (rnd != ROUND_RNE && rnd != ROUND_HALF_AWAY))
        return hipErrorNotSupported;
    const float *p = static_cast<const float *>(src);
    switch (fmt) {
        case FP8_E4M3: return launch_row_f32_r<FP8_E4M3>(rnd, p, n, elems, scales, st);
        case FP8_E5M2: return launch_row_f32_r<FP8_E5M2>(rnd, p, n, elems, scales, st);
        case FP6_E3M2: return launch_row_f32_r<FP6_E3M2>(rnd, p, n, elems, scales, st);
        case FP6_E2M3: return launch_row_f32_r<FP6_E2M3>(rnd, p, n, elems, scales, st);
        case FP4_E2M1: return launch_row_f32_r<FP4_E2M1>(rnd, p, n, elems, scales, st);
        default:       return launch_row_f32_r<INT8>(rnd, p, n, elems, scales, st);
    }
}

// Float32 source, blocks along dimension 0, whole 128 x 64 tiles, round to nearest
hipError_t launch_cast_col_f32_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd, uint8_t *elems,
                                    uint8_t *scales, hipStream_t st)
{
    if (rows % COL_TILE_R || cols % COL_TILE_C || rows == 0 || cols == 0 || (rnd != ROUND_RNE && rnd != ROUND_HALF_AWAY))
        return hipErrorNotSupported;
    const float *p = static_cast<const float *>(src);
    switch (fmt) {
        case FP8_E4M3: return launch_col_f32_r<FP8_E4M3>(rnd, p, rows, cols, ld, elems, scales, st);
        case FP8_E5M2: return launch_col_f32_r<FP8_E5M2>(rnd, p, rows, cols, ld, elems, scales, st);
        case FP6_E3M2: return launch_col_f32_r<FP6_E3M2>(rnd, p, rows, cols, ld, elems, scales, st);
        case FP6_E2M3: return launch_col_f32_r<FP6_E2M3>(rnd, p, rows, cols, ld, elems, scales, st);
        case FP4_E2M1: return launch_col_f32_r<FP4_E2M1>(rnd, p, rows, cols, ld, elems, scales, st);
        default:       return launch_col_f32_r<INT8>(rnd, p, rows, cols, ld, elems, scales, st);
    }
}

template <int FMT, int RND>
static hipError_t launch_fast_t(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *elems,
                                uint8_t *scales, hipStream_t st)
{
    const uint16_t *s16 = static_cast<const uint16_t *>(src);
    if (axis == 1) {
        const int64_t n = rows * cols;
        const int64_t waves = (n + ROW_WAVE_ELEMS - 1) / ROW_WAVE_ELEMS;
        const int64_t nb = (waves + 3) / 4;
        if (nb > 0x7FFFFFFF) return hipErrorNotSupported;
        if (ld == cols && n % (4 * ROW_WAVE_ELEMS) == 0)
            hipLaunchKernelGGL((cast_row_bf16_kernel<FMT, RND, true, true>), dim3((unsigned)nb), dim3(256), 0, st, s16, cols, ld,
                               elems, scales, n);
        else if (ld == cols)
            hipLaunchKernelGGL((cast_row_bf16_kernel<FMT, RND, true>), dim3((unsigned)nb), dim3(256), 0, st, s16, cols, ld,
                               elems, scales, n);
        else
            hipLaunchKernelGGL((cast_row_bf16_kernel<FMT, RND, false>), dim3((unsigned)nb), dim3(256), 0, st, s16, cols, ld,
                               elems, scales, n);
        return hipGetLastError();
    }
    const int64_t row_tiles = (rows + COL_TILE_R - 1) / COL_TILE_R;
    // 128-column tiles once they still give every compute unit several work-groups
    const bool wide = row_tiles * ((cols + 127) / 128) >= 1024;
    const int64_t n_tiles = row_tiles * (wide ? (cols + 127) / 128 : (cols + 63) / 64);
    const int64_t per_xcd = (n_tiles + 7) / 8;
    if (per_xcd * 8 > 0x7FFFFFFF) return hipErrorNotSupported;
    const bool whole = rows % COL_TILE_R == 0 && cols % (wide ? 128 : 64) == 0;
#define MX_COL_GO(TC_, WHOLE_)                                                                                               \
    hipLaunchKernelGGL((cast_col_bf16_kernel<FMT, RND, TC_, WHOLE_>), dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, s16, rows, cols, \
                       ld, elems, scales, row_tiles, n_tiles, per_xcd)
    if (wide) { if (whole) MX_COL_GO(128, true); else MX_COL_GO(128, false); }
    else      { if (whole) MX_COL_GO(64, true); else MX_COL_GO(64, false); }
#undef MX_COL_GO
    return hipGetLastError();
}

template <int FMT>
static hipError_t launch_fast_r(int rnd, const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, uint8_t *elems,
                                uint8_t *scales, hipStream_t st)
{
    return rnd == ROUND_RNE ? launch_fast_t<FMT, ROUND_RNE>(src, rows, cols, ld, axis, elems, scales, st)
                            : launch_fast_t<FMT, ROUND_HALF_AWAY>(src, rows, cols, ld, axis, elems, scales, st);
}

hipError_t launch_cast_bf16_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, int fmt, int rnd,
                                 uint8_t *elems, uint8_t *scales, hipStream_t st)
{
    if ((axis == 1 ? cols : rows) % BLOCK) return hipErrorNotSupported;   // whole blocks only
    switch (fmt) {
        case FP8_E4M3: return launch_fast_r<FP8_E4M3>(rnd, src, rows, cols, ld, axis, elems, scales, st);
        case FP8_E5M2: return launch_fast_r<FP8_E5M2>(rnd, src, rows, cols, ld, axis, elems, scales, st);
        case FP6_E3M2: return launch_fast_r<FP6_E3M2>(rnd, src, rows, cols, ld, axis, elems, scales, st);
        case FP6_E2M3: return launch_fast_r<FP6_E2M3>(rnd, src, rows, cols, ld, axis, elems, scales, st);
        case FP4_E2M1: return launch_fast_r<FP4_E2M1>(rnd, src, rows, cols, ld, axis, elems, scales, st);
        default:       return launch_fast_r<INT8>(rnd, src, rows, cols, ld, axis, elems, scales, st);
    }
}

}  // namespace mx
