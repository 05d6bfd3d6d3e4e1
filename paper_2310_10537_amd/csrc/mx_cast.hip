// MX cast kernels (Algorithm 1, Section 3 of arXiv 2310.10537) for gfx950.
//
//   cast_row_kernel  blocks of 32 along the contiguous axis.  A lane owns EPL
//                    consecutive elements (8, 16 or 32), 32/EPL adjacent lanes
//                    share a block; the block maximum is an integer max over
//                    the magnitude bits combined across lanes with DPP.
//   cast_col_kernel  blocks of 32 along dimension 0, output stored as the cast
//                    of the transpose.  A work-group stages a [128 x 64] tile
//                    in LDS with coalesced row loads; each lane then walks one
//                    column of one 32-row block, so the maximum is in-lane, and
//                    four adjacent lanes write one contiguous output line.
#include "mx_cast_generic.hpp"
#include "mx_launch.hpp"

namespace mx {

// ---------------------------------------------------------------------------
// Row cast.  unit = one lane-iteration = EPL elements; units are numbered in
// row-major order over the tensor with its rows filled up to whole blocks
// (pcols columns), so unit u belongs to block u / G.  Elements at or beyond
// cols read as zero.
// ---------------------------------------------------------------------------
template <int SRC, int FMT, int RND, int EPL>
__global__ __launch_bounds__(256) void cast_row_kernel(const void *__restrict__ src, int64_t cols, int64_t pcols, int64_t ld,
                                                       uint8_t *__restrict__ elems, uint8_t *__restrict__ scales,
                                                       int64_t n_units, uint64_t seed)
{
    constexpr int G = BLOCK / EPL;
    constexpr int w = Fmt<FMT>::bits;
    constexpr int esz = SRC == DT_BF16 ? 2 : 4;
    constexpr int ND = EPL * w / 32;
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t units_per_row = pcols / EPL;
    const bool flat = (ld == cols && cols == pcols);

    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < n_units; u += stride) {
        int64_t off;     // element offset of this lane's first element in the source
        int64_t e0;      // its number in the tensor, row * cols + col
        int n_valid = EPL;
        if (flat) {
            off = e0 = u * EPL;
        } else {
            const int64_t r = u / units_per_row, c0 = (u - r * units_per_row) * EPL;
            off = r * ld + c0;
            e0 = r * cols + c0;
            n_valid = cols - c0 >= EPL ? EPL : cols - c0 > 0 ? (int)(cols - c0) : 0;
        }
        uint32_t rr[EPL] = {};
        if (RND == ROUND_STOCHASTIC) {
            if ((cols & 3) == 0) {
                sr_offsets_run<EPL>(seed, e0, rr);      // e0 is a multiple of 4: one generator call per 4 elements
            } else {
#pragma unroll
                for (int i = 0; i < EPL; i++) rr[i] = sr_offset(seed, e0 + i);
            }
        }
        uint32_t v[EPL];
        if (n_valid == EPL) load_as_f32_bits<SRC, EPL>(reinterpret_cast<const char *>(src) + off * esz, v);
        else load_head_as_f32_bits<SRC, EPL>(reinterpret_cast<const char *>(src) + off * esz, n_valid, v);

        uint32_t amax = 0;
#pragma unroll
        for (int i = 0; i < EPL; i++) {
            uint32_t k = amax_key<FMT>(v[i]);
            amax = amax > k ? amax : k;
        }
        amax = group_max<G>(amax);
        const uint32_t s = scale_byte<FMT>(amax);

        uint32_t packed[ND];
        encode_lane<FMT, RND, EPL>(v, s, rr, packed);
        store_dwords<ND>(elems + u * (EPL * w / 8), packed);
        if (G == 1 || (threadIdx.x & (G - 1)) == 0) scales[u / G] = (uint8_t)s;
    }
}

// ---------------------------------------------------------------------------
// Column cast (blocks along dimension 0), simple form: one lane per
// (32-row block, column), adjacent lanes take adjacent columns so that every
// load instruction of a wave reads one contiguous run of a source row.
// ---------------------------------------------------------------------------
template <int SRC, int FMT, int RND>
__global__ __launch_bounds__(256) void cast_col_simple_kernel(const void *__restrict__ src, int64_t rows, int64_t cols,
                                                              int64_t ld, uint8_t *__restrict__ elems,
                                                              uint8_t *__restrict__ scales, uint64_t seed)
{
    constexpr int w = Fmt<FMT>::bits;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rb = blockIdx.y;
    if (c >= cols) return;
    uint32_t rr[BLOCK] = {};
    if (RND == ROUND_STOCHASTIC) {
        if ((cols & 3) == 0) {
            // The four lanes of a quad hold columns 4j .. 4j+3, i.e. the four words of one generator
            // call per row (cols is a multiple of 4, so a quad is never cut by the c >= cols exit):
            // lane l of the quad runs the generator for rows l, l+4, ... and the quad swaps the words.
            const int ql = threadIdx.x & 3;
            Philox4 p[BLOCK / 4];
#pragma unroll
            for (int k = 0; k < BLOCK / 4; k++)
                p[k] = philox4x32_10(seed, (uint64_t)(((rb * BLOCK + 4 * k + ql) * cols + (c & ~(int64_t)3)) >> 2));
#pragma unroll
            for (int i = 0; i < BLOCK; i++) {
                uint32_t b[4];
#pragma unroll
                for (int m = 0; m < 4; m++) {
                    const int src = (int)p[i >> 2].w[m];
                    // quad_perm with all four selectors equal: every lane reads quad lane i % 4
                    b[m] = (uint32_t)((i & 3) == 0   ? __builtin_amdgcn_update_dpp(0, src, 0x00, 0xF, 0xF, false)
                                      : (i & 3) == 1 ? __builtin_amdgcn_update_dpp(0, src, 0x55, 0xF, 0xF, false)
                                      : (i & 3) == 2 ? __builtin_amdgcn_update_dpp(0, src, 0xAA, 0xF, 0xF, false)
                                                     : __builtin_amdgcn_update_dpp(0, src, 0xFF, 0xF, 0xF, false));
                }
                rr[i] = (ql == 0 ? b[0] : ql == 1 ? b[1] : ql == 2 ? b[2] : b[3]) >> 7;
            }
        } else {
#pragma unroll
            for (int i = 0; i < BLOCK; i++) rr[i] = sr_offset(seed, (rb * BLOCK + i) * cols + c);
        }
    }
    uint32_t v[BLOCK];
#pragma unroll
    for (int i = 0; i < BLOCK; i++) {
        const int64_t row = rb * BLOCK + i, idx = row * ld + c;
        uint32_t x = 0;                                   // rows beyond the tensor: the fill of a partial last block
        if (row < rows) x = SRC == DT_BF16 ? (uint32_t)reinterpret_cast<const uint16_t *>(src)[idx] << 16 : reinterpret_cast<const uint32_t *>(src)[idx];
        v[i] = x;
    }
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < BLOCK; i++) {
        uint32_t k = amax_key<FMT>(v[i]);
        amax = amax > k ? amax : k;
    }
    const uint32_t s = scale_byte<FMT>(amax);
    uint32_t packed[w];
    encode_lane<FMT, RND, BLOCK>(v, s, rr, packed);
    const int64_t nrb = (rows + BLOCK - 1) / BLOCK;
    store_dwords<w>(elems + (c * nrb + rb) * (BLOCK * w / 8), packed);
    scales[c * nrb + rb] = (uint8_t)s;
}

// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------
template <int SRC, int FMT, int RND>
static hipError_t launch_row(const void *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *elems, uint8_t *scales,
                             uint64_t seed, hipStream_t st)
{
    // FP6 needs at least 16 elements per lane to store whole dwords
    constexpr int EPL = (Fmt<FMT>::bits == 6) ? 16 : 8;
    const int64_t pcols = (cols + BLOCK - 1) / BLOCK * BLOCK;
    const int64_t n_units = rows * pcols / EPL;
    int64_t nb = (n_units + 255) / 256;
    const int64_t cap = 256 * 32;   // enough work-groups to fill 256 CUs several times over
    if (nb > cap) nb = cap;
    hipLaunchKernelGGL((cast_row_kernel<SRC, FMT, RND, EPL>), dim3((unsigned)nb), dim3(256), 0, st, src, cols, pcols, ld,
                       elems, scales, n_units, seed);
    return hipGetLastError();
}

template <int SRC, int FMT, int RND>
static hipError_t launch_col(const void *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *elems, uint8_t *scales,
                             uint64_t seed, hipStream_t st)
{
    dim3 grid((unsigned)((cols + 255) / 256), (unsigned)((rows + BLOCK - 1) / BLOCK));
    hipLaunchKernelGGL((cast_col_simple_kernel<SRC, FMT, RND>), grid, dim3(256), 0, st, src, rows, cols, ld, elems, scales,
                       seed);
    return hipGetLastError();
}

template <int SRC, int FMT>
static hipError_t dispatch_rnd(int rnd, uint64_t seed, int axis, const void *src, int64_t rows, int64_t cols, int64_t ld,
                               uint8_t *elems, uint8_t *scales, hipStream_t st)
{
    if (axis == 1) {
        switch (rnd) {
            case ROUND_RNE:         return launch_row<SRC, FMT, ROUND_RNE>(src, rows, cols, ld, elems, scales, seed, st);
            case ROUND_HALF_AWAY:   return launch_row<SRC, FMT, ROUND_HALF_AWAY>(src, rows, cols, ld, elems, scales, seed, st);
            case ROUND_TOWARD_ZERO: return launch_row<SRC, FMT, ROUND_TOWARD_ZERO>(src, rows, cols, ld, elems, scales, seed, st);
            default:                return launch_row<SRC, FMT, ROUND_STOCHASTIC>(src, rows, cols, ld, elems, scales, seed, st);
        }
    }
    switch (rnd) {
        case ROUND_RNE:         return launch_col<SRC, FMT, ROUND_RNE>(src, rows, cols, ld, elems, scales, seed, st);
        case ROUND_HALF_AWAY:   return launch_col<SRC, FMT, ROUND_HALF_AWAY>(src, rows, cols, ld, elems, scales, seed, st);
        case ROUND_TOWARD_ZERO: return launch_col<SRC, FMT, ROUND_TOWARD_ZERO>(src, rows, cols, ld, elems, scales, seed, st);
        default:                return launch_col<SRC, FMT, ROUND_STOCHASTIC>(src, rows, cols, ld, elems, scales, seed, st);
    }
}

template <int SRC>
static hipError_t dispatch_fmt(int fmt, int rnd, uint64_t seed, int axis, const void *src, int64_t rows, int64_t cols,
                               int64_t ld, uint8_t *elems, uint8_t *scales, hipStream_t st)
{
    switch (fmt) {
        case FP8_E4M3: return dispatch_rnd<SRC, FP8_E4M3>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
        case FP8_E5M2: return dispatch_rnd<SRC, FP8_E5M2>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
        case FP6_E3M2: return dispatch_rnd<SRC, FP6_E3M2>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
        case FP6_E2M3: return dispatch_rnd<SRC, FP6_E2M3>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
        case FP4_E2M1: return dispatch_rnd<SRC, FP4_E2M1>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
        default:       return dispatch_rnd<SRC, INT8>(rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
    }
}

hipError_t launch_cast(const void *src, int src_dt, int64_t rows, int64_t cols, int64_t ld, int axis, int fmt, int rnd,
                       uint8_t *elems, uint8_t *scales, hipStream_t st, uint64_t seed)
{
    // The fast kernels store scale bytes 4 and 16 at a time; a scale array that starts at an odd
    // address (a slice of a larger output, see launch_cast_3d) takes the generic kernels, which
    // store them one by one.
    const bool scales_aligned = (reinterpret_cast<uintptr_t>(scales) & 15u) == 0;
    // the kernels built on the hardware converts round to nearest only
    if (scales_aligned && src_dt == DT_BF16 && (rnd == ROUND_RNE || rnd == ROUND_HALF_AWAY)) {
        hipError_t e = launch_cast_bf16_fast(src, rows, cols, ld, axis, fmt, rnd, elems, scales, st);
        if (e != hipErrorNotSupported) return e;
    }
    if (scales_aligned && src_dt == DT_F32) {
        hipError_t e = axis == 0 ? launch_cast_col_f32_fast(src, rows, cols, ld, fmt, rnd, elems, scales, st)
                                 : launch_cast_row_f32_fast(src, rows, cols, ld, fmt, rnd, elems, scales, st);
        if (e != hipErrorNotSupported) return e;
    }
    return src_dt == DT_BF16 ? dispatch_fmt<DT_BF16>(fmt, rnd, seed, axis, src, rows, cols, ld, elems, scales, st)
                             : dispatch_fmt<DT_F32>(fmt, rnd, seed, axis, src, rows, cols, ld, elems, scales, st);
}

}  // namespace mx
