// Algorithm 1 along any axis of a strided 3-D tensor (Section 3 of arXiv 2310.10537: the
// "principal axis" of a multi-dimensional tensor), in two output layouts.
//   block-major   the block axis is moved last (the 2-D cast of the permuted tensor): served by
//                 the 2-D cast kernels, one launch per slice where the strides do not let one
//                 launch cover everything;
//   source order  codes stay where their elements are, packed along the last axis, and the scale
//                 array is the source shape with the block axis replaced by its block count:
//                 cast_keep_kernel below (blocks along the last axis are the same in both layouts).
#include "mx_cast_generic.hpp"
#include "mx_launch.hpp"

namespace mx {

// Blocks run down the rows of a [rows][cols] slice with row pitch ld (elements); a lane owns 16
// adjacent columns of one 32-row block: a first pass over the 32 rows finds the 16 block maxima,
// a second pass (the rows are still in cache) encodes row by row and writes 16 codes -- 16, 12 or
// 8 bytes -- at the element's own place.  blockIdx.z walks a batch of slices.
constexpr int KEEP_G = 16;

template <int SRC, int FMT, int RND>
__global__ __launch_bounds__(256) void cast_keep_kernel(const void *__restrict__ src, int64_t rows, int64_t cols, int64_t ld,
                                                        int64_t src_bs, uint8_t *__restrict__ elems, int64_t out_rp,
                                                        int64_t out_bs, uint8_t *__restrict__ scales, int64_t sc_rp, int64_t sc_bs)
{
    constexpr int w = Fmt<FMT>::bits;
    constexpr int esz = SRC == DT_BF16 ? 2 : 4;
    constexpr int ND = KEEP_G * w / 32;
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * KEEP_G;
    if (c0 >= cols) return;
    const int64_t rb = blockIdx.y, z = blockIdx.z;
    const int n = cols - c0 >= KEEP_G ? KEEP_G : (int)(cols - c0);
    const char *base = reinterpret_cast<const char *>(src) + (z * src_bs + c0) * esz;

    uint32_t amax[KEEP_G];
#pragma unroll
    for (int i = 0; i < KEEP_G; i++) amax[i] = 0;
#pragma unroll 4
    for (int r = 0; r < BLOCK; r++) {
        const int64_t row = rb * BLOCK + r;
        if (row >= rows) break;
        uint32_t v[KEEP_G];
        if (n == KEEP_G) load_as_f32_bits<SRC, KEEP_G>(base + row * ld * esz, v);
        else load_head_as_f32_bits<SRC, KEEP_G>(base + row * ld * esz, n, v);
#pragma unroll
        for (int i = 0; i < KEEP_G; i++) {
            const uint32_t k = amax_key<FMT>(v[i]);
            amax[i] = amax[i] > k ? amax[i] : k;
        }
    }
    uint32_t s[KEEP_G];
#pragma unroll
    for (int i = 0; i < KEEP_G; i++) s[i] = scale_byte<FMT>(amax[i]);

    {
        uint8_t *sp = scales + z * sc_bs + rb * sc_rp + c0;
        if (n == KEEP_G && (reinterpret_cast<uintptr_t>(sp) & 15u) == 0) {
            uint32_t q[4];
#pragma unroll
            for (int i = 0; i < 4; i++) q[i] = s[4 * i] | (s[4 * i + 1] << 8) | (s[4 * i + 2] << 16) | (s[4 * i + 3] << 24);
            st16(sp, make_uint4(q[0], q[1], q[2], q[3]));
        } else {
#pragma unroll
            for (int i = 0; i < KEEP_G; i++)
                if (i < n) sp[i] = (uint8_t)s[i];
        }
    }

#pragma unroll 2
    for (int r = 0; r < BLOCK; r++) {
        const int64_t row = rb * BLOCK + r;
        if (row >= rows) break;
        uint32_t v[KEEP_G], c[KEEP_G], packed[ND];
        if (n == KEEP_G) load_as_f32_bits<SRC, KEEP_G>(base + row * ld * esz, v);
        else load_head_as_f32_bits<SRC, KEEP_G>(base + row * ld * esz, n, v);
#pragma unroll
        for (int i = 0; i < KEEP_G; i++)
            c[i] = (!Fmt<FMT>::elem_nan && s[i] == SCALE_NAN) ? 0u : encode_elem<FMT, RND>(v[i], s[i], 0u);
        pack_codes<FMT, KEEP_G>(c, packed);
        uint8_t *o = elems + z * out_bs + row * out_rp + c0 * w / 8;
        if (n == KEEP_G && (reinterpret_cast<uintptr_t>(o) & 15u) == 0) {
            store_dwords_any<ND>(o, packed);
        } else {
            const int nbytes = n * w / 8;                   // whole bytes: cols * w and c0 * w are multiples of 8
            for (int b = 0; b < nbytes; b++) o[b] = (uint8_t)(packed[b >> 2] >> (8 * (b & 3)));
        }
    }
}

// Source-order layout with the blocks along the last axis and a length that is not a multiple of
// 32: the codes of a row are packed without the fill that the block-major layout stores.  One lane
// per block; rare shape, plain code.
template <int SRC, int FMT, int RND>
__global__ __launch_bounds__(256) void cast_keep_last_kernel(const void *__restrict__ src, int64_t d1, int64_t d2, int64_t stride0,
                                                             int64_t stride1, int64_t n_units, uint8_t *__restrict__ elems,
                                                             uint8_t *__restrict__ scales)
{
    constexpr int w = Fmt<FMT>::bits;
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= n_units) return;
    const int64_t nblk = (d2 + BLOCK - 1) / BLOCK;
    const int64_t r = u / nblk, b = u - r * nblk, i0 = r / d1, i1 = r - i0 * d1;
    const int64_t off = i0 * stride0 + i1 * stride1 + b * BLOCK;
    const int n = d2 - b * BLOCK >= BLOCK ? BLOCK : (int)(d2 - b * BLOCK);
    uint32_t v[BLOCK], rr[BLOCK] = {};
#pragma unroll
    for (int i = 0; i < BLOCK; i++) {
        uint32_t x = 0;
        if (i < n) x = SRC == DT_BF16 ? (uint32_t)reinterpret_cast<const uint16_t *>(src)[off + i] << 16 : reinterpret_cast<const uint32_t *>(src)[off + i];
        v[i] = x;
    }
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < BLOCK; i++) {
        const uint32_t k = amax_key<FMT>(v[i]);
        amax = amax > k ? amax : k;
    }
    const uint32_t s = scale_byte<FMT>(amax);
    uint32_t packed[w];
    encode_lane<FMT, RND, BLOCK>(v, s, rr, packed);
    uint8_t *o = elems + r * (d2 * w / 8) + b * (BLOCK * w / 8);
    const int nbytes = n * w / 8;
    for (int k = 0; k < nbytes; k++) o[k] = (uint8_t)(packed[k >> 2] >> (8 * (k & 3)));
    scales[u] = (uint8_t)s;
}

template <int SRC, int FMT>
static hipError_t keep_last_rnd(int rnd, unsigned grid, hipStream_t st, const void *src, int64_t d1, int64_t d2, int64_t stride0,
                                int64_t stride1, int64_t n_units, uint8_t *elems, uint8_t *scales)
{
#define MX_GO(R) hipLaunchKernelGGL((cast_keep_last_kernel<SRC, FMT, R>), dim3(grid), dim3(256), 0, st, src, d1, d2, stride0, stride1, n_units, elems, scales)
    if (rnd == ROUND_RNE) MX_GO(ROUND_RNE);
    else if (rnd == ROUND_HALF_AWAY) MX_GO(ROUND_HALF_AWAY);
    else MX_GO(ROUND_TOWARD_ZERO);
#undef MX_GO
    return hipGetLastError();
}

template <int SRC>
static hipError_t keep_last_fmt(int fmt, int rnd, unsigned grid, hipStream_t st, const void *src, int64_t d1, int64_t d2, int64_t stride0,
                                int64_t stride1, int64_t n_units, uint8_t *elems, uint8_t *scales)
{
#define MX_F(F) return keep_last_rnd<SRC, F>(rnd, grid, st, src, d1, d2, stride0, stride1, n_units, elems, scales)
    switch (fmt) {
        case FP8_E4M3: MX_F(FP8_E4M3);
        case FP8_E5M2: MX_F(FP8_E5M2);
        case FP6_E3M2: MX_F(FP6_E3M2);
        case FP6_E2M3: MX_F(FP6_E2M3);
        case FP4_E2M1: MX_F(FP4_E2M1);
        default:       MX_F(INT8);
    }
#undef MX_F
}

template <int SRC, int FMT>
static hipError_t keep_rnd(int rnd, dim3 grid, hipStream_t st, const void *src, int64_t rows, int64_t cols, int64_t ld, int64_t src_bs,
                           uint8_t *elems, int64_t out_rp, int64_t out_bs, uint8_t *scales, int64_t sc_rp, int64_t sc_bs)
{
#define MX_GO(R) hipLaunchKernelGGL((cast_keep_kernel<SRC, FMT, R>), grid, dim3(256), 0, st, src, rows, cols, ld, src_bs, elems, out_rp, \
                                    out_bs, scales, sc_rp, sc_bs)
    if (rnd == ROUND_RNE) MX_GO(ROUND_RNE);
    else if (rnd == ROUND_HALF_AWAY) MX_GO(ROUND_HALF_AWAY);
    else MX_GO(ROUND_TOWARD_ZERO);
#undef MX_GO
    return hipGetLastError();
}

template <int SRC>
static hipError_t keep_fmt(int fmt, int rnd, dim3 grid, hipStream_t st, const void *src, int64_t rows, int64_t cols, int64_t ld,
                           int64_t src_bs, uint8_t *elems, int64_t out_rp, int64_t out_bs, uint8_t *scales, int64_t sc_rp, int64_t sc_bs)
{
#define MX_F(F) return keep_rnd<SRC, F>(rnd, grid, st, src, rows, cols, ld, src_bs, elems, out_rp, out_bs, scales, sc_rp, sc_bs)
    switch (fmt) {
        case FP8_E4M3: MX_F(FP8_E4M3);
        case FP8_E5M2: MX_F(FP8_E5M2);
        case FP6_E3M2: MX_F(FP6_E3M2);
        case FP6_E2M3: MX_F(FP6_E2M3);
        case FP4_E2M1: MX_F(FP4_E2M1);
        default:       MX_F(INT8);
    }
#undef MX_F
}

// a batch of `batch` slices [rows][cols]; at most 65535 per launch
static hipError_t launch_keep(const void *src, int src_dt, int64_t batch, int64_t rows, int64_t cols, int64_t ld, int64_t src_bs,
                              int fmt, int rnd, uint8_t *elems, int64_t out_rp, int64_t out_bs, uint8_t *scales, int64_t sc_rp,
                              int64_t sc_bs, hipStream_t st)
{
    const int64_t gx = (cols + 256 * KEEP_G - 1) / (256 * KEEP_G), gy = (rows + BLOCK - 1) / BLOCK;
    if (gx > 0x7FFFFFFF || gy > 65535) return hipErrorNotSupported;
    const int esz = src_dt == DT_BF16 ? 2 : 4;
    for (int64_t b0 = 0; b0 < batch; b0 += 65535) {
        const int64_t nb = batch - b0 < 65535 ? batch - b0 : 65535;
        const dim3 grid((unsigned)gx, (unsigned)gy, (unsigned)nb);
        const char *sp = static_cast<const char *>(src) + b0 * src_bs * esz;
        const hipError_t e = src_dt == DT_BF16
            ? keep_fmt<DT_BF16>(fmt, rnd, grid, st, sp, rows, cols, ld, src_bs, elems + b0 * out_bs, out_rp, out_bs, scales + b0 * sc_bs, sc_rp, sc_bs)
            : keep_fmt<DT_F32>(fmt, rnd, grid, st, sp, rows, cols, ld, src_bs, elems + b0 * out_bs, out_rp, out_bs, scales + b0 * sc_bs, sc_rp, sc_bs);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_cast_3d(const void *src, int src_dt, int64_t d0, int64_t d1, int64_t d2, int64_t stride0, int64_t stride1,
                          int axis, int fmt, int rnd, bool keep_order, uint8_t *elems, uint8_t *scales, hipStream_t st)
{
    const int w = fmt_bits(fmt);
    const int esz = src_dt == DT_BF16 ? 2 : 4;
    const char *s8 = static_cast<const char *>(src);
    const int64_t dim[3] = {d0, d1, d2};
    const int64_t nblk = (dim[axis] + BLOCK - 1) / BLOCK, line_bytes = nblk * BLOCK * w / 8;
    if (axis == 2 && keep_order && d2 % BLOCK) {     // the block-major layout would store the fill of the last block
        const int64_t n_units = d0 * d1 * nblk, nb = (n_units + 255) / 256;
        if (nb > 0x7FFFFFFF) return hipErrorNotSupported;
        return src_dt == DT_BF16 ? keep_last_fmt<DT_BF16>(fmt, rnd, (unsigned)nb, st, src, d1, d2, stride0, stride1, n_units, elems, scales)
                                 : keep_last_fmt<DT_F32>(fmt, rnd, (unsigned)nb, st, src, d1, d2, stride0, stride1, n_units, elems, scales);
    }
    if (axis == 2) {        // whole blocks along the last axis: both layouts coincide
        if (stride0 == d1 * stride1) return launch_cast(src, src_dt, d0 * d1, d2, stride1, 1, fmt, rnd, elems, scales, st);
        for (int64_t i = 0; i < d0; i++) {
            const hipError_t e = launch_cast(s8 + i * stride0 * esz, src_dt, d1, d2, stride1, 1, fmt, rnd, elems + i * d1 * line_bytes,
                                             scales + i * d1 * nblk, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (keep_order) {
        const int64_t row_bytes = d2 * w / 8;
        if (axis == 1)      // per i0: blocks down the d1 rows of the slice; scales [d0][nblk][d2]
            return launch_keep(src, src_dt, d0, d1, d2, stride1, stride0, fmt, rnd, elems, row_bytes, d1 * row_bytes, scales, d2, nblk * d2, st);
        // axis 0, per i1: blocks down the d0 "rows" (pitch stride0); output row (i0, i1); scales [nblk][d1][d2]
        return launch_keep(src, src_dt, d1, d0, d2, stride0, stride1, fmt, rnd, elems, d1 * row_bytes, row_bytes, scales, d1 * d2, d2, st);
    }
    if (axis == 1) {        // per i0 the axis-0 cast of the [d1][d2] slice: elems [d0][d2][line], scales [d0][d2][nblk]
        for (int64_t i = 0; i < d0; i++) {
            const hipError_t e = launch_cast(s8 + i * stride0 * esz, src_dt, d1, d2, stride1, 0, fmt, rnd, elems + i * d2 * line_bytes,
                                             scales + i * d2 * nblk, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    // axis 0: elems [d1][d2][line]; with dense inner rows the tensor is the 2-D [d0][d1 * d2]
    if (stride1 == d2) return launch_cast(src, src_dt, d0, d1 * d2, stride0, 0, fmt, rnd, elems, scales, st);
    for (int64_t i = 0; i < d1; i++) {
        const hipError_t e = launch_cast(s8 + i * stride1 * esz, src_dt, d0, d2, stride0, 0, fmt, rnd, elems + i * d2 * line_bytes,
                                         scales + i * d2 * nblk, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace mx
