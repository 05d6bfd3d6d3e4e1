// MXINT8 x MXINT8 GEMM (Section 4.1 of arXiv 2310.10537; MXINT8 is the format of Table 1
// with two's-complement elements and an implied scale of 2^-6).  The block-scaled matrix
// instruction has no integer form, so each 32-element block is one plain
// V_MFMA_I32_32X32X32_I8 -- its 32 products and their sum are exact integers -- and
// the block's contribution X_A * X_B * sum is added in Float32 with an exact
// power-of-two scaling (a Float32 factor where the scales allow it, ldexp otherwise):
//   C[m][n] += float(sum_j qa[m][32b+j] * qb[n][32b+j]) * 2^(sA[m][b] + sB[n][b] - 254 - 12).
// Operand layout of the instruction (the same as each 32-wide half of the 8-bit f8f6f4 form):
// lane l holds, for row / column l % 32, the 16 consecutive K bytes [16 * (l / 32), + 16);
// result register t of lane l is C[8*(t/4) + 4*(l/32) + t%4][l % 32].
// One wave per 32 x 32 output tile, operands straight from global memory, any shape.  The
// A scale of a block is needed per output row, i.e. per result register: the 32 row bytes
// go through a wave-private LDS line and come back as the sixteen dwords a lane needs.
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

// Adds one block's contribution to the 16 accumulators of a lane: acc[t] += p[t] * 2^(sA[row t] + sB - 266).
// sa / sb are the scale bytes of the lane's own row / column (lane i = row i and column i of the tile);
// the per-row bytes travel through the wave's 32-dword LDS line.  When every scale byte of the block is
// within [70, 196] (or the NaN byte) the two factors 2^(s - 133) and their product are normal Float32
// numbers (exponent sum in [-126, 126]), so is every scaled sum: one multiply and one fused
// multiply-add per entry, the row factor arriving ready-made.  Any other scale byte in the wave's block
// sends the whole wave through the exact power-of-two scaling of ldexp (3 more instructions per entry).
__device__ __forceinline__ uint32_t i8_factor_bits(uint32_t s) { return s == SCALE_NAN ? 0x7FC00000u : (s - 6u) << 23; }
__device__ __forceinline__ bool i8_factor_ok(uint32_t s) { return s - 70u <= 126u || s == SCALE_NAN; }

__device__ __forceinline__ void i8_accumulate(float (&acc)[16], const v16i_t &p, uint32_t sa, uint32_t sb, uint32_t *line,
                                              int i, int g)
{
    const bool plain = i8_factor_ok(sa) && i8_factor_ok(sb);
    const bool fast = __builtin_amdgcn_ballot_w64(!plain) == 0;   // uniform over the wave
    if (g == 0) line[i] = fast ? i8_factor_bits(sa) : sa;
    wave_lds_sync8();
    uint32_t w[16];
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const uint4 r = *reinterpret_cast<const uint4 *>(line + 8 * q + 4 * g);   // rows 8q + 4g .. + 3 = registers 4q .. 4q + 3
        w[4 * q] = r.x; w[4 * q + 1] = r.y; w[4 * q + 2] = r.z; w[4 * q + 3] = r.w;
    }
    if (fast) {
        const float fb = __uint_as_float(i8_factor_bits(sb));
#pragma unroll
        for (int t = 0; t < 16; t++) acc[t] = fmaf((float)p[t], __uint_as_float(w[t]) * fb, acc[t]);
    } else {
#pragma unroll
        for (int t = 0; t < 16; t++) {
            float term = ldexpf((float)p[t], (int)w[t] + (int)sb - 254 - 12);
            if (w[t] == SCALE_NAN || sb == SCALE_NAN) term = __uint_as_float(0x7FC00000u);
            acc[t] += term;
        }
    }
    wave_lds_sync8();   // the line is rewritten for the next block
}

// Clears the split route's flag word.  A kernel rather than a memset node, so that a caller who captures the
// stream into a graph replays an ordinary launch.
__global__ void int8_clear_flag_kernel(uint32_t *flag) { *flag = 0u; }

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
    __shared__ __attribute__((aligned(16))) uint32_t lds_all[4 * 32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t *lds = lds_all + wave * 32;
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
        const v4i_t a = rv ? v4i_t{(int)qa.x, (int)qa.y, (int)qa.z, (int)qa.w} : v4i_t{0, 0, 0, 0};
        const v4i_t b = cv ? v4i_t{(int)qb.x, (int)qb.y, (int)qb.z, (int)qb.w} : v4i_t{0, 0, 0, 0};
        v16i_t z;
#pragma unroll
        for (int t = 0; t < 16; t++) z[t] = 0;
        const v16i_t p = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, z, 0, 0, 0);
        i8_accumulate(acc, p, sa, sb, lds, i, g);
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
    __shared__ __attribute__((aligned(16))) uint32_t lds_all[I8_WAVES * 32];
    __shared__ float red[I8_WAVES - 1][16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t *lds = lds_all + wave * 32;
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
            const v4i_t a = rv ? v4i_t{(int)qa[u].x, (int)qa[u].y, (int)qa[u].z, (int)qa[u].w} : v4i_t{0, 0, 0, 0};
            const v4i_t b = cv ? v4i_t{(int)qb[u].x, (int)qb[u].y, (int)qb[u].z, (int)qb[u].w} : v4i_t{0, 0, 0, 0};
            v16i_t z;
#pragma unroll
            for (int t = 0; t < 16; t++) z[t] = 0;
            const v16i_t p = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, z, 0, 0, 0);
            i8_accumulate(acc, p, sa[u], sb[u], lds, i, g);
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

// The same with the operands staged through LDS (K a multiple of 128).  Above, every lane of an operand
// load addresses a different matrix row, so one load instruction touches 64 cache lines and uses 16 bytes
// of each; here a wave fetches 128 bytes of each row at a time with loads whose adjacent lanes read
// adjacent 16 bytes (every line touched once), parks the pieces in a private LDS tile -- rows of 128
// bytes, 16-byte piece c of row r in slot c ^ ((r / 2) % 8), which keeps both the parking stores and the
// operand reads free of bank conflicts -- and multiplies its four blocks from there while the next 128
// bytes are in flight.  MT tiles of 32 rows share the B tile of the work-group's 32 columns.  Rows beyond
// M and columns beyond N read the last valid one instead: their results are never stored.
// QN: groups of 8 rows of a tile that are scaled and stored (result registers 4q .. 4q + 3 are rows
// 8q + 4g .. + 3); a decoding step of at most 8 or 16 rows skips the rest.
template <int MT, int QN, int CDT>
__global__ __launch_bounds__(64 * I8_WAVES) void gemm_int8_lds_kernel(int64_t M, int64_t N, int64_t K,
                                                                       const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                                       const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                                       void *__restrict__ C, int64_t ldc)
{
    constexpr int T_BYTES = 32 * 128, W_BYTES = (MT + 1) * T_BYTES;
    constexpr int RED_BYTES = (I8_WAVES - 1) * MT * 16 * 64 * 4;
    static_assert(I8_WAVES * W_BYTES >= RED_BYTES, "the partial sums reuse the staging tiles");
    __shared__ __attribute__((aligned(16))) uint8_t lds[I8_WAVES * W_BYTES];
    __shared__ __attribute__((aligned(16))) uint32_t lines[I8_WAVES * MT * 4 * 32];   // per wave, tile and block: 32 row words
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 31, g = lane >> 5;
    const int64_t n0 = (int64_t)blockIdx.x * 32, m0 = (int64_t)blockIdx.y * (32 * MT);
    const int64_t nkb = K / BLOCK, chunks = K / 128;
    const int64_t per_wave = (chunks + I8_WAVES - 1) / I8_WAVES;
    const int64_t c_begin = wave * per_wave, c_end = c_begin + per_wave < chunks ? c_begin + per_wave : chunks;
    uint8_t *tA = lds + wave * W_BYTES, *tB = tA + MT * T_BYTES;
    uint32_t *line = lines + wave * (MT * 4 * 32);

    const int lr = lane >> 3, lp = lane & 7;            // a wave-wide load: 8 rows x eight 16-byte pieces
    auto slot = [](int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); };
    auto clampi = [](int64_t v, int64_t hi) { return v < hi ? v : hi; };
    uint4 ra[MT][4], rb[4];
    uint32_t sa_d[MT], sb_d;
    auto request = [&](int64_t c) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int j = 0; j < 4; j++) ra[x][j] = ld16(Ae + clampi(m0 + 32 * x + 8 * j + lr, M - 1) * K + c * 128 + lp * 16);
#pragma unroll
        for (int j = 0; j < 4; j++) rb[j] = ld16(Be + clampi(n0 + 8 * j + lr, N - 1) * K + c * 128 + lp * 16);
#pragma unroll
        for (int x = 0; x < MT; x++) sa_d[x] = *reinterpret_cast<const uint32_t *>(As + clampi(m0 + 32 * x + i, M - 1) * nkb + c * 4);
        sb_d = *reinterpret_cast<const uint32_t *>(Bs + clampi(n0 + i, N - 1) * nkb + c * 4);
    };

    float acc[MT][16];
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 16; t++) acc[x][t] = 0.f;

    if (c_begin < c_end) request(c_begin);
    for (int64_t c = c_begin; c < c_end; c++) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int j = 0; j < 4; j++) *reinterpret_cast<uint4 *>(tA + x * T_BYTES + slot(8 * j + lr, lp)) = ra[x][j];
#pragma unroll
        for (int j = 0; j < 4; j++) *reinterpret_cast<uint4 *>(tB + slot(8 * j + lr, lp)) = rb[j];
        // The four scale bytes of row i (one per block of the chunk) go to the wave's lines next to the
        // operands, under the same wait: as ready-made Float32 factors when every scale byte of the chunk,
        // rows and columns, allows it (see i8_accumulate), as plain bytes otherwise.  The lower half-wave
        // writes blocks 0 and 1, the upper one blocks 2 and 3 (both hold row i's dword).
        uint32_t sa_c[MT];
#pragma unroll
        for (int x = 0; x < MT; x++) sa_c[x] = sa_d[x];
        const uint32_t sb_c = sb_d;
        bool plain = true;
#pragma unroll
        for (int b = 0; b < 4; b++) {
            plain = plain && i8_factor_ok((sb_c >> (8 * b)) & 0xFFu);
#pragma unroll
            for (int x = 0; x < MT; x++) plain = plain && i8_factor_ok((sa_c[x] >> (8 * b)) & 0xFFu);
        }
        const bool fast = __builtin_amdgcn_ballot_w64(!plain) == 0;   // uniform over the wave
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int b = 2 * g + h;
                const uint32_t sbyte = (sa_c[x] >> (8 * b)) & 0xFFu;
                line[(x * 4 + b) * 32 + i] = fast ? i8_factor_bits(sbyte) : sbyte;
            }
        wave_lds_sync8();
        if (c + 1 < c_end) request(c + 1);
#pragma unroll
        for (int b = 0; b < 4; b++) {
            // lane (i, g) of the instruction: bytes [16 g, 16 g + 16) of block b of row / column i
            const uint4 qb = *reinterpret_cast<const uint4 *>(tB + slot(i, 2 * b + g));
            const v4i_t bv = {(int)qb.x, (int)qb.y, (int)qb.z, (int)qb.w};
            const uint32_t sbb = (sb_c >> (8 * b)) & 0xFFu;
            const float fb = __uint_as_float(i8_factor_bits(sbb));
#pragma unroll
            for (int x = 0; x < MT; x++) {
                const uint4 qa = *reinterpret_cast<const uint4 *>(tA + x * T_BYTES + slot(i, 2 * b + g));
                const v4i_t av = {(int)qa.x, (int)qa.y, (int)qa.z, (int)qa.w};
                uint32_t w[4 * QN];
#pragma unroll
                for (int q = 0; q < QN; q++) {
                    const uint4 r = *reinterpret_cast<const uint4 *>(line + (x * 4 + b) * 32 + 8 * q + 4 * g);   // rows 8q + 4g .. + 3
                    w[4 * q] = r.x; w[4 * q + 1] = r.y; w[4 * q + 2] = r.z; w[4 * q + 3] = r.w;
                }
                v16i_t z;
#pragma unroll
                for (int t = 0; t < 16; t++) z[t] = 0;
                const v16i_t p = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, z, 0, 0, 0);
                if (fast) {
#pragma unroll
                    for (int t = 0; t < 4 * QN; t++) acc[x][t] = fmaf((float)p[t], __uint_as_float(w[t]) * fb, acc[x][t]);
                } else {
#pragma unroll
                    for (int t = 0; t < 4 * QN; t++) {
                        float term = ldexpf((float)p[t], (int)w[t] + (int)sbb - 254 - 12);
                        if (w[t] == SCALE_NAN || sbb == SCALE_NAN) term = __uint_as_float(0x7FC00000u);
                        acc[x][t] += term;
                    }
                }
            }
        }
        wave_lds_sync8();   // tiles and lines are read before the next chunk is parked in them
    }

    // ---- the eight partial sums, always w0 + w1 + ... + w7; the staging tiles are done with
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
    if (wave > 0) {
#pragma unroll
        for (int x = 0; x < MT; x++)
#pragma unroll
            for (int t = 0; t < 4 * QN; t++) red[(((wave - 1) * MT + x) * 16 + t) * 64 + lane] = acc[x][t];
    }
    __syncthreads();
    if (wave != 0) return;
    const int64_t col = n0 + i;
#pragma unroll
    for (int x = 0; x < MT; x++)
#pragma unroll
        for (int t = 0; t < 4 * QN; t++) {
            float v = acc[x][t];
#pragma unroll
            for (int w = 0; w < I8_WAVES - 1; w++) v += red[((w * MT + x) * 16 + t) * 64 + lane];
            const int64_t r = m0 + 32 * x + 8 * (t / 4) + 4 * g + (t % 4);
            if (r < M && col < N) {
                if (CDT == DT_F32) reinterpret_cast<float *>(C)[r * ldc + col] = v;
                else reinterpret_cast<uint16_t *>(C)[r * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
            }
        }
}

template <int MT, int QN>
static hipError_t launch_int8_lds(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                                  const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 32 * MT - 1) / (32 * MT)));
    if (c_dt == DT_F32)
        hipLaunchKernelGGL((gemm_int8_lds_kernel<MT, QN, DT_F32>), grid, dim3(64 * I8_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    else
        hipLaunchKernelGGL((gemm_int8_lds_kernel<MT, QN, DT_BF16>), grid, dim3(64 * I8_WAVES), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc);
    return hipGetLastError();
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
    // Four routes, picked by measurement (same box, bf16 output; TOP/s = 2 M N K / time):
    //  - the split route: whole 256 x 256 tiles and a depth the tiled kernel takes (4K a multiple of 128, >= 512).
    //    It wins once the tiles fill most of the chip: 4096^3 505 TOP/s, 8192 x 4096 x 4096 631, 2048 x 8192 x 1024
    //    363, 4096 x 4096 x 512 272 -- against 250, 257, 136, 74 for the staged kernel;
    //  - the LDS-staged shared-K kernel (K a multiple of 128): about 230 TOP/s when K is long, falling with K
    //    (each tile's eight partial sums cost the same whatever K is): 512 x 4096 x 4096 77 us against the
    //    direct kernel's 128, 256 x 11008 x 4096 112 against 189, 1000 x 1000 x 1024 19 against 25; with 64 tiles
    //    and a long K it is ahead of the split route too (2048^3 95 against 116 us, 1024 x 4096 x 4096 146 against
    //    196; level at 2048 x 2048 x 512), and few rows (decoding) are 1.2-1.7 times faster than unstaged;
    //  - the unstaged shared-K kernel for few rows or few tiles when K is not a multiple of 128;
    //  - the direct kernel for everything else (short K, odd shapes): 80-170 TOP/s.
    const int64_t tiles256 = (M / 256) * (N / 256);
    const bool split = M > 0 && N > 0 && K >= 128 && (tiles256 >= 96 || (tiles256 >= 64 && K < 1024)) &&
                       gemm_tiled_applies(M, N, 4 * K, FP6_E2M3, FP6_E2M3);
    if (split) {
        const size_t nba = (size_t)M * (size_t)(K / BLOCK), nbb = (size_t)N * (size_t)(K / BLOCK);
        const size_t off_ea = 256, off_eb = off_ea + nba * 96, off_sa = off_eb + nbb * 96, off_sb = off_sa + nba * 4;
        uint8_t *ws = nullptr;
        hipError_t e = ws_acquire(off_sb + nbb * 4, st, &ws);
        if (e != hipSuccess) return e;
        {
            uint32_t *flag = reinterpret_cast<uint32_t *>(ws);
            hipLaunchKernelGGL(int8_clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
            e = hipGetLastError();
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
            const hipError_t f = ws_release(ws, st);
            return e != hipSuccess ? e : f;
        }
    }
    if (M > 0 && N > 0 && K % 128 == 0 && (M <= 128 ? K >= 8 * BLOCK : K >= 1024) && (M + 63) / 64 <= 65535)
        return M <= 8    ? launch_int8_lds<1, 1>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
               : M <= 16 ? launch_int8_lds<1, 2>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
               : M <= 32 ? launch_int8_lds<1, 4>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st)
                         : launch_int8_lds<2, 4>(M, N, K, Ae, As, Be, Bs, C, c_dt, ldc, st);
    // K not in whole 128-byte pieces: few rows, or so few tiles that the direct kernel would put at most one
    // wave on a SIMD while K is long (256 x 4096 x 4096 81 -> 66 us; with 2048 tiles of 32 x 32 the direct
    // kernel is ahead again, 114 vs 124 us)
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
