/*
 * mx_oracle.c -- reference CPU implementation of the MX cast (Algorithm 1 of
 * arXiv 2310.10537), of v = X * P (Section 2) and of the MX dot product
 * (Section 4.1).  TEST INFRASTRUCTURE: plain, slow, written to be read next
 * to the paper.  Shares nothing with the GPU library.
 *
 * Arithmetic: every real number that occurs (a Float32 or BFloat16 input, a
 * power of two between 2^-127 and 2^127, their quotient, an element value) is
 * exactly representable in IEEE double, and all scalings are by powers of two
 * through ldexp, so no step before the one explicit rounding is inexact.
 */
#include "mx_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------
 * Element formats (Table 1 gives name and width; "ExMy" fixes the rest:
 * sign-magnitude, x exponent bits with bias 2^(x-1)-1, y mantissa bits,
 * exponent field 0 = subnormals).  Special codes: FP8 E5M2 keeps IEEE Inf and
 * NaN in its top exponent; FP8 E4M3 has no Inf and a single NaN mantissa
 * pattern (all ones); the 6- and 4-bit formats have neither (Section 2.1:
 * Inf/NaN per element only "depending on the element format").
 * ---------------------------------------------------------------------- */
typedef struct {
    int bits;    /* total width                                   */
    int ebits;   /* exponent field width (0 for INT8)             */
    int mbits;   /* mantissa field width                          */
    int bias;    /* exponent bias                                 */
    int emax;    /* exponent of the largest normal (Algorithm 1)  */
    int has_inf; /* element codes for +-Inf exist                 */
    int has_nan; /* element codes for NaN exist                   */
} fmt_t;

static const fmt_t FMT[MXO_NUM_FORMATS] = {
    /* FP8 E4M3 */ {8, 4, 3, 7, 8, 0, 1},
    /* FP8 E5M2 */ {8, 5, 2, 15, 15, 1, 1},
    /* FP6 E3M2 */ {6, 3, 2, 3, 4, 0, 0},
    /* FP6 E2M3 */ {6, 2, 3, 1, 2, 0, 0},
    /* FP4 E2M1 */ {4, 2, 1, 1, 2, 0, 0},
    /* INT8     */ {8, 0, 0, 0, 0, 0, 0},
};

static int fmt_ok(int fmt) { return fmt >= 0 && fmt < MXO_NUM_FORMATS; }

int mxo_elem_bits(int fmt) { return fmt_ok(fmt) ? FMT[fmt].bits : -1; }
int mxo_emax(int fmt) { return fmt_ok(fmt) ? FMT[fmt].emax : -1; }

int mxo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* floor(log2(a)) for finite a > 0 */
static int floor_log2(double a)
{
    int e;
    (void)frexp(a, &e); /* a = f * 2^e with f in [0.5, 1) */
    return e - 1;
}

/* Largest normal magnitude of a floating-point element format. */
static double fp_max_normal(const fmt_t *f)
{
    int top_e = (1 << f->ebits) - 1;
    int top_m = (1 << f->mbits) - 1;
    if (f->has_inf) top_e -= 1;            /* E5M2: top exponent is Inf/NaN */
    else if (f->has_nan) top_m -= 1;       /* E4M3: only S.1111.111 is NaN  */
    return ldexp((double)((1 << f->mbits) + top_m), top_e - f->bias - f->mbits);
}

/* ------------------------------------------------------------------------
 * decode: element code -> P
 * ---------------------------------------------------------------------- */
double mxo_decode(int fmt, unsigned code)
{
    if (!fmt_ok(fmt)) return NAN;
    const fmt_t *f = &FMT[fmt];
    code &= (1u << f->bits) - 1u;

    if (fmt == MXO_INT8) {
        /* two's complement integer with an implied scale of 2^-6 */
        int v = (code & 0x80u) ? (int)code - 256 : (int)code;
        return ldexp((double)v, -6);
    }

    unsigned sign = code >> (f->bits - 1);
    unsigned E = (code >> f->mbits) & ((1u << f->ebits) - 1u);
    unsigned M = code & ((1u << f->mbits) - 1u);
    double s = sign ? -1.0 : 1.0;

    if (f->has_inf && E == (1u << f->ebits) - 1u)     /* E5M2 top exponent */
        return M == 0 ? s * INFINITY : NAN;
    if (!f->has_inf && f->has_nan &&                   /* E4M3 S.1111.111  */
        E == (1u << f->ebits) - 1u && M == (1u << f->mbits) - 1u)
        return NAN;

    if (E == 0) /* subnormal: 0.M * 2^(1-bias) */
        return s * ldexp((double)M, 1 - f->bias - f->mbits);
    /* normal: 1.M * 2^(E-bias) */
    return s * ldexp((double)((1u << f->mbits) + M), (int)E - f->bias - f->mbits);
}

/* Round the non-negative exact quotient q to an integer.  u in [0, 1) is used
 * by the stochastic mode only: the magnitude goes up when the discarded
 * fraction plus u reaches 1, i.e. with probability equal to that fraction.
 * u is a multiple of 2^-25 and q has at most 24 significant bits, so whenever
 * the double sum q + u is not exact, q is far too small to move it across an
 * integer: the floor is that of the exact sum. */
static double round_q(double q, int rnd, double u)
{
    double fl = floor(q);
    double d = q - fl; /* exact: q has at most 53 significant bits */
    if (rnd == MXO_ROUND_TOWARD_ZERO) {
        /* magnitude truncated */
    } else if (rnd == MXO_ROUND_STOCHASTIC) {
        fl = floor(q + u);
    } else if (rnd == MXO_ROUND_HALF_AWAY) {
        if (d >= 0.5) fl += 1.0;
    } else { /* ties to even */
        if (d > 0.5 || (d == 0.5 && fmod(fl, 2.0) != 0.0)) fl += 1.0;
    }
    return fl;
}

/* ------------------------------------------------------------------------
 * encode: quantize_to_element_format (Algorithm 1 line 4 and the notes
 * after it), applied to x = V / X.
 * ---------------------------------------------------------------------- */
unsigned mxo_encode(int fmt, int rnd, double x)
{
    return mxo_encode_u(fmt, rnd, x, 0.0);
}

unsigned mxo_encode_u(int fmt, int rnd, double x, double u)
{
    if (!fmt_ok(fmt)) return 0;
    const fmt_t *f = &FMT[fmt];
    unsigned sign = signbit(x) ? 1u : 0u;
    unsigned signbit_code = sign << (f->bits - 1);

    if (isnan(x)) {
        if (fmt == MXO_FP8_E4M3) return signbit_code | 0x7Fu;
        if (fmt == MXO_FP8_E5M2) return signbit_code | 0x7Eu; /* S.11111.10 */
        return 0;
    }
    if (isinf(x)) { /* never clamped */
        if (fmt == MXO_FP8_E5M2) return signbit_code | 0x7Cu;
        if (fmt == MXO_FP8_E4M3) return signbit_code | 0x7Fu; /* no Inf code */
        return 0;
    }

    double a = fabs(x);

    if (fmt == MXO_INT8) {
        double q = round_q(ldexp(a, 6), rnd, u); /* grid step 2^-6 */
        if (q > 127.0) q = 127.0;             /* symmetric clamp */
        int iq = (int)q;
        if (sign) iq = -iq;
        return (unsigned)iq & 0xFFu;
    }

    if (a == 0.0) return signbit_code;

    int emin = 1 - f->bias; /* exponent of the smallest normal */
    int step_exp;           /* grid step is 2^step_exp around a  */
    if (a < ldexp(1.0, emin))
        step_exp = emin - f->mbits; /* subnormal grid */
    else
        step_exp = floor_log2(a) - f->mbits;

    double q = round_q(ldexp(a, -step_exp), rnd, u);
    double r = ldexp(q, step_exp);
    double vmax = fp_max_normal(f);
    if (r > vmax) r = vmax; /* clamp normals, keep sign */

    /* write r (exactly on the grid now) as sign / exponent / mantissa */
    if (r == 0.0) return signbit_code;
    unsigned E, M;
    if (r < ldexp(1.0, emin)) {
        E = 0;
        M = (unsigned)ldexp(r, -(emin - f->mbits));
    } else {
        int e = floor_log2(r);
        E = (unsigned)(e + f->bias);
        M = (unsigned)ldexp(r, -(e - f->mbits)) - (1u << f->mbits);
    }
    return signbit_code | (E << f->mbits) | M;
}

/* ------------------------------------------------------------------------
 * Algorithm 1 on one block.
 * ---------------------------------------------------------------------- */
#define F32_MIN_NORMAL 0x1p-126 /* smallest normal Float32 */

void mxo_quantize_block(const double v[MXO_BLOCK], int fmt, int rnd,
                        uint8_t *scale, unsigned codes[MXO_BLOCK])
{
    mxo_quantize_block_u(v, fmt, rnd, NULL, scale, codes);
}

void mxo_quantize_block_u(const double v[MXO_BLOCK], int fmt, int rnd,
                          const double *u, uint8_t *scale,
                          unsigned codes[MXO_BLOCK])
{
    const fmt_t *f = &FMT[fmt];
    int any_nonfinite = 0;
    double m = 0.0; /* max |V_i| over normal finite inputs */

    for (int i = 0; i < MXO_BLOCK; i++) {
        if (isnan(v[i]) || isinf(v[i])) { any_nonfinite = 1; continue; }
        double a = fabs(v[i]);
        if (a < F32_MIN_NORMAL) continue; /* Float32 subnormal or zero */
        if (a > m) m = a;
    }

    /* formats with no element Inf/NaN: the only NaN encoding left is X = NaN */
    if (any_nonfinite && !f->has_nan) {
        *scale = MXO_SCALE_NAN;
        for (int i = 0; i < MXO_BLOCK; i++) codes[i] = 0;
        return;
    }

    /* line 1: shared_exp = floor(log2(max |V_i|)) - emax_elem,
     * kept inside what E8M0 can hold as a number (bytes 0..254) */
    int s;
    if (m == 0.0) {
        s = 0; /* log2(0) = -inf, clamped */
    } else {
        int shared_exp = floor_log2(m) - f->emax;
        s = shared_exp + 127;
        if (s < 0) s = 0;
        if (s > 254) s = 254;
    }
    *scale = (uint8_t)s;

    /* lines 3-5: P_i = quantize(V_i / X), X = 2^(s-127) */
    for (int i = 0; i < MXO_BLOCK; i++) {
        double x;
        if (isnan(v[i]) || isinf(v[i]))
            x = v[i];
        else if (fabs(v[i]) < F32_MIN_NORMAL)
            x = copysign(0.0, v[i]); /* Float32 subnormal -> P_i = 0 */
        else
            x = ldexp(v[i], 127 - s);
        codes[i] = mxo_encode_u(fmt, rnd, x, u ? u[i] : 0.0);
    }
}

/* ------------------------------------------------------------------------
 * Random offsets of the stochastic mode: Philox4x32-10 (Salmon, Moraes, Dror,
 * Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC 2011), a counter
 * based generator, so the number that belongs to a tensor element depends on
 * (seed, element index) only and not on who computes it.
 * One round: (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1,
 * lo(M0*c0)); the key goes up by the two Weyl constants before every round
 * after the first.
 * ---------------------------------------------------------------------- */
void mxo_philox4x32(uint64_t key, uint64_t counter, uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c[4] = { (uint32_t)counter, (uint32_t)(counter >> 32), 0u, 0u };
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
    for (int round = 0; round < 10; round++) {
        if (round > 0) { k0 += W0; k1 += W1; }
        uint64_t p0 = (uint64_t)M0 * c[0];
        uint64_t p1 = (uint64_t)M1 * c[2];
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
    }
    for (int i = 0; i < 4; i++) out[i] = c[i];
}

/* same with a full 128-bit counter and 64-bit key given as words (used to
 * check the generator against its published known answers) */
void mxo_philox4x32_words(const uint32_t ctr[4], const uint32_t key[2],
                          uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; round++) {
        if (round > 0) { k0 += W0; k1 += W1; }
        uint64_t p0 = (uint64_t)M0 * c[0];
        uint64_t p1 = (uint64_t)M1 * c[2];
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
    }
    for (int i = 0; i < 4; i++) out[i] = c[i];
}

/* u of tensor element number e (row * cols + col of the source tensor):
 * word e mod 4 of the generator's output for counter e / 4, top 25 bits. */
double mxo_sr_uniform(uint64_t seed, int64_t e)
{
    uint32_t w[4];
    mxo_philox4x32(seed, (uint64_t)e >> 2, w);
    return ldexp((double)(w[e & 3] >> 7), -25);
}

/* ------------------------------------------------------------------------
 * Tensor level
 * ---------------------------------------------------------------------- */
static double load_scalar(const void *src, int dt, int64_t idx)
{
    if (dt == MXO_DT_F32) {
        float fv;
        memcpy(&fv, (const char *)src + 4 * idx, 4);
        return (double)fv;
    } else { /* bf16 = upper half of a Float32 */
        uint16_t h;
        memcpy(&h, (const char *)src + 2 * idx, 2);
        uint32_t u = (uint32_t)h << 16;
        float fv;
        memcpy(&fv, &u, 4);
        return (double)fv;
    }
}

/* element j of a packed row: bits [j*w, (j+1)*w), little-endian */
static void put_code(uint8_t *row, int64_t j, int w, unsigned code)
{
    int64_t bit = j * w;
    for (int b = 0; b < w; b++, bit++) {
        uint8_t mask = (uint8_t)(1u << (bit & 7));
        if ((code >> b) & 1u) row[bit >> 3] |= mask;
        else row[bit >> 3] &= (uint8_t)~mask;
    }
}

static unsigned get_code(const uint8_t *row, int64_t j, int w)
{
    int64_t bit = j * w;
    unsigned code = 0;
    for (int b = 0; b < w; b++, bit++)
        code |= (unsigned)((row[bit >> 3] >> (bit & 7)) & 1u) << b;
    return code;
}

/* The block axis may have any length: the last block of a line is then filled
 * up with zeros (which neither move the block maximum nor produce a non-zero
 * code), and the stored line holds whole blocks. */
static int shape_ok(int64_t rows, int64_t cols, int axis)
{
    if (rows <= 0 || cols <= 0) return 0;
    return axis == 0 || axis == 1;
}

int mxo_quantize(const void *src, int src_dt, int64_t rows, int64_t cols,
                 int64_t ld, int axis, int fmt, int rnd,
                 uint8_t *elems_out, uint8_t *scales_out)
{
    if (rnd == MXO_ROUND_STOCHASTIC) return MXO_ERR_ARG; /* needs a seed */
    return mxo_quantize_seeded(src, src_dt, rows, cols, ld, axis, fmt, rnd, 0,
                               elems_out, scales_out);
}

int mxo_quantize_seeded(const void *src, int src_dt, int64_t rows, int64_t cols,
                        int64_t ld, int axis, int fmt, int rnd, uint64_t seed,
                        uint8_t *elems_out, uint8_t *scales_out)
{
    if (!src || !elems_out || !scales_out || !fmt_ok(fmt)) return MXO_ERR_ARG;
    if (src_dt != MXO_DT_F32 && src_dt != MXO_DT_BF16) return MXO_ERR_ARG;
    if (rnd < MXO_ROUND_RNE || rnd > MXO_ROUND_STOCHASTIC) return MXO_ERR_ARG;
    if (!shape_ok(rows, cols, axis) || ld < cols) return MXO_ERR_ARG;

    int w = FMT[fmt].bits;
    /* the output is indexed [o][l]: o = the axis that is not blocked,
     * l = position along the block axis */
    int64_t n_out = axis == 1 ? rows : cols;
    int64_t len = axis == 1 ? cols : rows;
    int64_t nblk = (len + MXO_BLOCK - 1) / MXO_BLOCK;
    int64_t row_bytes = nblk * MXO_BLOCK * w / 8;

#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n_out; o++) {
        uint8_t *erow = elems_out + o * row_bytes;
        for (int64_t b = 0; b < nblk; b++) {
            double v[MXO_BLOCK], u[MXO_BLOCK];
            unsigned codes[MXO_BLOCK];
            for (int i = 0; i < MXO_BLOCK; i++) {
                int64_t l = b * MXO_BLOCK + i;
                int64_t row = axis == 1 ? o : l, col = axis == 1 ? l : o;
                if (l >= len) { v[i] = 0.0; u[i] = 0.0; continue; } /* fill */
                v[i] = load_scalar(src, src_dt, row * ld + col);
                u[i] = rnd == MXO_ROUND_STOCHASTIC
                           ? mxo_sr_uniform(seed, row * cols + col) : 0.0;
            }
            mxo_quantize_block_u(v, fmt, rnd, u, &scales_out[o * nblk + b], codes);
            for (int i = 0; i < MXO_BLOCK; i++)
                put_code(erow, b * MXO_BLOCK + i, w, codes[i]);
        }
    }
    return MXO_OK;
}

/* Section 3, "principal axis" of a multi-dimensional tensor: Algorithm 1 applied to every
 * 1-D fibre of a 3-D tensor [d0][d1][d2] along `axis`, one block of 32 after the other.
 * Element (i0, i1, i2) lives at src[i0*stride0 + i1*stride1 + i2].
 * keep_order = 0: the block axis is moved last and the other two keep their order; with
 *     (o1, o2) the two remaining indices in source order and L the block-axis length,
 *     elems [o1][o2][ceil(L/32)*32*w/8], scales [o1][o2][ceil(L/32)]  (fill = code 0).
 * keep_order = 1: codes stay in source order, densely packed along d2 (d2*w a multiple of 8):
 *     elems [d0][d1][d2*w/8]; the scales array is the source shape with the block axis
 *     replaced by its block count: [d0][d1][ceil(d2/32)], [d0][ceil(d1/32)][d2] or
 *     [ceil(d0/32)][d1][d2]. */
int mxo_quantize_3d(const void *src, int src_dt, int64_t d0, int64_t d1, int64_t d2,
                    int64_t stride0, int64_t stride1, int axis, int fmt, int rnd,
                    int keep_order, uint8_t *elems_out, uint8_t *scales_out)
{
    if (!src || !elems_out || !scales_out || !fmt_ok(fmt)) return MXO_ERR_ARG;
    if (src_dt != MXO_DT_F32 && src_dt != MXO_DT_BF16) return MXO_ERR_ARG;
    if (rnd < MXO_ROUND_RNE || rnd > MXO_ROUND_TOWARD_ZERO) return MXO_ERR_ARG;
    if (d0 <= 0 || d1 <= 0 || d2 <= 0 || axis < 0 || axis > 2) return MXO_ERR_ARG;
    int w = FMT[fmt].bits;
    if (keep_order && (d2 * w) % 8) return MXO_ERR_ARG;
    const int64_t dim[3] = {d0, d1, d2};
    const int64_t L = dim[axis], nblk = (L + MXO_BLOCK - 1) / MXO_BLOCK;
    /* the two axes that are not blocked, in source order */
    const int a1 = axis == 0 ? 1 : 0, a2 = axis == 2 ? 1 : 2;
    const int64_t n1 = dim[a1], n2 = dim[a2];
    const int64_t line_bytes = nblk * MXO_BLOCK * w / 8, row_bytes = d2 * w / 8;

    for (int64_t o1 = 0; o1 < n1; o1++)
        for (int64_t o2 = 0; o2 < n2; o2++)
            for (int64_t b = 0; b < nblk; b++) {
                double v[MXO_BLOCK];
                unsigned codes[MXO_BLOCK];
                int64_t idx[3];
                uint8_t sc;
                idx[a1] = o1; idx[a2] = o2;
                for (int i = 0; i < MXO_BLOCK; i++) {
                    int64_t l = b * MXO_BLOCK + i;
                    if (l >= L) { v[i] = 0.0; continue; }
                    idx[axis] = l;
                    v[i] = load_scalar(src, src_dt, idx[0] * stride0 + idx[1] * stride1 + idx[2]);
                }
                mxo_quantize_block(v, fmt, rnd, &sc, codes);
                if (!keep_order) {
                    uint8_t *line = elems_out + (o1 * n2 + o2) * line_bytes;
                    for (int i = 0; i < MXO_BLOCK; i++) put_code(line, b * MXO_BLOCK + i, w, codes[i]);
                    scales_out[(o1 * n2 + o2) * nblk + b] = sc;
                } else {
                    for (int i = 0; i < MXO_BLOCK; i++) {
                        int64_t l = b * MXO_BLOCK + i;
                        if (l >= L) break;
                        idx[axis] = l;
                        put_code(elems_out + (idx[0] * d1 + idx[1]) * row_bytes, idx[2], w, codes[i]);
                    }
                    /* the scale sits where the block sits: the block axis index is b */
                    idx[axis] = b;
                    int64_t sd1 = axis == 1 ? nblk : d1, sd2 = axis == 2 ? nblk : d2;
                    scales_out[(idx[0] * sd1 + idx[1]) * sd2 + idx[2]] = sc;
                }
            }
    return MXO_OK;
}

/* X * P as a double; X = NaN gives NaN (Section 2) */
static double block_value(int fmt, unsigned code, uint8_t s)
{
    if (s == MXO_SCALE_NAN) return NAN;
    return ldexp(mxo_decode(fmt, code), (int)s - 127);
}

/* double -> bf16 bits, round to nearest even, done on the bf16 grid directly */
static uint16_t to_bf16_bits(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isinf(a)) return sign | 0x7F80;
    if (a == 0.0) return sign;
    int step_exp = (a < F32_MIN_NORMAL) ? -126 - 7 : floor_log2(a) - 7;
    double r = ldexp(round_q(ldexp(a, -step_exp), MXO_ROUND_RNE, 0.0), step_exp);
    if (r > 0x1.FEp127) return sign | 0x7F80; /* above the largest bf16 */
    float fr = (float)r; /* exact: r is on the bf16 grid */
    uint32_t u;
    memcpy(&u, &fr, 4);
    return sign | (uint16_t)(u >> 16);
}

static void store_scalar(void *dst, int dt, int64_t idx, double v)
{
    if (dt == MXO_DT_F32) {
        float fv = (float)v; /* beyond Float32 range -> +-Inf */
        uint32_t u;
        memcpy(&u, &fv, 4);
        if (isnan(v)) u = 0x7FC00000u; /* one canonical quiet NaN */
        memcpy((char *)dst + 4 * idx, &u, 4);
    } else {
        uint16_t h = to_bf16_bits(v);
        memcpy((char *)dst + 2 * idx, &h, 2);
    }
}

int mxo_dequantize(const uint8_t *elems, const uint8_t *scales, int fmt,
                   int64_t rows, int64_t cols, int axis,
                   void *dst, int dst_dt, int64_t ld)
{
    if (!elems || !scales || !dst || !fmt_ok(fmt)) return MXO_ERR_ARG;
    if (dst_dt != MXO_DT_F32 && dst_dt != MXO_DT_BF16) return MXO_ERR_ARG;
    if (!shape_ok(rows, cols, axis) || ld < cols) return MXO_ERR_ARG;

    int w = FMT[fmt].bits;
    int64_t n_out = axis == 1 ? rows : cols;
    int64_t len = axis == 1 ? cols : rows;
    int64_t nblk = (len + MXO_BLOCK - 1) / MXO_BLOCK;
    int64_t row_bytes = nblk * MXO_BLOCK * w / 8; /* whole blocks are stored */

#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n_out; o++) {
        const uint8_t *erow = elems + o * row_bytes;
        for (int64_t l = 0; l < len; l++) {
            uint8_t s = scales[o * nblk + l / MXO_BLOCK];
            double v = block_value(fmt, get_code(erow, l, w), s);
            int64_t idx = axis == 1 ? o * ld + l : l * ld + o;
            store_scalar(dst, dst_dt, idx, v);
        }
    }
    return MXO_OK;
}

/* Inverse of mxo_quantize_3d (Section 2: v_i = X * P_i), for both of its layouts: element
 * (i0, i1, i2) of the [d0][d1][d2] result, written at dst[i0*stride0 + i1*stride1 + i2], is the
 * code that mxo_quantize_3d put there times the scale of the block it lies in. */
int mxo_dequantize_3d(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t d0, int64_t d1,
                      int64_t d2, int axis, int keep_order, void *dst, int dst_dt,
                      int64_t stride0, int64_t stride1)
{
    if (!elems || !scales || !dst || !fmt_ok(fmt)) return MXO_ERR_ARG;
    if (dst_dt != MXO_DT_F32 && dst_dt != MXO_DT_BF16) return MXO_ERR_ARG;
    if (d0 <= 0 || d1 <= 0 || d2 <= 0 || axis < 0 || axis > 2) return MXO_ERR_ARG;
    int w = FMT[fmt].bits;
    if (keep_order && (d2 * w) % 8) return MXO_ERR_ARG;
    const int64_t dim[3] = {d0, d1, d2};
    const int64_t L = dim[axis], nblk = (L + MXO_BLOCK - 1) / MXO_BLOCK;
    const int a1 = axis == 0 ? 1 : 0, a2 = axis == 2 ? 1 : 2;
    const int64_t n2 = dim[a2];
    const int64_t line_bytes = nblk * MXO_BLOCK * w / 8, row_bytes = d2 * w / 8;
    const int64_t sd1 = axis == 1 ? nblk : d1, sd2 = axis == 2 ? nblk : d2;

    for (int64_t i0 = 0; i0 < d0; i0++)
        for (int64_t i1 = 0; i1 < d1; i1++)
            for (int64_t i2 = 0; i2 < d2; i2++) {
                const int64_t idx[3] = {i0, i1, i2};
                const int64_t l = idx[axis], b = l / MXO_BLOCK;
                unsigned code;
                uint8_t sc;
                if (!keep_order) {
                    const int64_t line = idx[a1] * n2 + idx[a2];
                    code = get_code(elems + line * line_bytes, l, w);
                    sc = scales[line * nblk + b];
                } else {
                    int64_t sidx[3] = {i0, i1, i2};
                    sidx[axis] = b;
                    code = get_code(elems + (i0 * d1 + i1) * row_bytes, i2, w);
                    sc = scales[(sidx[0] * sd1 + sidx[1]) * sd2 + sidx[2]];
                }
                store_scalar(dst, dst_dt, i0 * stride0 + i1 * stride1 + i2, block_value(fmt, code, sc));
            }
    return MXO_OK;
}

/* ------------------------------------------------------------------------
 * MX dot product.  Because every X is a power of two, sum over blocks of
 * X_A * X_B * sum_j a_j * b_j equals the plain sum of products of the
 * dequantized values; each product is exact in double.
 * ---------------------------------------------------------------------- */
static void dequant_row(const uint8_t *elems, const uint8_t *scales, int fmt,
                        int64_t K, int64_t r, double *out)
{
    int w = FMT[fmt].bits;
    const uint8_t *erow = elems + r * (K * w / 8);
    const uint8_t *srow = scales + r * (K / MXO_BLOCK);
    for (int64_t k = 0; k < K; k++)
        out[k] = block_value(fmt, get_code(erow, k, w), srow[k / MXO_BLOCK]);
}

static int gemm_args_ok(int64_t M, int64_t N, int64_t K, const void *a,
                        const void *as, int fa, const void *b, const void *bs,
                        int fb, const void *C)
{
    if (!a || !as || !b || !bs || !C) return 0;
    if (!fmt_ok(fa) || !fmt_ok(fb)) return 0;
    if (M <= 0 || N <= 0 || K <= 0 || K % MXO_BLOCK) return 0;
    return 1;
}

int mxo_gemm(int64_t M, int64_t N, int64_t K,
             const uint8_t *A_elems, const uint8_t *A_scales, int fmtA,
             const uint8_t *B_elems, const uint8_t *B_scales, int fmtB,
             double *C, double *Cabs)
{
    if (!gemm_args_ok(M, N, K, A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, C))
        return MXO_ERR_ARG;

    /* working copies of the operands as doubles (freed before returning) */
    double *Ad = (double *)malloc((size_t)M * K * sizeof(double));
    double *Bd = (double *)malloc((size_t)N * K * sizeof(double));
    if (!Ad || !Bd) { free(Ad); free(Bd); return MXO_ERR_ARG; }

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++)
        dequant_row(A_elems, A_scales, fmtA, K, m, Ad + m * K);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++)
        dequant_row(B_elems, B_scales, fmtB, K, n, Bd + n * K);

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++) {
        for (int64_t n = 0; n < N; n++) {
            double acc = 0.0, accabs = 0.0;
            for (int64_t k = 0; k < K; k++) {
                double p = Ad[m * K + k] * Bd[n * K + k];
                acc += p;
                accabs += fabs(p);
            }
            C[m * N + n] = acc;
            if (Cabs) Cabs[m * N + n] = accabs;
        }
    }
    free(Ad);
    free(Bd);
    return MXO_OK;
}

int mxo_gemm_entries(int64_t M, int64_t N, int64_t K,
                     const uint8_t *A_elems, const uint8_t *A_scales, int fmtA,
                     const uint8_t *B_elems, const uint8_t *B_scales, int fmtB,
                     int64_t n, const int64_t *mi, const int64_t *ni,
                     double *C, double *Cabs)
{
    if (!gemm_args_ok(M, N, K, A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, C))
        return MXO_ERR_ARG;
    if (n < 0 || !mi || !ni) return MXO_ERR_ARG;
    for (int64_t t = 0; t < n; t++)
        if (mi[t] < 0 || mi[t] >= M || ni[t] < 0 || ni[t] >= N) return MXO_ERR_ARG;

    int wa = FMT[fmtA].bits, wb = FMT[fmtB].bits;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; t++) {
        const uint8_t *ea = A_elems + mi[t] * (K * wa / 8);
        const uint8_t *sa = A_scales + mi[t] * (K / MXO_BLOCK);
        const uint8_t *eb = B_elems + ni[t] * (K * wb / 8);
        const uint8_t *sb = B_scales + ni[t] * (K / MXO_BLOCK);
        double acc = 0.0, accabs = 0.0;
        for (int64_t k = 0; k < K; k++) {
            double a = block_value(fmtA, get_code(ea, k, wa), sa[k / MXO_BLOCK]);
            double b = block_value(fmtB, get_code(eb, k, wb), sb[k / MXO_BLOCK]);
            double p = a * b;
            acc += p;
            accabs += fabs(p);
        }
        C[t] = acc;
        if (Cabs) Cabs[t] = accabs;
    }
    return MXO_OK;
}
