/*
 * mx_oracle.h -- reference CPU implementation of the Microscaling (MX) cast,
 * its inverse, and the MX dot product (arXiv 2310.10537, Sections 2, 3, 4.1).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow on purpose: every function is the
 * definition written out in double precision and integer arithmetic, with no
 * blocking, fusion or reordering, so that it can be checked against the paper
 * by eye.  It shares no code with the GPU library and must never be linked
 * into, or called from, the product path.
 *
 * All pointers are HOST pointers and caller-owned; nothing is retained.
 * Only mxo_gemm allocates (working copies of its operands, freed on return).
 *
 * Parity unpinned (conventions of this build, the paper leaves them open):
 *   - the scale byte of a block with no normal finite value (0x00);
 *   - Inf/NaN inputs to element formats that have no Inf/NaN code
 *     (whole block marked NaN by scale byte 0xFF, element codes 0);
 *   - Inf input to FP8 E4M3 (encoded as the element NaN, sign kept).
 */
#ifndef MX_ORACLE_H
#define MX_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element data formats of Table 1.  Numbering is part of the interface. */
enum {
    MXO_FP8_E4M3 = 0,
    MXO_FP8_E5M2 = 1,
    MXO_FP6_E3M2 = 2,
    MXO_FP6_E2M3 = 3,
    MXO_FP4_E2M1 = 4,
    MXO_INT8     = 5,
    MXO_NUM_FORMATS = 6
};

/* Rounding used by quantize_to_element_format (Section 4.3: ties to even;
 * Section 4.5: ties away from zero).  The paper studies only those two; the
 * other two are extensions of this build: the magnitude truncated, and the
 * magnitude rounded up with probability equal to the discarded fraction
 * (u in [0, 1), a multiple of 2^-25, is added to |x| / step before the floor). */
enum { MXO_ROUND_RNE = 0, MXO_ROUND_HALF_AWAY = 1, MXO_ROUND_TOWARD_ZERO = 2,
       MXO_ROUND_STOCHASTIC = 3 };

/* Scalar float types of tensors handed to the cast. */
enum { MXO_DT_F32 = 0, MXO_DT_BF16 = 1 };

enum { MXO_OK = 0, MXO_ERR_ARG = 1 };

#define MXO_BLOCK 32          /* block size k of every concrete format (Table 1) */
#define MXO_SCALE_NAN 0xFF    /* E8M0 code of X = NaN (Section 2.1)              */

/* Bit width of one element (Table 1); -1 for an unknown format. */
int mxo_elem_bits(int fmt);

/* emax_elem of Algorithm 1: exponent of the largest normal number. */
int mxo_emax(int fmt);

/* Value of one element code P (Section 2: v = X * P, this is P).
 * May return +-Inf or NaN for FP8 codes that encode them. */
double mxo_decode(int fmt, unsigned code);

/* quantize_to_element_format of Algorithm 1, line 4, for one already scaled
 * value x = V / X.  x may be any double including +-0, +-Inf and NaN.
 * Finite magnitudes beyond the largest normal are clamped to it, sign kept;
 * Inf and NaN are never clamped.  For formats without Inf/NaN codes the
 * caller handles non-finite inputs at block level and this returns 0. */
unsigned mxo_encode(int fmt, int rnd, double x);

/* Same with the random offset u of the stochastic mode (ignored by the other
 * modes; mxo_encode passes 0, which makes that mode truncate). */
unsigned mxo_encode_u(int fmt, int rnd, double x, double u);

/* Algorithm 1 on one block of 32 values, already widened (exactly) from
 * Float32 or BFloat16 to double.  Inputs below 2^-126 in magnitude are
 * Float32 subnormals and become P_i = 0.  Writes the E8M0 byte and the 32
 * element codes. */
void mxo_quantize_block(const double v[MXO_BLOCK], int fmt, int rnd,
                        uint8_t *scale, unsigned codes[MXO_BLOCK]);

/* Same with one random offset per element (u may be NULL = all 0). */
void mxo_quantize_block_u(const double v[MXO_BLOCK], int fmt, int rnd,
                          const double *u, uint8_t *scale,
                          unsigned codes[MXO_BLOCK]);

/* Philox4x32-10 (Salmon et al., SC 2011) with counter words
 * (lo32(counter), hi32(counter), 0, 0) and key words (lo32(key), hi32(key));
 * the _words form takes all six words. */
void mxo_philox4x32(uint64_t key, uint64_t counter, uint32_t out[4]);
void mxo_philox4x32_words(const uint32_t ctr[4], const uint32_t key[2],
                          uint32_t out[4]);

/* Random offset of tensor element e = row * cols + col under `seed`:
 * (word e mod 4 of philox(key = seed, counter = e / 4)) >> 7, times 2^-25. */
double mxo_sr_uniform(uint64_t seed, int64_t e);

/* Cast a row-major [rows, cols] tensor (leading dimension ld, in elements).
 * axis = 1: blocks of 32 along the last dimension;
 *           elems [rows][cols*bits/8], scales [rows][cols/32].
 * axis = 0: blocks of 32 along dimension 0, output written as the cast of the
 *           transpose: elems [cols][rows*bits/8], scales [cols][rows/32].
 * Elements are densely bit-packed little-endian: element j of an output row
 * occupies bits [j*w, (j+1)*w) of that row's byte string.
 * The block axis may have any length L: the paper does not say what happens to
 * a last, partial block; here it is filled up with zeros, and every stored row
 * holds ceil(L/32) whole blocks (elems [..][ceil(L/32)*32*bits/8], scales
 * [..][ceil(L/32)]; the fill positions hold code 0). */
int mxo_quantize(const void *src, int src_dt, int64_t rows, int64_t cols,
                 int64_t ld, int axis, int fmt, int rnd,
                 uint8_t *elems_out, uint8_t *scales_out);

/* Same for every rounding mode; the stochastic one draws element (row, col)'s
 * offset as mxo_sr_uniform(seed, row * cols + col), whatever the axis. */
int mxo_quantize_seeded(const void *src, int src_dt, int64_t rows, int64_t cols,
                        int64_t ld, int axis, int fmt, int rnd, uint64_t seed,
                        uint8_t *elems_out, uint8_t *scales_out);

/* Algorithm 1 along any axis of a 3-D tensor [d0][d1][d2] (Section 3: the principal axis
 * of a multi-dimensional tensor); element (i0, i1, i2) at src[i0*stride0 + i1*stride1 + i2].
 * keep_order = 0: block axis moved last, the other two axes keep their order:
 *     elems [o1][o2][ceil(L/32)*32*bits/8], scales [o1][o2][ceil(L/32)].
 * keep_order = 1: codes in source order packed along d2 (d2*bits a multiple of 8):
 *     elems [d0][d1][d2*bits/8], scales = source shape with the block axis replaced by its
 *     block count.  Rounding: not the stochastic mode. */
int mxo_quantize_3d(const void *src, int src_dt, int64_t d0, int64_t d1, int64_t d2,
                    int64_t stride0, int64_t stride1, int axis, int fmt, int rnd,
                    int keep_order, uint8_t *elems_out, uint8_t *scales_out);

/* Inverse: v = X * P (Section 2), X = NaN makes the whole block NaN, results
 * beyond Float32 range become +-Inf.  Writes row-major [rows, cols]; with a
 * block-axis length that is not a multiple of 32 the stored rows hold whole
 * blocks (as mxo_quantize writes them) and the fill positions are skipped. */
/* inverse of mxo_quantize_3d for both layouts; dst [d0][d1][d2] with element strides (stride0, stride1, 1) */
int mxo_dequantize_3d(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t d0, int64_t d1,
                      int64_t d2, int axis, int keep_order, void *dst, int dst_dt,
                      int64_t stride0, int64_t stride1);
int mxo_dequantize(const uint8_t *elems, const uint8_t *scales, int fmt,
                   int64_t rows, int64_t cols, int axis,
                   void *dst, int dst_dt, int64_t ld);

/* MX dot products (Section 4.1): C[m][n] = sum_k A[m][k] * B[n][k] with both
 * operands MX tensors whose blocks run along K (A: [M][K], B: [N][K], as
 * written by mxo_quantize with axis = 1).  Accumulated in double in plain k
 * order.  Cabs (may be NULL) receives sum_k |A[m][k]| * |B[n][k]|. */
int mxo_gemm(int64_t M, int64_t N, int64_t K,
             const uint8_t *A_elems, const uint8_t *A_scales, int fmtA,
             const uint8_t *B_elems, const uint8_t *B_scales, int fmtB,
             double *C, double *Cabs);

/* Same dot product for a list of n (m, n) output coordinates only. */
int mxo_gemm_entries(int64_t M, int64_t N, int64_t K,
                     const uint8_t *A_elems, const uint8_t *A_scales, int fmtA,
                     const uint8_t *B_elems, const uint8_t *B_scales, int fmtB,
                     int64_t n, const int64_t *mi, const int64_t *ni,
                     double *C, double *Cabs);

/* Number of threads the loops over rows use (OpenMP); 1 if built without. */
int mxo_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
