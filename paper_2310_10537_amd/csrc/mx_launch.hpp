// Host-side launch entry points shared between the kernel files and the C ABI.
// Each returns the hipError_t of the launch; arguments are validated by the caller.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mx {

// seed: read by the stochastic rounding mode only
hipError_t launch_cast(const void *src, int src_dt, int64_t rows, int64_t cols, int64_t ld, int axis, int fmt, int rnd,
                       uint8_t *elems, uint8_t *scales, hipStream_t st, uint64_t seed = 0);

// Algorithm 1 along axis 0, 1 or 2 of a 3-D tensor [d0][d1][d2] with element strides (stride0, stride1, 1);
// keep_order = false: block axis moved last; true: codes in source order packed along d2
hipError_t launch_cast_3d(const void *src, int src_dt, int64_t d0, int64_t d1, int64_t d2, int64_t stride0, int64_t stride1,
                          int axis, int fmt, int rnd, bool keep_order, uint8_t *elems, uint8_t *scales, hipStream_t st);

// bf16 sources and the two round-to-nearest modes only; hipErrorNotSupported when the shape is
// outside what the fast kernels take
hipError_t launch_cast_bf16_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int axis, int fmt, int rnd,
                                 uint8_t *elems, uint8_t *scales, hipStream_t st);

// Float32 sources, axis 0, whole 128 x 64 tiles, the two round-to-nearest modes; else hipErrorNotSupported
hipError_t launch_cast_col_f32_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd, uint8_t *elems,
                                    uint8_t *scales, hipStream_t st);

// Float32 sources, axis 1, dense rows of whole blocks, a whole number of 2048-element runs, round to nearest
hipError_t launch_cast_row_f32_fast(const void *src, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd, uint8_t *elems,
                                    uint8_t *scales, hipStream_t st);

// both axes in one pass over the source: (e1, s1) as launch_cast with axis 1, (e0, s0) with axis 0
hipError_t launch_cast_dual(const void *src, int src_dt, int64_t rows, int64_t cols, int64_t ld, int fmt, int rnd,
                            uint8_t *e1, uint8_t *s1, uint8_t *e0, uint8_t *s0, hipStream_t st);

hipError_t launch_dequant(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t rows, int64_t cols, int axis,
                          void *dst, int dst_dt, int64_t ld, hipStream_t st);

// inverse of launch_cast_3d for both layouts; dst [d0][d1][d2] with element strides (stride0, stride1, 1)
hipError_t launch_dequant_3d(const uint8_t *elems, const uint8_t *scales, int fmt, int64_t d0, int64_t d1, int64_t d2, int axis,
                             bool keep_order, void *dst, int dst_dt, int64_t stride0, int64_t stride1, hipStream_t st);

// Scratch memory of the GEMM routes that need it (the MX form of a bf16 operand, the two E2M3 halves of
// MXINT8 operands, a Float32 C that is cast afterwards).  Inside a WorkspaceScope -- opened by the
// entry points that take a caller-owned workspace -- ws_acquire carves 256-byte aligned pieces off
// that workspace (hipErrorOutOfMemory when it is too small); outside one it takes the piece from
// the device's memory pool in stream order.  ws_release returns the piece (last acquired first).
// A refused request is an error of the call; no route falls back to another kernel because of it.
struct WorkspaceScope {
    WorkspaceScope(void *p, size_t bytes);
    ~WorkspaceScope();
    WorkspaceScope(const WorkspaceScope &) = delete;
    WorkspaceScope &operator=(const WorkspaceScope &) = delete;
};
hipError_t ws_acquire(size_t bytes, hipStream_t st, uint8_t **out);
hipError_t ws_release(uint8_t *p, hipStream_t st);
// upper bounds of what mx_gemm / mx_gemm_qa / mx_gemm_q can ask for (0: the call never needs scratch)
size_t gemm_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);
size_t gemm_qa_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);
size_t gemm_q_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);

// a_bf16 != nullptr selects the quantize-on-load form (A_elems / A_scales unused).
hipError_t launch_gemm(int64_t M, int64_t N, int64_t K, const uint8_t *A_elems, const uint8_t *A_scales,
                       const void *a_bf16, int64_t lda, int rnd, int fmtA, const uint8_t *B_elems,
                       const uint8_t *B_scales, int fmtB, void *C, int c_dt, int64_t ldc, hipStream_t st);

// MXINT8 x MXINT8: integer matrix instruction per block, Float32 accumulation of the scaled block sums
hipError_t launch_gemm_int8(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                            const uint8_t *Bs, void *C, int c_dt, int64_t ldc, hipStream_t st);

// true when the LDS-tiled kernel takes the problem: FP8 / FP6 / FP4 operands, whole 256 x 256
// tiles, K a multiple of 128 and at least 512
bool gemm_tiled_applies(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);
// true when the tiled kernel can cast a bf16 A operand inside its K loop (8-bit pairs)
bool gemm_tiled_fuses_cast(int fmtA, int fmtB);

// LDS-tiled kernel (a_bf16 != nullptr: A is raw bf16 and cast on load); hipErrorNotSupported
// when the problem does not qualify.
hipError_t launch_gemm_tiled(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const void *a_bf16,
                             int64_t lda, int rnd, int fmtA, const uint8_t *Be, const uint8_t *Bs, int fmtB, void *C,
                             int c_dt, int64_t ldc, hipStream_t st);

// At most 128 rows of A: eight waves per 32 columns of C share the K range (FP8 / FP6 / FP4 operands)
bool gemm_skinny_applies(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);
hipError_t launch_gemm_skinny(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA, const uint8_t *Be,
                              const uint8_t *Bs, int fmtB, void *C, int c_dt, int64_t ldc, hipStream_t st);

// The same product with C written as an MX tensor (blocks of 32 along N) by the tiled kernel's
// epilogue; hipErrorNotSupported when the shape, the formats or the rounding are outside it.
bool gemm_tiled_casts_output(int fmtC, int rndC);
hipError_t launch_gemm_tiled_mx(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA,
                                const uint8_t *Be, const uint8_t *Bs, int fmtB, uint8_t *Ce, uint8_t *Cs, int fmtC, int rndC,
                                hipStream_t st);

// mx_gemm followed by the axis-1 cast of its Float32 result, fused where the tiled kernel applies
hipError_t launch_gemm_q(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA, const uint8_t *Be,
                         const uint8_t *Bs, int fmtB, uint8_t *Ce, uint8_t *Cs, int fmtC, int rndC, hipStream_t st);

}  // namespace mx
