// C ABI of the MX library (see include/mx.h): argument validation and dispatch.  Every call
// enqueues on the caller's stream.  The library keeps no tensor pointers; the routes that need
// a workspace are named in include/mx.h, and mx_gemm_qa_noalloc below keeps its workspace in a
// static device array instead of taking it from the memory pool.
#include "../../include/mx.h"

#include <atomic>

#include "mx_device.hpp"
#include "mx_launch.hpp"

namespace {

bool fmt_ok(int f) { return f >= 0 && f < mx::NUM_FORMATS; }
bool dt_ok(int d) { return d == MX_DT_F32 || d == MX_DT_BF16; }
// the modes that need no seed
bool rnd_ok(int r) { return r == MX_ROUND_RNE || r == MX_ROUND_HALF_AWAY || r == MX_ROUND_TOWARD_ZERO; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int esize(int dt) { return dt == MX_DT_BF16 ? 2 : 4; }

// whole_blocks: the block axis must be a multiple of 32 (entry points without a partial-block path)
int tensor_shape_status(int64_t rows, int64_t cols, int axis, int64_t ld, bool whole_blocks = false)
{
    if (rows < 0 || cols < 0) return MX_ERR_SHAPE;
    if (whole_blocks && (axis == 1 ? cols : rows) % mx::BLOCK) return MX_ERR_SHAPE;
    if (ld < cols) return MX_ERR_SHAPE;
    return MX_OK;
}

int64_t blocks_of(int64_t len) { return (len + mx::BLOCK - 1) / mx::BLOCK; }

// a GEMM route that could not get its scratch memory (caller workspace too small, or the pool refused)
int gemm_status(hipError_t e) { return e == hipSuccess ? MX_OK : e == hipErrorOutOfMemory ? MX_ERR_WORKSPACE : MX_ERR_LAUNCH; }

}  // namespace

extern "C" {

size_t mx_elem_bytes(mx_format_t fmt, int64_t rows, int64_t cols, int axis)
{
    if (!fmt_ok(fmt) || rows < 0 || cols < 0 || (axis != 0 && axis != 1)) return 0;
    const int64_t lines = axis == 1 ? rows : cols, len = axis == 1 ? cols : rows;
    return (size_t)lines * (size_t)blocks_of(len) * (size_t)(mx::BLOCK * mx::fmt_bits(fmt) / 8);
}

size_t mx_scale_bytes(int64_t rows, int64_t cols, int axis)
{
    if (rows < 0 || cols < 0 || (axis != 0 && axis != 1)) return 0;
    const int64_t lines = axis == 1 ? rows : cols, len = axis == 1 ? cols : rows;
    return (size_t)lines * (size_t)blocks_of(len);
}

static int quantize_common(const void *src, mx_dtype_t src_dt, int64_t rows, int64_t cols, int64_t ld, int axis,
                           mx_format_t fmt, int rnd, uint64_t seed, void *elems_out, uint8_t *scales_out, void *hip_stream)
{
    if (!fmt_ok(fmt) || !dt_ok(src_dt) || (axis != 0 && axis != 1)) return MX_ERR_ENUM;
    if (int st = tensor_shape_status(rows, cols, axis, ld)) return st;
    if (rows == 0 || cols == 0) return MX_OK;
    if (!src || !elems_out || !scales_out) return MX_ERR_NULL;
    if (!aligned16(src) || !aligned16(elems_out) || !aligned16(scales_out) || (ld * esize(src_dt)) % 16)
        return MX_ERR_ALIGN;
    hipError_t e = mx::launch_cast(src, src_dt, rows, cols, ld, axis, fmt, rnd, static_cast<uint8_t *>(elems_out),
                                   scales_out, static_cast<hipStream_t>(hip_stream), seed);
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

int mx_quantize(const void *src, mx_dtype_t src_dt, int64_t rows, int64_t cols, int64_t ld, int axis, mx_format_t fmt,
                mx_round_t rnd, void *elems_out, uint8_t *scales_out, void *hip_stream)
{
    if (!rnd_ok(rnd)) return MX_ERR_ENUM;   // the stochastic mode needs a seed: mx_quantize_sr
    return quantize_common(src, src_dt, rows, cols, ld, axis, fmt, rnd, 0, elems_out, scales_out, hip_stream);
}

int mx_quantize_sr(const void *src, mx_dtype_t src_dt, int64_t rows, int64_t cols, int64_t ld, int axis, mx_format_t fmt,
                   uint64_t seed, void *elems_out, uint8_t *scales_out, void *hip_stream)
{
    return quantize_common(src, src_dt, rows, cols, ld, axis, fmt, MX_ROUND_STOCHASTIC, seed, elems_out, scales_out,
                           hip_stream);
}

int mx_quantize_dual(const void *src, mx_dtype_t src_dt, int64_t rows, int64_t cols, int64_t ld, mx_format_t fmt,
                     mx_round_t rnd, void *elems_axis1, uint8_t *scales_axis1, void *elems_axis0, uint8_t *scales_axis0,
                     void *hip_stream)
{
    if (!fmt_ok(fmt) || !dt_ok(src_dt) || !rnd_ok(rnd)) return MX_ERR_ENUM;
    if (int st = tensor_shape_status(rows, cols, 1, ld, true)) return st;
    if (int st = tensor_shape_status(rows, cols, 0, ld, true)) return st;
    if (rows == 0 || cols == 0) return MX_OK;
    if (!src || !elems_axis1 || !scales_axis1 || !elems_axis0 || !scales_axis0) return MX_ERR_NULL;
    if (!aligned16(src) || !aligned16(elems_axis1) || !aligned16(scales_axis1) || !aligned16(elems_axis0) ||
        !aligned16(scales_axis0) || (ld * esize(src_dt)) % 16)
        return MX_ERR_ALIGN;
    hipError_t e = mx::launch_cast_dual(src, src_dt, rows, cols, ld, fmt, rnd, static_cast<uint8_t *>(elems_axis1), scales_axis1,
                                        static_cast<uint8_t *>(elems_axis0), scales_axis0, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

int mx_quantize_3d(const void *src, mx_dtype_t src_dt, int64_t d0, int64_t d1, int64_t d2, int64_t stride0, int64_t stride1,
                   int axis, mx_format_t fmt, mx_round_t rnd, int keep_order, void *elems_out, uint8_t *scales_out, void *hip_stream)
{
    if (!fmt_ok(fmt) || !dt_ok(src_dt) || !rnd_ok(rnd) || axis < 0 || axis > 2 || (keep_order != 0 && keep_order != 1)) return MX_ERR_ENUM;
    if (d0 < 0 || d1 < 0 || d2 < 0 || stride1 < d2 || stride0 < d1 * stride1) return MX_ERR_SHAPE;
    if (keep_order && (d2 * mx::fmt_bits(fmt)) % 8) return MX_ERR_SHAPE;
    if (d0 == 0 || d1 == 0 || d2 == 0) return MX_OK;
    if (!src || !elems_out || !scales_out) return MX_ERR_NULL;
    if (!aligned16(src) || !aligned16(elems_out) || !aligned16(scales_out) || (stride0 * esize(src_dt)) % 16 || (stride1 * esize(src_dt)) % 16)
        return MX_ERR_ALIGN;
    hipError_t e = mx::launch_cast_3d(src, src_dt, d0, d1, d2, stride0, stride1, axis, fmt, rnd, keep_order != 0,
                                      static_cast<uint8_t *>(elems_out), scales_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MX_OK : e == hipErrorNotSupported ? MX_ERR_UNSUPPORTED : MX_ERR_LAUNCH;
}

int mx_dequantize(const void *elems, const uint8_t *scales, mx_format_t fmt, int64_t rows, int64_t cols, int axis,
                  void *dst, mx_dtype_t dst_dt, int64_t ld, void *hip_stream)
{
    if (!fmt_ok(fmt) || !dt_ok(dst_dt) || (axis != 0 && axis != 1)) return MX_ERR_ENUM;
    if (int st = tensor_shape_status(rows, cols, axis, ld)) return st;
    if (rows == 0 || cols == 0) return MX_OK;
    if (!elems || !scales || !dst) return MX_ERR_NULL;
    if (!aligned16(elems) || !aligned16(scales) || !aligned16(dst) || (ld * esize(dst_dt)) % 16) return MX_ERR_ALIGN;
    hipError_t e = mx::launch_dequant(static_cast<const uint8_t *>(elems), scales, fmt, rows, cols, axis, dst, dst_dt, ld,
                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

int mx_dequantize_3d(const void *elems, const uint8_t *scales, mx_format_t fmt, int64_t d0, int64_t d1, int64_t d2, int axis,
                     int keep_order, void *dst, mx_dtype_t dst_dt, int64_t stride0, int64_t stride1, void *hip_stream)
{
    if (!fmt_ok(fmt) || !dt_ok(dst_dt) || axis < 0 || axis > 2 || (keep_order != 0 && keep_order != 1)) return MX_ERR_ENUM;
    if (d0 < 0 || d1 < 0 || d2 < 0 || stride1 < d2 || stride0 < d1 * stride1) return MX_ERR_SHAPE;
    if (keep_order && (d2 * mx::fmt_bits(fmt)) % 8) return MX_ERR_SHAPE;
    if (d0 == 0 || d1 == 0 || d2 == 0) return MX_OK;
    if (!elems || !scales || !dst) return MX_ERR_NULL;
    if (!aligned16(elems) || !aligned16(scales) || !aligned16(dst) || (stride0 * esize(dst_dt)) % 16 || (stride1 * esize(dst_dt)) % 16)
        return MX_ERR_ALIGN;
    hipError_t e = mx::launch_dequant_3d(static_cast<const uint8_t *>(elems), scales, fmt, d0, d1, d2, axis, keep_order != 0, dst, dst_dt,
                                         stride0, stride1, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

static int gemm_common(bool qa, int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales,
                       const void *A_bf16, int64_t lda, int rnd, mx_format_t fmtA, const void *B_elems, const uint8_t *B_scales,
                       mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc, void *hip_stream, void *workspace = nullptr,
                       size_t workspace_bytes = 0)
{
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB) || !dt_ok(c_dt)) return MX_ERR_ENUM;
    if (qa && !rnd_ok(rnd)) return MX_ERR_ENUM;
    if (M < 0 || N < 0 || K < 0 || K % mx::BLOCK || ldc < N || (qa && lda < K)) return MX_ERR_SHAPE;
    if ((fmtA == MX_INT8) != (fmtB == MX_INT8)) return MX_ERR_UNSUPPORTED;   // MXINT8 only pairs with MXINT8
    if (M == 0 || N == 0) return MX_OK;
    if (!C || (K > 0 && ((qa ? !A_bf16 : (!A_elems || !A_scales)) || !B_elems || !B_scales))) return MX_ERR_NULL;
    if (!aligned16(B_elems) || !aligned16(B_scales) || !aligned16(C)) return MX_ERR_ALIGN;
    if (qa ? (!aligned16(A_bf16) || (lda * 2) % 16) : (!aligned16(A_elems) || !aligned16(A_scales))) return MX_ERR_ALIGN;
    if (workspace) {
        if (!aligned16(workspace)) return MX_ERR_ALIGN;
        const size_t need = qa ? mx::gemm_qa_workspace_bound(M, N, K, fmtA, fmtB) : mx::gemm_workspace_bound(M, N, K, fmtA, fmtB);
        if (workspace_bytes < need) return MX_ERR_WORKSPACE;
    }
    mx::WorkspaceScope scope(workspace, workspace_bytes);
    hipError_t e = mx::launch_gemm(M, N, K, static_cast<const uint8_t *>(A_elems), A_scales, qa ? A_bf16 : nullptr, lda, rnd, fmtA,
                                   static_cast<const uint8_t *>(B_elems), B_scales, fmtB, C, c_dt, ldc,
                                   static_cast<hipStream_t>(hip_stream));
    return gemm_status(e);
}

size_t mx_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, mx_format_t fmtA, mx_format_t fmtB)
{
    return fmt_ok(fmtA) && fmt_ok(fmtB) ? mx::gemm_workspace_bound(M, N, K, fmtA, fmtB) : 0;
}

size_t mx_gemm_qa_workspace_bytes(int64_t M, int64_t N, int64_t K, mx_format_t fmtA, mx_format_t fmtB)
{
    return fmt_ok(fmtA) && fmt_ok(fmtB) ? mx::gemm_qa_workspace_bound(M, N, K, fmtA, fmtB) : 0;
}

size_t mx_gemm_q_workspace_bytes(int64_t M, int64_t N, int64_t K, mx_format_t fmtA, mx_format_t fmtB)
{
    return fmt_ok(fmtA) && fmt_ok(fmtB) ? mx::gemm_q_workspace_bound(M, N, K, fmtA, fmtB) : 0;
}

int mx_gemm_ws(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
               const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc,
               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return gemm_common(false, M, N, K, A_elems, A_scales, nullptr, 0, MX_ROUND_RNE, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc,
                       hip_stream, workspace, workspace_bytes);
}

int mx_gemm_qa_ws(int64_t M, int64_t N, int64_t K, const void *A_bf16, int64_t lda, mx_format_t fmtA, mx_round_t rnd,
                  const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc,
                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return gemm_common(true, M, N, K, nullptr, nullptr, A_bf16, lda, rnd, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc,
                       hip_stream, workspace, workspace_bytes);
}

int mx_gemm(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
            const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc,
            void *hip_stream)
{
    return gemm_common(false, M, N, K, A_elems, A_scales, nullptr, 0, MX_ROUND_RNE, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc,
                       hip_stream);
}

int mx_gemm_qa(int64_t M, int64_t N, int64_t K, const void *A_bf16, int64_t lda, mx_format_t fmtA, mx_round_t rnd,
               const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc,
               void *hip_stream)
{
    return gemm_common(true, M, N, K, nullptr, nullptr, A_bf16, lda, rnd, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc,
                       hip_stream);
}

static int gemm_q_common(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
                         const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, mx_format_t fmtC, mx_round_t rnd,
                         void *C_elems, uint8_t *C_scales, void *hip_stream, void *workspace, size_t workspace_bytes)
{
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB) || !fmt_ok(fmtC) || !rnd_ok(rnd)) return MX_ERR_ENUM;
    if (M < 0 || N < 0 || K < 0 || K % mx::BLOCK) return MX_ERR_SHAPE;
    if ((fmtA == MX_INT8) != (fmtB == MX_INT8)) return MX_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return MX_OK;
    if (!C_elems || !C_scales || (K > 0 && (!A_elems || !A_scales || !B_elems || !B_scales))) return MX_ERR_NULL;
    if (!aligned16(A_elems) || !aligned16(A_scales) || !aligned16(B_elems) || !aligned16(B_scales) || !aligned16(C_elems) ||
        !aligned16(C_scales))
        return MX_ERR_ALIGN;
    if (workspace) {
        if (!aligned16(workspace)) return MX_ERR_ALIGN;
        if (workspace_bytes < mx::gemm_q_workspace_bound(M, N, K, fmtA, fmtB)) return MX_ERR_WORKSPACE;
    }
    mx::WorkspaceScope scope(workspace, workspace_bytes);
    hipError_t e = mx::launch_gemm_q(M, N, K, static_cast<const uint8_t *>(A_elems), A_scales, fmtA,
                                     static_cast<const uint8_t *>(B_elems), B_scales, fmtB, static_cast<uint8_t *>(C_elems),
                                     C_scales, fmtC, rnd, static_cast<hipStream_t>(hip_stream));
    return gemm_status(e);
}

int mx_gemm_q(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
              const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, mx_format_t fmtC, mx_round_t rnd, void *C_elems,
              uint8_t *C_scales, void *hip_stream)
{
    return gemm_q_common(M, N, K, A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, fmtC, rnd, C_elems, C_scales, hip_stream, nullptr, 0);
}

int mx_gemm_q_ws(int64_t M, int64_t N, int64_t K, const void *A_elems, const uint8_t *A_scales, mx_format_t fmtA,
                 const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, mx_format_t fmtC, mx_round_t rnd, void *C_elems,
                 uint8_t *C_scales, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return gemm_q_common(M, N, K, A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, fmtC, rnd, C_elems, C_scales, hip_stream, workspace,
                         workspace_bytes);
}

// ---------------------------------------------------------------------------------------------
// mx_gemm_qa for callers that cannot allocate.  The MX form of A goes into a static device array
// instead of a pool workspace.  Host code never uses the array's name as an address: the address
// is looked up once per device with hipGetSymbolAddress and kept per device.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[MX_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<unsigned char *> scratch_ptr[MAX_DEVICES];

// device address of this device's copy of the array (nullptr on failure); the current device
// must be `dev`.  Looking the symbol up allocates nothing.
unsigned char *scratch_of(int dev)
{
    if (dev < 0 || dev >= MAX_DEVICES) return nullptr;
    unsigned char *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
        (void)hipGetLastError();
        return nullptr;
    }
    scratch_ptr[dev].store(static_cast<unsigned char *>(sym), std::memory_order_release);
    return static_cast<unsigned char *>(sym);
}
}  // namespace

int mx_gemm_qa_noalloc(int64_t M, int64_t N, int64_t K, const void *A_bf16, int64_t lda, mx_format_t fmtA, mx_round_t rnd,
                       const void *B_elems, const uint8_t *B_scales, mx_format_t fmtB, void *C, mx_dtype_t c_dt, int64_t ldc,
                       void *hip_stream)
{
    if (!fmt_ok(fmtA) || !fmt_ok(fmtB) || !dt_ok(c_dt) || !rnd_ok(rnd)) return MX_ERR_ENUM;
    if (M < 0 || N < 0 || K < 0 || K % mx::BLOCK || ldc < N || lda < K) return MX_ERR_SHAPE;
    if (fmtA == MX_INT8 || fmtB == MX_INT8) return MX_ERR_UNSUPPORTED;   // the MXINT8 routes take pool workspaces
    if (M == 0 || N == 0) return MX_OK;
    if (!C || (K > 0 && (!A_bf16 || !B_elems || !B_scales))) return MX_ERR_NULL;
    if (!aligned16(B_elems) || !aligned16(B_scales) || !aligned16(C) || !aligned16(A_bf16) || (lda * 2) % 16) return MX_ERR_ALIGN;
    // A as an MX tensor: element bytes (rounded up to 256), then scale bytes
    const size_t eb = ((size_t)M * (size_t)K * (size_t)mx::fmt_bits(fmtA) / 8 + 255) & ~(size_t)255;
    const size_t sbytes = (size_t)M * (size_t)(K / mx::BLOCK);
    if (eb + sbytes > (size_t)MX_NOALLOC_SCRATCH_BYTES) return MX_ERR_TOO_LARGE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (K == 0)
        return mx::launch_gemm(M, N, 0, nullptr, nullptr, nullptr, 0, MX_ROUND_RNE, fmtA, nullptr, nullptr, fmtB, C, c_dt, ldc, st) ==
                       hipSuccess ? MX_OK : MX_ERR_LAUNCH;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return MX_ERR_LAUNCH;
    unsigned char *ws = scratch_of(dev);
    if (!ws) return MX_ERR_LAUNCH;
    hipError_t e = mx::launch_cast(A_bf16, MX_DT_BF16, M, K, lda, 1, fmtA, rnd, ws, ws + eb, st);
    if (e == hipSuccess)
        e = mx::launch_gemm(M, N, K, ws, ws + eb, nullptr, 0, MX_ROUND_RNE, fmtA, static_cast<const uint8_t *>(B_elems), B_scales,
                            fmtB, C, c_dt, ldc, st);
    return e == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

const char *mx_strerror(int status)
{
    switch (status) {
        case MX_OK: return "ok";
        case MX_ERR_NULL: return "a required pointer is NULL";
        case MX_ERR_ENUM: return "format, rounding, dtype or axis out of range";
        case MX_ERR_SHAPE: return "bad shape: negative size, block axis not a multiple of 32, or leading dimension too small";
        case MX_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
        case MX_ERR_UNSUPPORTED: return "the GEMM pairs MX_INT8 only with MX_INT8";
        case MX_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case MX_ERR_WORKSPACE: return "scratch memory: the caller's workspace is too small, or the memory pool refused the request";
        case MX_ERR_TOO_LARGE: return "the problem needs more scratch memory than the entry point's static buffer holds";
        default: return "unknown status";
    }
}

}  // extern "C"
