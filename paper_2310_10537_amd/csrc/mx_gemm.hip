// MX GEMM kernels (Section 4.1 of arXiv 2310.10537) on gfx950's block-scaled
// f8f6f4 matrix instruction:
//   C[m][n] = sum_b X_A[m][b] * X_B[n][b] * sum_j a[m][32b+j] * b[n][32b+j].
//
// V_MFMA_SCALE_F32_32X32X64_F8F6F4 register layout, established by one-hot and
// random-operand probes on the hardware (l = lane, i = l % 32, g = l / 32):
//   6- and 4-bit operands: lane l holds, for matrix row (A) / column (B) i, the
//     32 consecutive K elements [32g, 32g+32) densely bit-packed from bit 0
//     (FP6: 6 dwords, FP4: 4 dwords) -- one lane = one MX block;
//   8-bit operands: dwords 0-3 hold K [16g, 16g+16) and dwords 4-7 hold
//     K [32+16g, 32+16g+16), so a lane carries half of each of the two blocks;
//   scales: lane l supplies the E8M0 byte of row/column i, K block g (byte 0 of
//     the scale register with op_sel 0), whatever the element width;
//   result: lane l, register t holds C[8*(t/4) + 4*g + t%4][i].
// The 32x32x64 form is used for every format pair: it runs 6- and 4-bit pairs
// at twice the 8-bit rate, which the 16x16x128 form does not.
#include "mx_gemm_frag.hpp"
#include "mx_launch.hpp"

namespace mx {

// ---------------------------------------------------------------------------
// Workspace of the routes that need scratch memory (see mx_launch.hpp)
// ---------------------------------------------------------------------------
namespace {
struct WsState { uint8_t *base; size_t bytes, used; bool active; };
thread_local WsState g_ws = {nullptr, 0, 0, false};
size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }
}  // namespace

WorkspaceScope::WorkspaceScope(void *p, size_t bytes) { g_ws = {static_cast<uint8_t *>(p), bytes, 0, p != nullptr}; }
WorkspaceScope::~WorkspaceScope() { g_ws = {nullptr, 0, 0, false}; }

hipError_t ws_acquire(size_t bytes, hipStream_t st, uint8_t **out)
{
    *out = nullptr;
    if (g_ws.active) {
        const size_t need = up256(bytes);
        if (g_ws.used + need > g_ws.bytes) return hipErrorOutOfMemory;
        *out = g_ws.base + g_ws.used;
        g_ws.used += need;
        return hipSuccess;
    }
    const hipError_t e = hipMallocAsync(reinterpret_cast<void **>(out), bytes, st);
    if (e != hipSuccess) (void)hipGetLastError();
    return e;
}

hipError_t ws_release(uint8_t *p, hipStream_t st)
{
    if (g_ws.active) {
        g_ws.used = (size_t)(p - g_ws.base);     // pieces are released in reverse order of acquisition
        return hipSuccess;
    }
    return hipFreeAsync(p, st);
}

static size_t cast_ws_bytes(int64_t M, int64_t K, int fmtA)
{
    const size_t bits = fmtA == FP4_E2M1 ? 4 : (fmtA == FP6_E3M2 || fmtA == FP6_E2M3) ? 6 : 8;
    return up256((size_t)M * (size_t)K * bits / 8 + 16) + up256((size_t)M * (size_t)(K / BLOCK));
}

size_t gemm_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    if (fmtA != INT8 || fmtB != INT8 || M <= 0 || N <= 0 || K <= 0) return 0;
    return up256(256 + (size_t)(M + N) * (size_t)(K / BLOCK) * 100);      // the two E2M3 halves of both operands + scales
}

size_t gemm_qa_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return cast_ws_bytes(M, K, fmtA) + gemm_workspace_bound(M, N, K, fmtA, fmtB);
}

size_t gemm_q_workspace_bound(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    if (M <= 0 || N <= 0) return 0;
    return up256((size_t)M * (size_t)((N + 3) & ~(int64_t)3) * sizeof(float)) + gemm_workspace_bound(M, N, K, fmtA, fmtB);
}

// ---------------------------------------------------------------------------
// Direct kernel: operands go from global memory straight into MFMA registers.
// Work-group = 4 waves, each wave one 32 x 32 output tile, K step 64.
// Handles every shape (ragged M, N; K any multiple of 32).
// ---------------------------------------------------------------------------
template <int FA, int FB, bool QA, int RND, int CDT>
__global__ __launch_bounds__(256) void gemm_direct_kernel(int64_t M, int64_t N, int64_t K,
                                                          const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                          const uint16_t *__restrict__ Abf, int64_t lda,
                                                          const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                          void *__restrict__ C, int64_t ldc)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t m0 = (int64_t)blockIdx.y * 64 + (wave >> 1) * 32;
    const int64_t n0 = (int64_t)blockIdx.x * 64 + (wave & 1) * 32;
    direct_tile<FA, FB, QA, RND, CDT>(M, N, K, Ae, As, Abf, lda, Be, Bs, C, ldc, m0, n0, lane);
}

// ---------------------------------------------------------------------------
// Dispatch over (fmtA, fmtB, quantize-on-load, rounding, output type)
// ---------------------------------------------------------------------------
struct GemmArgs {
    int64_t M, N, K;
    const uint8_t *Ae, *As;
    const uint16_t *Abf;
    int64_t lda;
    const uint8_t *Be, *Bs;
    void *C;
    int64_t ldc;
    hipStream_t st;
};

template <int FA, int FB, bool QA, int RND, int CDT>
static hipError_t launch_direct(const GemmArgs &g)
{
    dim3 grid((unsigned)((g.N + 63) / 64), (unsigned)((g.M + 63) / 64));
    hipLaunchKernelGGL((gemm_direct_kernel<FA, FB, QA, RND, CDT>), grid, dim3(256), 0, g.st, g.M, g.N, g.K, g.Ae, g.As,
                       g.Abf, g.lda, g.Be, g.Bs, g.C, g.ldc);
    return hipGetLastError();
}

template <int FA, int FB>
static hipError_t dispatch_mode(const GemmArgs &g, int rnd, int c_dt)
{
    if (g.Abf) {
        if (rnd == ROUND_RNE)
            return c_dt == DT_F32 ? launch_direct<FA, FB, true, ROUND_RNE, DT_F32>(g)
                                  : launch_direct<FA, FB, true, ROUND_RNE, DT_BF16>(g);
        return c_dt == DT_F32 ? launch_direct<FA, FB, true, ROUND_HALF_AWAY, DT_F32>(g)
                              : launch_direct<FA, FB, true, ROUND_HALF_AWAY, DT_BF16>(g);
    }
    return c_dt == DT_F32 ? launch_direct<FA, FB, false, ROUND_RNE, DT_F32>(g)
                          : launch_direct<FA, FB, false, ROUND_RNE, DT_BF16>(g);
}

template <int FA>
static hipError_t dispatch_b(const GemmArgs &g, int fmtB, int rnd, int c_dt)
{
    switch (fmtB) {
        case FP8_E4M3: return dispatch_mode<FA, FP8_E4M3>(g, rnd, c_dt);
        case FP8_E5M2: return dispatch_mode<FA, FP8_E5M2>(g, rnd, c_dt);
        case FP6_E3M2: return dispatch_mode<FA, FP6_E3M2>(g, rnd, c_dt);
        case FP6_E2M3: return dispatch_mode<FA, FP6_E2M3>(g, rnd, c_dt);
        default:       return dispatch_mode<FA, FP4_E2M1>(g, rnd, c_dt);
    }
}

// Whether a problem goes to the kernel that shares the K range of 32 columns among eight waves
// rather than to 256 x 256 tiles: few rows of A (a decoding step), shapes that are not whole tiles,
// and so few tiles that most compute units would idle.  A tiled launch of fewer than 256 tiles
// takes as long as its K loop, about 0.0095 us per element of K; the other kernel runs at 400
// TFLOP/s on the whole chip (600 for long K).  Measured: 256 x 4096 x 4096 24 against 40 us, 256 x
// 4096 x 11008 40 against 104 us, 512 x 4096 x 11008 77 against 105 us; but 512 x 4096 x 4096 44
// against 42 us and 256 x 11008 x 4096 65 against 43 us.
static bool shares_k_among_waves(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    if (!gemm_skinny_applies(M, N, K, fmtA, fmtB)) return false;
    if (M <= 128 || !gemm_tiled_applies(M, N, K, fmtA, fmtB)) return true;
    const int64_t tiles = (M / 256) * (N / 256);
    return tiles < 32 || (tiles < 44 && K >= 8192);
}

// whether the fused quantize-on-load tiled kernel beats cast + plain tiled kernel (256 x 256 tiles)
static bool qa_fused_pays(int64_t M, int64_t N) { return N / 256 <= 2 && (M / 256) * (N / 256) >= 256; }

// one problem, one kernel route
static hipError_t launch_gemm_part(int64_t M, int64_t N, int64_t K, const uint8_t *A_elems, const uint8_t *A_scales,
                                   const void *a_bf16, int64_t lda, int rnd, int fmtA, const uint8_t *B_elems,
                                   const uint8_t *B_scales, int fmtB, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    if (fmtA == INT8 && fmtB == INT8) {
        if (!a_bf16) return launch_gemm_int8(M, N, K, A_elems, A_scales, B_elems, B_scales, C, c_dt, ldc, st);
        // quantize-on-load: cast A into a stream-ordered workspace first (the bytes mx_quantize writes)
        const size_t eb = (size_t)M * (size_t)K, sb = eb / BLOCK;
        if (eb == 0) return launch_gemm_int8(M, N, K, nullptr, nullptr, B_elems, B_scales, C, c_dt, ldc, st);
        uint8_t *ws = nullptr;
        hipError_t e = ws_acquire(eb + sb + 16, st, &ws);
        if (e != hipSuccess) return e;
        uint8_t *wss = ws + ((eb + 15) & ~(size_t)15);
        e = launch_cast(a_bf16, DT_BF16, M, K, lda, 1, INT8, rnd, ws, wss, st);
        if (e == hipSuccess) e = launch_gemm_int8(M, N, K, ws, wss, B_elems, B_scales, C, c_dt, ldc, st);
        const hipError_t f = ws_release(ws, st);
        return e != hipSuccess ? e : f;
    }
    // Quantize-on-load casts A into a workspace first (the bytes mx_quantize writes).
    if (shares_k_among_waves(M, N, K, fmtA, fmtB)) {
        if (!a_bf16) return launch_gemm_skinny(M, N, K, A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
        const size_t bits = fmtA <= FP8_E5M2 ? 8 : fmtA <= FP6_E2M3 ? 6 : 4;
        const size_t eb = ((size_t)M * (size_t)K * bits / 8 + 15) & ~(size_t)15, sb = (size_t)M * (size_t)K / BLOCK;
        uint8_t *ws = nullptr;
        hipError_t e = ws_acquire(eb + sb, st, &ws);
        if (e != hipSuccess) return e;
        e = launch_cast(a_bf16, DT_BF16, M, K, lda, 1, fmtA, rnd, ws, ws + eb, st);
        if (e == hipSuccess)
            e = launch_gemm_skinny(M, N, K, ws, ws + eb, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
        const hipError_t f = ws_release(ws, st);
        return e != hipSuccess ? e : f;
    }
    // Quantize-on-load on whole tiles.  The fused kernel casts each A tile once per column of
    // output tiles and reads it as bf16 that often, so it pays only for narrow outputs (measured:
    // up to two tile columns), and only when there are enough tiles to fill the chip, since the
    // stand-alone cast always runs on every compute unit.  Every other problem casts A once into
    // a stream-ordered workspace (the same cast kernel, hence the same bytes, as mx_quantize)
    // and runs the plain tiled kernel on it.
    if (a_bf16 && gemm_tiled_applies(M, N, K, fmtA, fmtB) && !(gemm_tiled_fuses_cast(fmtA, fmtB) && qa_fused_pays(M, N))) {
        const size_t bits = fmtA <= FP8_E5M2 ? 8 : fmtA <= FP6_E2M3 ? 6 : 4;
        const size_t eb = (size_t)M * (size_t)K * bits / 8, sb = (size_t)M * (size_t)K / BLOCK;
        uint8_t *ws = nullptr;
        hipError_t e = ws_acquire(eb + sb, st, &ws);
        if (e != hipSuccess) return e;
        e = launch_cast_bf16_fast(a_bf16, M, K, lda, 1, fmtA, rnd, ws, ws + eb, st);
        if (e == hipSuccess)
            e = launch_gemm_tiled(M, N, K, ws, ws + eb, nullptr, 0, rnd, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
        const hipError_t f = ws_release(ws, st);
        return e != hipSuccess ? e : f;
    }
    {
        hipError_t e = launch_gemm_tiled(M, N, K, A_elems, A_scales, a_bf16, lda, rnd, fmtA, B_elems, B_scales, fmtB, C,
                                         c_dt, ldc, st);
        if (e != hipErrorNotSupported) return e;
    }
    GemmArgs g{M, N, K, A_elems, A_scales, reinterpret_cast<const uint16_t *>(a_bf16), lda, B_elems, B_scales, C, ldc, st};
    switch (fmtA) {
        case FP8_E4M3: return dispatch_b<FP8_E4M3>(g, fmtB, rnd, c_dt);
        case FP8_E5M2: return dispatch_b<FP8_E5M2>(g, fmtB, rnd, c_dt);
        case FP6_E3M2: return dispatch_b<FP6_E3M2>(g, fmtB, rnd, c_dt);
        case FP6_E2M3: return dispatch_b<FP6_E2M3>(g, fmtB, rnd, c_dt);
        default:       return dispatch_b<FP4_E2M1>(g, fmtB, rnd, c_dt);
    }
}

// A problem whose M or N is not a multiple of the 256 x 256 tile is cut into the largest interior
// of whole tiles, which takes the tiled kernel, and an L-shaped fringe of fewer than 256 rows /
// columns, which takes the kernel for shapes that are not whole tiles (or the direct kernel when
// K is not a multiple of 128).  Every output entry is computed by exactly one launch; which one
// depends on the shape only, so a result is reproducible, and quantize-on-load follows the same cut.
hipError_t launch_gemm(int64_t M, int64_t N, int64_t K, const uint8_t *A_elems, const uint8_t *A_scales,
                       const void *a_bf16, int64_t lda, int rnd, int fmtA, const uint8_t *B_elems,
                       const uint8_t *B_scales, int fmtB, void *C, int c_dt, int64_t ldc, hipStream_t st)
{
    if (a_bf16 && rnd != ROUND_RNE && rnd != ROUND_HALF_AWAY && M * K > 0) {
        // the in-kernel casts round to nearest only: any other mode casts A into a workspace first
        const size_t bits = fmtA == FP4_E2M1 ? 4 : (fmtA == FP6_E3M2 || fmtA == FP6_E2M3) ? 6 : 8;
        const size_t eb = ((size_t)M * (size_t)K * bits / 8 + 15) & ~(size_t)15, sb = (size_t)M * (size_t)K / BLOCK;
        uint8_t *ws = nullptr;
        hipError_t e = ws_acquire(eb + sb, st, &ws);
        if (e != hipSuccess) return e;
        e = launch_cast(a_bf16, DT_BF16, M, K, lda, 1, fmtA, rnd, ws, ws + eb, st);
        if (e == hipSuccess)
            e = launch_gemm(M, N, K, ws, ws + eb, nullptr, 0, ROUND_RNE, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
        const hipError_t f = ws_release(ws, st);
        return e != hipSuccess ? e : f;
    }
    const int64_t M0 = M & ~(int64_t)255, N0 = N & ~(int64_t)255;
    // small ragged problems: one launch of the kernel for such shapes instead of three
    if (fmtA != INT8 && K % 128 == 0 && (M0 / 256) * (N0 / 256) < 32 && gemm_skinny_applies(M, N, K, fmtA, fmtB))
        return launch_gemm_part(M, N, K, A_elems, A_scales, a_bf16, lda, rnd, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
    if ((M0 == M && N0 == N) || M0 == 0 || N0 == 0 || fmtA == INT8 || !gemm_tiled_applies(M0, N0, K, fmtA, fmtB))
        return launch_gemm_part(M, N, K, A_elems, A_scales, a_bf16, lda, rnd, fmtA, B_elems, B_scales, fmtB, C, c_dt, ldc, st);
    const int64_t bitsA = fmtA <= FP8_E5M2 ? 8 : fmtA <= FP6_E2M3 ? 6 : 4, bitsB = fmtB <= FP8_E5M2 ? 8 : fmtB <= FP6_E2M3 ? 6 : 4;
    const int64_t nkb = K / BLOCK, esz = c_dt == DT_F32 ? 4 : 2;
    const uint8_t *a16 = static_cast<const uint8_t *>(a_bf16);
    auto part = [&](int64_t r0, int64_t rows, int64_t c0, int64_t cols) {
        return launch_gemm_part(rows, cols, K, A_elems ? A_elems + r0 * (K * bitsA / 8) : nullptr,
                                A_scales ? A_scales + r0 * nkb : nullptr, a16 ? a16 + r0 * lda * 2 : nullptr, lda, rnd, fmtA,
                                B_elems + c0 * (K * bitsB / 8), B_scales + c0 * nkb, fmtB,
                                static_cast<uint8_t *>(C) + (r0 * ldc + c0) * esz, c_dt, ldc, st);
    };
    hipError_t e = part(0, M0, 0, N0);
    if (e == hipSuccess && M > M0) e = part(M0, M - M0, 0, N);
    if (e == hipSuccess && N > N0) e = part(0, M0, N0, N - N0);
    return e;
}

// C as an MX tensor.  Whole-tile problems cast the accumulators in the tiled kernel's epilogue;
// every other problem (MXINT8 operands, truncated output) writes C as Float32 into a stream-ordered
// workspace and casts that -- the same accumulators and the same Algorithm 1, hence the same bytes.
hipError_t launch_gemm_q(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA, const uint8_t *Be,
                         const uint8_t *Bs, int fmtB, uint8_t *Ce, uint8_t *Cs, int fmtC, int rndC, hipStream_t st)
{
    // (only where mx_gemm runs the tiled kernel too: the two must see the same accumulators)
    if (fmtA != INT8 && !shares_k_among_waves(M, N, K, fmtA, fmtB)) {
        const hipError_t e = launch_gemm_tiled_mx(M, N, K, Ae, As, fmtA, Be, Bs, fmtB, Ce, Cs, fmtC, rndC, st);
        if (e != hipErrorNotSupported) return e;
    }
    float *ws = nullptr;
    const int64_t ldw = (N + 3) & ~(int64_t)3;   // rows of the workspace stay 16-byte aligned
    uint8_t *ws8 = nullptr;
    hipError_t e = ws_acquire((size_t)M * (size_t)ldw * sizeof(float), st, &ws8);
    if (e != hipSuccess) return e;
    ws = reinterpret_cast<float *>(ws8);
    e = launch_gemm(M, N, K, Ae, As, nullptr, 0, ROUND_RNE, fmtA, Be, Bs, fmtB, ws, DT_F32, ldw, st);
    if (e == hipSuccess) e = launch_cast(ws, DT_F32, M, N, ldw, 1, fmtC, rndC, Ce, Cs, st);
    const hipError_t f = ws_release(ws8, st);
    return e != hipSuccess ? e : f;
}

}  // namespace mx
