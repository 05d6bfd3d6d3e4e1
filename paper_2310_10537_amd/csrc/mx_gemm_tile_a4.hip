// LDS-tiled MX GEMM, A operand FP4 (E2M1): every B format; and the entry point that picks the
// translation unit by A width.
#include "mx_gemm_tile.hpp"

namespace mx {

hipError_t launch_gemm_tiled_a4(const TileArgs &a, int, int fmtB) { return launch_a<FP4_E2M1>(a, fmtB); }

bool gemm_tiled_applies(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB)
{
    return fmtA >= FP8_E4M3 && fmtA <= FP4_E2M1 && fmtB >= FP8_E4M3 && fmtB <= FP4_E2M1 && M % TM == 0 && N % TN == 0 &&
           K % TK == 0 && K >= TK * SCL_GROUP && K <= (1 << 23) /* 32-bit byte offsets inside a tile */ && M > 0 && N > 0 &&
           (M / TM) * (N / TN) <= (1 << 24);
}

bool gemm_tiled_fuses_cast(int fmtA, int fmtB) { return fmtA <= FP8_E5M2 && fmtB <= FP8_E5M2; }

hipError_t launch_gemm_tiled(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const void *a_bf16,
                             int64_t lda, int rnd, int fmtA, const uint8_t *Be, const uint8_t *Bs, int fmtB, void *C,
                             int c_dt, int64_t ldc, hipStream_t st)
{
    if (!gemm_tiled_applies(M, N, K, fmtA, fmtB)) return hipErrorNotSupported;
    if (a_bf16 && !gemm_tiled_fuses_cast(fmtA, fmtB)) return hipErrorNotSupported;
    const TileArgs a{M, N, K, Ae, As, static_cast<const uint16_t *>(a_bf16), lda, rnd, Be, Bs, C, c_dt, ldc, st};
    switch (fmtA) {
        case FP8_E4M3: case FP8_E5M2: return launch_gemm_tiled_a8(a, fmtA, fmtB);
        case FP6_E3M2: case FP6_E2M3: return launch_gemm_tiled_a6(a, fmtA, fmtB);
        default:                      return launch_gemm_tiled_a4(a, fmtA, fmtB);
    }
}

}  // namespace mx
