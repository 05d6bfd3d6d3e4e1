// LDS-tiled MX GEMM on the 16 x 16 x 128 matrix instruction: both operands FP8 (E4M3 / E5M2), Float32 / bf16 output.
#include "mx_gemm_tile16.hpp"

namespace mx {

template <int FA, int FB>
static hipError_t launch_pair16(const TileArgs &a)
{
    return a.c_dt == DT_F32 ? launch_t16<FA, FB, DT_F32>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st)
                            : launch_t16<FA, FB, DT_BF16>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st);
}

hipError_t launch_gemm_tiled16_a8(const TileArgs &a, int fmtA, int fmtB)
{
    if (a.Abf || (a.c_dt != DT_F32 && a.c_dt != DT_BF16) || a.K < 1024) return hipErrorNotSupported;
    if (fmtA == FP8_E4M3) return fmtB == FP8_E4M3 ? launch_pair16<FP8_E4M3, FP8_E4M3>(a) : launch_pair16<FP8_E4M3, FP8_E5M2>(a);
    return fmtB == FP8_E4M3 ? launch_pair16<FP8_E5M2, FP8_E4M3>(a) : launch_pair16<FP8_E5M2, FP8_E5M2>(a);
}

}  // namespace mx
