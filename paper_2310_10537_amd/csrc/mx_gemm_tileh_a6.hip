// Half-width (256 x 128, four waves) LDS-tiled MX GEMM, A operand 6-bit: every B format.
#include "mx_gemm_tile8.hpp"

namespace mx {

hipError_t launch_gemm_tiledh_a6(const TileArgs &a, int fmtA, int fmtB)
{
    return fmtA == FP6_E3M2 ? launch_a_half<FP6_E3M2>(a, fmtB) : launch_a_half<FP6_E2M3>(a, fmtB);
}

}  // namespace mx
