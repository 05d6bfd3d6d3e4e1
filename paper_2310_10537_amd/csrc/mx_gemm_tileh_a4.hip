// Half-width (256 x 128, four waves) LDS-tiled MX GEMM, A operand 4-bit: every B format.
#include "mx_gemm_tile8.hpp"

namespace mx {

hipError_t launch_gemm_tiledh_a4(const TileArgs &a, int fmtA, int fmtB)
{
    (void)fmtA;
    return launch_a_half<FP4_E2M1>(a, fmtB);
}

}  // namespace mx
