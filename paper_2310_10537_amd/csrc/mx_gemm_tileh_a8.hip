// Half-width (256 x 128, four waves) LDS-tiled MX GEMM, A operand 8-bit: every B format.
#include "mx_gemm_tile8.hpp"

namespace mx {

hipError_t launch_gemm_tiledh_a8(const TileArgs &a, int fmtA, int fmtB)
{
    return fmtA == FP8_E4M3 ? launch_a_half<FP8_E4M3>(a, fmtB) : launch_a_half<FP8_E5M2>(a, fmtB);
}

}  // namespace mx
