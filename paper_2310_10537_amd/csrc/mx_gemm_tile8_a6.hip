// Eight-wave LDS-tiled MX GEMM, A operand 6-bit: every B format.
#include "mx_gemm_tile8.hpp"

namespace mx {

hipError_t launch_gemm_tiled8_a6(const TileArgs &a, int fmtA, int fmtB)
{
    (void)fmtA;
    return fmtA == FP6_E3M2 ? launch_a8w<FP6_E3M2>(a, fmtB) : launch_a8w<FP6_E2M3>(a, fmtB);
}

}  // namespace mx
