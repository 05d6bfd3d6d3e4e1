// LDS-tiled MX GEMM, A operand FP6 (E3M2 / E2M3): every B format.
#include "mx_gemm_tile.hpp"

namespace mx {

hipError_t launch_gemm_tiled_a6(const TileArgs &a, int fmtA, int fmtB)
{
    return fmtA == FP6_E3M2 ? launch_a<FP6_E3M2>(a, fmtB) : launch_a<FP6_E2M3>(a, fmtB);
}

}  // namespace mx
