// LDS-tiled MX GEMM, A operand FP8 (E4M3 / E5M2): every B format, and the fused cast of a bf16 A.
#include "mx_gemm_tile.hpp"

namespace mx {

hipError_t launch_gemm_tiled_a8(const TileArgs &a, int fmtA, int fmtB)
{
    return fmtA == FP8_E4M3 ? launch_a<FP8_E4M3>(a, fmtB) : launch_a<FP8_E5M2>(a, fmtB);
}

}  // namespace mx
