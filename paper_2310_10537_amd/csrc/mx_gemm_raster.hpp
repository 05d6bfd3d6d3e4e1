// XCD-aware order of the output tiles of the LDS-tiled GEMM kernels (Section 4.1 of arXiv
// 2310.10537: the dot-product workload; the order decides how often operand slabs are re-read).
//
// Work-groups are dealt round-robin to the 8 XCDs, each with its own L2, and the first 32 an XCD
// receives run at the same time (one per compute unit), in step over K.  What such a group
// misses in its L2 per K step is one A slab per distinct tile row plus one B slab per distinct
// tile column, so the 32 tiles should form a patch that is as square as the operand widths ask:
// h rows x w columns costs h * bitsA + w * bitsB.  The 8 XCDs therefore share the tile grid as
// an xm x xn arrangement of regions (xm * xn = 8, regions of rm x rn tiles), and each XCD walks
// its region in bands of h tile rows, column by column.  The host picks (xm, h) with the least
// cost among the arrangements that divide the grid evenly; a grid that none divides is walked
// linearly (row-major, one eighth per XCD).
#pragma once

#include <hip/hip_runtime.h>

namespace mx {

struct Raster {
    int xn;       // regions per row of the XCD arrangement; 0: linear walk
    int rm, rn;   // tiles per region
    int h;        // tile rows per band
};

inline Raster choose_raster(int tiles_m, int tiles_n, int bits_a, int bits_b)
{
    Raster best = {0, 0, 0, 0};
    long best_cost = -1;
    for (int xm = 8; xm >= 1; xm >>= 1) {
        const int xn = 8 / xm;
        if (tiles_m % xm || tiles_n % xn) continue;
        const int rm = tiles_m / xm, rn = tiles_n / xn;
        for (int h = 1; h <= 32; h <<= 1) {
            if (rm % h) continue;
            const int per_band = 32 / h;                           // columns of a full patch
            const int cols = rn < per_band ? rn : per_band;
            int rows = h * ((32 + h * cols - 1) / (h * cols));     // a short band lets the group spill into the next one
            if (rows > rm) rows = rm;
            // cost per tile of the group, scaled to avoid fractions
            const long tiles = (long)rows * cols < 32 ? (long)rows * cols : 32;
            const long cost = ((long)rows * bits_a + (long)cols * bits_b) * 1024 / tiles;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = {xn, rm, rn, h}; }
        }
    }
    return best;
}

// number of work-groups to launch: 8 x (tiles per XCD)
inline unsigned raster_grid(const Raster &r, int tiles_m, int tiles_n)
{
    return r.xn ? 8u * (unsigned)(r.rm * r.rn) : 8u * (unsigned)((tiles_m * tiles_n + 7) / 8);
}

// tile of work-group b; false when b has none (the linear walk pads the grid to a multiple of 8)
__host__ __device__ __forceinline__ bool raster_tile(const Raster &r, int b, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int xcd = b & 7, idx = b >> 3;
    if (r.xn == 0) {
        const int n_tiles = tiles_m * tiles_n, per_xcd = (n_tiles + 7) >> 3;
        const int tile_id = xcd * per_xcd + idx;
        if (idx >= per_xcd || tile_id >= n_tiles) return false;
        tm = tile_id / tiles_n;
        tn = tile_id % tiles_n;
        return true;
    }
    if (idx >= r.rm * r.rn) return false;
    const int xr = xcd / r.xn, xc = xcd - xr * r.xn;
    const int band = r.h * r.rn;
    const int sub = idx / band, q = idx - sub * band;
    tm = xr * r.rm + sub * r.h + q % r.h;
    tn = xc * r.rn + q / r.h;
    return true;
}

}  // namespace mx
