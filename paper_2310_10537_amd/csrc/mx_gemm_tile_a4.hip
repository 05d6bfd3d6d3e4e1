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

// whole 256 x 256 tiles: four waves, on the 16 x 16 x 128 instruction for plain pairs of 8-bit formats with
// K >= 1024 (mx_gemm_tile16.hpp: its scale bytes travel in groups of eight K steps), or eight waves for pairs without an 8-bit operand (mx_gemm_tile8.hpp)
static hipError_t launch_whole(const TileArgs &a, int fmtA, int fmtB)
{
    if (!a.Abf && fmtA <= FP8_E5M2 && fmtB <= FP8_E5M2 && a.K >= 1024) return launch_gemm_tiled16_a8(a, fmtA, fmtB);
    if (!a.Abf && fmtA >= FP6_E3M2 && fmtB >= FP6_E3M2)
        return fmtA <= FP6_E2M3 ? launch_gemm_tiled8_a6(a, fmtA, fmtB) : launch_gemm_tiled8_a4(a, fmtA, fmtB);
    switch (fmtA) {
        case FP8_E4M3: case FP8_E5M2: return launch_gemm_tiled_a8(a, fmtA, fmtB);
        case FP6_E3M2: case FP6_E2M3: return launch_gemm_tiled_a6(a, fmtA, fmtB);
        default:                      return launch_gemm_tiled_a4(a, fmtA, fmtB);
    }
}

static hipError_t launch_half(const TileArgs &a, int fmtA, int fmtB)
{
    switch (fmtA) {
        case FP8_E4M3: case FP8_E5M2: return launch_gemm_tiledh_a8(a, fmtA, fmtB);
        case FP6_E3M2: case FP6_E2M3: return launch_gemm_tiledh_a6(a, fmtA, fmtB);
        default:                      return launch_gemm_tiledh_a4(a, fmtA, fmtB);
    }
}

hipError_t launch_gemm_tiled(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const void *a_bf16,
                             int64_t lda, int rnd, int fmtA, const uint8_t *Be, const uint8_t *Bs, int fmtB, void *C,
                             int c_dt, int64_t ldc, hipStream_t st)
{
    if (!gemm_tiled_applies(M, N, K, fmtA, fmtB)) return hipErrorNotSupported;
    if (a_bf16 && !gemm_tiled_fuses_cast(fmtA, fmtB)) return hipErrorNotSupported;
    const TileArgs a{M, N, K, Ae, As, static_cast<const uint16_t *>(a_bf16), lda, rnd, Be, Bs, C, c_dt, ldc, st};
    if (a_bf16) return launch_whole(a, fmtA, fmtB);
    // Whole tiles run in rounds of one per compute unit.  Where that leaves most of the chip idle, 256 x 128
    // half tiles (0.6 of a whole tile's time each) fill it better: a problem of at most 128 tiles, and the
    // last round of a larger one when it is at most half full -- the leading tile columns that make up whole
    // rounds go to the whole-tile kernel, the remaining columns to the half-tile kernel behind it.  (An
    // entry's K chain does not depend on the tile it lies in: same bits either way.)
    constexpr int64_t CUS = 256;
    const int64_t tiles_m = M / TM, tiles_n = N / TN, tiles = tiles_m * tiles_n;
    if (tiles <= CUS / 2) return launch_half(a, fmtA, fmtB);
    const int64_t rounds = tiles / CUS, rem = tiles % CUS;
    const int64_t lead = rounds * CUS / tiles_m;             // whole-tile columns
    if (rem == 0 || rem > CUS / 2 || lead < 1 || lead >= tiles_n) return launch_whole(a, fmtA, fmtB);
    const int wa = fmtA <= FP8_E5M2 ? 8 : fmtA <= FP6_E2M3 ? 6 : 4, wb = fmtB <= FP8_E5M2 ? 8 : fmtB <= FP6_E2M3 ? 6 : 4;
    (void)wa;
    const int64_t n1 = lead * TN, esz = c_dt == DT_F32 ? 4 : 2;
    TileArgs p1 = a, p2 = a;
    p1.N = n1;
    p2.N = N - n1;
    p2.Be = Be + n1 * (K * wb / 8);
    p2.Bs = Bs + n1 * (K / BLOCK);
    p2.C = static_cast<uint8_t *>(C) + n1 * esz;
    const hipError_t e = launch_whole(p1, fmtA, fmtB);
    return e != hipSuccess ? e : launch_half(p2, fmtA, fmtB);
}

// C written as an MX tensor by the kernel's epilogue: every element format, round to nearest
bool gemm_tiled_casts_output(int fmtC, int rndC)
{
    return fmtC >= FP8_E4M3 && fmtC <= INT8 && (rndC == ROUND_RNE || rndC == ROUND_HALF_AWAY);
}

hipError_t launch_gemm_tiled_mx(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, int fmtA,
                                const uint8_t *Be, const uint8_t *Bs, int fmtB, uint8_t *Ce, uint8_t *Cs, int fmtC, int rndC,
                                hipStream_t st)
{
    if (!gemm_tiled_applies(M, N, K, fmtA, fmtB) || !gemm_tiled_casts_output(fmtC, rndC)) return hipErrorNotSupported;
    TileArgs a{M, N, K, Ae, As, nullptr, 0, ROUND_RNE, Be, Bs, Ce, DT_MX, 0, st};
    a.Cs = Cs;
    a.fcr = fmtC | (rndC << 4);
    switch (fmtA) {
        case FP8_E4M3: case FP8_E5M2: return launch_gemm_tiled_a8(a, fmtA, fmtB);
        case FP6_E3M2: case FP6_E2M3: return launch_gemm_tiled_a6(a, fmtA, fmtB);
        default:                      return launch_gemm_tiled_a4(a, fmtA, fmtB);
    }
}

}  // namespace mx
