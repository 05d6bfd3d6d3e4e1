// LDS-tiled MX GEMM for pairs of 8-bit formats on the 16 x 16 x 128 form of the block-scaled matrix
// instruction (Section 4.1: C[m,n] = sum_b X_A[m,b] X_B[n,b] sum_j a[m,32b+j] b[n,32b+j]).
//
// Same work-group tile (256 x 256, K step 128), LDS layout, direct loads, scale staging and raster as
// gemm_tile_kernel (mx_gemm_tile.hpp); what differs is the instruction and everything shaped by it.
// For 8-bit operands the 16 x 16 x 128 form does the same work per clock as the 32 x 32 x 64 form
// (32 clocks for half the flops) but needs less energy per flop, and on this chip an FP8 GEMM on real
// data runs at the board's power limit, so energy is time: from registers alone it sustains 9 % more
// than the 32 x 32 x 64 form on the same operand values.  One instruction adds the 128 products of an
// entry in the order of two chained 32 x 32 x 64 instructions -- passes of 16 K positions, increasing
// K -- with the same rounding (checked on the GPU against the instruction model over a million
// entries with random scales and accumulator inputs), so this kernel returns the same bits as the one
// it replaces.
//
// Register layout (one-hot probes): lane l, i = l % 16, q = l / 16.  Operand: dwords 0-3 hold K
// [16q, 16q+16), dwords 4-7 hold K [64+16q, +16) of row i; scale: byte for row i, block q.  Result
// register t holds D[4q + t][i], rows taken from the first operand.  The B fragment goes first, so a
// lane ends up with four consecutive columns of one row of C: one 8-byte (bf16) or 16-byte (Float32)
// store per instruction result.
//
// Pipeline.  A wave owns 128 x 128 = 8 x 8 instruction tiles and splits each K step into four
// quadrants of 16 instructions: (rows 0-63 | 64-127) x (columns 0-63 | 64-127).  A quadrant uses one
// set of four A fragments and one of four B fragments (32 registers each); there are four sets, aL, aH,
// bL, bH, and the quadrants of a step are walked so that consecutive quadrants share a set and the set
// that fell free is refilled for the quadrant after next:
//     even step:  (aL,bL) (aL,bH) | barrier | (aH,bH) (aH,bL)      reading  bH, aH | aL', bH'
//     odd step:   (aL,bH) (aL,bL) | barrier | (aH,bL) (aH,bH)      reading  bL, aH | aL', bL'
// (primed: of the next stage).  By the barrier every wave has issued its last read of the stage and
// the next stage has landed; behind it the stage after next is requested into the vacated buffer, one
// direct load per two instructions.
#pragma once
#include "mx_gemm_tile.hpp"

namespace mx {

typedef float v4f_t __attribute__((ext_vector_type(4)));

// One instruction, accumulator updated in place in the accumulation registers.  Written as assembly so that
// destination and addend are the same registers by construction: given the choice the register allocator
// assigns them apart and then rotates all 256 accumulator registers at the loop's back edge.  cbsz / blgp
// carry the formats of the first / second operand; both scale operands use byte 0 of their register.
template <int H1, int H2>
__device__ __forceinline__ void mfma16(v4f_t &acc, const v8i_t &op1, const v8i_t &op2, uint32_t s1, uint32_t s2)
{
    asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0,0,0] cbsz:%5 blgp:%6"
                 : "+a"(acc)
                 : "v"(op1), "v"(op2), "v"(s1), "v"(s2), "n"(H1), "n"(H2));
}

template <int FA, int FB, int CDT, bool PROBE = false>
__global__ __launch_bounds__(256, 1) void gemm_tile16_kernel(int64_t M, int64_t N, int64_t K,
                                                              const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                              const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                              void *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n, Raster rast,
                                                              unsigned long long *__restrict__ probe)
{
    unsigned long long probe_c0 = 0, probe_r0 = 0;
    if constexpr (PROBE) { probe_c0 = __builtin_readcyclecounter(); probe_r0 = __builtin_amdgcn_s_memrealtime(); }
    static_assert(Fmt<FA>::bits == 8 && Fmt<FB>::bits == 8, "pairs of 8-bit formats");
    static_assert(CDT == DT_F32 || CDT == DT_BF16, "plain output types only");
    typedef TileFmt<8> TF;
    constexpr int A_BYTES = TM * TF::ROW, B_BYTES = TN * TF::ROW, STAGE_BYTES = A_BYTES + B_BYTES;
    // {A tile, B tile} x two stages, then {A scale dwords, B scale dwords} x two groups
    // Scale bytes travel in groups of eight K steps: 32 bytes per row, fetched by two lanes, so a wave-wide
    // load touches 32 cache lines; each four-step trip of the loop below requests half of the next group's rows
    // (no branch in the loop: with one, the register allocator moves every accumulator at the back edge).  The load path's cost is per line, and with 16 bytes per row (64 lines
    // per load, one load pair per four steps) the scale loads took 260 clocks per K step, 9 % of the loop,
    // for 3 % of its bytes; the 160 KB of LDS have room for exactly this doubling, no more.
    constexpr int SG = 8, SG_ROW = 4 * SG, SG_BYTES = (TM + TN) * SG_ROW;
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE_BYTES + 2 * SG_BYTES];
    static_assert(sizeof(lds) <= 160 * 1024, "LDS of a compute unit");
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int i = lane & 15, q = lane >> 4;

    int tm, tn;
    if (!raster_tile(rast, (int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int64_t m0 = (int64_t)tm * TM, n0 = (int64_t)tn * TN;
    const int64_t nkb = K / BLOCK;
    const int T = (int)(K / TK);                  // K steps; at least 8
    const int Tfull = T & ~3;                     // the loop below takes four steps per trip
    const int Tg = T & ~(SG - 1);                 // steps in whole scale groups; the rest form a last, partial group

    // ---- staging map (as in gemm_tile_kernel): wave w, load j fills rows (4j + w) * 8 .. + 7; lane l
    // writes slot l % 8 of row l / 8 of that group and fetches the chunk the swizzle keeps there
    const int s_r = lane >> 3;
    const int s_u = (lane & 7) ^ (((wave * 8 + s_r) >> 1) & 7);
    const uint8_t *gA = Ae + (m0 + wave * TF::RPI + s_r) * K + s_u * TF::UNIT;
    const uint8_t *gB = Be + (n0 + wave * TF::RPI + s_r) * K + s_u * TF::UNIT;
    const int st_l = wave * 1024;
    // scale staging: wave w fetches the rows 64w .. 64w+63 of A and of B, 32 rows per load, lane l the
    // half l / 32 (steps 0-3 | 4-7 of the group) of row l % 32.  A load's 1 KB of LDS is therefore
    // [half][32 rows][16 bytes]: rows stay at a 16-byte pitch, as the byte reads below want them (at a
    // 32-byte pitch they cost three times the LDS cycles)
    const uint8_t *sA = As + (m0 + wave * 64 + (lane & 31)) * nkb + (lane >> 5) * 16;
    const uint8_t *sB = Bs + (n0 + wave * 64 + (lane & 31)) * nkb + (lane >> 5) * 16;
    // ---- operand reads: tile row wm*128 + 16x + i (A) / wn*128 + 16y + i (B), chunks q and q + 4
    const int ra0 = (wm * 128 + i) * 128 + ((q ^ ((i >> 1) & 7)) << 4);
    const int rb0 = (wn * 128 + i) * 128 + ((q ^ ((i >> 1) & 7)) << 4);
    // ---- scale reads: byte q of the step's dword of the same rows
    const int rsa = wm * 4096 + i * 16 + q, rsb = TM * SG_ROW + wn * 4096 + i * 16 + q;   // 16-row block x: + (x / 2) * 1024 + (x % 2) * 256

    v4f_t acc[8][8];
#pragma unroll
    for (int x = 0; x < 8; x++)
#pragma unroll
        for (int y = 0; y < 8; y++) acc[x][y] = v4f_t{0.f, 0.f, 0.f, 0.f};

    typedef __attribute__((address_space(3))) void lds_ptr_t;
    constexpr int NJ = A_BYTES / 4096;            // direct loads per wave per operand tile (1 KB each)
    // LDS address of this wave's 1 KB slot in the first A tile, as the scalar the direct loads put into M0
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)lds) + st_l;
    // (dst: byte offset of the destination tile inside the LDS array)
    auto stage_a1 = [&](int ts, int dst, int j) {
        const uint8_t *gp = gA + (int64_t)ts * TK + j * (4 * TF::RPI) * K;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gp), "s"(lds0 + dst + j * 4096) : "m0");
    };
    auto stage_b1 = [&](int ts, int dst, int j) {
        const uint8_t *gp = gB + (int64_t)ts * TK + j * (4 * TF::RPI) * K;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gp), "s"(lds0 + dst + j * 4096) : "m0");
    };
    // direct load number k of a stage: A's eight, then B's eight
    auto stage_one = [&](int k, int ts, int dstA, int dstB) {
        if (k < NJ) stage_a1(ts, dstA, k);
        else stage_b1(ts, dstB, k - NJ);
    };
    uint8_t *const scl = lds + 2 * STAGE_BYTES;
    const int n_groups = (T + SG - 1) / SG;
    // Byte offset of the scale dword of K step ts from that of the group's first step (same row).  The partial last group
    // is loaded as the row's LAST 32 scale bytes (steps T-8 .. T-1), so that the load never reaches past the
    // row, and its steps sit further back in the slot accordingly.
    auto scl_ofs = [&](int ts) {
        const int hh = ts < Tg ? (ts & (SG - 1)) : ts - (T - SG);      // position in the group, 0..7
        return (hh >> 2) * 512 + (hh & 3) * 4;
    };
    // scale bytes of K steps 8G .. 8G+7 (group G, clamped to the last) into slot G & 1, for the 32 rows j (0 / 1)
    // of this wave's 64 rows of A and of B
    auto stage_scales = [&](int G, int j) {
        G = G < n_groups ? G : n_groups - 1;
        const uint32_t l0 = lds0 + 2 * STAGE_BYTES + (G & 1) * SG_BYTES + wave * (64 * SG_ROW - 1024) + j * 1024;   // lds0 holds wave * 1024
        const int64_t src_ofs = (G * SG + SG <= T ? (int64_t)G * SG_ROW : (int64_t)T * 4 - SG_ROW) + j * 32 * nkb;
        const uint8_t *pa = sA + src_ofs, *pb = sB + src_ofs;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(pa), "s"(l0) : "m0");
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(pb), "s"(l0 + TM * SG_ROW) : "m0");
    };
    // fragment of 16-row block xb of the tile at buf
    auto frag = [&](const uint8_t *buf, int ofs, int xb) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(buf + ofs + xb * 2048);
        const uint4 hi = *reinterpret_cast<const uint4 *>(buf + (ofs ^ 64) + xb * 2048);
        return v8i_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };

    v8i_t aL[4], aH[4], bL[4], bH[4];
    // Scale bytes of the step, one register per 16-row block.  Each half of them (rows / columns 0-63,
    // 64-127) is refilled in place for the next step as soon as its last quadrant is over: no second set.
    uint32_t sa[8], sb[8];
    // byte offset, from the scale area, of the dword row 0 holds for K step ts (clamped to the last step)
    auto scale_ofs = [&](int ts) {
        ts = ts < T ? ts : T - 1;
        return ((ts / SG) & 1) * SG_BYTES + scl_ofs(ts);
    };
    auto read_sa = [&](int so, int x0) {
#pragma unroll
        for (int x = 0; x < 4; x++) sa[x0 + x] = scl[so + rsa + ((x0 + x) >> 1) * 1024 + ((x0 + x) & 1) * 256];
    };
    auto read_sb = [&](int so, int y0) {
#pragma unroll
        for (int y = 0; y < 4; y++) sb[y0 + y] = scl[so + rsb + ((y0 + y) >> 1) * 1024 + ((y0 + y) & 1) * 256];
    };

#define MX_FENCE() __builtin_amdgcn_sched_barrier(0)
    // instruction (x, y) of the wave's 8 x 8: B fragment first (see the header)
#define MX_MF(AS, BS, X0, Y0, XX, YY) mfma16<HB, HA>(acc[X0 + XX][Y0 + YY], BS[YY], AS[XX], sb[Y0 + YY], sa[X0 + XX])
    // a quadrant whose 16 instructions run beside the refill of set RS (four fragments, two per group of
    // four instructions, none in the last two groups) from tile RBUF at offset ROFS, blocks RB0 .. RB0+3
#define MX_QUAD_READ(AS, BS, X0, Y0, RS, RBUF, ROFS, RB0, EXTRA)                                                            \
    RS[0] = frag(RBUF, ROFS, RB0 + 0); RS[1] = frag(RBUF, ROFS, RB0 + 1);                                              \
    MX_MF(AS, BS, X0, Y0, 0, 0); MX_MF(AS, BS, X0, Y0, 1, 0); MX_MF(AS, BS, X0, Y0, 2, 0); MX_MF(AS, BS, X0, Y0, 3, 0); MX_FENCE(); \
    RS[2] = frag(RBUF, ROFS, RB0 + 2); RS[3] = frag(RBUF, ROFS, RB0 + 3);                                              \
    MX_MF(AS, BS, X0, Y0, 0, 1); MX_MF(AS, BS, X0, Y0, 1, 1); MX_MF(AS, BS, X0, Y0, 2, 1); MX_MF(AS, BS, X0, Y0, 3, 1); MX_FENCE(); \
    EXTRA;                                                                                                             \
    MX_MF(AS, BS, X0, Y0, 0, 2); MX_MF(AS, BS, X0, Y0, 1, 2); MX_MF(AS, BS, X0, Y0, 2, 2); MX_MF(AS, BS, X0, Y0, 3, 2); MX_FENCE(); \
    MX_MF(AS, BS, X0, Y0, 0, 3); MX_MF(AS, BS, X0, Y0, 1, 3); MX_MF(AS, BS, X0, Y0, 2, 3); MX_MF(AS, BS, X0, Y0, 3, 3); MX_FENCE()
    // the same with eight direct loads (numbers L0 .. L0+7 of stage TS into DA / DB), one per two
    // instructions: a burst would fill the memory pipeline's queue and stall the wave in front of its
    // next matrix instruction
#define MX_PAIR(AS, BS, X0, Y0, XX, YY, LK, TS, DA, DB)                                                                \
    stage_one(LK, TS, DA, DB); MX_MF(AS, BS, X0, Y0, XX, YY); MX_MF(AS, BS, X0, Y0, XX + 1, YY); MX_FENCE()
#define MX_QUAD_LOAD(AS, BS, X0, Y0, RS, RBUF, ROFS, RB0, L0, TS, DA, DB, EXTRA)                                       \
    RS[0] = frag(RBUF, ROFS, RB0 + 0); RS[1] = frag(RBUF, ROFS, RB0 + 1);                                              \
    MX_PAIR(AS, BS, X0, Y0, 0, 0, L0 + 0, TS, DA, DB); MX_PAIR(AS, BS, X0, Y0, 2, 0, L0 + 1, TS, DA, DB);              \
    RS[2] = frag(RBUF, ROFS, RB0 + 2); RS[3] = frag(RBUF, ROFS, RB0 + 3);                                              \
    MX_PAIR(AS, BS, X0, Y0, 0, 1, L0 + 2, TS, DA, DB); MX_PAIR(AS, BS, X0, Y0, 2, 1, L0 + 3, TS, DA, DB);              \
    EXTRA;                                                                                                             \
    MX_PAIR(AS, BS, X0, Y0, 0, 2, L0 + 4, TS, DA, DB); MX_PAIR(AS, BS, X0, Y0, 2, 2, L0 + 5, TS, DA, DB);              \
    MX_PAIR(AS, BS, X0, Y0, 0, 3, L0 + 6, TS, DA, DB); MX_PAIR(AS, BS, X0, Y0, 2, 3, L0 + 7, TS, DA, DB)

    // ---- prologue: stage 0 and the first scale group, then stage 1, on their way to LDS
    {
        const int t1 = T > 1 ? 1 : 0;
#pragma unroll
        for (int j = 0; j < NJ; j++) stage_b1(0, A_BYTES, j);
        stage_scales(0, 0);
        stage_scales(0, 1);
#pragma unroll
        for (int j = 0; j < NJ; j++) stage_a1(0, 0, j);
#pragma unroll
        for (int j = 0; j < NJ; j++) stage_a1(t1, STAGE_BYTES, j);
#pragma unroll
        for (int j = 0; j < NJ; j++) stage_b1(t1, STAGE_BYTES + A_BYTES, j);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NJ) : "memory");   // all but stage 1
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; x++) { aL[x] = frag(lds, ra0, x); bL[x] = frag(lds + A_BYTES, rb0, x); }
    read_sa(scale_ofs(0), 0); read_sa(scale_ofs(0), 4); read_sb(scale_ofs(0), 0); read_sb(scale_ofs(0), 4);

    // One K step; h is a literal at every call, so the parity of the step picks its half at compile time.
    // so / so1: scale_ofs of this step and of the next one
    auto k_step = [&](const int tt, const int h, const int so, const int so1) __attribute__((always_inline)) {
        const int t = tt + h;
        uint8_t *bufA = lds + (h & 1) * STAGE_BYTES, *bufB = bufA + A_BYTES;
        uint8_t *nxtA = lds + ((h & 1) ^ 1) * STAGE_BYTES, *nxtB = nxtA + A_BYTES;
        const int dA = (h & 1) * STAGE_BYTES, dB = dA + A_BYTES;   // where stage t+2 goes
        const int t2 = t + 2 < T ? t + 2 : T - 1;             // the stage requested during this step
        MX_FENCE();
        if ((h & 1) == 0) {
            MX_QUAD_READ(aL, bL, 0, 0, bH, bufB, rb0, 4, read_sa(so, 4); read_sb(so, 4));
            MX_QUAD_READ(aL, bH, 0, 4, aH, bufA, ra0, 4, (void)0);
        } else {
            MX_QUAD_READ(aL, bH, 0, 4, bL, bufB, rb0, 0, read_sa(so, 4); read_sb(so, 0));
            MX_QUAD_READ(aL, bL, 0, 0, aH, bufA, ra0, 4, (void)0);
        }
        // stage t+1 must be in LDS, and every wave must have finished its reads of stage t, before the
        // buffers change roles (the barrier waits for this wave's LDS reads as well)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        MX_FENCE();
        // (the scale bytes of the rows 0-63 and of the columns whose last quadrant of this step is the first
        // one behind the barrier are refilled for step t+1 in the last quadrant; the other halves follow in
        // the first quadrant of step t+1, see below)
        if ((h & 1) == 0) {
            MX_QUAD_LOAD(aH, bH, 4, 4, aL, nxtA, ra0, 0, 0, t2, dA, dB, if (h == 0) stage_scales(tt / SG + 1, (tt >> 2) & 1));
            MX_QUAD_LOAD(aH, bL, 4, 0, bH, nxtB, rb0, 4, 8, t2, dA, dB, read_sa(so1, 0); read_sb(so1, 4));
        } else {
            MX_QUAD_LOAD(aH, bL, 4, 0, aL, nxtA, ra0, 0, 0, t2, dA, dB, (void)0);
            MX_QUAD_LOAD(aH, bH, 4, 4, bL, nxtB, rb0, 0, 8, t2, dA, dB, read_sa(so1, 0); read_sb(so1, 0));
        }
        MX_FENCE();
    };
    // four steps per trip (the steps of the partial last group do not sit at consecutive offsets, so every
    // step's is worked out: scalar arithmetic, once per trip)
    for (int tt = 0; tt < Tfull; tt += 4) {
        const int so0 = scale_ofs(tt), so1 = scale_ofs(tt + 1), so2 = scale_ofs(tt + 2), so3 = scale_ofs(tt + 3), so4 = scale_ofs(tt + 4);
        k_step(tt, 0, so0, so1);
        k_step(tt, 1, so1, so2);
        k_step(tt, 2, so2, so3);
        k_step(tt, 3, so3, so4);
    }
    // the last one to three steps (Tfull is a multiple of four: the parity of a step is that of h)
    if (T - Tfull > 0) k_step(Tfull, 0, scale_ofs(Tfull), scale_ofs(Tfull + 1));
    if (T - Tfull > 1) k_step(Tfull, 1, scale_ofs(Tfull + 1), scale_ofs(Tfull + 2));
    if (T - Tfull > 2) k_step(Tfull, 2, scale_ofs(Tfull + 2), scale_ofs(Tfull + 3));
#undef MX_QUAD_LOAD
#undef MX_PAIR
#undef MX_QUAD_READ
#undef MX_MF
#undef MX_FENCE
    // The compiler does not know that the assembly above is matrix instructions, so it leaves no wait
    // states between the last of them (8 passes) and the first read of an accumulator register.  The
    // waits are written here, and every accumulator passes through a statement behind them (volatile
    // statements keep their order), so that no read of one can move in front.
#define MX_ACC_ROW(X)                                                                                                  \
    "+a"(acc[X][0]), "+a"(acc[X][1]), "+a"(acc[X][2]), "+a"(acc[X][3]), "+a"(acc[X][4]), "+a"(acc[X][5]), "+a"(acc[X][6]), "+a"(acc[X][7])
    asm volatile("s_nop 15\n\ts_nop 15" : MX_ACC_ROW(0), MX_ACC_ROW(1));
    asm volatile("" : MX_ACC_ROW(2), MX_ACC_ROW(3));
    asm volatile("" : MX_ACC_ROW(4), MX_ACC_ROW(5));
    asm volatile("" : MX_ACC_ROW(6), MX_ACC_ROW(7));
#undef MX_ACC_ROW
    if constexpr (PROBE) {
        if (threadIdx.x == 0) {
            probe[2 * blockIdx.x] = __builtin_readcyclecounter() - probe_c0;
            probe[2 * blockIdx.x + 1] = __builtin_amdgcn_s_memrealtime() - probe_r0;
        }
    }

    // ---- epilogue: lane (i, q), register t of instruction tile (x, y) -> C[16x + i][16y + 4q + t]: four
    // consecutive columns per lane, stored 16 bytes at a time where the row pitch keeps them aligned.  bf16
    // output uses the hardware's packed Float32 -> bf16 convert: round to nearest even, a NaN stays a NaN.
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t_ __attribute__((ext_vector_type(2)));
    auto pack2 = [](float lo, float hi) {
        const f32x2_t v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t_));
    };
    const int64_t r0 = m0 + wm * 128 + i, c0 = n0 + wn * 128 + 4 * q;
    if constexpr (CDT == DT_F32) {
        if ((ldc & 3) == 0) {
#pragma unroll
            for (int x = 0; x < 8; x++)
#pragma unroll
                for (int y = 0; y < 8; y++)
                    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(C) + (r0 + x * 16) * ldc + c0 + y * 16) =
                        make_float4(acc[x][y][0], acc[x][y][1], acc[x][y][2], acc[x][y][3]);
        } else {
#pragma unroll
            for (int x = 0; x < 8; x++)
#pragma unroll
                for (int y = 0; y < 8; y++) {
                    float *o = reinterpret_cast<float *>(C) + (r0 + x * 16) * ldc + c0 + y * 16;
                    o[0] = acc[x][y][0]; o[1] = acc[x][y][1]; o[2] = acc[x][y][2]; o[3] = acc[x][y][3];
                }
        }
    } else if ((ldc & 7) == 0) {
        // Four bf16 are 8 bytes per lane and 32 bytes per row and instruction.  Lanes q and q ^ 1 hold
        // neighbouring column groups of the same rows, so they trade: the even one hands over its four
        // columns of tile y + 1 and takes the odd one's of tile y (the row swap of the lane-permute unit
        // does exactly this exchange between 16-lane rows), and each stores 8 consecutive columns, 16
        // bytes -- 64 contiguous bytes per row and instruction, half as many instructions.
        const int64_t c1 = n0 + wn * 128 + 16 * (q & 1) + 4 * (q & 2);
#pragma unroll
        for (int x = 0; x < 8; x++)
#pragma unroll
            for (int y = 0; y < 8; y += 2) {
                const auto lo = __builtin_amdgcn_permlane16_swap(pack2(acc[x][y][0], acc[x][y][1]), pack2(acc[x][y + 1][0], acc[x][y + 1][1]), false, false);
                const auto hi = __builtin_amdgcn_permlane16_swap(pack2(acc[x][y][2], acc[x][y][3]), pack2(acc[x][y + 1][2], acc[x][y + 1][3]), false, false);
                *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(C) + (r0 + x * 16) * ldc + c1 + y * 16) = make_uint4(lo[0], hi[0], lo[1], hi[1]);
            }
    } else {
#pragma unroll
        for (int x = 0; x < 8; x++)
#pragma unroll
            for (int y = 0; y < 8; y++) {
                const uint32_t p0 = pack2(acc[x][y][0], acc[x][y][1]), p1 = pack2(acc[x][y][2], acc[x][y][3]);
                uint16_t *o = reinterpret_cast<uint16_t *>(C) + (r0 + x * 16) * ldc + c0 + y * 16;
                o[0] = (uint16_t)p0; o[1] = (uint16_t)(p0 >> 16); o[2] = (uint16_t)p1; o[3] = (uint16_t)(p1 >> 16);
            }
    }
    // The last steps requested stages beyond the end of K (clamped to the last one: harmless, branch-free);
    // those direct loads must have landed before this work-group's LDS is handed to another one.  The
    // epilogue above does not touch LDS, so the wait stands here, behind the stores, where it costs nothing.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int FA, int FB, int CDT>
static hipError_t launch_t16(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                             const uint8_t *Bs, void *C, int64_t ldc, hipStream_t st)
{
    auto kern = gemm_tile16_kernel<FA, FB, CDT>;
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
    const Raster rast = choose_raster(tiles_m, tiles_n, 8, 8);
    hipLaunchKernelGGL(kern, dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(256), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc, tiles_m, tiles_n,
                       rast, static_cast<unsigned long long *>(nullptr));
    return hipGetLastError();
}

}  // namespace mx
