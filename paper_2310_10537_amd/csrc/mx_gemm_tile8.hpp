// LDS-tiled MX GEMM (Section 4.1 of arXiv 2310.10537), eight-wave form: the 256 x 256 x 128 tile,
// the LDS layouts, the direct global-to-LDS staging and the XCD-aware tile order of
// mx_gemm_tile.hpp, but with 512 threads = 8 waves per work-group, each wave owning a 128 x 64
// sub-tile (4 x 2 matrix-instruction tiles, 128 accumulator registers).  Two waves then share
// every SIMD, so while one of them is held up issuing its direct loads, waiting at the barrier
// or waiting for LDS, the other keeps the matrix pipe fed.  The price is LDS traffic: a wave
// reads 4 + 2 operand fragments per 8 matrix instructions instead of 4 + 4 per 16.
// Measured against the four-wave kernel on one box (bf16 out, random operands): 6- and 4-bit
// pairs, whose K step holds half the matrix work of an 8-bit pair and which therefore wait more,
// gain 3-8 % (config 5: 254 / 220 / 210 -> 241 / 208 / 193 us); pairs with an 8-bit operand do
// not (115.1 -> 115.7 us on 8192 x 4096 x 4096, 417 -> 425 us on 8192^3): with real operands
// those run into the chip's power limit, not into issue stalls -- the same launch on all-zero
// operands takes 92 us.  So the dispatcher sends only pairs without an 8-bit operand here.
// Plain operands and Float32 / bf16 output only; quantize-on-load and the MX epilogue stay with
// the four-wave kernel.
//
// Half-width form (NW = 4): the same kernel with four waves and a 256 x 128 tile (two 64-column
// quarters), for every format pair.  A half tile costs about 0.6 of a whole one (it needs the whole A
// tile for half the products), so it pays where whole tiles leave most compute units idle: the last,
// partly filled round of a large problem, and problems of at most 128 tiles (launch_gemm_tiled
// decides).  An entry's K chain is the same in every form, so the results are bit-identical.
#pragma once

#include "mx_gemm_tile.hpp"

namespace mx {

template <int FA, int FB, int CDT, bool PROBE = false, int NW8 = 8>   // PROBE: as in the four-wave kernel; NW8: waves (8 or 4)
__global__ __launch_bounds__(64 * NW8, 1) void gemm_tile8_kernel(int64_t M, int64_t N, int64_t K,
                                                             const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                             const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                             void *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n, Raster rast,
                                                             unsigned long long *__restrict__ probe)
{
    unsigned long long probe_c0 = 0, probe_r0 = 0;
    if constexpr (PROBE) { probe_c0 = __builtin_readcyclecounter(); probe_r0 = __builtin_amdgcn_s_memrealtime(); }
    static_assert(CDT == DT_F32 || CDT == DT_BF16, "plain output types only");
    constexpr int WA = Fmt<FA>::bits, WB = Fmt<FB>::bits;
    typedef TileFmt<WA> TA;
    typedef TileFmt<WB> TB;
    static_assert(NW8 == 8 || NW8 == 4, "eight waves (256 x 256) or four (256 x 128)");
    constexpr int TNW = 32 * NW8;                        // tile width: 64 columns per pair of waves
    constexpr int A_BYTES = TM * TA::ROW, B_BYTES = TNW * TB::ROW, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int NSTAGE = (WA < 8 && WB < 8 && 3 * STAGE_BYTES + 2 * SCL_BYTES <= 160 * 1024) ? 3 : 2;
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES + 2 * SCL_BYTES];
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: everything derived from it stays in scalar registers
    const int wm = wave / (NW8 / 2), wn = wave % (NW8 / 2);   // 128-row half, 64-column quarter
    const int li = lane & 31, g = lane >> 5;

    // XCD-aware order of the tiles (mx_gemm_raster.hpp)
    int tm, tn;
    if (!raster_tile(rast, (int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int64_t m0 = (int64_t)tm * TM;
    const int64_t n0 = (int64_t)tn * TNW;
    const int64_t nkb = K / BLOCK;
    const int T = (int)(K / TK);
    const int Tfull = T & ~(SCL_GROUP - 1);

    // ---- staging map: wave w, load j fills LDS bytes (NW8 * j + w) * 1024 .. + 1023 of an operand tile
    const int a_r = WA == 4 ? lane >> 2 : lane >> 3, b_r = WB == 4 ? lane >> 2 : lane >> 3;
    const int a_u = WA == 4 ? (lane & 3) ^ ((a_r >> 2) & 3) : (lane & 7) ^ (((wave * 8 + a_r) >> 1) & 7);
    const int b_u = WB == 4 ? (lane & 3) ^ ((b_r >> 2) & 3) : (lane & 7) ^ (((wave * 8 + b_r) >> 1) & 7);
    const int64_t a_row_bytes = K * WA / 8, b_row_bytes = K * WB / 8;
    // A direct load takes a wave-uniform 64-bit base (scalar registers: tile origin, the wave's row group,
    // the K step, the load number) plus one 32-bit offset per lane that never changes (6-bit: one per load
    // number), so staging costs no vector arithmetic and two / four vector registers.
    const uint8_t *sA = WA == 6 ? Ae + m0 * a_row_bytes : Ae + (m0 + wave * TA::RPI) * a_row_bytes;
    const uint8_t *sB = WB == 6 ? Be + n0 * b_row_bytes : Be + (n0 + wave * TB::RPI) * b_row_bytes;
    const uint32_t vA = (uint32_t)(a_r * a_row_bytes + a_u * TA::UNIT), vB = (uint32_t)(b_r * b_row_bytes + b_u * TB::UNIT);
    constexpr int NJA = A_BYTES / (NW8 * 1024), NJB = B_BYTES / (NW8 * 1024);   // direct loads per wave per stage
    constexpr int N6A = WA == 6 ? NJA : 1, N6B = WB == 6 ? NJB : 1;   // 6-bit: one lane offset per load number
    uint32_t a6[N6A] = {}, b6[N6B] = {};
    if (WA == 6 || WB == 6) {
#pragma unroll
        for (int j = 0; j < (N6A > N6B ? N6A : N6B); j++) {
            const uint32_t q = (uint32_t)((NW8 * j + wave) * 64 + lane), row = q / 6, c = (q - row * 6) ^ ((row >> 3) & 1);
            if (WA == 6 && j < N6A) a6[j] = row * (uint32_t)a_row_bytes + c * 16;
            if (WB == 6 && j < N6B) b6[j] = row * (uint32_t)b_row_bytes + c * 16;
        }
    }
    const int st_l = wave * 1024;
    // ---- scale staging: 64 rows per wave-wide load, A's four groups then B's (TNW / 64); wave w takes
    // groups w and w + NW8 (eight waves: one each; four waves: A's group w, and B's for w < 2)
    constexpr int N_SCL = 4 + TNW / 64;
    auto scl_src = [&](int idx) { return idx < 4 ? As + (m0 + idx * 64) * nkb : Bs + (n0 + (idx - 4) * 64) * nkb; };
    const uint8_t *sS0 = scl_src(wave), *sS1 = scl_src(wave + NW8 < N_SCL ? wave + NW8 : wave);
    const uint32_t vS = (uint32_t)(lane * nkb);
    const int rsa = (wm * 128 + li) * 16, rsb = TM * 16 + (wn * 64 + li) * 16;
    const FragOfs<WA> ra0 = frag_ofs<WA>(wm * 128 + li, g);
    const FragOfs<WB> rb0 = frag_ofs<WB>(wn * 64 + li, g);

    v16f_t acc[4][2];
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 2; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][y][t] = 0.f;

    typedef __attribute__((address_space(3))) void lds_ptr_t;
    uint32_t sa[4], sb[2], sa_n[4], sb_n[2];
    v8i_t af[4], b0[2], b1[2];   // A fragments (one set, refilled in place), B fragments of sub-step 0 / 1

    auto stage_a1 = [&](int ts, uint8_t *dst, int j) {
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + st_l));
        const uint8_t *sp = WA == 6 ? sA + (int64_t)ts * (TK * WA / 8) : sA + (int64_t)ts * (TK * WA / 8) + j * (NW8 * TA::RPI) * a_row_bytes;
        const uint32_t vo = WA == 6 ? a6[j < N6A ? j : 0] : vA;
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(vo), "s"(sp), "s"(l0 + j * (NW8 * 1024)) : "m0");
    };
    auto stage_b1 = [&](int ts, uint8_t *dst, int j) {
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + st_l));
        const uint8_t *sp = WB == 6 ? sB + (int64_t)ts * (TK * WB / 8) : sB + (int64_t)ts * (TK * WB / 8) + j * (NW8 * TB::RPI) * b_row_bytes;
        const uint32_t vo = WB == 6 ? b6[j < N6B ? j : 0] : vB;
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(vo), "s"(sp), "s"(l0 + j * (NW8 * 1024)) : "m0");
    };
    auto stage_all = [&](int ts, uint8_t *dst) {
#pragma unroll
        for (int j = 0; j < NJA; j++) stage_a1(ts, dst, j);
#pragma unroll
        for (int j = 0; j < NJB; j++) stage_b1(ts, dst + A_BYTES, j);
    };
    static_assert(NJA + NJB <= 12, "the second half of a step has twelve slots for direct loads");
    // Three stages: a stage's buffer is free from the barrier of the step that read it until two steps later,
    // so its refill need not be crammed into the half step behind that barrier, where the eight waves' loads
    // together ask more of the load path than it gives (12 loads x 8 waves x 16 clocks against the 1024 clocks
    // of the half step).  The first NLY loads are requested there, the rest in the first half of the next step.
    constexpr int NL = NJA + NJB, NLY = NSTAGE == 3 ? (NL + 1) / 2 : NL;
    auto stage_one = [&](int k, int ts, uint8_t *dstA, uint8_t *dstB) {
        if (k < NJA) stage_a1(ts, dstA, k);
        else if (k - NJA < NJB) stage_b1(ts, dstB, k - NJA);
    };
    auto stage_y = [&](int k, int ts, uint8_t *dstA, uint8_t *dstB) {
        if (k < NLY) stage_one(k, ts, dstA, dstB);
    };
    uint8_t *const scl = lds + NSTAGE * STAGE_BYTES;
    const int n_groups = (T + SCL_GROUP - 1) / SCL_GROUP;
    auto scl_ofs = [&](int ts) { return ts < Tfull ? (ts & (SCL_GROUP - 1)) * 4 : (ts - (T - SCL_GROUP)) * 4; };
    auto stage_scales = [&](int G) {
        G = G < n_groups ? G : n_groups - 1;
        uint8_t *dst = scl + (G & 1) * SCL_BYTES;
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + wave * 1024));
        const int64_t src_ofs = G * SCL_GROUP + SCL_GROUP <= T ? (int64_t)G * 16 : (int64_t)T * 4 - 16;
        const uint8_t *p = sS0 + src_ofs;
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(vS), "s"(p), "s"(l0) : "m0");
        if (NW8 < N_SCL && wave + NW8 < N_SCL) {            // wave-uniform
            const uint8_t *p1 = sS1 + src_ofs;
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(vS), "s"(p1), "s"(l0 + NW8 * 1024) : "m0");
        }
    };
    // Scale bytes.  A row's 16-byte LDS slot holds the dwords of the four K steps of a scale group.  Reading
    // one dword per step from 32 consecutive slots conflicts four ways (16-byte pitch: 16 banks for 32 rows,
    // and the two half-waves do not merge), a quarter of this kernel's LDS cycles; so a group's slots are
    // read whole, 16 bytes per row block and conflict-free, once per group, and a step takes its dword from
    // registers.  The registers of a group are dead once the dwords of its last step have been taken (one
    // step ahead), which is when the next group's are read into them.
    u32x4_t qa4[4], qb4[2];
    auto read_group = [&](int ts) {          // the group holding K step ts (clamped to the last step)
        ts = ts < T ? ts : T - 1;
        const uint8_t *src = scl + ((ts / SCL_GROUP) & 1) * SCL_BYTES;
#pragma unroll
        for (int x = 0; x < 4; x++) qa4[x] = *reinterpret_cast<const u32x4_t *>(src + rsa + x * 512);
#pragma unroll
        for (int y = 0; y < 2; y++) qb4[y] = *reinterpret_cast<const u32x4_t *>(src + rsb + y * 512);
    };
    // dword d (0..3, a literal wherever the steps are unrolled) of the group in registers -> next step's scales
    auto take_scales = [&](int d) {
#pragma unroll
        for (int x = 0; x < 4; x++) {
            const uint32_t da = d == 0 ? qa4[x][0] : d == 1 ? qa4[x][1] : d == 2 ? qa4[x][2] : qa4[x][3];
            sa_n[x] = g ? da >> 8 : da;
        }
#pragma unroll
        for (int y = 0; y < 2; y++) {
            const uint32_t db = d == 0 ? qb4[y][0] : d == 1 ? qb4[y][1] : d == 2 ? qb4[y][2] : qb4[y][3];
            sb_n[y] = g ? db >> 8 : db;
        }
    };
    // The scales of step t+1, taken during step t = tt + h.  In the unrolled loop over whole groups (MAIN, h
    // a literal) the dword number is h + 1 for the first three steps; the fourth reads the group that step
    // tt + 4 belongs to (the next whole one, the partial last one, or -- behind the last step -- its own
    // again) and takes that step's dword, whose number only the run-time K decides.
    auto next_scales = [&](const int tt, const int h, const bool MAIN) __attribute__((always_inline)) {
        if (MAIN && h < SCL_GROUP - 1) {
            take_scales(h + 1);
        } else {
            const int ts = tt + h + 1 < T ? tt + h + 1 : T - 1;
            if (MAIN) read_group(ts);
            take_scales(scl_ofs(ts) >> 2);
        }
    };
#define MX8_FENCE() __builtin_amdgcn_sched_barrier(0)
#define MX8_MFMA(AF, BF, X, Y, OPS)                                                                                   \
    acc[X][Y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(AF[X], BF[Y], acc[X][Y], HA, HB, OPS, (int)sa[X], OPS, (int)sb[Y])

    // ---- prologue
    stage_scales(0);
    stage_all(0, lds);
    {
        const int t1 = T > 1 ? 1 : 0;
        stage_all(t1, lds + STAGE_BYTES);
        if (NSTAGE == 3) {      // stage 2: the share of the second half step; the first step brings the rest
#pragma unroll
            for (int k = 0; k < NLY; k++) stage_one(k, T > 2 ? 2 : T - 1, lds + 2 * STAGE_BYTES, lds + 2 * STAGE_BYTES + A_BYTES);
        }
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NSTAGE == 3 ? NL + NLY : NL) : "memory");
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; x++) af[x] = read_frag<WA>(lds, ra0, 0, x);
#pragma unroll
    for (int y = 0; y < 2; y++) b0[y] = read_frag<WB>(lds + A_BYTES, rb0, 0, y);
    read_group(0);
    take_scales(0);
#pragma unroll
    for (int x = 0; x < 4; x++) sa[x] = sa_n[x];
#pragma unroll
    for (int y = 0; y < 2; y++) sb[y] = sb_n[y];

    int ring = 0;
    auto k_step = [&](const int tt, const int h, const bool MAIN) __attribute__((always_inline)) {
        const int t = tt + h;
        const int cur = NSTAGE == 2 ? (h & 1) : ring;
        uint8_t *bufA = lds + cur * STAGE_BYTES;
        uint8_t *nxt = lds + (NSTAGE == 2 ? (cur ^ 1) : (cur == 2 ? 0 : cur + 1)) * STAGE_BYTES;
        uint8_t *bufB = bufA + A_BYTES;
        const int t2 = t + NSTAGE < T ? t + NSTAGE : T - 1;
        // three stages: the rest of stage t+2 goes into the buffer stage t-1 vacated at the previous barrier
        uint8_t *prvA = lds + (cur == 0 ? 2 : cur - 1) * STAGE_BYTES, *prvB = prvA + A_BYTES;
        const int t2x = t + 2 < T ? t + 2 : T - 1;
#define MX8_XLOAD(I) do { if (NSTAGE == 3) stage_one(NLY + (I), t2x, prvA, prvB); } while (0)
        MX8_FENCE();
        // ---- X: sub-step 0 (8 matrix instructions, A fragment by A fragment).  An A fragment is dead
        // after its two instructions and is refilled at once with the same rows of sub-step 1, so only
        // one set of A fragments is ever live; the two B fragments of sub-step 1 are read meanwhile.
        b1[0] = read_frag<WB>(bufB, rb0, 1, 0);
        MX8_XLOAD(0); MX8_MFMA(af, b0, 0, 0, 0); MX8_XLOAD(1); MX8_MFMA(af, b0, 0, 1, 0);
        af[0] = read_frag<WA>(bufA, ra0, 1, 0);
        MX8_FENCE();
        b1[1] = read_frag<WB>(bufB, rb0, 1, 1);
        MX8_XLOAD(2); MX8_MFMA(af, b0, 1, 0, 0); MX8_XLOAD(3); MX8_MFMA(af, b0, 1, 1, 0);
        af[1] = read_frag<WA>(bufA, ra0, 1, 1);
        MX8_FENCE();
        MX8_XLOAD(4); MX8_MFMA(af, b0, 2, 0, 0); MX8_XLOAD(5); MX8_MFMA(af, b0, 2, 1, 0);
        af[2] = read_frag<WA>(bufA, ra0, 1, 2);
        MX8_FENCE();
        MX8_MFMA(af, b0, 3, 0, 0); MX8_MFMA(af, b0, 3, 1, 0);
        af[3] = read_frag<WA>(bufA, ra0, 1, 3);
        MX8_FENCE();
#undef MX8_XLOAD
        // Stage t+1 must be in LDS, and every wave must have issued its last read of stage t,
        // before the buffers change roles.
        if (NSTAGE == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NJA + NJB) : "memory");
        __syncthreads();
        MX8_FENCE();
        // ---- Y: sub-step 1; stage t+NSTAGE is requested into the buffer stage t just vacated, one direct
        // load per matrix instruction, and the fragments of sub-step 0 of stage t+1 are read
        b0[0] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 0);
        // (stage_y: load k of the stage, if it belongs to this half step)
        stage_y(0, t2, bufA, bufB); stage_y(0 + 8, t2, bufA, bufB); MX8_MFMA(af, b1, 0, 0, 2); MX8_FENCE();
        stage_y(1, t2, bufA, bufB); stage_y(1 + 8, t2, bufA, bufB); MX8_MFMA(af, b1, 0, 1, 2);
        af[0] = read_frag<WA>(nxt, ra0, 0, 0);
        MX8_FENCE();
        b0[1] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 1);
        stage_y(2, t2, bufA, bufB); stage_y(2 + 8, t2, bufA, bufB); MX8_MFMA(af, b1, 1, 0, 2); MX8_FENCE();
        stage_y(3, t2, bufA, bufB); stage_y(3 + 8, t2, bufA, bufB); MX8_MFMA(af, b1, 1, 1, 2);
        af[1] = read_frag<WA>(nxt, ra0, 0, 1);
        MX8_FENCE();
        if (h == 0) stage_scales(tt / SCL_GROUP + 1);
        next_scales(tt, h, MAIN);
        stage_y(4, t2, bufA, bufB); MX8_MFMA(af, b1, 2, 0, 2); MX8_FENCE();
        stage_y(5, t2, bufA, bufB); MX8_MFMA(af, b1, 2, 1, 2);
        af[2] = read_frag<WA>(nxt, ra0, 0, 2);
        MX8_FENCE();
        stage_y(6, t2, bufA, bufB); MX8_MFMA(af, b1, 3, 0, 2); MX8_FENCE();
        stage_y(7, t2, bufA, bufB); MX8_MFMA(af, b1, 3, 1, 2);
        af[3] = read_frag<WA>(nxt, ra0, 0, 3);
        MX8_FENCE();
#pragma unroll
        for (int x = 0; x < 4; x++) sa[x] = sa_n[x];
#pragma unroll
        for (int y = 0; y < 2; y++) sb[y] = sb_n[y];
        if (NSTAGE == 3) ring = ring == 2 ? 0 : ring + 1;
        MX8_FENCE();
    };
    for (int tt = 0; tt < Tfull; tt += SCL_GROUP) {
#pragma unroll
        for (int h = 0; h < SCL_GROUP; h++) k_step(tt, h, true);
    }
#pragma unroll 1
    for (int h = 0; h < T - Tfull; h++) k_step(Tfull, h, false);
#undef MX8_MFMA
    if constexpr (PROBE) {
        if (threadIdx.x == 0) {
            probe[2 * blockIdx.x] = __builtin_readcyclecounter() - probe_c0;
            probe[2 * blockIdx.x + 1] = __builtin_amdgcn_s_memrealtime() - probe_r0;
        }
    }
#undef MX8_FENCE

    // ---- epilogue: lane (li, g), register t of tile (x, y) -> C[8*(t/4) + 4g + t%4][li]
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 2; y++) {
            const int64_t c = n0 + wn * 64 + y * 32 + li;
            if constexpr (CDT == DT_F32) {
#pragma unroll
                for (int t = 0; t < 16; t++) {
                    const int64_t r = m0 + wm * 128 + x * 32 + 8 * (t / 4) + 4 * g + (t % 4);
                    reinterpret_cast<float *>(C)[r * ldc + c] = acc[x][y][t];
                }
            } else {
                typedef float f32x2_t __attribute__((ext_vector_type(2)));
                typedef __bf16 bf16x2_t_ __attribute__((ext_vector_type(2)));
#pragma unroll
                for (int t = 0; t < 16; t += 2) {
                    const int64_t r = m0 + wm * 128 + x * 32 + 8 * (t / 4) + 4 * g + (t % 4);
                    const f32x2_t v = {acc[x][y][t], acc[x][y][t + 1]};
                    const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t_));
                    uint16_t *o = reinterpret_cast<uint16_t *>(C) + r * ldc + c;
                    o[0] = (uint16_t)pk;
                    o[ldc] = (uint16_t)(pk >> 16);
                }
            }
        }
    // The last steps requested stages beyond the end of K (clamped to the last one: harmless, branch-free);
    // those direct loads must have landed before this work-group's LDS is handed to another one.  The
    // epilogue above does not touch LDS, so the wait stands here, behind the stores, where it costs nothing.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int FA, int FB, int CDT, int NW = 8>
static hipError_t launch_t8(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint8_t *Be,
                            const uint8_t *Bs, void *C, int64_t ldc, hipStream_t st)
{
    auto kern = gemm_tile8_kernel<FA, FB, CDT, false, NW>;
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / (32 * NW));
    // (a half tile's B slab is half as heavy as its A slab)
    const Raster rast = choose_raster(tiles_m, tiles_n, Fmt<FA>::bits * 8, Fmt<FB>::bits * NW);
    hipLaunchKernelGGL(kern, dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(64 * NW), 0, st, M, N, K, Ae, As, Be, Bs, C, ldc, tiles_m, tiles_n,
                       rast, static_cast<unsigned long long *>(nullptr));
    return hipGetLastError();
}

template <int FA, int FB>
static hipError_t launch_pair8(const TileArgs &a)
{
    return a.c_dt == DT_F32 ? launch_t8<FA, FB, DT_F32>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st)
                            : launch_t8<FA, FB, DT_BF16>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st);
}

// the half-width form: 256 x 128 tiles, four waves, every format pair
template <int FA, int FB>
static hipError_t launch_pair_half(const TileArgs &a)
{
    return a.c_dt == DT_F32 ? launch_t8<FA, FB, DT_F32, 4>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st)
                            : launch_t8<FA, FB, DT_BF16, 4>(a.M, a.N, a.K, a.Ae, a.As, a.Be, a.Bs, a.C, a.ldc, a.st);
}

template <int FA>
static hipError_t launch_a_half(const TileArgs &a, int fmtB)
{
    switch (fmtB) {
        case FP8_E4M3: return launch_pair_half<FA, FP8_E4M3>(a);
        case FP8_E5M2: return launch_pair_half<FA, FP8_E5M2>(a);
        case FP6_E3M2: return launch_pair_half<FA, FP6_E3M2>(a);
        case FP6_E2M3: return launch_pair_half<FA, FP6_E2M3>(a);
        case FP4_E2M1: return launch_pair_half<FA, FP4_E2M1>(a);
        default:       return hipErrorNotSupported;
    }
}

template <int FA>
static hipError_t launch_a8w(const TileArgs &a, int fmtB)
{
    switch (fmtB) {
        case FP6_E3M2: return launch_pair8<FA, FP6_E3M2>(a);
        case FP6_E2M3: return launch_pair8<FA, FP6_E2M3>(a);
        case FP4_E2M1: return launch_pair8<FA, FP4_E2M1>(a);
        default:       return hipErrorNotSupported;
    }
}

}  // namespace mx
