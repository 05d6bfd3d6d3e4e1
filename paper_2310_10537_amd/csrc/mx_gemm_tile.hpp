// LDS-tiled MX GEMM (Section 4.1 of arXiv 2310.10537) on gfx950's block-scaled
// 32x32x64 f8f6f4 matrix instruction, for every pair of FP8 / FP6 / FP4 formats.
//
// Work-group: 256 threads = 4 waves in a 2 x 2 arrangement, output tile
// 256 x 256, K step 128 (four MX blocks).  Each wave owns a 128 x 128 sub-tile:
// 4 x 4 matrix-instruction tiles of 32 x 32, i.e. 256 accumulator registers.
// Per K step the work-group stages 256 rows x 128 elements of A and of B in LDS
// (double buffered) with direct global-to-LDS loads (no register staging, no LDS
// store instructions: measured, the LDS pipe cannot carry the operand reads of
// this tile shape and store instructions as well).  A direct load writes its 64
// lanes to consecutive 16-byte LDS slots, so any layout that permutes 16-byte
// slots is free: the permutation is applied on the global side.
// LDS has 64 banks of 4 bytes (measured: a 16-byte wave read takes 4 clocks when each group
// of 16 lanes covers 256 distinct bytes, 8 clocks with the 32-bank swizzle c ^ (r & 7)).
//   8-bit: a row is 128 bytes = 8 slots, two rows per bank sweep; chunk c of
//          row r sits in slot c ^ ((r >> 1) & 7), so the operand reads (rows r ..
//          r+15, same chunk) touch 16 different 16-byte bank groups.  A lane's
//          operand is chunks {4s+g, 4s+g+2} of sub-step s.
//   6-bit: a row is 96 bytes = 6 slots and the tile is stored densely, row after
//          row (slot number 6r + c'), so that it takes 6 wave-wide loads per wave
//          instead of the 8 that 12-byte pieces in 16-byte slots would need --
//          the number of load instructions, not their bytes, is what limits this
//          kernel.  A wave-wide load then covers 10 2/3 rows: lane l of load
//          number n holds slot 64n + l and works out its row and chunk once.  A
//          lane's operand (one MX block, 24 bytes at byte 48s + 24g of the row) is
//          read as three 8-byte pieces.  The 32 rows of an operand read, 96 bytes
//          apart, would meet in 8 of the 16 bank groups; chunk c of row r sits in
//          slot c ^ ((r >> 3) & 1) of its row, which spreads them over all 16
//          (two rows per bank group is the minimum for 8-byte reads of one half).
//   4-bit: a row is 64 bytes = 4 slots, four rows per bank sweep, slot
//          c ^ ((r >> 2) & 3); a lane's operand is the single chunk 2s+g.
// Scale bytes travel the same way, four K steps at a time: a row's scale bytes
// for 512 elements are 16 consecutive bytes, so one 16-byte direct load per row
// brings four steps' worth and touches its cache line once instead of four
// times (a row's scales and its neighbours' are 128 bytes apart -- per-step
// dword loads doubled the number of L2 requests of the whole kernel).  Two such
// groups (256 + 256 rows x 16 bytes each) sit in LDS behind the element tiles.
// Lanes 32..63 shift their dword by one byte so that a single op_sel value
// addresses block 2*sub + g for every lane.
//
// Quantize-on-load (QA = true): the A operand arrives as raw bf16.  Each thread
// owns four MX blocks of a stage (lane l of wave w: tile row 16w + l/4 + 64p for
// p < 4, block l % 4 of the row's four), fetches them into registers during the
// second half of a step, casts them with the hardware converts of the stand-alone
// cast kernels during the first half of the next step and writes elements and
// scale bytes into the LDS stage that the B operand reaches by direct load.  The
// hot loop has no exact path: a block the converts cannot take (non-finite value,
// or a scale byte so small that Float32 subnormals matter) only raises a flag, and
// a work-group that saw one recomputes its whole tile afterwards, 32 x 32 tile by
// tile, with the exact cast of the direct kernel and in the same K order -- so the
// result is bit-identical to mx_quantize followed by mx_gemm either way.
#pragma once

#include "mx_convert.hpp"
#include "mx_gemm_frag.hpp"
#include "mx_gemm_raster.hpp"
#include "mx_launch.hpp"

namespace mx {

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));


constexpr int TM = 256, TN = 256, TK = 128;      // work-group tile (TK in elements)
constexpr int SCL_GROUP = 4;                     // K steps per scale group
constexpr int SCL_BYTES = (TM + TN) * 4 * SCL_GROUP;   // one group: 16 scale bytes per row

// How an operand of element width W travels through LDS.
template <int W> struct TileFmt;
template <> struct TileFmt<8> { static constexpr int ROW = 128, UNIT = 16, RPI = 8; };   // LDS bytes per row, global bytes per
template <> struct TileFmt<6> { static constexpr int ROW = 96, UNIT = 16, RPI = 0; };    // lane of a direct load, tile rows per
template <> struct TileFmt<4> { static constexpr int ROW = 64, UNIT = 16, RPI = 16; };   // wave-wide direct load (1 KB of LDS;
                                                                                         // 6-bit: 10 2/3 rows, see above)

// LDS byte offset of 16-byte chunk c (0..7) of tile row r, 8-bit operand
__device__ __forceinline__ int swz(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

// Where lane (li, g) finds its operand of tile row r (a multiple of 32 rows further down only adds
// a constant).  8- / 4-bit: the byte offset of the first slot for sub-step 0; the other slots follow
// by XOR.  6-bit: the byte offsets of the three 8-byte pieces of either sub-step.
template <int W> struct FragOfs { int o; };
template <> struct FragOfs<6> { int o[2][3]; };
template <int W>
__device__ __forceinline__ FragOfs<W> frag_ofs(int r, int g)
{
    FragOfs<W> f;
    if constexpr (W == 8) f.o = r * 128 + ((g ^ ((r >> 1) & 7)) << 4);
    else if constexpr (W == 4) f.o = r * 64 + ((g ^ ((r >> 2) & 3)) << 4);
    else {
#pragma unroll
        for (int s = 0; s < 2; s++)
#pragma unroll
            for (int k = 0; k < 3; k++) {
                const int t = 48 * s + 24 * g + 8 * k;          // byte of the row
                f.o[s][k] = r * 96 + (((t >> 4) ^ ((r >> 3) & 1)) << 4) + (t & 8);
            }
    }
    return f;
}

// One operand fragment: tile row block x (32 rows each), sub-step sub, from the tile at buf.
template <int W>
__device__ __forceinline__ v8i_t read_frag(const uint8_t *buf, const FragOfs<W> &f, int sub, int x)
{
    if constexpr (W == 8) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(buf + (f.o ^ (sub << 6)) + x * 4096);
        const uint4 hi = *reinterpret_cast<const uint4 *>(buf + (f.o ^ (sub << 6) ^ 32) + x * 4096);
        return v8i_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    } else if constexpr (W == 6) {
        const uint2 p0 = *reinterpret_cast<const uint2 *>(buf + f.o[sub][0] + x * 3072);
        const uint2 p1 = *reinterpret_cast<const uint2 *>(buf + f.o[sub][1] + x * 3072);
        const uint2 p2 = *reinterpret_cast<const uint2 *>(buf + f.o[sub][2] + x * 3072);
        return v8i_t{(int)p0.x, (int)p0.y, (int)p1.x, (int)p1.y, (int)p2.x, (int)p2.y, 0, 0};
    } else {
        const uint4 lo = *reinterpret_cast<const uint4 *>(buf + (f.o ^ (sub << 5)) + x * 2048);
        return v8i_t{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, 0, 0, 0, 0};
    }
}

// ---------------------------------------------------------------------------------------------
// Epilogue that writes C as an MX tensor (blocks of 32 along N): Algorithm 1 applied to the
// Float32 accumulators, i.e. the cast that would otherwise read C back from memory (Figure 2:
// the output of one MatMul is cast for the next).  An accumulator block -- one row of a 32 x 32
// matrix-instruction tile -- is spread over 32 lanes, so each wave passes its accumulators through
// a 32-row patch of LDS (free once the K loop is over) and gets whole blocks per lane back.
// ---------------------------------------------------------------------------------------------
constexpr int DT_MX = 2;                 // internal output kind next to DT_F32 / DT_BF16
constexpr int EP_PITCH = 544;            // bytes per patch row: 128 Float32 + 32 bytes, so that rows 4 apart
                                         // (the two halves of a wave) start 32 banks apart

// the same for a run-time format and rounding mode; stores the block (4 * bits bytes at dst, a
// multiple of 8) and returns the scale byte
template <int FMT, int RND>
__device__ __forceinline__ uint32_t quantize_store_block(const uint32_t *src, uint8_t *dst)
{
    constexpr int w = Fmt<FMT>::bits;
    uint32_t pk[w];
    const uint32_t s = quantize_block_lds<FMT, RND>(src, 1, pk);
    if constexpr (w == 8) {
        st16(dst, make_uint4(pk[0], pk[1], pk[2], pk[3]));
        st16(dst + 16, make_uint4(pk[4], pk[5], pk[6], pk[7]));
    } else if constexpr (w == 6) {
#pragma unroll
        for (int i = 0; i < 3; i++) *reinterpret_cast<uint2 *>(dst + 8 * i) = make_uint2(pk[2 * i], pk[2 * i + 1]);
    } else {
        st16(dst, make_uint4(pk[0], pk[1], pk[2], pk[3]));
    }
    return s;
}

__device__ __forceinline__ uint32_t quantize_store_block_rt(int fc, int rc, const uint32_t *src, uint8_t *dst)
{
#define MX_QS(F) (rc == ROUND_RNE ? quantize_store_block<F, ROUND_RNE>(src, dst) : quantize_store_block<F, ROUND_HALF_AWAY>(src, dst))
    switch (fc) {
        case FP8_E4M3: return MX_QS(FP8_E4M3);
        case FP8_E5M2: return MX_QS(FP8_E5M2);
        case FP6_E3M2: return MX_QS(FP6_E3M2);
        case FP6_E2M3: return MX_QS(FP6_E2M3);
        case FP4_E2M1: return MX_QS(FP4_E2M1);
        default:       return MX_QS(INT8);
    }
#undef MX_QS
}

// PROBE (measurement aid): thread 0 of every work-group also records how long it took from its start
// to the end of its K loop, in shader clocks and in ticks of the constant 100 MHz counter, at
// probe[2 * blockIdx.x] and [.. + 1]: what the shader clock was under this load, and how many
// clocks a K step took.
template <int FA, int FB, int CDT, bool QA, int RND, bool PROBE = false>
__global__ __launch_bounds__(256, 1) void gemm_tile_kernel(int64_t M, int64_t N, int64_t K,
                                                            const uint8_t *__restrict__ Ae, const uint8_t *__restrict__ As,
                                                            const uint16_t *__restrict__ Abf, int64_t lda,
                                                            const uint8_t *__restrict__ Be, const uint8_t *__restrict__ Bs,
                                                            void *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n,
                                                            uint8_t *__restrict__ Cs, int fcr, Raster rast,
                                                            unsigned long long *__restrict__ probe)
{
    unsigned long long probe_c0 = 0, probe_r0 = 0;
    if constexpr (PROBE) { probe_c0 = __builtin_readcyclecounter(); probe_r0 = __builtin_amdgcn_s_memrealtime(); }
    static_assert(!(QA && CDT == DT_MX), "the MX epilogue is built for plain operands");
    constexpr int WA = Fmt<FA>::bits, WB = Fmt<FB>::bits;
    static_assert(!QA || WA == 8, "the fused cast is written for 8-bit A operands");
    typedef TileFmt<WA> TA;
    typedef TileFmt<WB> TB;
    constexpr int A_BYTES = TM * TA::ROW, B_BYTES = TN * TB::ROW, STAGE_BYTES = A_BYTES + B_BYTES;
    // Stages in flight.  A stage is requested NSTAGE - 1 steps before it is read.  With 6- / 4-bit
    // operands a step holds only 1024 clocks of matrix instructions, less than the latency of a
    // load under this traffic, so two stages leave the matrix pipe waiting for memory every step;
    // wherever three stages fit in the 160 KB of LDS, three are used.
    // (measured: +9 % for a 6-bit x 4-bit pair, +1.5 % for 4 x 4; an 8-bit operand brings enough
    // matrix work per step, and such pairs ran 7 % slower with three stages)
    constexpr int NSTAGE = (!QA && WA < 8 && WB < 8 && 3 * STAGE_BYTES + 2 * SCL_BYTES <= 160 * 1024) ? 3 : 2;
    // {A tile, B tile} x NSTAGE stages, then {A scale dwords, B scale dwords} x two groups
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES + 2 * SCL_BYTES];
    constexpr int HA = hw_fmt(FA), HB = hw_fmt(FB);   // must reach the builtin as literal constants
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, g = lane >> 5;

    // XCD-aware order of the tiles (mx_gemm_raster.hpp)
    int tm, tn;
    if (!raster_tile(rast, (int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int64_t m0 = (int64_t)tm * TM;
    const int64_t n0 = (int64_t)tn * TN;
    const int64_t nkb = K / BLOCK;
    const int T = (int)(K / TK);          // K steps; at least 4
    const int Tfull = T & ~(SCL_GROUP - 1);   // steps in whole scale groups; the rest form a last, partial group

    // ---- staging map: one direct load of a wave fills 1 KB of LDS = RPI tile rows; wave w, load j
    // covers rows (4j + w) * RPI .. + RPI-1.  Lane l writes slot l % S of row l / S of that group
    // (S slots per row) and therefore fetches the unit that the layout keeps in that slot.
    // (tile row of the lane = a multiple of 32 rows + wave * RPI + a_r, which fixes the swizzle term)
    // (6-bit tiles are dense: lane l of the wave's load j holds slot (4j + wave) * 64 + l = 6 * row + c',
    // and fetches chunk c' ^ ((row >> 3) & 1) of that row; its byte offset from the tile's first row
    // differs from load to load, one register each)
    const int a_r = WA == 4 ? lane >> 2 : lane >> 3, b_r = WB == 4 ? lane >> 2 : lane >> 3;
    const int a_u = WA == 4 ? (lane & 3) ^ ((a_r >> 2) & 3) : (lane & 7) ^ (((wave * 8 + a_r) >> 1) & 7);
    const int b_u = WB == 4 ? (lane & 3) ^ ((b_r >> 2) & 3) : (lane & 7) ^ (((wave * 8 + b_r) >> 1) & 7);
    const int64_t a_row_bytes = K * WA / 8, b_row_bytes = K * WB / 8;
    const uint8_t *gA = QA ? nullptr : WA == 6 ? Ae + m0 * a_row_bytes : Ae + (m0 + wave * TA::RPI + a_r) * a_row_bytes + a_u * TA::UNIT;
    const uint8_t *gB = WB == 6 ? Be + n0 * b_row_bytes : Be + (n0 + wave * TB::RPI + b_r) * b_row_bytes + b_u * TB::UNIT;
    uint32_t a6[6] = {}, b6[6] = {};
    if (WA == 6 || WB == 6) {
#pragma unroll
        for (int j = 0; j < 6; j++) {
            const uint32_t q = (uint32_t)((4 * j + wave) * 64 + lane), row = q / 6, c = (q - row * 6) ^ ((row >> 3) & 1);
            if (WA == 6) a6[j] = row * (uint32_t)a_row_bytes + c * 16;
            if (WB == 6) b6[j] = row * (uint32_t)b_row_bytes + c * 16;
        }
    }
    const int st_l = wave * 1024;                  // LDS offset of this wave's 1 KB slot within a 4 KB group
    // ---- scale staging: wave w fetches the dwords of rows 64w .. 64w+63 of A and of B
    const uint8_t *sA = As + (m0 + wave * 64 + lane) * nkb;
    const uint8_t *sB = Bs + (n0 + wave * 64 + lane) * nkb;
    // ---- scale reads: dword of tile row wm*128 + 32x + li (A) / wn*128 + 32y + li (B)
    const int rsa = (wm * 128 + li) * 16, rsb = TM * 16 + (wn * 128 + li) * 16;
    // ---- operand read offsets inside a stage's tile (sub-step 0, row block 0)
    const FragOfs<WA> ra0 = frag_ofs<WA>(wm * 128 + li, g);
    const FragOfs<WB> rb0 = frag_ofs<WB>(wn * 128 + li, g);

    v16f_t acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++)
#pragma unroll
            for (int t = 0; t < 16; t++) acc[x][y][t] = 0.f;

    // Software pipeline (one work-group barrier per K step), buffer cur = t & 1 holds stage t:
    //   X : 16 MFMA of sub-step 0 | read a1[0..3], b1[0..3] (sub-step 1 of stage t)
    //   wait for the direct loads of stage t+1, barrier: every read of stage t was issued before it
    //   Y : 16 MFMA of sub-step 1 | request stage t+2 into the buffer stage t just vacated,
    //                               read a0[0..3], b0[0..3] (sub-step 0 of stage t+1)
    // Four LDS reads per four matrix instructions throughout, so the LDS pipe is loaded evenly.
    // LDS reads are written in program order between the matrix instructions and the compiler is
    // fenced group by group, so the LDS pipe and the matrix pipe work at the same time.
    // Stages beyond the last are clamped to the last one (harmless extra loads, no branches).
    typedef __attribute__((address_space(3))) void lds_ptr_t;
    uint32_t sa[4], sb[4];   // scale dwords of the current stage, already shifted for this lane
    uint32_t sa_n[4], sb_n[4];   // ... and of the next one, read early in the second half of a step
    v8i_t a0[4], a1[4], b0[4], b1[4];   // operand fragments of sub-step 0 / 1, double-buffered in time

    // Direct loads of one operand tile for K offset kofs into LDS tile dst.  Written as inline
    // assembly on purpose: the compiler makes every later LDS read wait for a direct load it knows
    // about (it cannot tell that the two stage buffers never overlap), which serialises the whole
    // pipeline.  Here the only consumer-side wait is the explicit vmcnt(0) before the barrier.
    // M0 carries the wave-uniform LDS destination; lane l lands at destination + 16 * l.
    constexpr int NJA = QA ? 0 : A_BYTES / 4096, NJB = B_BYTES / 4096;   // direct loads per wave per stage (1 KB each)
    auto stage_a1 = [&](int ts, uint8_t *dst, int j) {
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + st_l));
        const uint8_t *gp = WA == 6 ? gA + (int64_t)ts * (TK * WA / 8) + a6[j < 6 ? j : 0]
                                    : gA + (int64_t)ts * (TK * WA / 8) + j * (4 * TA::RPI) * a_row_bytes;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gp), "s"(l0 + j * 4096) : "m0");
    };
    auto stage_b1 = [&](int ts, uint8_t *dst, int j) {
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + st_l));
        const uint8_t *gp = WB == 6 ? gB + (int64_t)ts * (TK * WB / 8) + b6[j < 6 ? j : 0]
                                    : gB + (int64_t)ts * (TK * WB / 8) + j * (4 * TB::RPI) * b_row_bytes;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gp), "s"(l0 + j * 4096) : "m0");
    };
    auto stage_a = [&](int ts, uint8_t *dst) {
#pragma unroll
        for (int j = 0; j < NJA; j++) stage_a1(ts, dst, j);
    };
    auto stage_b = [&](int ts, uint8_t *dst) {
#pragma unroll
        for (int j = 0; j < NJB; j++) stage_b1(ts, dst, j);
    };
    // direct load number k of a stage (A's first, then B's), one per matrix instruction of the
    // second half of a step: a burst of them would fill the memory pipeline's queue and stall the
    // wave -- in-order issue -- in front of its next matrix instruction
    auto stage_one = [&](int k, int ts, uint8_t *dstA, uint8_t *dstB) {
        if (k < NJA) stage_a1(ts, dstA, k);
        else if (k - NJA < NJB) stage_b1(ts, dstB, k - NJA);
    };
    uint8_t *const scl = lds + NSTAGE * STAGE_BYTES;
    const int n_groups = (T + SCL_GROUP - 1) / SCL_GROUP;
    // Byte offset, inside a row's 16-byte LDS slot, of the scale dword of K step ts.  The partial
    // last group is loaded as the row's LAST 16 scale bytes (steps T-4 .. T-1), so that the load
    // never reaches past the row, and its steps sit further back in the slot accordingly.
    auto scl_ofs = [&](int ts) { return ts < Tfull ? (ts & (SCL_GROUP - 1)) * 4 : (ts - (T - SCL_GROUP)) * 4; };
    // scale bytes of K steps 4G .. 4G+3 (group G, clamped to the last) into slot G & 1: A rows, then B rows
    auto stage_scales = [&](int G) {
        G = G < n_groups ? G : n_groups - 1;
        uint8_t *dst = scl + (G & 1) * SCL_BYTES;
        const uint32_t l0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t *)(dst + wave * 1024));
        const int64_t src_ofs = G * SCL_GROUP + SCL_GROUP <= T ? (int64_t)G * 16 : (int64_t)T * 4 - 16;
        const uint8_t *pa = sA + src_ofs, *pb = sB + src_ofs;
        if (!QA) asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(pa), "s"(l0) : "m0");
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(pb), "s"(l0 + TM * 16) : "m0");
    };

    // ---- quantize-on-load of A: registers for the thread's four blocks of one stage
    u32x4_t qa[4][4];
    uint32_t bad = 0;   // set when a block of this thread cannot take the hardware converts
    const int q_row = wave * 16 + (lane >> 2), q_kb = lane & 3;
    const uint16_t *gQ = QA ? Abf + (m0 + q_row) * lda + q_kb * BLOCK : nullptr;
    // request the four blocks of pass p (tile row q_row + 64p) of K step ts.  Ordinary loads: the
    // compiler places their waits itself (the direct loads it cannot see only make them stricter).
    auto qa_request = [&](int ts, int p) {
        ts = ts < T ? ts : T - 1;
        const u32x4_t *gp = reinterpret_cast<const u32x4_t *>(gQ + (int64_t)ts * TK + (int64_t)p * 64 * lda);
#pragma unroll
        for (int i = 0; i < 4; i++) qa[p][i] = gp[i];
    };
    // cast pass p (already in registers) as K step ts and write it into the A tile `dst`
    auto qa_commit = [&](int ts, int p, uint8_t *dst) {
        uint32_t d[16], out[8];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            d[4 * i] = qa[p][i][0]; d[4 * i + 1] = qa[p][i][1]; d[4 * i + 2] = qa[p][i][2]; d[4 * i + 3] = qa[p][i][3];
        }
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < 16; i++) m = pk_absmax(m, d[i]);
        const uint32_t amax16 = pk_hmax(m);
        const uint32_t sbyte = scale_from_bf16_max<FA>(amax16);
        // an all-zero block is safe with any scale: the converts keep (signed) zero
        bad |= (uint32_t)(amax16 != 0 && !fast_ok(amax16, sbyte));
        // the converts clamp finite overflow to the largest normal only in saturate mode, and the
        // matrix instructions must not run in it (they would clamp NaN / Inf operands of B too)
        fp8_saturate_mode(true);
        convert_bf16_fast<FA, RND, 16>(d, sbyte, out);
        fp8_saturate_mode(false);
        const int r = q_row + 64 * p;
        *reinterpret_cast<uint4 *>(dst + swz(r, 2 * q_kb)) = make_uint4(out[0], out[1], out[2], out[3]);
        *reinterpret_cast<uint4 *>(dst + swz(r, 2 * q_kb + 1)) = make_uint4(out[4], out[5], out[6], out[7]);
        const int tsc = ts < T ? ts : T - 1;
        scl[((tsc / SCL_GROUP) & 1) * SCL_BYTES + r * 16 + scl_ofs(tsc) + q_kb] = (uint8_t)sbyte;
    };
    // scale dwords of K step ts for this lane's rows
    auto read_scales = [&](int ts) {
        ts = ts < T ? ts : T - 1;
        const uint8_t *src = scl + ((ts / SCL_GROUP) & 1) * SCL_BYTES + scl_ofs(ts);
#pragma unroll
        for (int x = 0; x < 4; x++) {
            const uint32_t da = *reinterpret_cast<const uint32_t *>(src + rsa + x * 512);
            const uint32_t db = *reinterpret_cast<const uint32_t *>(src + rsb + x * 512);
            sa_n[x] = g ? da >> 8 : da;
            sb_n[x] = g ? db >> 8 : db;
        }
    };
#define MX_FENCE() __builtin_amdgcn_sched_barrier(0)
#define MX_MFMA1(AF, BF, X, Y, OPS)                                                                                   \
    acc[X][Y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(AF[X], BF, acc[X][Y], HA, HB, OPS, (int)sa[X], OPS, (int)sb[Y])
#define MX_MFMA4(AF, BF, Y, OPS)                                                                                      \
    _Pragma("unroll") for (int x = 0; x < 4; x++)                                                                     \
        acc[x][Y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(AF[x], BF, acc[x][Y], HA, HB, OPS, (int)sa[x], OPS, (int)sb[Y])

    // ---- prologue: stage 0 (and the first scale group), then stages 1 .. NSTAGE-1, on their way
    // to LDS; the first half step only needs stage 0, so the others may stay in flight
    stage_b(0, lds + A_BYTES);
    stage_scales(0);
    {
        const int t1 = T > 1 ? 1 : 0;
        if (!QA) {
            stage_a(0, lds);
            stage_a(t1, lds + STAGE_BYTES);
            stage_b(t1, lds + STAGE_BYTES + A_BYTES);
            if (NSTAGE == 3) {
                const int t2 = T > 2 ? 2 : T - 1;
                stage_a(t2, lds + 2 * STAGE_BYTES);
                stage_b(t2, lds + 2 * STAGE_BYTES + A_BYTES);
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 1) * (NJA + NJB)) : "memory");   // all but the later stages
        } else {
            stage_b(t1, lds + STAGE_BYTES + A_BYTES);
#pragma unroll
            for (int p = 0; p < 4; p++) qa_request(0, p);
#pragma unroll
            for (int p = 0; p < 4; p++) qa_commit(0, p, lds);
#pragma unroll
            for (int p = 0; p < 4; p++) qa_request(1, p);   // committed during the first step
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; x++) { a0[x] = read_frag<WA>(lds, ra0, 0, x); b0[x] = read_frag<WB>(lds + A_BYTES, rb0, 0, x); }
    read_scales(0);
#pragma unroll
    for (int x = 0; x < 4; x++) { sa[x] = sa_n[x]; sb[x] = sb_n[x]; }

    // four K steps (one scale group) per trip, so that the scale request sits in a fixed place of
    // straight-line code (a branch inside the step would undo the interleaving)
    // (the body is a lambda so that the partial last group can run it with a run-time step index)
    int ring = 0;   // three stages: buffer of the current step (wave-uniform, run-time)
    auto k_step = [&](const int tt, const int h) __attribute__((always_inline)) {
        const int t = tt + h;
        const int cur = NSTAGE == 2 ? (h & 1) : ring;
        uint8_t *bufA = lds + cur * STAGE_BYTES;
        uint8_t *nxt = lds + (NSTAGE == 2 ? (cur ^ 1) : (cur == 2 ? 0 : cur + 1)) * STAGE_BYTES;
        uint8_t *bufB = bufA + A_BYTES;
        const int t2 = t + NSTAGE < T ? t + NSTAGE : T - 1;   // the stage requested during this step
        MX_FENCE();

        // ---- X: the 16 matrix instructions of sub-step 0; meanwhile all fragments of sub-step 1
        // are read, two fragments (four LDS reads) per group of four matrix instructions
        // Quantize-on-load: the registers hold stage t+1 of A (requested half a step ago); one
        // pass per group is cast and written to the other buffer, whose last readers passed the
        // previous barrier.
        a1[0] = read_frag<WA>(bufA, ra0, 1, 0); b1[0] = read_frag<WB>(bufB, rb0, 1, 0); a1[1] = read_frag<WA>(bufA, ra0, 1, 1);
        MX_MFMA4(a0, b0[0], 0, 0);
        if (QA) qa_commit(t + 1, 0, nxt);
        MX_FENCE();
        a1[2] = read_frag<WA>(bufA, ra0, 1, 2); a1[3] = read_frag<WA>(bufA, ra0, 1, 3); b1[1] = read_frag<WB>(bufB, rb0, 1, 1);
        MX_MFMA4(a0, b0[1], 1, 0);
        if (QA) qa_commit(t + 1, 1, nxt);
        MX_FENCE();
        b1[2] = read_frag<WB>(bufB, rb0, 1, 2); b1[3] = read_frag<WB>(bufB, rb0, 1, 3);
        MX_MFMA4(a0, b0[2], 2, 0);
        if (QA) qa_commit(t + 1, 2, nxt);
        MX_FENCE();
        // (no reads in the last group: the barrier below waits for every read of this half step)
        MX_MFMA4(a0, b0[3], 3, 0);
        if (QA) qa_commit(t + 1, 3, nxt);
        MX_FENCE();
        // Stage t+1 must be in LDS, and every wave must have issued its last read of stage t,
        // before the buffers change roles.  With three stages the loads issued during the previous
        // step (stage t+2: NJA + NJB of them, and at most the two scale loads in their midst, which
        // this count then forces to land early) may stay in flight: loads complete in order.
        if (NSTAGE == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NJA + NJB) : "memory");
        __syncthreads();
        MX_FENCE();

        // ---- Y: the 16 matrix instructions of sub-step 1; meanwhile stage t+NSTAGE is requested
        // into the buffer stage t just vacated and the sub-step-0 fragments of stage t+1 are read
#define MX_Y_GROUP(GRP, READ0, READ1, BF, Y)                                                                             \
    stage_one(4 * GRP + 0, t2, bufA, bufB); READ0; MX_MFMA1(a1, BF, 0, Y, 2); MX_FENCE();                                   \
    stage_one(4 * GRP + 1, t2, bufA, bufB);        MX_MFMA1(a1, BF, 1, Y, 2); MX_FENCE();                                   \
    stage_one(4 * GRP + 2, t2, bufA, bufB); READ1; MX_MFMA1(a1, BF, 2, Y, 2); MX_FENCE();                                   \
    stage_one(4 * GRP + 3, t2, bufA, bufB);        MX_MFMA1(a1, BF, 3, Y, 2); MX_FENCE()
        if (QA) { qa_request(t + 2, 0); qa_request(t + 2, 1); }
        MX_Y_GROUP(0, a0[0] = read_frag<WA>(nxt, ra0, 0, 0), b0[0] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 0), b1[0], 0);
        if (QA) { qa_request(t + 2, 2); qa_request(t + 2, 3); }
        MX_Y_GROUP(1, a0[1] = read_frag<WA>(nxt, ra0, 0, 1), a0[2] = read_frag<WA>(nxt, ra0, 0, 2), b1[1], 1);
        if (h == 0) stage_scales(tt / SCL_GROUP + 1);   // next group, once every four steps
        read_scales(t + 1);
        MX_Y_GROUP(2, a0[3] = read_frag<WA>(nxt, ra0, 0, 3), b0[1] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 1), b1[2], 2);
        MX_Y_GROUP(3, b0[2] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 2), b0[3] = read_frag<WB>(nxt + A_BYTES, rb0, 0, 3), b1[3], 3);
#undef MX_Y_GROUP
        // the next step's scales were read two groups ago (their LDS latency is long past)
#pragma unroll
        for (int x = 0; x < 4; x++) { sa[x] = sa_n[x]; sb[x] = sb_n[x]; }
        if (NSTAGE == 3) ring = ring == 2 ? 0 : ring + 1;
        MX_FENCE();
    };
    for (int tt = 0; tt < Tfull; tt += SCL_GROUP) {
#pragma unroll
        for (int h = 0; h < SCL_GROUP; h++) k_step(tt, h);
    }
#pragma unroll 1
    for (int h = 0; h < T - Tfull; h++) k_step(Tfull, h);
#undef MX_MFMA4
#undef MX_MFMA1
    // every direct load (the last, clamped, stages included) must have landed before this
    // work-group's LDS can be handed to another one
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (PROBE) {
        if (threadIdx.x == 0) {
            probe[2 * blockIdx.x] = __builtin_readcyclecounter() - probe_c0;
            probe[2 * blockIdx.x + 1] = __builtin_amdgcn_s_memrealtime() - probe_r0;
        }
    }
#undef MX_FENCE

    // ---- quantize-on-load: exact recomputation of the tile if any block needed the exact cast
    if constexpr (QA) {
        if (__syncthreads_or((int)bad)) {
#pragma unroll 1
            for (int sub = 0; sub < 16; sub++)
                direct_tile<FA, FB, true, RND, CDT>(M, N, K, nullptr, nullptr, Abf, lda, Be, Bs, C, ldc,
                                                    m0 + wm * 128 + (sub >> 2) * 32, n0 + wn * 128 + (sub & 3) * 32, lane);
            return;
        }
    }

    // ---- MX output: C = element bytes [M][N*bits/8], Cs = scale bytes [M][N/32]; fcr = format | rounding << 4
    if constexpr (CDT == DT_MX) {
        __syncthreads();   // every wave's direct loads have landed and its operand reads are over: LDS is free
        const int fc = fcr & 15, rc = fcr >> 4;
        const int wbits = fmt_bits(fc);
        uint32_t *patch = reinterpret_cast<uint32_t *>(lds + wave * (32 * EP_PITCH));   // 32 rows x 128 columns of this wave
        const int64_t c_row_bytes = N * wbits / 8, nsb = N / BLOCK;
        if (fc <= FP8_E5M2) fp8_saturate_mode(true);   // no matrix instruction follows
#pragma unroll
        for (int x = 0; x < 4; x++) {
#pragma unroll
            for (int y = 0; y < 4; y++)
#pragma unroll
                for (int t = 0; t < 16; t++)
                    patch[(8 * (t / 4) + 4 * g + (t % 4)) * (EP_PITCH / 4) + 32 * y + li] = __float_as_uint(acc[x][y][t]);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_wave_barrier();
#pragma unroll 1
            for (int p = 0; p < 2; p++) {
                const int bq = lane + 64 * p, row = bq >> 2, blk = bq & 3;   // four lanes write one 128-column run
                const int64_t gr = m0 + wm * 128 + x * 32 + row, gb = (n0 + wn * 128) / BLOCK + blk;
                const uint32_t sb = quantize_store_block_rt(fc, rc, patch + row * (EP_PITCH / 4) + blk * 32,
                                                            static_cast<uint8_t *>(C) + gr * c_row_bytes + gb * (4 * wbits));
                Cs[gr * nsb + gb] = (uint8_t)sb;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // all reads of the patch are over before it is written again
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }

    // ---- epilogue: lane (li, g), register t of tile (x, y) -> C[8*(t/4) + 4g + t%4][li].
    // (Sending bf16 output through an LDS patch, as the MX output does, so that it leaves with 16-byte
    // stores that fill whole lines, measured 4-5 % slower on three problem shapes than these 2-byte
    // stores in 64-byte runs: the transposition costs more than the store pattern gains.)
    // bf16 output uses the hardware's packed Float32 -> bf16 convert (round to nearest even, two
    // values per instruction): the integer formulation costs some 2000 vector instructions per
    // lane here, most of the epilogue.  A NaN stays a NaN (its payload is the hardware's choice).
#pragma unroll
    for (int x = 0; x < 4; x++)
#pragma unroll
        for (int y = 0; y < 4; y++) {
            const int64_t c = n0 + wn * 128 + y * 32 + li;
            if constexpr (CDT == DT_MX) {
            } else if constexpr (CDT == DT_F32) {
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
                    o[0] = (uint16_t)pk;            // rows r and r + 1
                    o[ldc] = (uint16_t)(pk >> 16);
                }
            }
        }
}

template <int FA, int FB, int CDT, bool QA, int RND>
static hipError_t launch_t(int64_t M, int64_t N, int64_t K, const uint8_t *Ae, const uint8_t *As, const uint16_t *Abf,
                           int64_t lda, const uint8_t *Be, const uint8_t *Bs, void *C, int64_t ldc, hipStream_t st,
                           uint8_t *Cs = nullptr, int fcr = 0)
{
    auto kern = gemm_tile_kernel<FA, FB, CDT, QA, RND>;
    const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
    const Raster rast = choose_raster(tiles_m, tiles_n, Fmt<FA>::bits, Fmt<FB>::bits);
    hipLaunchKernelGGL(kern, dim3(raster_grid(rast, tiles_m, tiles_n)), dim3(256), 0, st, M, N, K, Ae, As, Abf, lda, Be, Bs, C, ldc,
                       tiles_m, tiles_n, Cs, fcr, rast, static_cast<unsigned long long *>(nullptr));
    return hipGetLastError();
}

// Arguments of a tiled launch (Abf != nullptr: A is raw bf16, cast inside the kernel).
struct TileArgs {
    int64_t M, N, K;
    const uint8_t *Ae, *As;
    const uint16_t *Abf;
    int64_t lda;
    int rnd;
    const uint8_t *Be, *Bs;
    void *C;
    int c_dt;
    int64_t ldc;
    hipStream_t st;
    uint8_t *Cs = nullptr;   // c_dt == DT_MX: C receives element bytes, Cs scale bytes,
    int fcr = 0;             // in format fcr & 15 with rounding fcr >> 4
};

template <int FA, int FB>
static hipError_t launch_pair(const TileArgs &a)
{
#define MX_GO(QA_, RND_)                                                                                                  \
    (a.c_dt == DT_F32 ? launch_t<FA, FB, DT_F32, QA_, RND_>(a.M, a.N, a.K, a.Ae, a.As, a.Abf, a.lda, a.Be, a.Bs, a.C, a.ldc, a.st) \
                      : launch_t<FA, FB, DT_BF16, QA_, RND_>(a.M, a.N, a.K, a.Ae, a.As, a.Abf, a.lda, a.Be, a.Bs, a.C, a.ldc, a.st))
    if (a.c_dt == DT_MX)
        return a.Abf ? hipErrorNotSupported
                     : launch_t<FA, FB, DT_MX, false, ROUND_RNE>(a.M, a.N, a.K, a.Ae, a.As, nullptr, 0, a.Be, a.Bs, a.C, 0, a.st, a.Cs, a.fcr);
    if (!a.Abf) return MX_GO(false, ROUND_RNE);
    // the fused cast exists for 8-bit pairs only
    if constexpr (Fmt<FA>::bits == 8 && Fmt<FB>::bits == 8)
        return a.rnd == ROUND_RNE ? MX_GO(true, ROUND_RNE) : MX_GO(true, ROUND_HALF_AWAY);
    else
        return hipErrorNotSupported;
#undef MX_GO
}

// all B formats for one A format
template <int FA>
static hipError_t launch_a(const TileArgs &a, int fmtB)
{
    switch (fmtB) {
        case FP8_E4M3: return launch_pair<FA, FP8_E4M3>(a);
        case FP8_E5M2: return launch_pair<FA, FP8_E5M2>(a);
        case FP6_E3M2: return launch_pair<FA, FP6_E3M2>(a);
        case FP6_E2M3: return launch_pair<FA, FP6_E2M3>(a);
        case FP4_E2M1: return launch_pair<FA, FP4_E2M1>(a);
        default:       return hipErrorNotSupported;
    }
}

// one translation unit per A element width (the instantiations are many and compile in parallel)
hipError_t launch_gemm_tiled_a8(const TileArgs &a, int fmtA, int fmtB);
hipError_t launch_gemm_tiled_a6(const TileArgs &a, int fmtA, int fmtB);
hipError_t launch_gemm_tiled_a4(const TileArgs &a, int fmtA, int fmtB);
// pairs of 8-bit formats on the 16 x 16 x 128 instruction (mx_gemm_tile16.hpp; plain operands, Float32 / bf16 output)
hipError_t launch_gemm_tiled16_a8(const TileArgs &a, int fmtA, int fmtB);
// the eight-wave form of the kernel (plain operands, Float32 / bf16 output), same split
hipError_t launch_gemm_tiled8_a6(const TileArgs &a, int fmtA, int fmtB);
hipError_t launch_gemm_tiled8_a4(const TileArgs &a, int fmtA, int fmtB);
// the half-width form (256 x 128 tiles, four waves), plain operands, Float32 / bf16 output, every pair
hipError_t launch_gemm_tiledh_a8(const TileArgs &a, int fmtA, int fmtB);
hipError_t launch_gemm_tiledh_a6(const TileArgs &a, int fmtA, int fmtB);
hipError_t launch_gemm_tiledh_a4(const TileArgs &a, int fmtA, int fmtB);

}  // namespace mx
