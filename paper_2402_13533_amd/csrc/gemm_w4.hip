// Four-wave bf16 GEMM for gfx950: 256 x 256 workgroup tile, one wave per SIMD, each wave
// owning a 128 x 128 block of the output in 256 accumulator registers.
//
// Why this shape.  A compute unit retires one 32x32x16 MFMA per SIMD every 32 cycles at best.
// With a 128 x 128 wave tile a 16-deep k slice costs 8 fragment reads (8 KiB) for 16 matrix
// instructions, i.e. 64 B/clk of LDS reads per CU at full matrix rate, plus 32 B/clk of
// global -> LDS writes for a 256 x 256 tile: three quarters of the 128 B/clk the LDS can
// move.  Any tile with half the area (or 128 x 64 wave tiles) needs more than the LDS has.
//
// Schedule.  K tiles of depth 32 travel through a ring of NS LDS stages filled by
// global -> LDS requests that bypass the register file.  Each wave software-pipelines its own
// work: while the 16 matrix instructions of one k slice issue, the fragments of the next
// slice are read from LDS into the other half of a double buffer and requests for the K tile
// NS ahead are posted, one memory instruction per matrix instruction.  One workgroup barrier
// per K tile (between its two slices) publishes the next tile and releases the stage of the
// current one.
#include "gemm_bf16.h"
#include "gemm_ring.h"
#include "profile.h"

#include <stdio.h>

namespace fhpc {
namespace w4 {

using namespace ring;

constexpr int NT = 256;

template <int NS, int A_MODE, int B_MODE, int OUT_MODE>
__global__ __launch_bounds__(NT) void gemm_w4_kernel(GemmArgs p)
{
    constexpr int BM = 256, BN = 256, BK = 32;
    constexpr int TM = 4, TN = 4;                              // 32 x 32 blocks per wave: 128 x 128
    constexpr int WTM = 128, WTN = 128;
    using FA = Feeder<A_MODE, BM, BK, 4>;
    using FB = Feeder<B_MODE, BN, BK, 4>;
    using TA = typename FA::Tile;
    using TB = typename FB::Tile;
    constexpr int TILE_A_BYTES = FA::TILE_BYTES, STAGE_BYTES = FA::TILE_BYTES + FB::TILE_BYTES;
    constexpr int L = FA::PER + FB::PER;                       // requests per wave per K tile
    static_assert(L == 8, "eight requests per wave per K tile");
    static_assert(NS * STAGE_BYTES <= 160 * 1024, "LDS ring");

    __shared__ __attribute__((aligned(1024))) unsigned char lds[NS * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m0 = (wave >> 1) * WTM;
    const int wave_n0 = (wave & 1) * WTN;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    int tm, tn, split;
    work_coords(blockIdx.x, tiles_m, tiles_n, p.splits > 1 ? p.splits : 1, tm, tn, split);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][i][v] = 0.f;

    const int kbeg = split * p.k_chunk;
    const int kend = (kbeg + p.k_chunk < p.K) ? kbeg + p.k_chunk : p.K;
    if (kbeg < kend) {
        FA fa;
        FB fb;
        fa.init(p.a, m0, p.M, p.K, wave, lane);
        fb.init(p.b, n0, p.N, p.K, wave, lane);
        const int kld = FHPC_DBG_NO_LOADS(p) ? kbeg : kend;             // diagnostics: nothing is in range
        const FragAddr aa = TA::make(wave_m0, lane);
        const FragAddr ab = TB::make(wave_n0, lane);

        // prologue: K tiles 0 .. NS-2 whole and the first half of tile NS-1's requests (the
        // loop posts every tile in two halves, see below)
#pragma unroll
        for (int u = 0; u < NS - 1; u++) {
            fa.issue(lds + u * STAGE_BYTES, kbeg + u * BK, kld, wave);
            fb.issue(lds + u * STAGE_BYTES + TILE_A_BYTES, kbeg + u * BK, kld, wave);
        }
        fa.issue(lds + (NS - 1) * STAGE_BYTES, kbeg + (NS - 1) * BK, kld, wave);
        static_assert(FA::PER == 4, "the first half of a tile's requests is its A part");
        FHPC_WAIT_VM((NS - 2) * L + 4);
        wg_barrier();

        bf16x8 ra[2][TM], rb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; i++) ra[0][i] = TA::frag(lds, aa, i, 0);
#pragma unroll
        for (int j = 0; j < TN; j++) rb[0][j] = TB::frag(lds + TILE_A_BYTES, ab, j, 0);

        // Fragment q of a k slice in the order the matrix instructions first need them:
        // B0 A0 A1 A2 A3 B1 B2 B3 (the instructions run j-major over acc[j][i]).
#define FHPC_READ(BUF, STAGE_PTR, SLICE, Q)                                                          \
    {                                                                                                \
        if ((Q) == 0) rb[BUF][0] = TB::frag((STAGE_PTR) + TILE_A_BYTES, ab, 0, SLICE);               \
        else if ((Q) <= 4) ra[BUF][(Q) - 1] = TA::frag((STAGE_PTR), aa, (Q) - 1, SLICE);             \
        else rb[BUF][(Q) - 4] = TB::frag((STAGE_PTR) + TILE_A_BYTES, ab, (Q) - 4, SLICE);            \
    }
#define FHPC_REQ(STAGE_PTR, KPOS, R)                                                                 \
    {                                                                                                \
        if ((R) < FA::PER) fa.issue_one((STAGE_PTR), (KPOS), kld, wave, (R));                        \
        else fb.issue_one((STAGE_PTR) + TILE_A_BYTES, (KPOS), kld, wave, (R) - FA::PER);             \
    }
        // One K tile (ring slot STAGE, k position KPOS).
        //   first half : matrix instructions of slice 0; reads of slice 1; the second four
        //                requests for the tile NS-1 ahead (slot of the previous tile, released
        //                by the previous barrier)
        //   barrier    : own requests for the next tile have landed, own reads of this tile
        //                are complete
        //   second half: matrix instructions of slice 1; reads of slice 0 of the next tile; the
        //                first four requests for the tile NS ahead (this tile's slot)
#define FHPC_TILE(STAGE, KPOS)                                                                       \
    {                                                                                                \
        constexpr int PREV = ((STAGE) + NS - 1) % NS, NEXT = ((STAGE) + 1) % NS;                     \
        unsigned char* cur = lds + (STAGE) * STAGE_BYTES;                                            \
        unsigned char* prv = lds + PREV * STAGE_BYTES;                                               \
        unsigned char* nxt = lds + NEXT * STAGE_BYTES;                                               \
        _Pragma("unroll") for (int q = 0; q < 16; q++) {                                             \
            acc[q / 4][q % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rb[0][q / 4], ra[0][q % 4], acc[q / 4][q % 4], 0, 0, 0); \
            if (q < 8) FHPC_READ(1, cur, 1, q)                                                       \
            else if (q % 2 == 0) FHPC_REQ(prv, (KPOS) + (NS - 1) * BK, 4 + (q - 8) / 2)              \
            __builtin_amdgcn_sched_barrier(0);                                                       \
        }                                                                                            \
        FHPC_WAIT_VM((NS - 2) * L);                                                                  \
        FHPC_WAIT_LGKM0();                                                                           \
        wg_barrier();                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                           \
        _Pragma("unroll") for (int q = 0; q < 16; q++) {                                             \
            acc[q / 4][q % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rb[1][q / 4], ra[1][q % 4], acc[q / 4][q % 4], 0, 0, 0); \
            if (q < 8) FHPC_READ(0, nxt, 0, q)                                                       \
            else if (q % 2 == 0) FHPC_REQ(cur, (KPOS) + NS * BK, (q - 8) / 2)                        \
            __builtin_amdgcn_sched_barrier(0);                                                       \
        }                                                                                            \
    }
        // The ring is walked with compile-time slot numbers, NS tiles per trip; tiles past the
        // end of the k range are zero tiles (their requests are out of range and arrive as
        // zeros).
        for (int k0 = kbeg; k0 < kend; k0 += NS * BK) {
            FHPC_TILE(0, k0)
            FHPC_TILE(1, k0 + BK)
            FHPC_TILE(2, k0 + 2 * BK)
            FHPC_TILE(3, k0 + 3 * BK)
            if constexpr (NS == 5) FHPC_TILE(4, k0 + 4 * BK)
        }
#undef FHPC_TILE
#undef FHPC_REQ
#undef FHPC_READ
        FHPC_WAIT_VM(0);                                        // zero-tile requests past the end may still be landing
        FHPC_WAIT_LGKM0();
        wg_barrier();
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32 x 32 block
    const float alpha = p.alpha;
    const int l32 = lane & 31, hi = lane >> 5;
    if constexpr (OUT_MODE == OUT_BF16) {
        // through LDS as [BM][BN] bf16 with row-swizzled 16-byte chunks, then whole chunks along rows
        constexpr int CPR = BN / 8;
        static_assert(BM * BN * 2 <= NS * STAGE_BYTES, "output tile must fit the ring");
#pragma unroll
        for (int j = 0; j < TN; j++) {
#pragma unroll
            for (int i = 0; i < TM; i++) {
                const int row = wave_m0 + i * 32 + l32;
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const int chunk = (wave_n0 + j * 32 + g * 8) >> 3;
                    u32x2 o;
                    o.x = pack_bf16(acc[j][i][4 * g + 0] * alpha, acc[j][i][4 * g + 1] * alpha);
                    o.y = pack_bf16(acc[j][i][4 * g + 2] * alpha, acc[j][i][4 * g + 3] * alpha);
                    *reinterpret_cast<u32x2*>(lds + row * (BN * 2) + (((chunk ^ row) & (CPR - 1)) << 4) + hi * 8) = o;
                }
            }
        }
        __syncthreads();
        constexpr int PASSES = BM * CPR / NT;
        const int c = tid % CPR, r0 = tid / CPR;
        const int col = n0 + c * 8;
#pragma unroll 8
        for (int q = 0; q < PASSES; q++) {
            const int row = r0 + q * (NT / CPR);
            const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * (BN * 2) + (((c ^ row) & (CPR - 1)) << 4));
            const int m = m0 + row;
            if (m < p.M && col < p.N)
                *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.c) + (size_t)m * (size_t)p.ldc + (size_t)col) = v;
        }
    } else {
        // fp32: this split's partial sum goes to its own slab, straight from the registers
        float* dst = reinterpret_cast<float*>(p.c) + (size_t)split * (size_t)p.split_stride;
#pragma unroll
        for (int j = 0; j < TN; j++) {
#pragma unroll
            for (int i = 0; i < TM; i++) {
                const int m = m0 + wave_m0 + i * 32 + l32;
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const int n = n0 + wave_n0 + j * 32 + g * 8 + hi * 4;
                    if (m < p.M && n < p.N) {
                        f32x4 o;
                        o.x = acc[j][i][4 * g + 0] * alpha;
                        o.y = acc[j][i][4 * g + 1] * alpha;
                        o.z = acc[j][i][4 * g + 2] * alpha;
                        o.w = acc[j][i][4 * g + 3] * alpha;
                        *reinterpret_cast<f32x4*>(dst + (size_t)m * (size_t)p.ldc + (size_t)n) = o;
                    }
                }
            }
        }
    }
}

template <int NS, int AM, int BMODE, int OUT>
static hipError_t launch_w4(const GemmArgs& a, hipStream_t s)
{
    const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    dim3 grid((unsigned)(tiles * (a.splits > 1 ? a.splits : 1)));
    int slot = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof(name), "gemm_w4<256x256x32,a%d,b%d,o%d>", AM, BMODE, OUT);
        slot = prof_begin(name, 2.0 * a.M * a.N * (double)a.K, 0.0, s);
    }
    hipLaunchKernelGGL((gemm_w4_kernel<NS, AM, BMODE, OUT>), grid, dim3(NT), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

constexpr int RING = 5;
template __global__ void gemm_w4_kernel<RING, OP_KC, OP_XC, OUT_BF16>(GemmArgs);
template __global__ void gemm_w4_kernel<RING, OP_KC, OP_KC, OUT_BF16>(GemmArgs);
template __global__ void gemm_w4_kernel<RING, OP_XC, OP_XC, OUT_F32>(GemmArgs);

}  // namespace w4

bool gemm_w4_supports(int a_mode, int b_mode, int b2_mode, int out_mode, int tile)
{
    if (b2_mode != OP_NONE || tile != TILE_256x256) return false;
    if (a_mode == OP_KC && b_mode == OP_XC && out_mode == OUT_BF16) return true;
    if (a_mode == OP_KC && b_mode == OP_KC && out_mode == OUT_BF16) return true;
    if (a_mode == OP_XC && b_mode == OP_XC && out_mode == OUT_F32) return true;
    return false;
}

hipError_t launch_gemm_w4(int a_mode, int b_mode, int out_mode, const GemmArgs& args, hipStream_t stream)
{
    using namespace w4;
    if (args.M <= 0 || args.N <= 0) return hipSuccess;
    if (args.splits > 1 && out_mode != OUT_F32) return hipErrorInvalidValue;
    if (a_mode == OP_KC && b_mode == OP_XC && out_mode == OUT_BF16) return launch_w4<RING, OP_KC, OP_XC, OUT_BF16>(args, stream);
    if (a_mode == OP_KC && b_mode == OP_KC && out_mode == OUT_BF16) return launch_w4<RING, OP_KC, OP_KC, OUT_BF16>(args, stream);
    if (a_mode == OP_XC && b_mode == OP_XC && out_mode == OUT_F32) return launch_w4<RING, OP_XC, OP_XC, OUT_F32>(args, stream);
    return hipErrorInvalidValue;
}

}  // namespace fhpc
