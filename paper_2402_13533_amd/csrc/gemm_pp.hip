// Eight-wave "ping-pong" bf16 GEMM for gfx950 with global -> LDS loads that bypass the
// register file (buffer_load ... lds), a ring of LDS stages, and the CDNA4 transposing LDS
// read for operands whose output index is the contiguous one.
//
// Schedule.  The workgroup is two groups of four waves (one wave of each group per SIMD).
// Time is cut into phases separated by workgroup barriers.  In odd phases group 0 reads the
// fragments of K tile t from LDS into registers while group 1 issues the matrix
// instructions of tile t-1; in even phases the roles swap.  A SIMD's matrix pipe is
// therefore fed by one wave at a time, from registers only, and the LDS / memory latency
// of the sibling wave is hidden behind it.  Every wave starts each odd phase by requesting
// K tile t+D (D = NSTAGE-1) straight into the LDS stage that tile t-1 has just vacated,
// and ends each even phase by waiting until its own requests for tile t+1 have landed, so
// a request has D full steps to complete and no staging registers are needed.
//
// Two workgroup shapes share the per-wave work (a 128 x 64 accumulator tile, 12 fragment
// reads and 16 MFMAs per phase pair):
//   spatial  256 x 256 x 32: the groups own different column halves of the output;
//   k-split  256 x 128 x 64: both groups cover the whole 256 x 128 tile and split each
//            64-deep K tile in two; group 1's accumulators are added to group 0's through
//            LDS at the end.  Used when the output is too narrow for 256 x 256 tiles to
//            fill the chip.
//
// The spatial shape runs as one workgroup per compute unit that walks over its output tiles
// (the same XCD-aware order as a plain launch would give): before the epilogue of a tile it
// posts the requests for the first K tiles of the next one, and the bf16 epilogue goes through
// small wave-private LDS patches outside the ring, so those requests land while the output
// is being stored.
#include "gemm_bf16.h"
#include "gemm_ring.h"
#include "profile.h"

#include <stdio.h>

namespace fhpc {
namespace pp {

using namespace ring;

constexpr int NT = 512;

template <int BM, int BN, int BK, bool KSPLIT, int NSTAGE, int A_MODE, int B_MODE, int OUT_MODE>
__global__ __launch_bounds__(NT) void gemm_pp_kernel(GemmArgs p)
{
    constexpr int TM = 4, TN = 2;                              // every wave: 128 x 64 accumulators
    constexpr int WTM = 128, WTN = 64;
    static_assert(KSPLIT ? (BM == 2 * WTM && BN == 2 * WTN && BK == 64) : (BM == 2 * WTM && BN == 4 * WTN && BK == 32),
                  "workgroup shape");
    using FA = Feeder<A_MODE, BM, BK>;
    using FB = Feeder<B_MODE, BN, BK>;
    using TA = typename FA::Tile;
    using TB = typename FB::Tile;
    constexpr int TILE_A_BYTES = FA::TILE_BYTES, STAGE_BYTES = FA::TILE_BYTES + FB::TILE_BYTES;
    constexpr int D = NSTAGE - 1;                              // prefetch distance in K tiles
    constexpr int L = FA::PER + FB::PER;                       // requests per wave per K tile
    constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;
    // bf16 output leaves through a 4 KiB LDS patch private to each writing wave, outside the ring
    constexpr int OUT_WAVES = KSPLIT ? 4 : 8;
    constexpr int PATCH_BYTES = 32 * WTN * 2;
    constexpr int LDS_BYTES = RING_BYTES + (OUT_MODE == OUT_BF16 ? OUT_WAVES * PATCH_BYTES : 0);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS ring and output patches");
    static_assert(!KSPLIT || 4 * 128 * 256 <= RING_BYTES, "LDS for the accumulator hand-over");
    // The spatial shape is launched with one workgroup per compute unit that walks over output
    // tiles: the requests for the first K tiles of the next output tile are posted before the
    // epilogue of the current one, so their latency hides behind the output stores.
    constexpr bool PERSISTENT = !KSPLIT;

    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = wave >> 2, wq = wave & 3;
    // k-split: 2 x 2 waves per group over 256 x 128; spatial: 2 x 4 waves over 256 x 256
    const int wave_m0 = KSPLIT ? (wq >> 1) * WTM : (wave >> 2) * WTM;
    const int wave_n0 = KSPLIT ? (wq & 1) * WTN : (wave & 3) * WTN;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const int nsplit = p.splits > 1 ? p.splits : 1;
    const int total = tiles_m * tiles_n * nsplit;
    const FragAddr aa = TA::make(wave_m0, lane);
    const FragAddr ab = TB::make(wave_n0, lane);

    FA fa;
    FB fb;
    fa.describe(p.a, p.M, p.K);
    fb.describe(p.b, p.N, p.K);
    int m0, n0, split, kbeg, kend, kld;
    // coordinates of work item `pid`, its feeders, and the requests for its first D K tiles
    auto begin_tile = [&](int pid) {
        int tm, tn;
        work_coords(pid, tiles_m, tiles_n, nsplit, tm, tn, split);
        m0 = tm * BM;
        n0 = tn * BN;
        kbeg = split * p.k_chunk;
        kend = (kbeg + p.k_chunk < p.K) ? kbeg + p.k_chunk : p.K;
        kld = FHPC_DBG_NO_LOADS(p) ? kbeg : kend;                       // diagnostics: nothing is in range
        if (kbeg < kend) {
            fa.set_tile(p.a, m0, p.M, wave, lane);
            fb.set_tile(p.b, n0, p.N, wave, lane);
#pragma unroll
            for (int u = 0; u < D; u++) {
                fa.issue(lds + u * STAGE_BYTES, kbeg + u * BK, kld, wave);
                fb.issue(lds + u * STAGE_BYTES + TILE_A_BYTES, kbeg + u * BK, kld, wave);
            }
        }
    };
    begin_tile(blockIdx.x);

    for (int pid = blockIdx.x; pid < total; pid += gridDim.x) {
    const int out_m0 = m0, out_n0 = n0, out_split = split;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][i][v] = 0.f;

    if (kbeg < kend) {
        FHPC_WAIT_VM((D - 1) * L);                             // (output stores of the previous tile, younger
        wg_barrier();                                          //  than these requests, only make this wait longer)

        bf16x8 ra[2][TM], rb[2][TN];
        // Memory phase of one wave: its 12 fragment reads of tile t (ring slot STAGE) interleaved
        // with its L requests for tile t+D (into the slot tile t-1 has just left).  A request
        // blocks the wave until the texture path accepts it, so spreading the requests between
        // the LDS reads lets the reads drain meanwhile.
#define FHPC_MEM(STAGE, KPOS)                                                                        \
    {                                                                                                \
        constexpr int REQ = ((STAGE) + NSTAGE - 1) % NSTAGE;                                         \
        const unsigned char* st = lds + (STAGE) * STAGE_BYTES;                                       \
        unsigned char* rq = lds + REQ * STAGE_BYTES;                                                 \
        int issued = 0;                                                                              \
        _Pragma("unroll") for (int s = 0; s < 2; s++) {                                              \
            _Pragma("unroll") for (int i = 0; i < TM; i++) {                                         \
                ra[s][i] = TA::frag(st, aa, i, SLICE0 + s);                             \
                if ((s * (TM + TN) + i) % 2 == 1 && issued < L) {                                    \
                    if (issued < FA::PER) fa.issue_one(rq, (KPOS) + D * BK, kld, wave, issued);      \
                    else fb.issue_one(rq + TILE_A_BYTES, (KPOS) + D * BK, kld, wave, issued - FA::PER); \
                    issued++;                                                                        \
                }                                                                                    \
                __builtin_amdgcn_sched_barrier(0);                                                   \
            }                                                                                        \
            _Pragma("unroll") for (int j = 0; j < TN; j++) {                                         \
                rb[s][j] = TB::frag(st + TILE_A_BYTES, ab, j, SLICE0 + s);              \
                if ((s * (TM + TN) + TM + j) % 2 == 1 && issued < L) {                               \
                    if (issued < FA::PER) fa.issue_one(rq, (KPOS) + D * BK, kld, wave, issued);      \
                    else fb.issue_one(rq + TILE_A_BYTES, (KPOS) + D * BK, kld, wave, issued - FA::PER); \
                    issued++;                                                                        \
                }                                                                                    \
                __builtin_amdgcn_sched_barrier(0);                                                   \
            }                                                                                        \
        }                                                                                            \
        static_assert(L <= 6, "one request per two fragment reads");                                 \
    }
#define FHPC_MMA()                                                                                   \
    {                                                                                                \
        __builtin_amdgcn_s_setprio(1);                                                               \
        _Pragma("unroll") for (int s = 0; s < 2; s++)                                                \
            _Pragma("unroll") for (int j = 0; j < TN; j++)                                           \
                _Pragma("unroll") for (int i = 0; i < TM; i++)                                       \
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rb[s][j], ra[s][i], acc[j][i], 0, 0, 0); \
        __builtin_amdgcn_s_setprio(0);                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                           \
    }
#define FHPC_END_ODD()                                                                               \
    {                                                                                                \
        FHPC_WAIT_LGKM0();                                                                           \
        wg_barrier();                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                           \
    }
#define FHPC_END_EVEN()                                                                              \
    {                                                                                                \
        FHPC_WAIT_VM((D - 1) * L);                                                                   \
        FHPC_WAIT_LGKM0();                                                                           \
        wg_barrier();                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                           \
    }
        // One K tile = an odd phase and an even phase.  Every wave opens the odd phase by
        // requesting tile t+D into the ring slot tile t-1 has just left, and closes the even
        // phase by waiting for its own requests for tile t+1.  The ring is walked with
        // compile-time slot numbers, NSTAGE tiles per trip; tiles past the end of the k range
        // are zero tiles (their requests are out of range and arrive as zeros).
#define FHPC_STEP_G0(STAGE, KPOS) { FHPC_MEM(STAGE, KPOS) FHPC_END_ODD() FHPC_MMA() FHPC_END_EVEN() }
#define FHPC_STEP_G1(STAGE, KPOS) { FHPC_MMA() FHPC_END_ODD() FHPC_MEM(STAGE, KPOS) FHPC_END_EVEN() }
#pragma unroll
        for (int s = 0; s < 2; s++) {
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int e = 0; e < 8; e++) ra[s][i][e] = (__bf16)0.f;
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int e = 0; e < 8; e++) rb[s][j][e] = (__bf16)0.f;
        }
        if (group == 0) {
            // group 0: fragments of tile t in the odd phase, its matrix instructions in the even phase
            constexpr int SLICE0 = 0;
            for (int k0 = kbeg; k0 < kend; k0 += NSTAGE * BK) {
                FHPC_STEP_G0(0, k0)
                FHPC_STEP_G0(1, k0 + BK)
                FHPC_STEP_G0(2, k0 + 2 * BK)
                if constexpr (NSTAGE == 4) FHPC_STEP_G0(3, k0 + 3 * BK)
            }
        } else {
            // group 1: one phase behind; its first odd phase multiplies zero fragments
            constexpr int SLICE0 = KSPLIT ? 2 : 0;
            for (int k0 = kbeg; k0 < kend; k0 += NSTAGE * BK) {
                FHPC_STEP_G1(0, k0)
                FHPC_STEP_G1(1, k0 + BK)
                FHPC_STEP_G1(2, k0 + 2 * BK)
                if constexpr (NSTAGE == 4) FHPC_STEP_G1(3, k0 + 3 * BK)
            }
            FHPC_MMA()                                          // the last tile
        }
#undef FHPC_STEP_G0
#undef FHPC_STEP_G1
#undef FHPC_END_ODD
#undef FHPC_END_EVEN
#undef FHPC_MMA
#undef FHPC_MEM
        FHPC_WAIT_VM(0);                                        // zero-tile requests past the end may still be landing
        wg_barrier();
    }
    if (PERSISTENT && pid + (int)gridDim.x < total) begin_tile(pid + (int)gridDim.x);

    // ---- k-split: group 1 hands its accumulators to group 0 through LDS
    if constexpr (KSPLIT) {
        float* red = reinterpret_cast<float*>(lds) + wq * (128 * 64);       // 32 KiB per wave pair
        if (group == 1) {
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int i = 0; i < TM; i++)
#pragma unroll
                    for (int v = 0; v < 16; v++) red[((j * TM + i) * 16 + v) * 64 + lane] = acc[j][i][v];
        }
        __syncthreads();
        if (group == 0) {
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int i = 0; i < TM; i++)
#pragma unroll
                    for (int v = 0; v < 16; v++) acc[j][i][v] += red[((j * TM + i) * 16 + v) * 64 + lane];
        }
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32 x 32 block
    const float alpha = p.alpha;
    const int l32 = lane & 31, hi = lane >> 5;
    const bool owner = !KSPLIT || group == 0;
    if constexpr (OUT_MODE == OUT_BF16) {
        // Each writing wave turns its tile around 32 rows at a time in its own LDS patch
        // ([32][64] bf16, 16-byte chunks XOR-swizzled by the row) and stores whole 128-byte
        // rows; no workgroup barrier, and the ring stays free for the next tile's requests.
        if (owner) {
            unsigned char* patch = lds + RING_BYTES + (KSPLIT ? wq : wave) * PATCH_BYTES;
            const int rc = lane & 7, rr = lane >> 3;
#pragma unroll
            for (int i = 0; i < TM; i++) {
#pragma unroll
                for (int j = 0; j < TN; j++) {
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const int chunk = j * 4 + g;
                        u32x2 o;
                        o.x = pack_bf16(acc[j][i][4 * g + 0] * alpha, acc[j][i][4 * g + 1] * alpha);
                        o.y = pack_bf16(acc[j][i][4 * g + 2] * alpha, acc[j][i][4 * g + 3] * alpha);
                        *reinterpret_cast<u32x2*>(patch + l32 * 128 + (((chunk ^ l32) & 7) << 4) + hi * 8) = o;
                    }
                }
                const int col = out_n0 + wave_n0 + rc * 8;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int row = rr + 8 * q;
                    const u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * 128 + (((rc ^ row) & 7) << 4));
                    const int m = out_m0 + wave_m0 + i * 32 + row;
                    if (m < p.M && col < p.N)
                        *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.c) + (size_t)m * (size_t)p.ldc + (size_t)col) = v;
                }
            }
        }
    } else {
        // fp32: this split's partial sum goes to its own slab, straight from the registers
        if (owner) {
            float* dst = reinterpret_cast<float*>(p.c) + (size_t)out_split * (size_t)p.split_stride;
#pragma unroll
            for (int j = 0; j < TN; j++) {
#pragma unroll
                for (int i = 0; i < TM; i++) {
                    const int m = out_m0 + wave_m0 + i * 32 + l32;
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const int n = out_n0 + wave_n0 + j * 32 + g * 8 + hi * 4;
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
    if (!PERSISTENT) break;
    }
}

}  // namespace pp

// compute units of the current device, rounded down to whole multiples of the eight XCDs (256 when no
// device can be asked: the planner also sizes workspaces on hosts without a GPU)
int compute_units()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n - n % 8 > 0 ? n - n % 8 : n;          // whole multiples of the eight XCDs keep the tile map aligned
    }
    return cached[dev];
}

namespace pp {

template <int BM, int BN, int BK, bool KSPLIT, int NSTAGE, int AM, int BMODE, int OUT>
static hipError_t launch_pp(const GemmArgs& a, hipStream_t s)
{
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    const int total = tiles * (a.splits > 1 ? a.splits : 1);
    const int cus = compute_units();
    dim3 grid((unsigned)((!KSPLIT && total > cus) ? cus : total));
    int slot = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof(name), "gemm_pp<%dx%dx%d,a%d,b%d,o%d>", BM, BN, BK, AM, BMODE, OUT);
        slot = prof_begin(name, 2.0 * a.M * a.N * (double)a.K, 0.0, s);
    }
    hipLaunchKernelGGL((gemm_pp_kernel<BM, BN, BK, KSPLIT, NSTAGE, AM, BMODE, OUT>), grid, dim3(NT), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

template <int AM, int BMODE, int OUT>
static hipError_t launch_pp_tile(int tile, const GemmArgs& a, hipStream_t s)
{
    if (tile == TILE_256x256) return launch_pp<256, 256, 32, false, 4, AM, BMODE, OUT>(a, s);
    if (tile == TILE_256x128) return launch_pp<256, 128, 64, true, 3, AM, BMODE, OUT>(a, s);
    return hipErrorInvalidValue;
}

// every instantiation the dispatcher below can reach
#define FHPC_PP_INSTANTIATE(AM, BMODE, OUT)                                                        \
    template __global__ void gemm_pp_kernel<256, 256, 32, false, 4, AM, BMODE, OUT>(GemmArgs);     \
    template __global__ void gemm_pp_kernel<256, 128, 64, true, 3, AM, BMODE, OUT>(GemmArgs);
FHPC_PP_INSTANTIATE(OP_KC, OP_XC, OUT_BF16)
FHPC_PP_INSTANTIATE(OP_KC, OP_KC, OUT_BF16)
FHPC_PP_INSTANTIATE(OP_XC, OP_XC, OUT_F32)
FHPC_PP_INSTANTIATE(OP_KC, OP_XC, OUT_F32)      // H = X A, Y = H B with the reduction split (fp32 slabs)
FHPC_PP_INSTANTIATE(OP_KC, OP_KC, OUT_F32)      // dH = dY B^T, dX = dH A^T likewise
#undef FHPC_PP_INSTANTIATE

}  // namespace pp

using namespace pp;

bool gemm_pp_supports(int a_mode, int b_mode, int b2_mode, int out_mode, int tile)
{
    if (b2_mode != OP_NONE) return false;
    if (tile != TILE_256x256 && tile != TILE_256x128) return false;
    if (a_mode == OP_KC && b_mode == OP_XC && out_mode == OUT_BF16) return true;
    if (a_mode == OP_KC && b_mode == OP_KC && out_mode == OUT_BF16) return true;
    if (a_mode == OP_XC && b_mode == OP_XC && out_mode == OUT_F32) return true;
    if (a_mode == OP_KC && (b_mode == OP_XC || b_mode == OP_KC) && out_mode == OUT_F32) return true;
    return false;
}

hipError_t launch_gemm_pp(int a_mode, int b_mode, int out_mode, int tile, const GemmArgs& args, hipStream_t stream)
{
    if (args.M <= 0 || args.N <= 0) return hipSuccess;
    if (args.splits > 1 && out_mode != OUT_F32) return hipErrorInvalidValue;
    if (a_mode == OP_KC && b_mode == OP_XC && out_mode == OUT_BF16) return launch_pp_tile<OP_KC, OP_XC, OUT_BF16>(tile, args, stream);
    if (a_mode == OP_KC && b_mode == OP_KC && out_mode == OUT_BF16) return launch_pp_tile<OP_KC, OP_KC, OUT_BF16>(tile, args, stream);
    if (a_mode == OP_XC && b_mode == OP_XC && out_mode == OUT_F32) return launch_pp_tile<OP_XC, OP_XC, OUT_F32>(tile, args, stream);
    if (a_mode == OP_KC && b_mode == OP_XC && out_mode == OUT_F32) return launch_pp_tile<OP_KC, OP_XC, OUT_F32>(tile, args, stream);
    if (a_mode == OP_KC && b_mode == OP_KC && out_mode == OUT_F32) return launch_pp_tile<OP_KC, OP_KC, OUT_F32>(tile, args, stream);
    return hipErrorInvalidValue;
}

}  // namespace fhpc
