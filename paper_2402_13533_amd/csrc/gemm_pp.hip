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
// (the same XCD-aware order as a plain launch would give).  The ring does not drain between
// tiles: the last steps of a tile's K loop request the first K tiles of the next one, the bf16
// epilogue goes through small wave-private LDS patches outside the ring, and the waits of the
// next tile's first steps allow for the output stores still in flight (a wave's memory
// operations complete in order) instead of waiting them out.
#include "gemm_bf16.h"
#include "gemm_ring.h"
#include "gate_math.h"
#include "profile.h"

#include <stdio.h>
#include <type_traits>

namespace fhpc {
namespace pp {

using namespace ring;

constexpr int NT = 512;

// Probe builds only (-DFHPC_TRACE): wave 0 of every workgroup stamps the 100 MHz clock at the phase boundaries of
// its first tiles, read back through fhpc_debug_read_ts.
#ifdef FHPC_TRACE
constexpr int TRACE_WGS = 256, TRACE_SLOTS = 40;
__device__ unsigned long long g_trace[TRACE_WGS * TRACE_SLOTS];
#define FHPC_TS(slot)                                                                                     \
    do {                                                                                                  \
        if (tid == 0 && blockIdx.x < TRACE_WGS && (slot) < TRACE_SLOTS)                                   \
            g_trace[blockIdx.x * TRACE_SLOTS + (slot)] = __builtin_amdgcn_s_memrealtime();                \
    } while (0)
#else
#define FHPC_TS(slot) do { } while (0)
#endif

template <int BM, int BN, int BK, bool KSPLIT, int NSTAGE, int A_MODE, int B_MODE, int OUT_MODE, int GATE = 0>
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
    // The spatial shape is launched with one workgroup per compute unit that walks over output tiles.
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
    const int per_product = tiles_m * tiles_n * nsplit;
    const int ngroups = p.groups > 1 ? p.groups : 1;
    const int total = per_product * ngroups;
    const FragAddr aa = TA::make(wave_m0, lane);
    const FragAddr ab = TB::make(wave_n0, lane);

    // Feeders and coordinates of the current work item and of the one this workgroup takes next.
    FA fa;
    FB fb;
    fa.describe(p.a, p.M, p.K);
    fb.describe(p.b, p.N, p.K);
    struct Item { int m0, n0, split, kbeg, kend, kld, grp; };
    Item cur = {}, nxt = {};                                   // (nxt is read, unused, when no item follows)
    auto item_of = [&](int pid, Item& it) {
        int tm, tn;
        const int id = xcd_contiguous(pid, total);
        it.grp = id / per_product;
        item_coords(id - it.grp * per_product, tiles_m, tiles_n, nsplit, tm, tn, it.split);
        it.m0 = tm * BM;
        it.n0 = tn * BN;
        it.kbeg = it.split * p.k_chunk;
        it.kend = (it.kbeg + p.k_chunk < p.K) ? it.kbeg + p.k_chunk : p.K;
        it.kld = FHPC_DBG_NO_LOADS(p) ? it.kbeg : it.kend;              // diagnostics: nothing is in range
    };
    // the D * L requests that fill the ring with the current item's first D K tiles
    auto first_requests = [&]() {
        if (cur.kbeg < cur.kend) {
#pragma unroll
            for (int u = 0; u < D; u++) {
                fa.issue(lds + u * STAGE_BYTES, cur.kbeg + u * BK, cur.kld, wave);
                fb.issue(lds + u * STAGE_BYTES + TILE_A_BYTES, cur.kbeg + u * BK, cur.kld, wave);
            }
        }
    };
    // The K loop of an item runs whole trips round the ring; where the item has a successor, the requests of
    // its last D steps (which would otherwise fetch zero tiles past the end of its k range) fetch the
    // successor's first D K tiles instead, into the very slots those will be read from: the ring never
    // drains between output tiles and the epilogue has only the output to move.  `chained` says this item's
    // first K tiles were requested that way.  A wave's memory operations complete in the order issued, so
    // when the predecessor's epilogue issued its STORES output stores unconditionally (a bf16 tile inside
    // the output: `relaxed`), the waits of the first D steps allow for them instead of waiting them out.
    constexpr int STORES = TM * 4;
    bool chained = false, relaxed = false;
    FHPC_TS(0);
    item_of(blockIdx.x, cur);
    int trace_tile = 0;
    (void)trace_tile;

    for (int pid = blockIdx.x; pid < total; pid += gridDim.x) {
    const int out_m0 = cur.m0, out_n0 = cur.n0, out_split = cur.split;
    void* const out_c = (p.groups > 1) ? p.gc[cur.grp] : p.c;
    const int kbeg = cur.kbeg, kend = cur.kend, kld = cur.kld;
    if (p.groups > 1) {
        // this item's product: its operands' descriptors (the lane offsets do not depend on the base address)
        GemmOperand ga = p.a, gb = p.b;
        ga.ptr = p.ga[cur.grp];
        gb.ptr = p.gb[cur.grp];
        fa.describe(ga, p.M, p.K);
        fb.describe(gb, p.N, p.K);
    }
    if (kbeg < kend) {
        fa.set_tile(p.a, cur.m0, p.M, wave, lane);
        fb.set_tile(p.b, cur.n0, p.N, wave, lane);
    }
    if (!chained) first_requests();
    const bool has_next = PERSISTENT && pid + (int)gridDim.x < total;
    if (has_next) item_of(pid + (int)gridDim.x, nxt);
    // whole trips: the first k position past this item's loop
    const int kpad = kbeg + (kend - kbeg + NSTAGE * BK - 1) / (NSTAGE * BK) * (NSTAGE * BK);
    // (the successor's requests use this item's operand descriptors: no chaining into another product)
    const bool chain = has_next && kbeg < kend && nxt.kbeg < nxt.kend && nxt.grp == cur.grp;
    const int nk0 = nxt.kbeg - kpad;                          // successor's k position = loop position + nk0

    f32x16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][i][v] = 0.f;

    if (kbeg < kend) {
        if (relaxed) FHPC_WAIT_VM((D - 1) * L + STORES);
        else FHPC_WAIT_VM((D - 1) * L);
        wg_barrier();
        FHPC_TS(1 + 4 * trace_tile);

        bf16x8 ra[2][TM], rb[2][TN];
        // request q (of L) of the K tile at loop position kpos.  NEXT marks the requests of an item's last
        // trip that reach past it: with a successor they fetch the successor's first K tiles, without one a
        // zero tile.  Only that trip carries the test; the trips before it request unconditionally.
#define FHPC_REQUEST(RQ, KP, Q, NEXT)                                                                                \
    {                                                                                                                \
        if ((NEXT) && chain) {                                                                                       \
            if ((Q) < FA::PER) fa.issue_one_for(p.a, nxt.m0, p.M, RQ, (KP) + nk0, nxt.kld, wave, lane, (Q));         \
            else fb.issue_one_for(p.b, nxt.n0, p.N, (RQ) + TILE_A_BYTES, (KP) + nk0, nxt.kld, wave, lane, (Q) - FA::PER); \
        } else {                                                                                                     \
            if ((Q) < FA::PER) fa.issue_one(RQ, (KP), kld, wave, (Q));                                               \
            else fb.issue_one((RQ) + TILE_A_BYTES, (KP), kld, wave, (Q) - FA::PER);                                  \
        }                                                                                                            \
    }
        // Memory phase of one wave: its 12 fragment reads of tile t (ring slot STAGE) interleaved
        // with its L requests for tile t+D (into the slot tile t-1 has just left).  A request
        // blocks the wave until the texture path accepts it, so spreading the requests between
        // the LDS reads lets the reads drain meanwhile.
#define FHPC_MEM(STAGE, KPOS, NEXT)                                                                  \
    {                                                                                                \
        constexpr int REQ = ((STAGE) + NSTAGE - 1) % NSTAGE;                                         \
        const unsigned char* st = lds + (STAGE) * STAGE_BYTES;                                       \
        unsigned char* rq = lds + REQ * STAGE_BYTES;                                                 \
        int issued = 0;                                                                              \
        _Pragma("unroll") for (int s = 0; s < 2; s++) {                                              \
            _Pragma("unroll") for (int i = 0; i < TM; i++) {                                         \
                ra[s][i] = TA::frag(st, aa, i, SLICE0 + s);                                          \
                if ((s * (TM + TN) + i) % 2 == 1 && issued < L) {                                    \
                    FHPC_REQUEST(rq, (KPOS) + D * BK, issued, NEXT)                                  \
                    issued++;                                                                        \
                }                                                                                    \
                __builtin_amdgcn_sched_barrier(0);                                                   \
            }                                                                                        \
            _Pragma("unroll") for (int j = 0; j < TN; j++) {                                         \
                rb[s][j] = TB::frag(st + TILE_A_BYTES, ab, j, SLICE0 + s);                           \
                if ((s * (TM + TN) + TM + j) % 2 == 1 && issued < L) {                               \
                    FHPC_REQUEST(rq, (KPOS) + D * BK, issued, NEXT)                                  \
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
        // End of step J of a trip: every wave waits for its own requests for the next K tile.  In an item's
        // FIRST trip the predecessor's output stores may still be in flight, younger than the requests the
        // first D - 1 steps wait for.
#define FHPC_END_EVEN(J, FIRST)                                                                      \
    {                                                                                                \
        if ((FIRST) && (J) + 1 < D && relaxed) FHPC_WAIT_VM((D - 1) * L + STORES);                   \
        else FHPC_WAIT_VM((D - 1) * L);                                                              \
        FHPC_WAIT_LGKM0();                                                                           \
        wg_barrier();                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                           \
    }
        // One K tile = an odd phase and an even phase.  Every wave opens the odd phase by
        // requesting tile t+D into the ring slot tile t-1 has just left, and closes the even
        // phase by waiting for its own requests for tile t+1.  The ring is walked with
        // compile-time slot numbers, NSTAGE tiles per trip; in the LAST trip the requests of the steps
        // from NSTAGE - D on reach past the item (FHPC_REQUEST).
#define FHPC_STEP_G0(S, K0, FIRST, LAST)                                                             \
    { FHPC_MEM(S, (K0) + (S) * BK, (LAST) && (S) >= NSTAGE - D) FHPC_END_ODD() FHPC_MMA() FHPC_END_EVEN(S, FIRST) }
#define FHPC_STEP_G1(S, K0, FIRST, LAST)                                                             \
    { FHPC_MMA() FHPC_END_ODD() FHPC_MEM(S, (K0) + (S) * BK, (LAST) && (S) >= NSTAGE - D) FHPC_END_EVEN(S, FIRST) }
#define FHPC_TRIP(G, K0, FIRST, LAST)                                                                \
    {                                                                                                \
        FHPC_STEP_##G(0, K0, FIRST, LAST)                                                            \
        FHPC_STEP_##G(1, K0, FIRST, LAST)                                                            \
        FHPC_STEP_##G(2, K0, FIRST, LAST)                                                            \
        if constexpr (NSTAGE == 4) FHPC_STEP_##G(3, K0, FIRST, LAST)                                 \
    }
        // first trip, middle trips, last trip (an item of a single trip: first and last at once)
#define FHPC_ITEM(G)                                                                                 \
    {                                                                                                \
        constexpr int TRIP_K = NSTAGE * BK;                                                          \
        if (kpad - kbeg == TRIP_K) {                                                                 \
            FHPC_TRIP(G, kbeg, true, true)                                                           \
        } else {                                                                                     \
            FHPC_TRIP(G, kbeg, true, false)                                                          \
            for (int k0 = kbeg + TRIP_K; k0 < kpad - TRIP_K; k0 += TRIP_K) FHPC_TRIP(G, k0, false, false) \
            FHPC_TRIP(G, kpad - TRIP_K, false, true)                                                 \
        }                                                                                            \
    }
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
            FHPC_ITEM(G0)
        } else {
            // group 1: one phase behind; its first odd phase multiplies zero fragments
            constexpr int SLICE0 = KSPLIT ? 2 : 0;
            FHPC_ITEM(G1)
            FHPC_MMA()                                          // the last tile
        }
#undef FHPC_ITEM
#undef FHPC_TRIP
#undef FHPC_STEP_G0
#undef FHPC_STEP_G1
#undef FHPC_END_ODD
#undef FHPC_END_EVEN
#undef FHPC_MMA
#undef FHPC_MEM
#undef FHPC_REQUEST
        FHPC_TS(2 + 4 * trace_tile);
        if (!chain) {
            // zero-tile requests past the end may still be landing in the ring: the k-split hand-over below
            // reuses it, and a workgroup must not end (and give its LDS up) with requests in flight
            FHPC_WAIT_VM(0);
            wg_barrier();
        }
        FHPC_TS(3 + 4 * trace_tile);
    }
    // (After the loop's last barrier no wave reads the ring any more; with a successor, the requests still
    // in flight are the successor's.)
    // A tile at or beyond p.n_split belongs to the launch's second output (c2): it takes the guarded stores.
    const bool second = p.n_split > 0 && out_n0 >= p.n_split;
    const bool inside = (out_m0 + BM <= p.M) && (out_n0 + BN <= p.N) && !second;
    chained = chain;
    relaxed = chain && inside && OUT_MODE == OUT_BF16 && GATE == 0;
#ifdef FHPC_DIAG
    if (p.dbg & 48) relaxed = false;                           // the probes that skip the stores
#endif

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
        // The vector ALU is what this costs (two waves share a SIMD, four cycles an instruction), so
        // the scale is skipped when it is 1, and a tile that lies inside the output stores through a
        // buffer descriptor with one lane offset for the whole tile: the row steps travel in the
        // scalar offset and nothing is compared or multiplied per store.
        if (owner) {
            unsigned char* patch = lds + RING_BYTES + (KSPLIT ? wq : wave) * PATCH_BYTES;
            const int rc = lane & 7, rr = lane >> 3;
            if (alpha != 1.f) {
#pragma unroll
                for (int j = 0; j < TN; j++)
#pragma unroll
                    for (int i = 0; i < TM; i++)
#pragma unroll
                        for (int v = 0; v < 16; v++) acc[j][i][v] *= alpha;
            }
            const __amdgpu_buffer_rsrc_t rs_c = __builtin_amdgcn_make_buffer_rsrc(out_c, 0, (int)((uint32_t)p.M * (uint32_t)p.ldc * 2u), 0x00020000);
            const uint32_t ldc_b = (uint32_t)p.ldc * 2u;
            const uint32_t lane_off = (uint32_t)(wave_m0 + rr) * ldc_b + (uint32_t)(wave_n0 + rc * 8) * 2u;
            const uint32_t tile_off = (uint32_t)out_m0 * ldc_b + (uint32_t)out_n0 * 2u;
            // (the 8-byte half a lane writes is flipped for rows 8 .. 15 and 24 .. 31, so that the 32 lanes of a
            // half wave spread over both halves of the 16-byte slots; the read-back below swaps them again)
            const uint32_t wr_off = (uint32_t)l32 * 128u + (uint32_t)((hi ^ (l32 >> 3)) & 1) * 8u;        // + swizzled chunk
            // The SiLU gate on a tile inside the output: the 16-byte pieces of G (and U) that match the pieces this
            // lane stores for a block of 32 rows are requested once the block's accumulators have gone to the patch,
            // and are on their way while the block is read back.  (Requesting one block ahead was measured: the 16 to
            // 32 registers it needs while all accumulators are live end in spills, and the launch gets slower.)
            const uint32_t gate_bytes = (uint32_t)p.M * ldc_b;
            const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(GATE ? p.gate_g : out_c), 0, (int)gate_bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t rs_u = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(GATE == 2 ? p.gate_u : out_c), 0, (int)gate_bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t rs_o1 = __builtin_amdgcn_make_buffer_rsrc(GATE ? p.gate_out1 : out_c, 0, (int)gate_bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t rs_o2 = __builtin_amdgcn_make_buffer_rsrc(GATE == 2 ? p.gate_out2 : out_c, 0, (int)gate_bytes, 0x00020000);
            u32x4 gq[4], uq[4];
            auto gate_requests = [&](int i, u32x4 (&g4)[4], u32x4 (&u4)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t soff = __builtin_amdgcn_readfirstlane(tile_off + (uint32_t)(i * 32 + 8 * q) * ldc_b);
                    g4[q] = __builtin_amdgcn_raw_buffer_load_b128(rs_g, lane_off, soff, 0);
                    if (GATE == 2) u4[q] = __builtin_amdgcn_raw_buffer_load_b128(rs_u, lane_off, soff, 0);
                }
            };
#pragma unroll
            for (int i = 0; i < TM; i++) {
#pragma unroll
                for (int j = 0; j < TN; j++) {
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const int chunk = j * 4 + g;
                        u32x2 o;
                        o.x = pack_bf16(acc[j][i][4 * g + 0], acc[j][i][4 * g + 1]);
                        o.y = pack_bf16(acc[j][i][4 * g + 2], acc[j][i][4 * g + 3]);
                        *reinterpret_cast<u32x2*>(patch + wr_off + (((chunk ^ l32) & 7) << 4)) = o;
                    }
                }
#ifdef FHPC_DIAG
                if (p.dbg & 16) continue;                      // probe: no read-back, no stores
#endif
                if (GATE != 0 && inside) gate_requests(i, gq, uq);
                if (inside && GATE != 0) {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int row = rr + 8 * q;
                        u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * 128 + (((rc ^ row) & 7) << 4));
                        if (q & 1) v = u32x4{v.z, v.w, v.x, v.y};
                        const uint32_t soff = __builtin_amdgcn_readfirstlane(tile_off + (uint32_t)(i * 32 + 8 * q) * ldc_b);
                        // A 16-byte store reads its data registers for some cycles after it has issued, and the
                        // arithmetic here would reuse them at once (measured: the first shift of the gate landed in
                        // the stored word of the lanes read last).  Both results are formed first, the two stores go
                        // out together, and four idle states follow them; nothing may be scheduled in between.
                        u32x4 o1, o2;
                        if (GATE == 1) {
                            o1 = v;
#pragma unroll
                            for (int e = 0; e < 4; e++) o2[e] = gate::fwd_pair(gq[q][e], v[e]);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                uint32_t a, b;
                                gate::bwd_pair(gq[q][e], uq[q][e], v[e], a, b);
                                o1[e] = a; o2[e] = b;
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        __builtin_amdgcn_raw_buffer_store_b128(o1, GATE == 1 ? rs_c : rs_o1, lane_off, soff, 0);
                        __builtin_amdgcn_raw_buffer_store_b128(o2, GATE == 1 ? rs_o1 : rs_o2, lane_off, soff, 0);
                        asm volatile("s_nop 3" ::: "memory");
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else if (inside) {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int row = rr + 8 * q;
                        u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * 128 + (((rc ^ row) & 7) << 4));
                        if (q & 1) v = u32x4{v.z, v.w, v.x, v.y};
#ifdef FHPC_DIAG
                        if (p.dbg & 32) { if (v.x == 0x12345678u && v.y == 0x9abcdef0u) reinterpret_cast<u32x4*>(out_c)[0] = v; continue; }
#endif
                        const uint32_t soff = __builtin_amdgcn_readfirstlane(tile_off + (uint32_t)(i * 32 + 8 * q) * ldc_b);
                        __builtin_amdgcn_raw_buffer_store_b128(v, rs_c, lane_off, soff, 0);
                    }
                } else {
                    // (edge tiles, and the tiles of a second output: its own base, leading dimension and width)
                    uint16_t* const eo = reinterpret_cast<uint16_t*>(second ? p.c2 : out_c);
                    const size_t eld = (size_t)(second ? p.ldc2 : p.ldc);
                    const int ecols = second ? p.N - p.n_split : (p.n_split > 0 ? p.n_split : p.N);
                    const int col = out_n0 - (second ? p.n_split : 0) + wave_n0 + rc * 8;
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int row = rr + 8 * q;
                        u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * 128 + (((rc ^ row) & 7) << 4));
                        if (q & 1) v = u32x4{v.z, v.w, v.x, v.y};
                        const int m = out_m0 + wave_m0 + i * 32 + row;
                        if (m < p.M && col < ecols) {
                            const size_t at = (size_t)m * eld + (size_t)col;
                            if (GATE == 0) {
                                *reinterpret_cast<u32x4*>(eo + at) = v;
                            } else {
                                // (results first, then the stores and the idle states: see the tiles inside the output)
                                const u32x4 gv = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.gate_g) + at);
                                u32x4 o1, o2;
                                if (GATE == 1) {
                                    o1 = v;
#pragma unroll
                                    for (int e = 0; e < 4; e++) o2[e] = gate::fwd_pair(gv[e], v[e]);
                                } else {
                                    const u32x4 uv = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.gate_u) + at);
#pragma unroll
                                    for (int e = 0; e < 4; e++) {
                                        uint32_t a, b;
                                        gate::bwd_pair(gv[e], uv[e], v[e], a, b);
                                        o1[e] = a; o2[e] = b;
                                    }
                                }
                                uint16_t* const d1 = GATE == 1 ? eo : static_cast<uint16_t*>(p.gate_out1);
                                uint16_t* const d2 = static_cast<uint16_t*>(GATE == 1 ? p.gate_out1 : p.gate_out2);
                                __builtin_amdgcn_sched_barrier(0);
                                *reinterpret_cast<u32x4*>(d1 + at) = o1;
                                *reinterpret_cast<u32x4*>(d2 + at) = o2;
                                asm volatile("s_nop 3" ::: "memory");
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
                }
            }
        }
    } else {
        // fp32: this split's partial sum goes to its own slab, straight from the registers
        if (owner) {
            float* dst = reinterpret_cast<float*>(out_c) + (size_t)out_split * (size_t)p.split_stride;
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
    FHPC_TS(4 + 4 * trace_tile);
    trace_tile++;
    if (!PERSISTENT) break;
    cur = nxt;
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

template <int BM, int BN, int BK, bool KSPLIT, int NSTAGE, int AM, int BMODE, int OUT, int GATE = 0>
static hipError_t launch_pp(const GemmArgs& a, hipStream_t s)
{
    if (a.gate != GATE) return hipErrorInvalidValue;
    if (a.n_split > 0 && (OUT != OUT_BF16 || a.groups > 1 || a.n_split % BN != 0 || a.n_split >= a.N || (a.N - a.n_split) % 8 != 0 || !a.c2))
        return hipErrorInvalidValue;
    if (a.gate != 0 && (OUT != OUT_BF16 || KSPLIT || a.groups > 1 || a.n_split > 0 || a.gate < 0 || a.gate > 2 || !a.gate_g ||
                        !a.gate_out1 || (a.gate == 2 && (!a.gate_u || !a.gate_out2)) || (a.N % 8) != 0 || (a.ldc % 8) != 0))
        return hipErrorInvalidValue;
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    const int total = tiles * (a.splits > 1 ? a.splits : 1) * (a.groups > 1 ? a.groups : 1);
    const int cus = compute_units();
    dim3 grid((unsigned)((!KSPLIT && total > cus) ? cus : total));
    int slot = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof(name), GATE ? "gemm_pp<%dx%dx%d,a%d,b%d,o%d,gate%d>" : "gemm_pp<%dx%dx%d,a%d,b%d,o%d>", BM, BN, BK, AM, BMODE, OUT, GATE);
        slot = prof_begin(name, 2.0 * a.M * a.N * (double)a.K * (a.groups > 1 ? a.groups : 1), 0.0, s);
    }
    hipLaunchKernelGGL((gemm_pp_kernel<BM, BN, BK, KSPLIT, NSTAGE, AM, BMODE, OUT, GATE>), grid, dim3(NT), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

template <int AM, int BMODE, int OUT>
static hipError_t launch_pp_tile(int tile, const GemmArgs& a, hipStream_t s)
{
    if (a.gate != 0) {
        // the gate epilogue exists where the FFN uses it: the up projection U = H B (forward) and the input
        // gradient of the down projection dZ = dH A^T (backward), on the 256 x 256 tile
        if constexpr (AM == OP_KC && BMODE == OP_XC && OUT == OUT_BF16) {
            if (tile == TILE_256x256 && a.gate == 1) return launch_pp<256, 256, 32, false, 4, AM, BMODE, OUT, 1>(a, s);
        }
        if constexpr (AM == OP_KC && BMODE == OP_KC && OUT == OUT_BF16) {
            if (tile == TILE_256x256 && a.gate == 2) return launch_pp<256, 256, 32, false, 4, AM, BMODE, OUT, 2>(a, s);
        }
        return hipErrorInvalidValue;
    }
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
template __global__ void gemm_pp_kernel<256, 256, 32, false, 4, OP_KC, OP_XC, OUT_BF16, 1>(GemmArgs);   // U = H B with Z = SiLU(G) U
template __global__ void gemm_pp_kernel<256, 256, 32, false, 4, OP_KC, OP_KC, OUT_BF16, 2>(GemmArgs);   // dZ = dH A^T into dG, dU

}  // namespace pp

using namespace pp;

#ifdef FHPC_TRACE
extern "C" int fhpc_debug_read_ts(unsigned long long* out, int n)
{
    if (n > TRACE_WGS * TRACE_SLOTS) n = TRACE_WGS * TRACE_SLOTS;
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_trace), sizeof(unsigned long long) * (size_t)n);
}
#endif

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
