// C ABI entry points: validation, workspace carving and the sequence of GEMM-core
// launches that makes up each pass of the layer.  See include/fingpt_hpc.h for the
// contract of every function.
#include "../../include/fingpt_hpc.h"
#include "gemm_bf16.h"
#include "kernels_misc.h"
#include "merge.h"
#include "qskinny.h"

#include <atomic>

using namespace fhpc;

namespace {

constexpr int64_t kMaxBytes = (int64_t)1 << 31;   // per-matrix limit of the 32-bit buffer offsets
// compute units of the current device: every plan below is sized for it
inline int num_cu() { return compute_units(); }
static_assert(QSKINNY_HEADER_BYTES == FHPC_WORKSPACE_HEADER_BYTES, "the header size is part of the ABI");

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// (hipErrorOutOfMemory is what the launch helpers below return when a split reduction asks for more
// partial-sum slabs than the workspace reserves: reported as a workspace error, nothing was launched for it)
#define FHPC_HIP(expr)                                                               \
    do {                                                                             \
        const hipError_t fhpc_e_ = (expr);                                           \
        if (fhpc_e_ != hipSuccess) {                                                 \
            (void)hipGetLastError();                                                 \
            return fhpc_e_ == hipErrorOutOfMemory ? FHPC_ERR_WORKSPACE : FHPC_ERR_HIP; \
        }                                                                            \
    } while (0)

// One pass over an entry point's launch sequence: the real one (launch on `st`; a split reduction whose
// slabs would not fit behind Scratch::part fails instead of writing past it) or a dry one (launch
// nothing, record the largest slab area any launch of the sequence asks for).
struct Run {
    hipStream_t st = nullptr;
    bool dry = false;
    int64_t part_cap = 0;        // bytes reserved for partial-sum slabs
    int64_t part_need = 0;       // dry pass: the most any launch asked for
    // true when `bytes` of slabs may be used (always in a dry pass, which only records)
    bool claim(int64_t bytes)
    {
        if (bytes > part_need) part_need = bytes;
        return dry || bytes <= part_cap;
    }
};
// a launch that uses no slabs: skipped in a dry pass
#define FHPC_LAUNCH(run, expr)                \
    do {                                      \
        if (!(run).dry) FHPC_HIP(expr);       \
    } while (0)

// Workspace carving: a bump allocator over the caller's buffer (or a dry run that
// only measures).
struct Carver {
    unsigned char* base;
    size_t used = 0;
    // a measuring pass (p == NULL) hands out addresses from a fake base: never dereferenced, but non-null, so
    // that code which asks "was this region carved" takes the same route as the real pass
    explicit Carver(void* p) : base(p ? static_cast<unsigned char*>(p) : reinterpret_cast<unsigned char*>((uintptr_t)1 << 20)) {}
    void* take(int64_t bytes)
    {
        void* p = bytes > 0 ? base + used : nullptr;
        used += (size_t)round_up(bytes > 0 ? bytes : 0, 256);
        return p;
    }
};

// Buffers an entry point may need, laid out identically by the measuring pass and the
// real pass.
struct Scratch {
    uint32_t* header = nullptr; // first QSKINNY_HEADER_BYTES of every workspace: arrival counters, zero between calls
    void* A_p = nullptr;    // bf16 [K][rp]   zero-padded copy of A when r % 8 != 0
    void* B_p = nullptr;    // bf16 [rp][N]
    void* H = nullptr;      // bf16 [M][rp]
    void* dH = nullptr;     // bf16 [M][rp]
    float* Hf = nullptr;    // fp32 [M][rp]   split-K accumulator for the rank-r products
    float* dA_t = nullptr;  // fp32 [K][rp]
    float* dB_t = nullptr;  // fp32 [rp][N]
    float* part = nullptr;  // fp32 partial sums of a split reduction, one slab per split
    int64_t part_bytes = 0; // what is reserved behind `part`
    void* Wm = nullptr;     // bf16 [K][N]    base_scale * deq(W) + scaling * A B, many tokens (see many_tokens)
    float* sk_part = nullptr;   // weight-streaming forward (few tokens): slabs of M x N
    float* sk_hpart = nullptr;  //                                        partial sums of X A
    float* sk_dxpart = nullptr; // weight-streaming input gradient (few tokens): slabs of M x K
    float* sk_dhpart = nullptr; //                                                partial sums of dY B^T
};

int64_t rank_pad(int64_t r) { return round_up(r, 8); }


// With many tokens the frozen-weight product dominates the finetuning layer, and the plain bf16 kernels
// (operands through global -> LDS requests) run it about 1.5 times faster than the kernels that
// dequantise the weight in their load path.  One pass that writes  base_scale * deq(W) + scaling * A B
// as bf16 [K][N] costs what about 600 token rows of that product cost, and removes the rank-r branch
// from the big product as well (W' x = W x + s B A x, Sec. 5.1).  288 GB of HBM make room for it.
// The forward and the backward call each merge for themselves; measured on 4096 x 4096 int8 and on a
// 13B decoder layer in int4, a whole step is faster this way from about 1152 tokens on.
// More than 16 tokens on one weight through the weight-streaming forward: the token rows in blocks of 16, every block a
// job of its own on the same weight (the 16-token kernel holds three workgroups per compute unit and its finishers
// gather a quarter of the slab rows each).  The plan of that launch.
static int token_blocks(int64_t M) { return (int)((M + 15) / 16); }
static QskinnyPlan qskinny_plan_token_blocks(int64_t M, int64_t K, int64_t r, int64_t N)
{
    int64_t Ns[QSKINNY_MAX_JOBS];
    const int tb = token_blocks(M);
    for (int t = 0; t < tb; t++) Ns[t] = N;
    return qskinny_plan(16, K, r, Ns, tb, num_cu());
}
// It pays while every (token block, 64-channel block) pair can still have three slices of the reduction in the one
// round of resident workgroups (measured at 64 tokens, forward, per call: 4096 x 4096 int8 29 -> 24 microseconds, at 32
// tokens 20 -> 18; 5120 x 5120 int4 the same either way; with more channel blocks than that the slices get so
// long that the blocks lose: 5120 x 13824 int4 59 -> 90 microseconds).
static bool token_blocks_pay(int64_t M, int64_t K, int64_t r, int64_t N)
{
    (void)K; (void)r;
    if (M <= 16 || token_blocks(M) > QSKINNY_MAX_JOBS) return false;
    const int64_t blocks = (N + 63) / 64 * token_blocks(M);
    return 3 * blocks <= 3 * (int64_t)num_cu();
}

bool many_tokens(int op, int64_t M, int64_t K, int64_t N);


int64_t tile_count(int tile, int64_t M, int64_t N)
{
    int bm, bn;
    gemm_tile_extent(tile, &bm, &bn);
    return ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
}

// How an fp32-output product whose reduction is split across workgroups is launched:
// the largest tile that fits the output (the splits, not the tiles, fill the chip) and
// as many slices of the reduction as it takes to occupy every compute unit.
struct SplitPlan {
    int tile, splits, k_chunk;
};

// `g` > 1: that many products of this shape share the launch (a grouped launch): their tiles fill the chip together,
// and every slice adds a slab per product.
SplitPlan plan_split_on(int tile, int64_t M, int64_t N, int64_t Kred, int g = 1)
{
    SplitPlan sp;
    sp.tile = tile;
    const int64_t tiles = tile_count(sp.tile, M, N) * g;
    const int64_t ksteps = (Kred + 63) / 64;
    // the eight-wave tiles occupy a compute unit alone; 128x128 runs two at a time.  The skinny tiles could
    // too, but their products are bound by streaming the long operand, and one workgroup per compute
    // unit with twice the depth measured faster than two (4096 x 5120 -> 16: 11.4 against 14.8 microseconds)
    // and leaves half as many slabs to add.
    const int64_t target = (sp.tile == TILE_128x128) ? 2 * num_cu() : num_cu();
    int64_t s = (target + tiles - 1) / tiles;
    if (s > ksteps) s = ksteps;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    if ((sp.tile == TILE_256x256 || sp.tile == TILE_256x128) && (tiles < target || (g > 1 && tiles % target != 0)) && ksteps >= 16) {
        // The eight-wave tiles run one workgroup per compute unit, so what a launch takes is the number of
        // rounds its tiles x slices need times the depth of a slice, plus a fixed part per round (ring fill,
        // fp32 epilogue) and the slabs it writes and the slab sum reads.  The rule above can leave a second
        // round nearly empty (96 tiles in 3 slices: 288 items, 235 microseconds for 4096 x 1536 over 16384
        // tokens; in 5 slices two full rounds of shorter slices); take the cheapest count instead.
        // (A grouped launch with more tiles than units is searched too: 344 tiles leave two thirds of the second
        // round empty, in two slices they are 2.7 rounds of half the depth.)
        // Units: 64-deep steps of a 256 x 256 tile (about 1.5 microseconds each).
        const double tile_steps = (sp.tile == TILE_256x256) ? 1.0 : 0.5;
        const double fixed_steps = 5.0;                                     // per round
        const double slab_steps = (double)g * (double)M * (double)N * 8.0 / 4.0e12 / 1.5e-6;   // one slab (per product) written and read at 4 TB/s
        double best = -1.0;
        for (int64_t c = 1; c <= 64 && c <= ksteps / 8; c++) {
            const int64_t rounds = (tiles * c + target - 1) / target;
            const int64_t per = (ksteps + c - 1) / c;
            const double cost = (double)rounds * ((double)per * tile_steps + fixed_steps) + (c > 1 ? (double)c * slab_steps : 0.0);
            if (best < 0.0 || cost < best) {
                best = cost;
                s = c;
            }
        }
    }
    const int64_t steps_per = (ksteps + s - 1) / s;
    sp.k_chunk = (int)(steps_per * 64);
    sp.splits = (int)((ksteps + steps_per - 1) / steps_per);
    return sp;
}

// `rows32`: 32-row tiles whatever M is (the only fp32-output shape of the products X A, H B, dY B^T, dH A^T)
SplitPlan plan_split(int64_t M, int64_t N, int64_t Kred, bool rows32 = false, int g = 1)
{
    int tile;
    if (N <= 32) tile = TILE_256x32;
    else if (M <= 32 || rows32) tile = TILE_32x256;
    else if (M > 128 && N > 128) tile = TILE_256x256;
    else if (M > 128) tile = TILE_256x128;
    else if (N > 128) tile = TILE_128x256;
    else tile = TILE_128x128;
    SplitPlan sp = plan_split_on(tile, M, N, Kred, g);
    if (tile == TILE_256x256 && sp.splits >= 8) {
        // Many slices mean many partial-sum slabs to write and re-read.  The 256x128 shape needs
        // half as many; measured, it wins from eight slices on (config 2: 4096x512 outputs over
        // 16384 tokens) and loses below (config 3: the 256x256 kernel is 25 % faster there).
        const SplitPlan alt = plan_split_on(TILE_256x128, M, N, Kred, g);
        if (alt.splits < sp.splits) sp = alt;
    }
    return sp;
}

// Bytes of partial-sum slabs for an M x N (leading dimension ldc) product reduced over Kred.
int64_t split_bytes(int64_t M, int64_t N, int64_t ldc, int64_t Kred, bool rows32 = false)
{
    const SplitPlan sp = plan_split(M, N, Kred, rows32);
    return sp.splits > 1 ? (int64_t)sp.splits * M * ldc * 4 : 0;
}

// A bf16 product M x Nout whose plain launch would put tiles on fewer than half of the compute units,
// while its reduction is long, is bound by streaming the long operand through those few units: it runs
// as a split reduction on 32-row tiles instead, as many slices as fill the chip, and the slab sum
// rounds to bf16.  Measured on one factorised layer 4096 -> 512 -> 4096, forward: 64 tokens 52 -> 28
// microseconds, 256 tokens 53 -> 30, 1024 tokens 54 -> 47; 11008 -> 1024 -> 4096 at 64 tokens 125 -> 30.
// (Outputs at most 32 wide have their own split shape, see rank_product.)
bool split_pays(int64_t M, int64_t Nout, int64_t Kred)
{
    if (Nout <= 32) return false;
    if (M > 32) {
        const int64_t tiles = ((M + 127) / 128) * ((Nout + 127) / 128);
        if (2 * tiles > num_cu() || Kred < 256) return false;
    }
    return plan_split(M, Nout, Kred, true).splits > 1;
}

// From 256 tokens on, an output that gives at most a quarter of the compute units a 256 x 128 tile, with a
// reduction of 1024 or more, takes the large request-fed tiles for its slices instead (slices of at least
// 512): one factorised layer 4096 -> 512 -> 4096 at 2048 tokens, forward 55 -> 43 microseconds and backward
// 107 -> 96 against the 32-row tiles; at 4096 tokens, where X A is 64 tiles in 4 slices, 69 -> 56 and
// 136 -> 125 against 128 unsplit tiles of 128 x 128.  At 8192 tokens (128 tiles) the slices and their slab
// sum take longer than the small tiles do: 54 + 8 against 57 microseconds.
SplitPlan plan_large_split(int64_t M, int64_t Nout, int64_t Kred)
{
    SplitPlan sp = plan_split(M, Nout, Kred);
    const int64_t ksteps = (Kred + 63) / 64;
    if (sp.k_chunk < 512) {
        // fewer slices, each 512 deep at least
        const int64_t s = ksteps / 8 > 0 ? ksteps / 8 : 1;
        const int64_t steps_per = (ksteps + s - 1) / s;
        sp.k_chunk = (int)(steps_per * 64);
        sp.splits = (int)((ksteps + steps_per - 1) / steps_per);
    }
    return sp;
}

bool large_split_pays(int64_t M, int64_t Nout, int64_t Kred)
{
    if (M < 256 || Nout <= 128 || Kred < 1024) return false;
    if (4 * tile_count(TILE_256x128, M, Nout) > num_cu()) return false;
    const SplitPlan sp = plan_large_split(M, Nout, Kred);
    // (with fewer workgroups than half the compute units the 32-row tiles do better)
    return sp.splits > 1 && 2 * sp.splits * tile_count(sp.tile, M, Nout) >= num_cu();
}

int64_t product_part_bytes(int64_t M, int64_t Nout, int64_t Kred)
{
    if (large_split_pays(M, Nout, Kred)) return (int64_t)plan_large_split(M, Nout, Kred).splits * M * Nout * 4;
    return split_pays(M, Nout, Kred) ? split_bytes(M, Nout, Nout, Kred, true) : 0;
}

// The products of the finetuning and blend layers that dequantise the frozen weight in their load path
// (65 .. 1151 tokens) read that weight once per row of output tiles: with few tiles the launch is bound by
// streaming the weight through few compute units.  Its reduction is then cut into slices of at least 512,
// as many as fit the chip at once (one slice more and a second, nearly empty round of workgroups costs more
// than the slices gain); the rank-r phase stays with slice 0 and a slab sum writes the bf16 output.
// Up to 256 tiles of 128 x 128 (two workgroups per compute unit) that tile is used; a larger output of at
// most 128 tiles of 256 x 256 (one workgroup per compute unit) takes those.  Measured on a 4-bit
// 5120 x 5120 weight: 65 tokens 76 -> 34 microseconds forward and 96 -> 49 backward, 256 tokens 86 -> 47 and
// 101 -> 63, 1024 tokens (80 tiles of 256 x 256, 3 slices) 107 -> 91 and 133 -> 108.
SplitPlan plan_fused_split(int64_t M, int64_t Nout, int64_t Kred)
{
    SplitPlan sp;
    sp.tile = TILE_128x128;
    sp.splits = 1;
    sp.k_chunk = (int)round_up(Kred, 64);
    const int64_t ksteps = (Kred + 63) / 64;
    const int64_t small = tile_count(TILE_128x128, M, Nout), large = tile_count(TILE_256x256, M, Nout);
    int64_t s;
    if (small <= num_cu()) {
        s = (2 * num_cu()) / small;
    } else {
        s = num_cu() / large;
        sp.tile = TILE_256x256;
    }
    if (s > ksteps / 8) s = ksteps / 8;
    if (s > 16) s = 16;
    if (s < 2) return sp;
    // two slices of a short reduction on the large tile do not pay for their slabs (4096 x 4096 at 1536 and
    // 2047 tokens: 86 against 79 and 99 against 89 microseconds unsplit); three do, and so do two of a long one
    if (sp.tile == TILE_256x256 && s == 2 && Kred < 8192) {
        sp.tile = TILE_128x128;
        return sp;
    }
    const int64_t steps_per = (ksteps + s - 1) / s;
    sp.k_chunk = (int)(steps_per * 64);
    sp.splits = (int)((ksteps + steps_per - 1) / steps_per);
    return sp;
}

int64_t fused_part_bytes(int64_t M, int64_t Nout, int64_t Kred)
{
    const SplitPlan sp = plan_fused_split(M, Nout, Kred);
    return sp.splits > 1 ? (int64_t)sp.splits * M * Nout * 4 : 0;
}

// How much of the chip the dequantising product M x Nout keeps busy: the share of workgroup slots its best
// launch fills over its rounds, times the per-flop standing of that tile shape (see pick_tile).
static double dequant_route_fill(int64_t M, int64_t Nout, int64_t Kred)
{
    const SplitPlan sp = plan_fused_split(M, Nout, Kred);
    if (sp.splits > 1) {
        const bool small = (sp.tile == TILE_128x128);
        return (double)(tile_count(sp.tile, M, Nout) * sp.splits) / (double)((small ? 2 : 1) * num_cu());
    }
    const int tiles[4] = {TILE_256x256, TILE_256x128, TILE_128x256, TILE_128x128};
    const double standing[4] = {1.0, 0.95, 0.8, 0.67};
    double best = 0.0;
    for (int i = 0; i < 4; i++) {
        const int64_t n = tile_count(tiles[i], M, Nout), slots = (i == 3 ? 2 : 1) * num_cu();
        const double f = (double)n / (double)(((n + slots - 1) / slots) * slots) * standing[i];
        if (f > best) best = f;
    }
    return best;
}

// From 1152 tokens on the finetuning and blend layers merge the weight and run plain products (see above):
// config 5's layer per step at 1280 / 1536 tokens 2478 / 2620 microseconds merged against 2557 / 2708
// dequantising, config 4's 656 against 705 at 1152; at 1024 tokens the dequantising route with its reduction
// in slices is ahead (1944 against 2157).  Between 1024 and 1151 tokens the layers merge only when the
// dequantising product would leave much of the chip idle for want of a tile shape that fits.
bool many_tokens(int op, int64_t M, int64_t K, int64_t N)
{
    if (M >= 1152) return true;
    if (M < 1024) return false;
    const bool fwd = (op == FHPC_OP_QLINEAR_FWD);
    return dequant_route_fill(M, fwd ? N : K, fwd ? K : N) < 0.7;
}

// The quantised layer's input gradient for at most 64 tokens is bound by reading the packed weight
// once: it then comes from the weight-streaming kernel (both schemes have the same shape limits).
bool stream_dx(int64_t M, int64_t K, int64_t r, int64_t N)
{
    return qskinny_dx_supports(M, K, r, N, FHPC_Q_INT4_BLOCK) && qskinny_dx_supports(M, K, r, N, FHPC_Q_INT8_PER_CHANNEL);
}

Scratch carve(Carver& c, int op, int64_t M, int64_t K, int64_t r, int64_t N, int dtype, bool quantised = true,
              bool premerged = false)
{
    Scratch s;
    s.header = static_cast<uint32_t*>(c.take(QSKINNY_HEADER_BYTES));
    if (dtype == FHPC_F32) {
        // fp32 path: H and dH in fp32, no padding
        s.H = c.take(M * r * 4);
        if (op == FHPC_OP_LOWRANK_BWD) s.dH = c.take(M * r * 4);
        return s;
    }
    if (op == FHPC_OP_QLINEAR_FWD && quantised && qskinny_supports(M, K, r, N, FHPC_Q_INT4_BLOCK)) {
        // a handful of tokens: the weight-streaming kernels need only their own slabs
        QskinnyPlan p = qskinny_plan(M, K, r, &N, 1, num_cu());
        if (M > 16) {                                  // (the same tokens in blocks of 16: whichever plan needs more)
            const QskinnyPlan pb = qskinny_plan_token_blocks(M, K, r, N);
            if (pb.part_bytes > p.part_bytes) p.part_bytes = pb.part_bytes;
            if (pb.hpart_bytes > p.hpart_bytes) p.hpart_bytes = pb.hpart_bytes;
        }
        s.sk_part = static_cast<float*>(c.take(p.part_bytes));
        s.sk_hpart = static_cast<float*>(c.take(p.hpart_bytes));
        return s;
    }
    const int64_t rp = rank_pad(r);
    const bool bwd = (op == FHPC_OP_LOWRANK_BWD || op == FHPC_OP_QLINEAR_BWD);
    if ((op == FHPC_OP_QLINEAR_FWD || op == FHPC_OP_QLINEAR_BWD) && !premerged && many_tokens(op, M, K, N))
        s.Wm = c.take((K + rp) * (N + MERGE_EXT_PAD) * 2);          // (room for the factor pair beside and below it, see rides_along)
    if (rp != r) {
        s.A_p = c.take(K * rp * 2);
        s.B_p = c.take(rp * N * 2);
    }
    s.H = c.take(M * rp * 2);
    if (bwd) s.dH = c.take(M * rp * 2);
    if (rp <= 32) s.Hf = static_cast<float*>(c.take(M * rp * 4));
    if (bwd && rp != r) {
        s.dA_t = static_cast<float*>(c.take(K * rp * 4));
        s.dB_t = static_cast<float*>(c.take(rp * N * 4));
    }
    if (op == FHPC_OP_QLINEAR_BWD && quantised && stream_dx(M, K, r, N)) {
        // a handful of tokens: dX comes from the weight-streaming kernel (sized for either scheme)
        const int64_t b4 = qskinny_dx_plan(M, K, N, FHPC_Q_INT4_BLOCK, num_cu()).part_bytes;
        const int64_t b8 = qskinny_dx_plan(M, K, N, FHPC_Q_INT8_PER_CHANNEL, num_cu()).part_bytes;
        s.sk_dxpart = static_cast<float*>(c.take(b4 > b8 ? b4 : b8));
        if (rp <= 16) {       // dH = dY B^T is then formed by the same launch, one partial sum per slice
            const int s4 = qskinny_dx_plan(M, K, N, FHPC_Q_INT4_BLOCK, num_cu()).slices;
            const int s8 = qskinny_dx_plan(M, K, N, FHPC_Q_INT8_PER_CHANNEL, num_cu()).slices;
            s.sk_dhpart = static_cast<float*>(c.take((int64_t)(s4 > s8 ? s4 : s8) * M * rp * 4));
        }
    }
    // split reductions of this entry point run one after another and share the slabs
    int64_t part = 0;
    auto upto = [&part](int64_t b) { if (b > part) part = b; };
    if (rp <= 32) {
        upto(split_bytes(M, rp, rp, K));               // H  = X A
        if (bwd) upto(split_bytes(M, rp, rp, N));      // dH = dY B^T
    } else {
        upto(product_part_bytes(M, rp, K));
        if (bwd) upto(product_part_bytes(M, rp, N));
    }
    if (op == FHPC_OP_QLINEAR_FWD) upto(fused_part_bytes(M, N, K));        // Y  = X deq(W) + s H B
    if (op == FHPC_OP_QLINEAR_BWD) upto(fused_part_bytes(M, K, N));        // dX = dY deq(W)^T + s dH A^T
    if (op == FHPC_OP_LOWRANK_FWD) upto(product_part_bytes(M, N, rp));     // Y  = H B
    if (op == FHPC_OP_LOWRANK_BWD) upto(product_part_bytes(M, K, rp));     // dX = dH A^T
    if (bwd) {
        upto(split_bytes(K, rp, rp, M) + split_bytes(rp, N, N, M));   // dA = X^T dH and dB = H^T dY, slabs side by side
    }
    s.part = static_cast<float*>(c.take(part));
    s.part_bytes = part;
    return s;
}

int check_common(int64_t M, int64_t K, int64_t r, int64_t N)
{
    if (M < 1 || K < 1 || r < 1 || N < 1) return FHPC_ERR_SHAPE;
    if ((K % 8) || (N % 8)) return FHPC_ERR_SHAPE;
    if (K > ((int64_t)1 << 20) || N > ((int64_t)1 << 20) || r > ((int64_t)1 << 16)) return FHPC_ERR_UNSUPPORTED;
    if (M > ((int64_t)1 << 30)) return FHPC_ERR_UNSUPPORTED;
    // the GEMM core addresses each operand with 32-bit byte offsets
    const int64_t rp = rank_pad(r);
    const int64_t widest = (K > N ? K : N) > rp ? (K > N ? K : N) : rp;
    if (M * widest * 2 >= kMaxBytes || K * rp * 2 >= kMaxBytes || rp * N * 2 >= kMaxBytes || K * N >= kMaxBytes)
        return FHPC_ERR_UNSUPPORTED;
    return FHPC_OK;
}

// Tile for an M x N output.  The narrow tiles exist only for the split rank-r products, so they are
// offered only when `allow_skinny`.  Among the four large tiles the choice follows the time the launch
// should take: rounds of resident workgroups x tile area x a per-flop penalty of the smaller shapes
// (measured on 4096-token products: 256x128 about 5 % behind 256x256 per flop, 128x256 25 %, 128x128
// 50 %; the 128x128 kernel runs two workgroups per compute unit).  What it decides in practice: an
// output of 320 tiles of 256x256 (4096 tokens x 5120 channels) would run two rounds, the second a
// quarter full; as 640 tiles of 256x128 it runs 2.5 (measured 196 against 217 microseconds).
int pick_tile(int64_t M, int64_t N, bool allow_skinny)
{
    if (allow_skinny && N <= 32) return TILE_256x32;
    if (allow_skinny && M <= 32) return TILE_32x256;
    const int order[4] = {TILE_256x256, TILE_256x128, TILE_128x256, TILE_128x128};
    const double penalty[4] = {1.0, 1.05, 1.25, 1.5};
    int best = TILE_128x128;
    double best_cost = -1.0;
    for (int i = 0; i < 4; i++) {
        int bm, bn;
        gemm_tile_extent(order[i], &bm, &bn);
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        // what the busiest compute unit has to work through, whether its tiles come one after the other or
        // share it (128 x 128 runs two at a time); a shape that leaves some units without a tile may still be
        // the fastest (12288 x 512: 192 tiles of 256 x 128 in 75 microseconds against 384 of 128 x 128 in 85)
        const double cost = (double)((tiles + num_cu() - 1) / num_cu()) * bm * bn * penalty[i];
        if (best_cost < 0.0 || cost < best_cost) {
            best = order[i];
            best_cost = cost;
        }
    }
    return best;
}

// What pick_tile minimises, for the tile it picks.
static double tile_cost(int64_t M, int64_t N, int* tile_out)
{
    const int tile = pick_tile(M, N, false);
    int bm, bn;
    gemm_tile_extent(tile, &bm, &bn);
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    if (tile_out) *tile_out = tile;
    return (double)((tiles + num_cu() - 1) / num_cu()) * bm * bn;
}

// The merged-weight products of the finetuning layer can carry a rank-r product along: with the merged weight in the
// extended layout of merge.h, X times it has H = X A in rp extra output columns, and dY times its transpose has
// dH = dY B^T there, written by the same launch through its second output (no pass over X or dY of their own, no
// slabs, no slab sum).  That costs one more column of tiles.  It is taken when that column does not add a round
// of workgroups (4096 tokens x 5120 channels: 656 tiles of 256 x 128 in the three rounds that 640 take; 4096 x 4096
// is exactly one round of 256 x 256 tiles and a 17th column would double it), when the request-fed kernels run
// the product on a tile whose width divides `width`, and for no more than 64 extra columns.
static bool rides_along(int a_mode, int b_mode, int64_t M, int64_t width, int64_t rp)
{
    if (rp > 64) return false;
    int tile = 0, tile0 = 0;
    const double with = tile_cost(M, width + rp, &tile), without = tile_cost(M, width, &tile0);
    if (with > without) return false;
    int bm, bn;
    gemm_tile_extent(tile, &bm, &bn);
    return width % bn == 0 && gemm_pp_supports(a_mode, b_mode, OP_NONE, OUT_BF16, tile);
}

// C[M][n_main] (ldc) and C2[M][n_all - n_main] (ldc2): one bf16 product whose trailing columns go to a second output.
static hipError_t gemm_two_outputs(int a_mode, int b_mode, GemmOperand a, GemmOperand b, void* C, int64_t ldc, void* C2, int64_t ldc2,
                                   int64_t M, int64_t n_main, int64_t n_all, int64_t Kred, Run& run)
{
    if (run.dry) return hipSuccess;
    GemmArgs g = {};
    g.a = a; g.b = b; g.c = C; g.ldc = ldc;
    g.c2 = C2; g.ldc2 = ldc2; g.n_split = (int)n_main;
    g.M = (int)M; g.N = (int)n_all; g.K = (int)Kred; g.K2 = 0;
    g.alpha = 1.f; g.mid_scale = 1.f; g.splits = 1; g.k_chunk = (int)round_up(Kred, 64);
    return launch_gemm_bf16(a_mode, b_mode, OP_NONE, OUT_BF16, pick_tile(M, n_all, false), g, run.st);
}

GemmOperand operand(const void* p, int64_t ld, const void* scales = nullptr, int64_t sld = 0)
{
    GemmOperand o;
    o.ptr = p;
    o.ld = ld;
    o.scales = scales;
    o.scale_ld = sld;
    return o;
}

// C[M,N] bf16 = A(KC or via a_mode) * B, whole reduction in one workgroup per tile.
hipError_t gemm_plain(int a_mode, int b_mode, GemmOperand a, GemmOperand b, void* C, int64_t ldc,
                      int64_t M, int64_t N, int64_t Kred, Run& run, float alpha = 1.f)
{
    if (run.dry) return hipSuccess;
    hipStream_t st = run.st;
    GemmArgs g = {};
    g.a = a; g.b = b; g.c = C; g.ldc = ldc;
    g.M = (int)M; g.N = (int)N; g.K = (int)Kred; g.K2 = 0;
    g.alpha = alpha; g.mid_scale = 1.f; g.splits = 1; g.k_chunk = (int)round_up(Kred, 64);
    return launch_gemm_bf16(a_mode, b_mode, OP_NONE, OUT_BF16, pick_tile(M, N, false), g, st);
}

// C[M,N] fp32 (ldc) = alpha * A * B with the reduction split across workgroups: every
// slice stores its partial sums to its own slab of `part` (no atomics, so the result does
// not depend on scheduling) and a second kernel adds the slabs into C.
// With `bf16_out` (dense, ldc == N) and more than one slice, the slab sum writes bf16 there and C is
// left alone: *wrote_bf16 tells the caller which happened.
hipError_t gemm_split_f32(int a_mode, int b_mode, GemmOperand a, GemmOperand b, float* C, int64_t ldc,
                          int64_t M, int64_t N, int64_t Kred, float alpha, float* part, Run& run,
                          void* bf16_out = nullptr, bool* wrote_bf16 = nullptr, bool rows32 = false,
                          const SplitPlan* plan = nullptr)
{
    if (wrote_bf16) *wrote_bf16 = false;
    const SplitPlan sp = plan ? *plan : plan_split(M, N, Kred, rows32);
    if (!run.claim(sp.splits > 1 ? (int64_t)sp.splits * M * ldc * 4 : 0)) return hipErrorOutOfMemory;
    if (run.dry) {
        if (wrote_bf16) *wrote_bf16 = (sp.splits > 1 && bf16_out);
        return hipSuccess;
    }
    hipStream_t st = run.st;
    GemmArgs g = {};
    g.a = a; g.b = b; g.ldc = ldc;
    g.M = (int)M; g.N = (int)N; g.K = (int)Kred; g.K2 = 0;
    g.alpha = alpha; g.mid_scale = 1.f;
    g.splits = sp.splits; g.k_chunk = sp.k_chunk;
    if (sp.splits == 1) {
        g.c = C;
        g.split_stride = 0;
        return launch_gemm_bf16(a_mode, b_mode, OP_NONE, OUT_F32, sp.tile, g, st);
    }
    g.c = part;
    g.split_stride = M * ldc;
    hipError_t e = launch_gemm_bf16(a_mode, b_mode, OP_NONE, OUT_F32, sp.tile, g, st);
    if (e != hipSuccess) return e;
    if (bf16_out && wrote_bf16) {
        *wrote_bf16 = true;
        return launch_sum_slabs(part, M * ldc, sp.splits, bf16_out, true, st);
    }
    return launch_sum_slabs(part, M * ldc, sp.splits, C, false, st);
}

// P[M][Nout] (bf16, row stride ldp) = L * R, L with k contiguous: the plain launch, or the split reduction on
// 32-row tiles when that pays (split_pays) and P is dense.
hipError_t product_bf16(int b_mode, GemmOperand a, GemmOperand b, void* P, int64_t ldp, int64_t Nout,
                        int64_t M, int64_t Kred, float* part, Run& run)
{
    const bool large = large_split_pays(M, Nout, Kred);
    if (ldp == Nout && (large || split_pays(M, Nout, Kred))) {
        bool done = false;
        // more than one slice (checked by both rules), so the slab sum writes P and no fp32 output is touched
        const SplitPlan lp = large ? plan_large_split(M, Nout, Kred) : SplitPlan();
        return gemm_split_f32(OP_KC, b_mode, a, b, nullptr, Nout, M, Nout, Kred, 1.f, part, run, P, &done, !large,
                              large ? &lp : nullptr);
    }
    return gemm_plain(OP_KC, b_mode, a, b, P, ldp, M, Nout, Kred, run);
}

// Whether a dense bf16 product M x Nout runs as one plain launch of the 256 x 256 request-fed kernel, the one
// whose epilogue can apply the FFN's SiLU gate to the tile it has just produced (GemmArgs::gate).
static bool gate_rides(int64_t M, int64_t Nout, int64_t Kred)
{
    if (large_split_pays(M, Nout, Kred) || split_pays(M, Nout, Kred)) return false;
    return pick_tile(M, Nout, false) == TILE_256x256;
}

// P[M][Nout] = a * b^(b_mode) (a with k contiguous) with the gate in the epilogue.  gate 1: P is stored and
// out1 = SiLU(G) * P; gate 2: P is not stored, out1 = dG and out2 = dU for dZ = P.  All dense, Nout wide.
static hipError_t gemm_gated(int b_mode, GemmOperand a, GemmOperand b, void* P, int64_t M, int64_t Nout, int64_t Kred,
                             int gate, const void* G, const void* U, void* out1, void* out2, Run& run)
{
    if (run.dry) return hipSuccess;
    GemmArgs g = {};
    g.a = a; g.b = b; g.c = P; g.ldc = Nout;
    g.M = (int)M; g.N = (int)Nout; g.K = (int)Kred; g.K2 = 0;
    g.alpha = 1.f; g.mid_scale = 1.f; g.splits = 1; g.k_chunk = (int)round_up(Kred, 64);
    g.gate = gate; g.gate_g = G; g.gate_u = U; g.gate_out1 = out1; g.gate_out2 = out2;
    return launch_gemm_bf16(OP_KC, b_mode, OP_NONE, OUT_BF16, TILE_256x256, g, run.st);
}

// A rank-r output of many rows whose operands both have the reduction contiguous (dH = dY B^T) goes out as one launch
// of 16-row workgroups that own the whole reduction, without slabs and their sum, once there are rows enough for
// half the compute units (C4's backward: 11.6 + 4.5 microseconds of product and slab sum become one launch, the step
// 1.262 -> 1.253 ms).
static bool tall_skinny_pays(int64_t M) { return M >= 8 * (int64_t)num_cu(); }

// Rank-r product P[M][rp] (bf16) = L * R where the output is only rp <= 32 wide:
// split the long reduction, accumulate in fp32, then round once to bf16.
hipError_t rank_product(int b_mode, GemmOperand a, GemmOperand b, void* P, int64_t rp, float* Pf, float* part,
                        int64_t M, int64_t Kred, Run& run)
{
    if (rp <= 32 && b_mode == OP_KC && (Kred % 32) == 0 && tall_skinny_pays(M)) {
        // many rows, both operands with the reduction contiguous (dH = dY B^T): one launch that owns the whole reduction
        if (run.dry) return hipSuccess;
        return launch_tall_skinny_kc(a.ptr, a.ld, b.ptr, b.ld, P, M, rp, Kred, run.st);
    }
    if (rp <= 32) {
        bool done = false;
        hipError_t e = gemm_split_f32(OP_KC, b_mode, a, b, Pf, rp, M, rp, Kred, 1.f, part, run, P, &done);
        if (e != hipSuccess || done || run.dry) return e;
        return launch_compact_f32(Pf, rp, P, rp, M, rp, 1.f, true, run.st);
    }
    return product_bf16(b_mode, a, b, P, rp, rp, M, Kred, part, run);
}

// C[M][Nout] (bf16, dense) = g.alpha * (g.mid_scale * A2 B2 + A deq(B)): whole, or split over the reduction
hipError_t fused_product(int b_mode, int b2_mode, GemmArgs g, void* C, int64_t M, int64_t Nout, int64_t Kred,
                         float* part, Run& run)
{
    const SplitPlan sp = plan_fused_split(M, Nout, Kred);
    if (!run.claim(sp.splits > 1 ? (int64_t)sp.splits * M * Nout * 4 : 0)) return hipErrorOutOfMemory;
    if (run.dry) return hipSuccess;
    hipStream_t st = run.st;
    g.ldc = Nout;
    if (sp.splits == 1) {
        g.c = C;
        g.splits = 1;
        g.k_chunk = (int)round_up(Kred, 64);
        return launch_gemm_bf16(OP_KC, b_mode, b2_mode, OUT_BF16, pick_tile(M, Nout, false), g, st);
    }
    g.c = part;
    g.splits = sp.splits;
    g.k_chunk = sp.k_chunk;
    g.split_stride = M * Nout;
    hipError_t e = launch_gemm_bf16(OP_KC, b_mode, b2_mode, OUT_F32, sp.tile, g, st);
    if (e != hipSuccess) return e;
    return launch_sum_slabs(part, M * Nout, sp.splits, C, true, st);
}

struct Factors {
    const void* A;   // bf16 [K][rp]
    const void* B;   // bf16 [rp][N]
};

// Zero-padded copies of A and B when the rank is not a multiple of 8.
int prepare_factors(const void* A, const void* B, int64_t K, int64_t r, int64_t rp, int64_t N,
                    const Scratch& s, Run& run, Factors* f)
{
    if (rp == r) {
        f->A = A;
        f->B = B;
        return FHPC_OK;
    }
    FHPC_LAUNCH(run, launch_pad2d_u16(A, r, K, r, s.A_p, rp, K, run.st));
    FHPC_LAUNCH(run, launch_pad2d_u16(B, N, r, N, s.B_p, N, rp, run.st));
    f->A = s.A_p;
    f->B = s.B_p;
    return FHPC_OK;
}

// dA[K][r] = alpha X^T dH and dB[r][N] = alpha H^T dY, both reductions over the M tokens.
int weight_grads(const void* X, const void* dY, const void* H, const void* dH, float* dA, float* dB,
                 int64_t M, int64_t K, int64_t r, int64_t rp, int64_t N, float alpha,
                 const Scratch& s, Run& run)
{
    hipStream_t st = run.st;
    // a handful of tokens: M-deep sums, both products in one launch of the vector-ALU kernel, until the sums
    // over the tokens outweigh writing the outputs once
    if ((dA || dB) && token_outer_supports(M) && (M <= 32 || rp * (K + N) <= ((int64_t)8 << 20))) {
        FHPC_LAUNCH(run, launch_token_outer_grads(X, dH, dA, H, dY, dB, M, K, r, rp, N, alpha, st));
        return FHPC_OK;
    }
    if (dA && dB) {
        // both reductions in slices, both sums small: the two slab sets sit side by side and one launch adds both
        const SplitPlan pa = plan_split(K, rp, M), pb = plan_split(rp, N, M);
        const int64_t na = K * rp, nb = rp * N;
        if (pa.splits > 1 && pb.splits > 1 && sum_slabs_is_small(na, pa.splits) && sum_slabs_is_small(nb, pb.splits) &&
            run.claim(((int64_t)pa.splits * na + (int64_t)pb.splits * nb) * 4)) {
            float* const da = (rp == r) ? dA : s.dA_t;
            float* const db = (rp == r) ? dB : s.dB_t;
            float* const part_b = s.part + (int64_t)pa.splits * na;
            if (!run.dry) {
                GemmArgs g = {};
                g.a = operand(X, K); g.b = operand(dH, rp); g.c = s.part; g.ldc = rp;
                g.M = (int)K; g.N = (int)rp; g.K = (int)M; g.alpha = alpha; g.mid_scale = 1.f;
                g.splits = pa.splits; g.k_chunk = pa.k_chunk; g.split_stride = na;
                FHPC_HIP(launch_gemm_bf16(OP_XC, OP_XC, OP_NONE, OUT_F32, pa.tile, g, st));
                g.a = operand(H, rp); g.b = operand(dY, N); g.c = part_b; g.ldc = N;
                g.M = (int)rp; g.N = (int)N;
                g.splits = pb.splits; g.k_chunk = pb.k_chunk; g.split_stride = nb;
                FHPC_HIP(launch_gemm_bf16(OP_XC, OP_XC, OP_NONE, OUT_F32, pb.tile, g, st));
                FHPC_HIP(launch_sum_slabs_pair(s.part, na, pa.splits, da, part_b, nb, pb.splits, db, st));
                if (rp != r) {
                    FHPC_HIP(launch_compact_f32(s.dA_t, rp, dA, r, K, r, 1.f, false, st));
                    FHPC_HIP(launch_compact_f32(s.dB_t, N, dB, N, r, N, 1.f, false, st));
                }
            }
            return FHPC_OK;
        }
    }
    if (dA) {
        float* dst = (rp == r) ? dA : s.dA_t;
        FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, operand(X, K), operand(dH, rp), dst, rp, K, rp, M, alpha, s.part, run));
        if (rp != r) FHPC_LAUNCH(run, launch_compact_f32(s.dA_t, rp, dA, r, K, r, 1.f, false, st));
    }
    if (dB) {
        float* dst = (rp == r) ? dB : s.dB_t;
        FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, operand(H, rp), operand(dY, N), dst, N, rp, N, M, alpha, s.part, run));
        if (rp != r) FHPC_LAUNCH(run, launch_compact_f32(s.dB_t, N, dB, N, r, N, 1.f, false, st));
    }
    return FHPC_OK;
}

int check_workspace(int op, void* ws, size_t ws_bytes, int64_t M, int64_t K, int64_t r, int64_t N, int dtype,
                    bool quantised = true, bool premerged = false)
{
    Carver dry(nullptr);
    carve(dry, op, M, K, r, N, dtype, quantised, premerged);
    if (dry.used == 0) return FHPC_OK;
    if (!ws || ws_bytes < dry.used) return FHPC_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return FHPC_ERR_ALIGN;
    return FHPC_OK;
}

// ---------------- fp32 path of the factorised layer ----------------
int lowrank_fwd_f32(const float* X, const float* A, const float* B, float* Y, float* H_out,
                    int64_t M, int64_t K, int64_t r, int64_t N, const Scratch& s, Run& run)
{
    if (run.dry) return FHPC_OK;
    hipStream_t st = run.st;
    if (lowrank_chain_f32_supports(r)) {
        // a rank that fits a workgroup's LDS: H = X A never leaves the chip on its way into Y = H B (one launch;
        // H is stored only if the caller asked for it)
        FHPC_HIP(launch_lowrank_chain_f32(X, K, A, r, 1, B, N, 1, Y, N, H_out, (int)M, (int)K, (int)r, (int)N, st));
        return FHPC_OK;
    }
    float* H = H_out ? H_out : static_cast<float*>(s.H);
    FHPC_HIP(launch_gemm_f32(X, K, 1, A, r, 1, H, r, (int)M, (int)r, (int)K, 1.f, st));
    FHPC_HIP(launch_gemm_f32(H, r, 1, B, N, 1, Y, N, (int)M, (int)N, (int)r, 1.f, st));
    return FHPC_OK;
}

int lowrank_bwd_f32(const float* X, const float* A, const float* B, const float* dY, const float* H_saved,
                    float* dX, float* dA, float* dB, int64_t M, int64_t K, int64_t r, int64_t N,
                    const Scratch& s, Run& run)
{
    if (run.dry) return FHPC_OK;
    hipStream_t st = run.st;
    const float* H = H_saved;
    if (!H && dB) {
        float* Hw = static_cast<float*>(s.H);
        FHPC_HIP(launch_gemm_f32(X, K, 1, A, r, 1, Hw, r, (int)M, (int)r, (int)K, 1.f, st));
        H = Hw;
    }
    float* dH = static_cast<float*>(s.dH);
    if (dX && lowrank_chain_f32_supports(r)) {
        // dH = dY B^T stays in LDS on its way into dX = dH A^T (and is stored for dA)
        FHPC_HIP(launch_lowrank_chain_f32(dY, N, B, 1, N, A, 1, r, dX, K, dA ? dH : nullptr, (int)M, (int)N, (int)r, (int)K, st));
    } else {
        if (dX || dA)   // dH[m][j] = sum_n dY[m][n] B[j][n]
            FHPC_HIP(launch_gemm_f32(dY, N, 1, B, 1, N, dH, r, (int)M, (int)r, (int)N, 1.f, st));
        if (dX)         // dX[m][k] = sum_j dH[m][j] A[k][j]
            FHPC_HIP(launch_gemm_f32(dH, r, 1, A, 1, r, dX, K, (int)M, (int)K, (int)r, 1.f, st));
    }
    if (dA)         // dA[k][j] = sum_m X[m][k] dH[m][j]
        FHPC_HIP(launch_gemm_f32(X, 1, K, dH, r, 1, dA, r, (int)K, (int)r, (int)M, 1.f, st));
    if (dB)         // dB[j][n] = sum_m H[m][j] dY[m][n]
        FHPC_HIP(launch_gemm_f32(H, 1, r, dY, N, 1, dB, N, (int)r, (int)N, (int)M, 1.f, st));
    return FHPC_OK;
}

size_t merge_workspace(int64_t K, int64_t r, int64_t N)
{
    (void)N;
    const int64_t rp = rank_pad(r);
    // a zero-padded copy of A, behind the header every workspace starts with
    return (rp != r) ? (size_t)QSKINNY_HEADER_BYTES + (size_t)round_up(K * rp * 2, 256) : 0;
}

// ---------------- rank-r factor pair of a pretrained weight ----------------
// Everything is a matrix product on the bf16 matrix cores plus r x r elementwise kernels.
struct DecompScratch {
    void* Yb;      // bf16 [K][r]
    void* Zb;      // bf16 [N][r]
    void* Qt;      // bf16 [max(K,N)][r]   orthonormalised Z
    float* F;      // fp32 [max(K,N)][r]   unsplit fp32 output before rounding
    float* G;      // fp32 [r][r]
    void* Gb;      // bf16 [r][r]
    void* G2b;     // bf16 [r][r]
    void* Sb;      // bf16 [r][r]
    float* Mf[6];  // fp32 [r][r] each: the r x r iteration of orthonormalise
    float* T;      // fp32 [r][N]
    void* Tb;      // bf16 [r][N]
    void* Cb;      // bf16 [r][N]
    float* part;   // partial-sum slabs of the split reductions
    int64_t part_bytes;
};

DecompScratch carve_decompose(Carver& c, int64_t K, int64_t r, int64_t N)
{
    DecompScratch d;
    (void)c.take(QSKINNY_HEADER_BYTES);                // every workspace starts with the header (unused here)
    const int64_t R = K > N ? K : N;
    d.Yb = c.take(K * r * 2);
    d.Zb = c.take(N * r * 2);
    d.Qt = c.take(R * r * 2);
    d.F = static_cast<float*>(c.take(R * r * 4));
    d.G = static_cast<float*>(c.take(r * r * 4));
    d.Gb = c.take(r * r * 2);
    d.G2b = c.take(r * r * 2);
    d.Sb = c.take(r * r * 2);
    for (int i = 0; i < 6; i++) d.Mf[i] = static_cast<float*>(c.take(r * r * 4));
    d.T = static_cast<float*>(c.take(r * N * 4));
    d.Tb = c.take(r * N * 2);
    d.Cb = c.take(r * N * 2);
    // Gram matrices over K (of Y, of A) and over N (of Z): the slice count is not monotone in the reduction
    // length, so each is sized for itself
    int64_t part = split_bytes(r, r, r, K);
    const int64_t p1 = split_bytes(r, r, r, N);
    const int64_t p2 = split_bytes(N, r, r, K);        // Z = W^T Y
    const int64_t p3 = split_bytes(r, N, N, K);        // T = A^T W
    if (p1 > part) part = p1;
    if (p2 > part) part = p2;
    if (p3 > part) part = p3;
    d.part = static_cast<float*>(c.take(part));
    d.part_bytes = part;
    return d;
}

// P[M][n] (bf16, dense) = sum_k a(m,k) b(j,k) with both operands stored reduction-major
int product_tn_bf16(GemmOperand a, GemmOperand b, void* P, int64_t M, int64_t n, int64_t Kred, const DecompScratch& d, Run& run)
{
    bool done = false;
    FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, a, b, d.F, n, M, n, Kred, 1.f, d.part, run, P, &done));
    if (!done) FHPC_LAUNCH(run, launch_compact_f32(d.F, n, P, n, M, n, 1.f, true, run.st));
    return FHPC_OK;
}

// fp32 r x r product C = A B (transpose_a: C = A^T B): fp32 operands and accumulation on the matrix cores
hipError_t small_mm(const float* A, bool transpose_a, const float* B, float* C, int64_t r, hipStream_t st)
{
    return launch_mm_f32(A, transpose_a, r, B, r, C, r, r, r, r, st);
}

// Columns of Y[R][r] (bf16) replaced by an orthonormal basis of their span: out = Y M with an r x r
// matrix M built by products only.  The iteration  Q <- Q (a I + b G + c G^2),  G = Q^T Q,  is run on M
// alone: with G0 = Y^T Y (one product over the long dimension, fp32) the Gram matrix of Q = Y M is
// M^T G0 M, so every step costs r x r products in fp32 and Y is touched twice in all (G0 and the final
// Y M).  That matters for accuracy, not only for time: Q rounded to bf16 after every step would drift out
// of the span of Y by 2^-9 per step, and the error of the factor pair is exactly that drift.
// `quintic` steps use coefficients that lift small singular values fast (they settle in about
// [0.7, 1.15] instead of converging), then `cubic` steps (1.5, -0.5) converge to 1 quadratically from
// there.  The first step divides by the Frobenius norm (trace of G0) so that no singular value starts
// above 1.
int orthonormalise(const void* Y, void* out, int64_t R, int64_t r, int quintic, int cubic, const DecompScratch& d, Run& run)
{
    hipStream_t st = run.st;
    float* const G0 = d.G;
    float* M = d.Mf[0];
    float* Mn = d.Mf[1];
    float* const P = d.Mf[2];
    float* const Gi = d.Mf[3];
    float* const G2 = d.Mf[4];
    float* const S = d.Mf[5];
    FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, operand(Y, r), operand(Y, r), G0, r, r, r, R, 1.f, d.part, run));
    for (int i = 0; i < quintic + cubic; i++) {
        const bool first = (i == 0), q5 = (i < quintic);
        const float* g = G0;
        if (!first) {
            FHPC_LAUNCH(run, small_mm(G0, false, M, P, r, st));            // P = G0 M
            FHPC_LAUNCH(run, small_mm(M, true, P, Gi, r, st));             // Gi = M^T G0 M
            g = Gi;
        }
        float* dst = first ? M : S;                                 // the first step's polynomial is M itself
        if (q5) {
            // the first step works on G0 / trace: Gi = that, G2 its square
            if (first) FHPC_LAUNCH(run, launch_gram_poly(G0, nullptr, Gi, false, r, 0.f, 1.f, 0.f, 1, st));
            FHPC_LAUNCH(run, small_mm(first ? Gi : g, false, first ? Gi : g, G2, r, st));
            FHPC_LAUNCH(run, launch_gram_poly(g, G2, dst, false, r, 3.4445f, -4.7750f, 2.0315f, first ? 2 : 0, st));
        } else {
            FHPC_LAUNCH(run, launch_gram_poly(g, nullptr, dst, false, r, 1.5f, -0.5f, 0.f, first ? 2 : 0, st));
        }
        if (!first) {
            FHPC_LAUNCH(run, small_mm(M, false, S, Mn, r, st));            // M <- M S
            float* t = M; M = Mn; Mn = t;
        }
    }
    FHPC_LAUNCH(run, launch_compact_f32(M, r, d.Sb, r, r, r, 1.f, true, st));
    FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(Y, r), operand(d.Sb, r), out, r, R, r, r, run));
    return FHPC_OK;
}

int check_q(int qscheme, int block, int64_t K)
{
    if (qscheme != FHPC_Q_INT8_PER_CHANNEL && qscheme != FHPC_Q_INT4_BLOCK) return FHPC_ERR_DTYPE;
    if (qscheme == FHPC_Q_INT4_BLOCK) {
        if (block != 64) return FHPC_ERR_UNSUPPORTED;
        if (K % 64) return FHPC_ERR_SHAPE;
    }
    return FHPC_OK;
}

// ---------------- launch sequences of the entry points ----------------
// Each takes validated arguments and the carved scratch, and is walked either for real or dry (see Run).

int seq_lowrank_fwd(Run& run, const Scratch& s, const void* X, const void* A, const void* B, void* Y, void* H_out,
                    int64_t M, int64_t K, int64_t r, int64_t N, int dtype)
{
    if (dtype == FHPC_F32)
        return lowrank_fwd_f32((const float*)X, (const float*)A, (const float*)B, (float*)Y, (float*)H_out, M, K, r, N, s, run);
    const int64_t rp = rank_pad(r);
    Factors f;
    int rc = prepare_factors(A, B, K, r, rp, N, s, run, &f);
    if (rc) return rc;
    void* H = (H_out && rp == r) ? H_out : s.H;
    FHPC_HIP(rank_product(OP_XC, operand(X, K), operand(f.A, rp), H, rp, s.Hf, s.part, M, K, run));
    FHPC_HIP(product_bf16(OP_XC, operand(H, rp), operand(f.B, N), Y, N, N, M, rp, s.part, run));
    if (H_out && rp != r) FHPC_LAUNCH(run, launch_pad2d_u16(H, rp, M, r, H_out, r, M, run.st));
    return FHPC_OK;
}

int seq_lowrank_bwd(Run& run, const Scratch& s, const void* X, const void* A, const void* B, const void* dY,
                    const void* H_saved, void* dX, float* dA, float* dB,
                    int64_t M, int64_t K, int64_t r, int64_t N, int dtype)
{
    if (dtype == FHPC_F32)
        return lowrank_bwd_f32((const float*)X, (const float*)A, (const float*)B, (const float*)dY,
                               (const float*)H_saved, (float*)dX, dA, dB, M, K, r, N, s, run);
    const int64_t rp = rank_pad(r);
    Factors f;
    int rc = prepare_factors(A, B, K, r, rp, N, s, run, &f);
    if (rc) return rc;
    const void* H = nullptr;
    if (dB) {
        if (H_saved && rp == r) {
            H = H_saved;
        } else if (H_saved) {
            FHPC_LAUNCH(run, launch_pad2d_u16(H_saved, r, M, r, s.H, rp, M, run.st));
            H = s.H;
        } else {
            FHPC_HIP(rank_product(OP_XC, operand(X, K), operand(f.A, rp), s.H, rp, s.Hf, s.part, M, K, run));
            H = s.H;
        }
    }
    if (dX || dA)
        FHPC_HIP(rank_product(OP_KC, operand(dY, N), operand(f.B, N), s.dH, rp, s.Hf, s.part, M, N, run));
    if (dX)
        FHPC_HIP(product_bf16(OP_KC, operand(s.dH, rp), operand(f.A, rp), dX, K, K, M, rp, s.part, run));
    return weight_grads(X, dY, H, s.dH, dA, dB, M, K, r, rp, N, 1.f, s, run);
}

}  // namespace

extern "C" {

size_t fhpc_workspace_bytes(int op, int64_t M, int64_t K, int64_t r, int64_t N, int dtype, int qscheme)
{
    if (op == FHPC_OP_DECOMPOSE) {
        if (check_common(1, K, r, N) != FHPC_OK || (r % 8) || r > K || r > N) return 0;
        Carver dry(nullptr);
        carve_decompose(dry, K, r, N);
        return dry.used;
    }
    if (op == FHPC_OP_MERGE) {
        // a zero-padded copy of A when the rank is not a multiple of 8; M, dtype and qscheme are ignored
        if (check_common(1, K, r, N) != FHPC_OK) return 0;
        return merge_workspace(K, r, N);
    }
    if (op < FHPC_OP_LOWRANK_FWD || op > FHPC_OP_QLINEAR_BWD) return 0;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return 0;
    if (check_common(M, K, r, N) != FHPC_OK) return 0;
    Carver dry(nullptr);
    carve(dry, op, M, K, r, N, dtype, qscheme != FHPC_W_BF16 && qscheme != FHPC_W_MERGED, qscheme == FHPC_W_MERGED);
    return dry.used;
}

int lowrank_linear_fwd(const void* X, const void* A, const void* B, void* Y, void* H_out,
                       int64_t M, int64_t K, int64_t r, int64_t N, int dtype,
                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !A || !B || !Y) return FHPC_ERR_NULL;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    int rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (!aligned(X, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(Y, 16) || !aligned(H_out, 16)) return FHPC_ERR_ALIGN;
    rc = check_workspace(FHPC_OP_LOWRANK_FWD, workspace, workspace_bytes, M, K, r, N, dtype);
    if (rc) return rc;
    Carver c(workspace);
    Scratch s = carve(c, FHPC_OP_LOWRANK_FWD, M, K, r, N, dtype);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_lowrank_fwd(run, s, X, A, B, Y, H_out, M, K, r, N, dtype);
}

int lowrank_linear_bwd(const void* X, const void* A, const void* B, const void* dY,
                       const void* H_saved, void* dX, float* dA, float* dB,
                       int64_t M, int64_t K, int64_t r, int64_t N, int dtype,
                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !A || !B || !dY) return FHPC_ERR_NULL;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    int rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (!aligned(X, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(dY, 16) || !aligned(H_saved, 16) ||
        !aligned(dX, 16) || !aligned(dA, 16) || !aligned(dB, 16))
        return FHPC_ERR_ALIGN;
    rc = check_workspace(FHPC_OP_LOWRANK_BWD, workspace, workspace_bytes, M, K, r, N, dtype);
    if (rc) return rc;
    Carver c(workspace);
    Scratch s = carve(c, FHPC_OP_LOWRANK_BWD, M, K, r, N, dtype);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_lowrank_bwd(run, s, X, A, B, dY, H_saved, dX, dA, dB, M, K, r, N, dtype);
}

// ---- g factorised layers on one X ------------------------------------------------------------------
// The first factors sit side by side in A_all [K][g r], so X A_all is one product g r wide, and the
// input gradient  sum_i dH_i A_i^T  is one product over the g r columns of dH_all = [dH_0 | ... ]: the
// g partial dX never exist and X is read once per pass instead of g times.

struct SharedScratch {
    void* H = nullptr;      // bf16 [M][g r]
    void* dH = nullptr;     // bf16 [M][g r]
    float* Pf = nullptr;    // fp32 [M][max(r, g r) when <= 32]  split accumulator of a narrow product
    float* part = nullptr;  // slabs of the split reductions
    int64_t part_bytes = 0;
};

static bool groupable_f32(int64_t M, int64_t N, int64_t Kred, int g);

static SharedScratch carve_shared(Carver& c, bool bwd, int64_t M, int64_t K, int64_t r, int64_t N, int g)
{
    SharedScratch s;
    const int64_t R = r * g;
    (void)c.take(QSKINNY_HEADER_BYTES);                // every workspace starts with the header (unused here)
    s.H = c.take(M * R * 2);
    if (bwd) s.dH = c.take(M * R * 2);
    if (r <= 32) s.Pf = static_cast<float*>(c.take(M * (R <= 32 ? R : r) * 4));
    int64_t part = 0;
    auto upto = [&part](int64_t b) { if (b > part) part = b; };
    upto(R <= 32 ? split_bytes(M, R, R, K) : product_part_bytes(M, R, K));      // H_all = X A_all
    if (!bwd) upto(product_part_bytes(M, N, r));       // Y_i = H_i B_i
    if (bwd) {
        upto(product_part_bytes(M, K, R));             // dX = dH_all A_all^T
        // dH_i = dY_i B_i^T: at most 32 wide it splits its reduction; wider, it is a column block of dH_all and
        // runs unsplit, except for g = 1, where the block is the whole (dense) matrix and may take the 32-row split
        if (r <= 32) upto(split_bytes(M, r, r, N));
        else if (g == 1) upto(product_part_bytes(M, r, N));
        upto(split_bytes(K, R, R, M));                 // dA_all = X^T dH_all
        // dB_i = H_i^T dY_i: one product's slabs, or all g products' when they go out in one launch
        if (groupable_f32(r, N, M, g)) {
            const SplitPlan gp = plan_split(r, N, M, false, g);
            upto(gp.splits > 1 ? (int64_t)g * gp.splits * r * N * 4 : 0);
        } else {
            upto(split_bytes(r, N, N, M));
        }
    }
    s.part = static_cast<float*>(c.take(part));
    s.part_bytes = part;
    return s;
}

static int check_shared(int64_t M, int64_t K, int64_t r, int64_t N, int g)
{
    if (g < 1 || g > FHPC_MAX_SHARED) return FHPC_ERR_SHAPE;
    int rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (r % 8) return FHPC_ERR_UNSUPPORTED;            // the column blocks of A_all and H_all must start 16-byte aligned
    return check_common(M, K, r * g, N);
}

size_t fhpc_workspace_bytes_lowrank_shared_x(int backward, int64_t M, int64_t K, int64_t r, int64_t N, int g)
{
    if (check_shared(M, K, r, N, g) != FHPC_OK) return 0;
    Carver dry(nullptr);
    carve_shared(dry, backward != 0, M, K, r, N, g);
    return dry.used;
}

// P[M][r] (bf16, row stride ldp) = L * R^(b_mode) over Kred; a product at most 32 wide splits its reduction.
static hipError_t narrow_product(int b_mode, GemmOperand a, GemmOperand b, void* P, int64_t ldp, int64_t r,
                                 float* Pf, float* part, int64_t M, int64_t Kred, Run& run)
{
    if (r > 32) return product_bf16(b_mode, a, b, P, ldp, r, M, Kred, part, run);
    hipError_t e = gemm_split_f32(OP_KC, b_mode, a, b, Pf, r, M, r, Kred, 1.f, part, run);
    if (e != hipSuccess || run.dry) return e;
    return launch_compact_f32(Pf, r, P, ldp, M, r, 1.f, true, run.st);
}

// column `col` of a row-major bf16 matrix
static inline void* bf16_col(const void* p, int64_t col)
{
    return const_cast<uint16_t*>(static_cast<const uint16_t*>(p)) + col;
}

// The g same-shaped products of a shared-X call (Y_i = H_i B_i, dH_i = dY_i B_i^T, dB_i = H_i^T dY_i) in one launch of
// the request-fed kernels: one ramp and one tail instead of g, and the workgroups of the persistent shape run on
// from one product into the next.  Whether that is possible for a product shape: unsplit bf16 output, or fp32
// output (split or not), on the tiles those kernels serve.
static bool groupable_bf16(int b_mode, int64_t M, int64_t Nout, int64_t ldp, int64_t Kred, int g)
{
    if (g < 2 || g > GEMM_MAX_GROUPS) return false;
    if (ldp == Nout && (large_split_pays(M, Nout, Kred) || split_pays(M, Nout, Kred))) return false;
    return gemm_pp_supports(OP_KC, b_mode, OP_NONE, OUT_BF16, pick_tile(M, Nout, false));
}

// P_i[M][Nout] (bf16, row stride ldp) = a_i * b_i^(b_mode), i < g; a_i has k contiguous
static hipError_t grouped_bf16(int b_mode, const GemmOperand* a, const GemmOperand* b, void* const* P, int64_t ldp,
                               int64_t Nout, int64_t M, int64_t Kred, int g, Run& run)
{
    if (run.dry) return hipSuccess;
    GemmArgs ga = {};
    ga.a = a[0]; ga.b = b[0]; ga.c = P[0]; ga.ldc = ldp;
    ga.M = (int)M; ga.N = (int)Nout; ga.K = (int)Kred; ga.K2 = 0;
    ga.alpha = 1.f; ga.mid_scale = 1.f; ga.splits = 1; ga.k_chunk = (int)round_up(Kred, 64);
    ga.groups = g;
    for (int i = 0; i < g; i++) { ga.ga[i] = a[i].ptr; ga.gb[i] = b[i].ptr; ga.gc[i] = P[i]; }
    return launch_gemm_bf16(OP_KC, b_mode, OP_NONE, OUT_BF16, pick_tile(M, Nout, false), ga, run.st);
}

// C_i[M][N] (fp32, dense) = a_i^T-type products reduced over Kred (both operands reduction-major), i < g: the g
// split reductions in one launch, slabs of product i behind those of product i - 1, then the g slab sums.
static bool groupable_f32(int64_t M, int64_t N, int64_t Kred, int g)
{
    if (g < 2 || g > GEMM_MAX_GROUPS) return false;
    return gemm_pp_supports(OP_XC, OP_XC, OP_NONE, OUT_F32, plan_split(M, N, Kred).tile);
}

static hipError_t grouped_split_f32(const GemmOperand* a, const GemmOperand* b, float* const* C, int64_t M, int64_t N,
                                    int64_t Kred, float* part, int g, Run& run)
{
    const SplitPlan sp = plan_split(M, N, Kred, false, g);
    const int64_t slab_area = sp.splits > 1 ? (int64_t)sp.splits * M * N : 0;      // floats per product
    if (!run.claim((int64_t)g * slab_area * 4)) return hipErrorOutOfMemory;
    if (run.dry) return hipSuccess;
    GemmArgs ga = {};
    ga.a = a[0]; ga.b = b[0]; ga.ldc = N;
    ga.M = (int)M; ga.N = (int)N; ga.K = (int)Kred; ga.K2 = 0;
    ga.alpha = 1.f; ga.mid_scale = 1.f; ga.splits = sp.splits; ga.k_chunk = sp.k_chunk;
    ga.split_stride = sp.splits > 1 ? M * N : 0;
    ga.groups = g;
    for (int i = 0; i < g; i++) {
        ga.ga[i] = a[i].ptr; ga.gb[i] = b[i].ptr;
        ga.gc[i] = sp.splits > 1 ? static_cast<void*>(part + (int64_t)i * slab_area) : static_cast<void*>(C[i]);
    }
    ga.c = ga.gc[0];
    hipError_t e = launch_gemm_bf16(OP_XC, OP_XC, OP_NONE, OUT_F32, sp.tile, ga, run.st);
    if (e != hipSuccess || sp.splits == 1) return e;
    for (int i = 0; i < g; i++) {
        e = launch_sum_slabs(part + (int64_t)i * slab_area, M * N, sp.splits, C[i], false, run.st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

static int seq_shared_fwd(Run& run, const SharedScratch& s, const void* X, const void* A_all, const void* const* B,
                          void* const* Y, void* H_all_out, int64_t M, int64_t K, int64_t r, int64_t N, int g)
{
    const int64_t R = r * g;
    void* H = H_all_out ? H_all_out : s.H;
    FHPC_HIP(narrow_product(OP_XC, operand(X, K), operand(A_all, R), H, R, R, s.Pf, s.part, M, K, run));
    if (groupable_bf16(OP_XC, M, N, N, r, g)) {
        GemmOperand a[GEMM_MAX_GROUPS], b[GEMM_MAX_GROUPS];
        for (int i = 0; i < g; i++) { a[i] = operand(bf16_col(H, i * r), R); b[i] = operand(B[i], N); }
        FHPC_HIP(grouped_bf16(OP_XC, a, b, Y, N, N, M, r, g, run));
        return FHPC_OK;
    }
    for (int i = 0; i < g; i++)
        FHPC_HIP(product_bf16(OP_XC, operand(bf16_col(H, i * r), R), operand(B[i], N), Y[i], N, N, M, r, s.part, run));
    return FHPC_OK;
}

static int seq_shared_bwd(Run& run, const SharedScratch& s, const void* X, const void* A_all, const void* const* B,
                          const void* const* dY, const void* H_all_saved, void* dX, float* dA_all, float* const* dB,
                          bool any_dB, int64_t M, int64_t K, int64_t r, int64_t N, int g)
{
    const int64_t R = r * g;
    const void* H = H_all_saved;
    if (any_dB && !H) {
        FHPC_HIP(narrow_product(OP_XC, operand(X, K), operand(A_all, R), s.H, R, R, s.Pf, s.part, M, K, run));
        H = s.H;
    }
    if ((dX || dA_all) && r > 32 && groupable_bf16(OP_KC, M, r, R, N, g)) {
        GemmOperand a[GEMM_MAX_GROUPS], b[GEMM_MAX_GROUPS];
        void* P[GEMM_MAX_GROUPS];
        for (int i = 0; i < g; i++) { a[i] = operand(dY[i], N); b[i] = operand(B[i], N); P[i] = bf16_col(s.dH, i * r); }
        FHPC_HIP(grouped_bf16(OP_KC, a, b, P, R, r, M, N, g, run));
    } else if (dX || dA_all) {
        for (int i = 0; i < g; i++)
            FHPC_HIP(narrow_product(OP_KC, operand(dY[i], N), operand(B[i], N), bf16_col(s.dH, i * r), R, r, s.Pf, s.part, M, N, run));
    }
    if (dX) FHPC_HIP(product_bf16(OP_KC, operand(s.dH, R), operand(A_all, R), dX, K, K, M, R, s.part, run));
    if (dA_all) FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, operand(X, K), operand(s.dH, R), dA_all, R, K, R, M, 1.f, s.part, run));
    bool all_dB = any_dB;
    for (int i = 0; i < g && all_dB; i++) all_dB = dB[i] != nullptr;
    if (all_dB && groupable_f32(r, N, M, g)) {
        GemmOperand a[GEMM_MAX_GROUPS], b[GEMM_MAX_GROUPS];
        for (int i = 0; i < g; i++) { a[i] = operand(bf16_col(H, i * r), R); b[i] = operand(dY[i], N); }
        FHPC_HIP(grouped_split_f32(a, b, dB, r, N, M, s.part, g, run));
        return FHPC_OK;
    }
    for (int i = 0; i < g && any_dB; i++)
        if (dB[i])
            FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, operand(bf16_col(H, i * r), R), operand(dY[i], N), dB[i], N, r, N, M, 1.f, s.part, run));
    return FHPC_OK;
}

int lowrank_linear_fwd_shared_x(const void* X, const void* A_all, const void* const* B, void* const* Y, void* H_all_out,
                                int64_t M, int64_t K, int64_t r, int64_t N, int g,
                                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !A_all || !B || !Y) return FHPC_ERR_NULL;
    int rc = check_shared(M, K, r, N, g);
    if (rc) return rc;
    if (!aligned(X, 16) || !aligned(A_all, 16) || !aligned(H_all_out, 16)) return FHPC_ERR_ALIGN;
    for (int i = 0; i < g; i++) {
        if (!B[i] || !Y[i]) return FHPC_ERR_NULL;
        if (!aligned(B[i], 16) || !aligned(Y[i], 16)) return FHPC_ERR_ALIGN;
    }
    const size_t need = fhpc_workspace_bytes_lowrank_shared_x(0, M, K, r, N, g);
    if (need && (!workspace || workspace_bytes < need)) return FHPC_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return FHPC_ERR_ALIGN;
    Carver c(workspace);
    const SharedScratch s = carve_shared(c, false, M, K, r, N, g);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_shared_fwd(run, s, X, A_all, B, Y, H_all_out, M, K, r, N, g);
}

int lowrank_linear_bwd_shared_x(const void* X, const void* A_all, const void* const* B, const void* const* dY,
                                const void* H_all_saved, void* dX, float* dA_all, float* const* dB,
                                int64_t M, int64_t K, int64_t r, int64_t N, int g,
                                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !A_all || !B || !dY) return FHPC_ERR_NULL;
    int rc = check_shared(M, K, r, N, g);
    if (rc) return rc;
    if (!aligned(X, 16) || !aligned(A_all, 16) || !aligned(H_all_saved, 16) || !aligned(dX, 16) || !aligned(dA_all, 16))
        return FHPC_ERR_ALIGN;
    bool any_dB = false;
    for (int i = 0; i < g; i++) {
        if (!B[i] || !dY[i]) return FHPC_ERR_NULL;
        if (!aligned(B[i], 16) || !aligned(dY[i], 16) || (dB && !aligned(dB[i], 16))) return FHPC_ERR_ALIGN;
        any_dB = any_dB || (dB && dB[i]);
    }
    const size_t need = fhpc_workspace_bytes_lowrank_shared_x(1, M, K, r, N, g);
    if (need && (!workspace || workspace_bytes < need)) return FHPC_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return FHPC_ERR_ALIGN;
    Carver c(workspace);
    const SharedScratch s = carve_shared(c, true, M, K, r, N, g);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_shared_bwd(run, s, X, A_all, B, dY, H_all_saved, dX, dA_all, dB, any_dB, M, K, r, N, g);
}

// ---- the FFN's gate (Sec. 3.1, eq. FFN) in the epilogue of the product that feeds it ------------------------------
// Forward: the gate and up projections read one X (the shared-X call with g = 2); U's tiles go through the gate
// on their way out, against G's finished tiles, so Z costs no pass of its own over G and U.
static int seq_ffn_gate_up_fwd(Run& run, const SharedScratch& s, const void* X, const void* A_all, const void* B_gate,
                               const void* B_up, void* G, void* U, void* Z, void* H_all_out,
                               int64_t M, int64_t K, int64_t r, int64_t N)
{
    const int64_t R = 2 * r;
    void* H = H_all_out ? H_all_out : s.H;
    FHPC_HIP(narrow_product(OP_XC, operand(X, K), operand(A_all, R), H, R, R, s.Pf, s.part, M, K, run));
    FHPC_HIP(product_bf16(OP_XC, operand(H, R), operand(B_gate, N), G, N, N, M, r, s.part, run));
    if (gate_rides(M, N, r)) {
        FHPC_HIP(gemm_gated(OP_XC, operand(bf16_col(H, r), R), operand(B_up, N), U, M, N, r, 1, G, nullptr, Z, nullptr, run));
        return FHPC_OK;
    }
    FHPC_HIP(product_bf16(OP_XC, operand(bf16_col(H, r), R), operand(B_up, N), U, N, N, M, r, s.part, run));
    FHPC_LAUNCH(run, launch_swiglu_fwd(G, U, Z, M * N, true, run.st));
    return FHPC_OK;
}

// Backward of the down projection Y = (Z A) B with its input gradient taken through the gate: the tiles of
// dZ = dH A^T leave as dG and dU, and dZ is never stored.  Without the gate epilogue (small or narrow outputs) dZ is
// written where dU will be and the streaming gate kernel turns it into dG and dU in place.
static int seq_ffn_down_bwd(Run& run, const Scratch& s, const void* Z, const void* A, const void* B, const void* dY,
                            const void* H_saved, const void* G, const void* U, void* dG, void* dU, float* dA, float* dB,
                            int64_t M, int64_t K, int64_t r, int64_t N)
{
    const int64_t rp = rank_pad(r);
    Factors f;
    int rc = prepare_factors(A, B, K, r, rp, N, s, run, &f);
    if (rc) return rc;
    const void* H = nullptr;
    if (dB) {
        if (H_saved && rp == r) {
            H = H_saved;
        } else if (H_saved) {
            FHPC_LAUNCH(run, launch_pad2d_u16(H_saved, r, M, r, s.H, rp, M, run.st));
            H = s.H;
        } else {
            FHPC_HIP(rank_product(OP_XC, operand(Z, K), operand(f.A, rp), s.H, rp, s.Hf, s.part, M, K, run));
            H = s.H;
        }
    }
    FHPC_HIP(rank_product(OP_KC, operand(dY, N), operand(f.B, N), s.dH, rp, s.Hf, s.part, M, N, run));
    if (gate_rides(M, K, rp)) {
        FHPC_HIP(gemm_gated(OP_KC, operand(s.dH, rp), operand(f.A, rp), nullptr, M, K, rp, 2, G, U, dG, dU, run));
    } else {
        FHPC_HIP(product_bf16(OP_KC, operand(s.dH, rp), operand(f.A, rp), dU, K, K, M, rp, s.part, run));
        FHPC_LAUNCH(run, launch_swiglu_bwd(G, U, dU, dG, dU, M * K, true, run.st));
    }
    return weight_grads(Z, dY, H, s.dH, dA, dB, M, K, r, rp, N, 1.f, s, run);
}

int lowrank_ffn_gate_up_fwd(const void* X, const void* A_all, const void* B_gate, const void* B_up,
                            void* G_out, void* U_out, void* Z_out, void* H_all_out,
                            int64_t M, int64_t K, int64_t r, int64_t N,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !A_all || !B_gate || !B_up || !G_out || !U_out || !Z_out) return FHPC_ERR_NULL;
    int rc = check_shared(M, K, r, N, 2);
    if (rc) return rc;
    if (!aligned(X, 16) || !aligned(A_all, 16) || !aligned(B_gate, 16) || !aligned(B_up, 16) || !aligned(G_out, 16) ||
        !aligned(U_out, 16) || !aligned(Z_out, 16) || !aligned(H_all_out, 16))
        return FHPC_ERR_ALIGN;
    const size_t need = fhpc_workspace_bytes_lowrank_shared_x(0, M, K, r, N, 2);
    if (need && (!workspace || workspace_bytes < need)) return FHPC_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return FHPC_ERR_ALIGN;
    Carver c(workspace);
    const SharedScratch s = carve_shared(c, false, M, K, r, N, 2);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_ffn_gate_up_fwd(run, s, X, A_all, B_gate, B_up, G_out, U_out, Z_out, H_all_out, M, K, r, N);
}

int lowrank_ffn_down_bwd(const void* Z, const void* A, const void* B, const void* dY, const void* H_saved,
                         const void* G, const void* U, void* dG_out, void* dU_out, float* dA, float* dB,
                         int64_t M, int64_t K, int64_t r, int64_t N,
                         void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!Z || !A || !B || !dY || !G || !U || !dG_out || !dU_out) return FHPC_ERR_NULL;
    int rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (!aligned(Z, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(dY, 16) || !aligned(H_saved, 16) || !aligned(G, 16) ||
        !aligned(U, 16) || !aligned(dG_out, 16) || !aligned(dU_out, 16) || !aligned(dA, 16) || !aligned(dB, 16))
        return FHPC_ERR_ALIGN;
    rc = check_workspace(FHPC_OP_LOWRANK_BWD, workspace, workspace_bytes, M, K, r, N, FHPC_BF16);
    if (rc) return rc;
    Carver c(workspace);
    Scratch s = carve(c, FHPC_OP_LOWRANK_BWD, M, K, r, N, FHPC_BF16);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_ffn_down_bwd(run, s, Z, A, B, dY, H_saved, G, U, dG_out, dU_out, dA, dB, M, K, r, N);
}

// Y = base_scale * X deq(W) + scaling * (X A) B
static int seq_qlinear_fwd(Run& run, const Scratch& s, const void* X, const void* Wq, const void* scales, int qscheme,
                           const void* A, const void* B, float base_scale, float scaling, void* Y, void* H_out,
                           int64_t M, int64_t K, int64_t r, int64_t N)
{
    const bool premerged = (qscheme == FHPC_W_MERGED);
    const bool dense = (qscheme == FHPC_W_BF16) || premerged;
    if (s.sk_part && token_blocks_pay(M, K, r, N)) {
        const QskinnyPlan p = qskinny_plan_token_blocks(M, K, r, N);
        const int tb = token_blocks(M);
        QskinnyJob jobs[QSKINNY_MAX_JOBS];
        for (int t = 0; t < tb; t++) {
            jobs[t] = QskinnyJob{Wq, scales, A, B, static_cast<uint16_t*>(Y) + (int64_t)16 * t * N,
                                 H_out ? static_cast<uint16_t*>(H_out) + (int64_t)16 * t * r : nullptr, N, base_scale, scaling,
                                 static_cast<const uint16_t*>(X) + (int64_t)16 * t * K, (M - 16 * t < 16) ? M - 16 * t : 16};
        }
        FHPC_LAUNCH(run, launch_qskinny_fwd(X, jobs, tb, qscheme, 16, K, r, p, s.sk_part, s.sk_hpart, s.header, run.st));
        return FHPC_OK;
    }
    if (s.sk_part) {
        const QskinnyPlan p = qskinny_plan(M, K, r, &N, 1, num_cu());
        const QskinnyJob job = {Wq, scales, A, B, Y, H_out, N, base_scale, scaling};
        FHPC_LAUNCH(run, launch_qskinny_fwd(X, &job, 1, qscheme, M, K, r, p, s.sk_part, s.sk_hpart, s.header, run.st));
        return FHPC_OK;
    }
    const int64_t rp = rank_pad(r);
    Factors f;
    int rc = prepare_factors(A, B, K, r, rp, N, s, run, &f);
    if (rc) return rc;
    void* H = (H_out && rp == r) ? H_out : s.H;
    const int w_kind = dense ? 1 : (qscheme == FHPC_Q_INT8_PER_CHANNEL) ? 2 : 3;
    if (premerged || (s.Wm && base_scale != 0.f)) {
        // many tokens (or a weight merged by the caller): one plain product with the merged weight; H only if
        // the caller wants it
        const void* Wm = Wq;
        if (!premerged && H_out && rides_along(OP_KC, OP_XC, M, N, rp)) {
            // H = X A out of the same product: A stands in rp extra columns of the merged weight
            FHPC_LAUNCH(run, launch_merge(Wq, scales, w_kind, f.A, rp, f.B, base_scale, scaling, s.Wm, false, K, rp, N, run.st, true));
            FHPC_HIP(gemm_two_outputs(OP_KC, OP_XC, operand(X, K), operand(s.Wm, N + MERGE_EXT_PAD), Y, N, H, rp, M, N, N + rp, K, run));
            if (rp != r) FHPC_LAUNCH(run, launch_pad2d_u16(H, rp, M, r, H_out, r, M, run.st));
            return FHPC_OK;
        }
        if (!premerged) {
            FHPC_LAUNCH(run, launch_merge(Wq, scales, w_kind, f.A, rp, f.B, base_scale, scaling, s.Wm, false, K, rp, N, run.st));
            Wm = s.Wm;
        }
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(X, K), operand(Wm, N), Y, N, M, N, K, run));
        if (H_out) {
            FHPC_HIP(rank_product(OP_XC, operand(X, K), operand(f.A, rp), H, rp, s.Hf, s.part, M, K, run));
            if (rp != r) FHPC_LAUNCH(run, launch_pad2d_u16(H, rp, M, r, H_out, r, M, run.st));
        }
        return FHPC_OK;
    }
    FHPC_HIP(rank_product(OP_XC, operand(X, K), operand(f.A, rp), H, rp, s.Hf, s.part, M, K, run));

    if (base_scale == 0.f) {
        // nothing of the frozen weight is left: the factorised layer alone
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(H, rp), operand(f.B, N), Y, N, M, N, rp, run, scaling));
    } else {
        // the kernel forms alpha * (mid_scale * H B + X deq(W))
        GemmArgs g = {};
        g.a = operand(X, K);
        g.b = dense ? operand(Wq, N) : operand(Wq, K, scales, K / 64);      // dense: W[K][N], element (n, k) at k*N + n
        g.a2 = operand(H, rp);
        g.b2 = operand(f.B, N);
        g.M = (int)M; g.N = (int)N; g.K = (int)K; g.K2 = (int)rp;
        g.alpha = base_scale; g.mid_scale = scaling / base_scale;
        const int b_mode = dense ? OP_XC : (qscheme == FHPC_Q_INT8_PER_CHANNEL) ? OP_Q8_KC : OP_Q4_KC;
        FHPC_HIP(fused_product(b_mode, OP_XC, g, Y, M, N, K, s.part, run));
    }
    if (H_out && rp != r) FHPC_LAUNCH(run, launch_pad2d_u16(H, rp, M, r, H_out, r, M, run.st));
    return FHPC_OK;
}

// Y = base_scale * X deq(W) + scaling * (X A) B: the finetuning layer (base_scale 1) and the blend
// layer (base_scale alpha, scaling 1 - alpha) share everything else.
static int qlinear_fwd_impl(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                            const void* A, const void* B, float base_scale, float scaling, void* Y, void* H_out,
                            int64_t M, int64_t K, int64_t r, int64_t N,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const bool premerged = (qscheme == FHPC_W_MERGED);    // Wq is the bf16 weight lowrank_merge wrote for this A, B, scaling
    const bool dense = (qscheme == FHPC_W_BF16) || premerged;      // (FHPC_W_BF16: blend layer with an unquantised frozen weight)
    if (!X || !Wq || (!scales && !dense) || !A || !B || !Y) return FHPC_ERR_NULL;
    int rc = dense ? FHPC_OK : check_q(qscheme, block, K);
    if (rc) return rc;
    rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (dense && K * N * 2 >= kMaxBytes) return FHPC_ERR_UNSUPPORTED;
    if (!aligned(X, 16) || !aligned(Wq, 16) || !aligned(scales, 16) || !aligned(A, 16) || !aligned(B, 16) ||
        !aligned(Y, 16) || !aligned(H_out, 16))
        return FHPC_ERR_ALIGN;
    rc = check_workspace(FHPC_OP_QLINEAR_FWD, workspace, workspace_bytes, M, K, r, N, FHPC_BF16, !dense, premerged);
    if (rc) return rc;
    Carver c(workspace);
    Scratch s = carve(c, FHPC_OP_QLINEAR_FWD, M, K, r, N, FHPC_BF16, !dense, premerged);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_qlinear_fwd(run, s, X, Wq, scales, qscheme, A, B, base_scale, scaling, Y, H_out, M, K, r, N);
}

int qlinear_lowrank_fwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                        const void* A, const void* B, float scaling, void* Y, void* H_out,
                        int64_t M, int64_t K, int64_t r, int64_t N,
                        void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (qscheme == FHPC_W_BF16) return FHPC_ERR_DTYPE;      // the finetuning layer's weight is quantised
    return qlinear_fwd_impl(X, Wq, scales, qscheme, block, A, B, 1.f, scaling, Y, H_out, M, K, r, N,
                            workspace, workspace_bytes, hip_stream);
}

// ---- the same forward for callers that cannot allocate --------------------------------------------
// The workspace is a fixed array in device memory that belongs to the library: every GPU the library runs on
// holds its own copy, at its own address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; what the kernels get is the address looked up once per device.
static __device__ __align__(256) unsigned char scratch[FHPC_NOALLOC_SCRATCH_BYTES];

// address of `scratch` on the current device (looked up on the first call on that device)
static int noalloc_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> addr[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return FHPC_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return FHPC_ERR_UNSUPPORTED;
    void* p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        // (two threads that race here look up the same address)
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return FHPC_ERR_HIP;
        }
        addr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return FHPC_OK;
}

int qlinear_lowrank_fwd_noalloc(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                                const void* A, const void* B, float scaling, void* Y, void* H_out,
                                int64_t M, int64_t K, int64_t r, int64_t N, void* hip_stream)
{
    if (qscheme == FHPC_W_BF16) return FHPC_ERR_DTYPE;
    if (!X || !Wq || !A || !B || !Y) return FHPC_ERR_NULL;
    int rc = check_common(M, K, r, N);
    if (rc) return rc;
    // what the call would carve, before anything else: a size beyond the fixed array is refused here
    const size_t need = fhpc_workspace_bytes(FHPC_OP_QLINEAR_FWD, M, K, r, N, FHPC_BF16, qscheme);
    if (need > (size_t)FHPC_NOALLOC_SCRATCH_BYTES) return FHPC_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = noalloc_scratch(&ws);
    if (rc) return rc;
    // every region the sequence reads is written earlier in the same call (slabs, H, the merged weight), so
    // nothing needs clearing between calls; the calls only must not overlap on one GPU
    return qlinear_fwd_impl(X, Wq, scales, qscheme, block, A, B, 1.f, scaling, Y, H_out, M, K, r, N,
                            ws, (size_t)FHPC_NOALLOC_SCRATCH_BYTES, hip_stream);
}

// workspace of the shared-X forward: the single-weight need of every weight (the fallback runs them one
// after another in the same workspace) and, when the weight-streaming kernels take all of them at
// once, that launch's slabs
static size_t shared_x_workspace(const int64_t* N, int count, int64_t M, int64_t K, int64_t r, int qscheme)
{
    size_t need = 0;
    for (int j = 0; j < count; j++) {
        Carver dry(nullptr);
        carve(dry, FHPC_OP_QLINEAR_FWD, M, K, r, N[j], FHPC_BF16, true);
        if (dry.used > need) need = dry.used;
    }
    if (count <= QSKINNY_MAX_JOBS && qskinny_supports(M, K, r, N[0], qscheme)) {
        const QskinnyPlan p = qskinny_plan(M, K, r, N, count, num_cu());
        const size_t fused = (size_t)QSKINNY_HEADER_BYTES + (size_t)round_up(p.part_bytes, 256) + (size_t)round_up(p.hpart_bytes, 256);
        if (fused > need) need = fused;
    }
    return need;
}

size_t fhpc_workspace_bytes_shared_x(const int64_t* N, int count, int64_t M, int64_t K, int64_t r, int qscheme)
{
    if (!N || count < 1 || count > 64) return 0;
    for (int j = 0; j < count; j++)
        if (check_common(M, K, r, N[j]) != FHPC_OK) return 0;
    return shared_x_workspace(N, count, M, K, r, qscheme);
}

int qlinear_lowrank_fwd_shared_x(const void* X, const fhpc_qlinear_weight* weights, int count, int qscheme, int block,
                                 int64_t M, int64_t K, int64_t r, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!X || !weights) return FHPC_ERR_NULL;
    if (count < 1 || count > 64) return FHPC_ERR_SHAPE;
    int rc = check_q(qscheme, block, K);
    if (rc) return rc;
    int64_t N[64];
    for (int j = 0; j < count; j++) {
        const fhpc_qlinear_weight& w = weights[j];
        if (!w.Wq || !w.scales || !w.A || !w.B || !w.Y) return FHPC_ERR_NULL;
        rc = check_common(M, K, r, w.N);
        if (rc) return rc;
        if (!aligned(w.Wq, 16) || !aligned(w.scales, 16) || !aligned(w.A, 16) || !aligned(w.B, 16) || !aligned(w.Y, 16) ||
            !aligned(w.H_out, 16))
            return FHPC_ERR_ALIGN;
        N[j] = w.N;
    }
    if (!aligned(X, 16)) return FHPC_ERR_ALIGN;
    const size_t need = shared_x_workspace(N, count, M, K, r, qscheme);
    if (need && (!workspace || workspace_bytes < need)) return FHPC_ERR_WORKSPACE;
    if (need && !aligned(workspace, 256)) return FHPC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (count <= QSKINNY_MAX_JOBS && qskinny_supports(M, K, r, N[0], qscheme)) {
        // few tokens: every weight in one launch
        const QskinnyPlan p = qskinny_plan(M, K, r, N, count, num_cu());
        Carver c(workspace);
        uint32_t* header = static_cast<uint32_t*>(c.take(QSKINNY_HEADER_BYTES));
        float* part = static_cast<float*>(c.take(p.part_bytes));
        float* hpart = static_cast<float*>(c.take(p.hpart_bytes));
        QskinnyJob jobs[QSKINNY_MAX_JOBS];
        for (int j = 0; j < count; j++) {
            const fhpc_qlinear_weight& w = weights[j];
            jobs[j] = QskinnyJob{w.Wq, w.scales, w.A, w.B, w.Y, w.H_out, w.N, 1.f, w.scaling};
        }
        FHPC_HIP(launch_qskinny_fwd(X, jobs, count, qscheme, M, K, r, p, part, hpart, header, st));
        return FHPC_OK;
    }
    // otherwise: the single-weight path, one weight after another on the stream
    for (int j = 0; j < count; j++) {
        const fhpc_qlinear_weight& w = weights[j];
        rc = qlinear_fwd_impl(X, w.Wq, w.scales, qscheme, block, w.A, w.B, 1.f, w.scaling, w.Y, w.H_out, M, K, r, w.N,
                              workspace, workspace_bytes, hip_stream);
        if (rc) return rc;
    }
    return FHPC_OK;
}

int qlinear_blend_fwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                      const void* A, const void* B, float alpha, void* Y, void* H_out,
                      int64_t M, int64_t K, int64_t r, int64_t N,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!(alpha >= 0.f && alpha <= 1.f)) return FHPC_ERR_SHAPE;
    if (qscheme == FHPC_W_MERGED) return FHPC_ERR_DTYPE;
    return qlinear_fwd_impl(X, Wq, scales, qscheme, block, A, B, alpha, 1.f - alpha, Y, H_out, M, K, r, N,
                            workspace, workspace_bytes, hip_stream);
}

// dX = base_scale * dY deq(W)^T + scaling * dH A^T, dA = scaling X^T dH, dB = scaling H^T dY
static int seq_qlinear_bwd(Run& run, const Scratch& s, const void* X, const void* Wq, const void* scales, int qscheme,
                           const void* A, const void* B, float base_scale, float scaling, const void* dY,
                           const void* H_saved, void* dX, float* dA, float* dB,
                           int64_t M, int64_t K, int64_t r, int64_t N)
{
    const bool premerged = (qscheme == FHPC_W_MERGED);
    const bool dense = (qscheme == FHPC_W_BF16) || premerged;
    const int64_t rp = rank_pad(r);
    Factors f;
    int rc = prepare_factors(A, B, K, r, rp, N, s, run, &f);
    if (rc) return rc;
    const void* H = nullptr;
    if (dB) {
        if (H_saved && rp == r) {
            H = H_saved;
        } else if (H_saved) {
            FHPC_LAUNCH(run, launch_pad2d_u16(H_saved, r, M, r, s.H, rp, M, run.st));
            H = s.H;
        } else {
            FHPC_HIP(rank_product(OP_XC, operand(X, K), operand(f.A, rp), s.H, rp, s.Hf, s.part, M, K, run));
            H = s.H;
        }
    }
    const bool merged_dx = premerged || (s.Wm != nullptr && base_scale != 0.f);   // then dX does not need dH
    const bool streamed_dx = dX && s.sk_dxpart && base_scale != 0.f;
    const bool dh_on_the_way = streamed_dx && s.sk_dhpart;                        // the streaming launch forms dH itself
    // (many tokens: dH = dY B^T can come out of the dX product itself, B standing in rp extra rows of the merged weight)
    const bool dh_rides = dX && merged_dx && !premerged && dA && rides_along(OP_KC, OP_KC, M, K, rp);
    if (!dh_on_the_way && !dh_rides && (dA || (dX && !merged_dx)))
        FHPC_HIP(rank_product(OP_KC, operand(dY, N), operand(f.B, N), s.dH, rp, s.Hf, s.part, M, N, run));
    if (dX && base_scale == 0.f) {
        FHPC_HIP(gemm_plain(OP_KC, OP_KC, operand(s.dH, rp), operand(f.A, rp), dX, K, M, K, rp, run, scaling));
    } else if (dX && merged_dx) {
        // many tokens: dX = dY W'^T with the merged weight W' = base_scale deq(W) + scaling A B
        const void* Wm = Wq;
        const int w_kind = dense ? 1 : (qscheme == FHPC_Q_INT8_PER_CHANNEL) ? 2 : 3;
        if (dh_rides) {
            FHPC_LAUNCH(run, launch_merge(Wq, scales, w_kind, f.A, rp, f.B, base_scale, scaling, s.Wm, false, K, rp, N, run.st, true));
            FHPC_HIP(gemm_two_outputs(OP_KC, OP_KC, operand(dY, N), operand(s.Wm, N + MERGE_EXT_PAD), dX, K, s.dH, rp, M, K, K + rp, N, run));
        } else {
            if (!premerged) {
                FHPC_LAUNCH(run, launch_merge(Wq, scales, w_kind, f.A, rp, f.B, base_scale, scaling, s.Wm, false, K, rp, N, run.st));
                Wm = s.Wm;
            }
            FHPC_HIP(gemm_plain(OP_KC, OP_KC, operand(dY, N), operand(Wm, N), dX, K, M, K, N, run));
        }
    } else if (streamed_dx) {
        // a handful of tokens: one pass over the packed weight (slabs; for r <= 16 also dH = dY B^T),
        // then slabs + rank-r branch -> bf16, and dH for dA
        const QskinnyDxPlan p = qskinny_dx_plan(M, K, N, qscheme, num_cu());
        QskinnyDxGrads grads = {X, H, dA, dB, r, scaling};
        const bool grads_ride = dh_on_the_way && (dA || dB);       // dA, dB in the finish launch
        FHPC_LAUNCH(run, launch_qskinny_dx(dY, Wq, scales, qscheme, f.B, f.A, rp, base_scale, scaling, dX, s.dH, M, K, N, p,
                                   s.sk_dxpart, s.sk_dhpart, grads_ride ? &grads : nullptr, run.st));
        if (grads_ride) return FHPC_OK;
    } else if (dX) {
        // dX[m][k] = base_scale * sum_n dY[m][n] deq(W)[k][n] + scaling * sum_j dH[m][j] A[k][j]
        GemmArgs g = {};
        g.a = operand(dY, N);
        g.b = dense ? operand(Wq, N) : operand(Wq, K, scales, K / 64);      // dense: element (k, n) at k*N + n
        g.a2 = operand(s.dH, rp);
        g.b2 = operand(f.A, rp);
        g.M = (int)M; g.N = (int)K; g.K = (int)N; g.K2 = (int)rp;
        g.alpha = base_scale; g.mid_scale = scaling / base_scale;
        const int b_mode = dense ? OP_KC : (qscheme == FHPC_Q_INT8_PER_CHANNEL) ? OP_Q8_XC : OP_Q4_XC;
        FHPC_HIP(fused_product(b_mode, OP_KC, g, dX, M, K, N, s.part, run));
    }
    return weight_grads(X, dY, H, s.dH, dA, dB, M, K, r, rp, N, scaling, s, run);
}

static int qlinear_bwd_impl(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                            const void* A, const void* B, float base_scale, float scaling, const void* dY,
                            const void* H_saved, void* dX, float* dA, float* dB,
                            int64_t M, int64_t K, int64_t r, int64_t N,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const bool premerged = (qscheme == FHPC_W_MERGED);
    const bool dense = (qscheme == FHPC_W_BF16) || premerged;
    if (!X || !Wq || (!scales && !dense) || !A || !B || !dY) return FHPC_ERR_NULL;
    int rc = dense ? FHPC_OK : check_q(qscheme, block, K);
    if (rc) return rc;
    rc = check_common(M, K, r, N);
    if (rc) return rc;
    if (dense && K * N * 2 >= kMaxBytes) return FHPC_ERR_UNSUPPORTED;
    if (!aligned(X, 16) || !aligned(Wq, 16) || !aligned(scales, 16) || !aligned(A, 16) || !aligned(B, 16) ||
        !aligned(dY, 16) || !aligned(H_saved, 16) || !aligned(dX, 16) || !aligned(dA, 16) || !aligned(dB, 16))
        return FHPC_ERR_ALIGN;
    rc = check_workspace(FHPC_OP_QLINEAR_BWD, workspace, workspace_bytes, M, K, r, N, FHPC_BF16, !dense, premerged);
    if (rc) return rc;
    Carver c(workspace);
    Scratch s = carve(c, FHPC_OP_QLINEAR_BWD, M, K, r, N, FHPC_BF16, !dense, premerged);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = s.part_bytes;
    return seq_qlinear_bwd(run, s, X, Wq, scales, qscheme, A, B, base_scale, scaling, dY, H_saved, dX, dA, dB, M, K, r, N);
}

int qlinear_lowrank_bwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                        const void* A, const void* B, float scaling, const void* dY,
                        const void* H_saved, void* dX, float* dA, float* dB,
                        int64_t M, int64_t K, int64_t r, int64_t N,
                        void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (qscheme == FHPC_W_BF16) return FHPC_ERR_DTYPE;
    return qlinear_bwd_impl(X, Wq, scales, qscheme, block, A, B, 1.f, scaling, dY, H_saved, dX, dA, dB, M, K, r, N,
                            workspace, workspace_bytes, hip_stream);
}

int qlinear_blend_bwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                      const void* A, const void* B, float alpha, const void* dY,
                      const void* H_saved, void* dX, float* dA, float* dB,
                      int64_t M, int64_t K, int64_t r, int64_t N,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!(alpha >= 0.f && alpha <= 1.f)) return FHPC_ERR_SHAPE;
    if (qscheme == FHPC_W_MERGED) return FHPC_ERR_DTYPE;
    return qlinear_bwd_impl(X, Wq, scales, qscheme, block, A, B, alpha, 1.f - alpha, dY, H_saved, dX, dA, dB, M, K, r, N,
                            workspace, workspace_bytes, hip_stream);
}

int swiglu_fwd(const void* G, const void* U, void* Z, int64_t n_elems, int dtype, void* hip_stream)
{
    if (!G || !U || !Z) return FHPC_ERR_NULL;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    if (n_elems < 0) return FHPC_ERR_SHAPE;
    if (!aligned(G, 16) || !aligned(U, 16) || !aligned(Z, 16)) return FHPC_ERR_ALIGN;
    FHPC_HIP(launch_swiglu_fwd(G, U, Z, n_elems, dtype == FHPC_BF16, static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

int swiglu_bwd(const void* G, const void* U, const void* dZ, void* dG, void* dU,
               int64_t n_elems, int dtype, void* hip_stream)
{
    if (!G || !U || !dZ || !dG || !dU) return FHPC_ERR_NULL;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    if (n_elems < 0) return FHPC_ERR_SHAPE;
    if (!aligned(G, 16) || !aligned(U, 16) || !aligned(dZ, 16) || !aligned(dG, 16) || !aligned(dU, 16)) return FHPC_ERR_ALIGN;
    FHPC_HIP(launch_swiglu_bwd(G, U, dZ, dG, dU, n_elems, dtype == FHPC_BF16, static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

int fhpc_add(const void* a, const void* b, void* out, int64_t n_elems, int dtype, void* hip_stream)
{
    if (!a || !b || !out) return FHPC_ERR_NULL;
    if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    if (n_elems < 0) return FHPC_ERR_SHAPE;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16)) return FHPC_ERR_ALIGN;
    FHPC_HIP(launch_add(a, b, out, n_elems, dtype == FHPC_BF16, static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

static int check_qweight(int qscheme, int block, int64_t K, int64_t N, bool needs_block)
{
    if (qscheme != FHPC_Q_INT8_PER_CHANNEL && qscheme != FHPC_Q_INT4_BLOCK) return FHPC_ERR_DTYPE;
    if (K < 1 || N < 1 || (K % 8) || (N % 8)) return FHPC_ERR_SHAPE;
    if (qscheme == FHPC_Q_INT4_BLOCK && needs_block) {
        if (block != 64) return FHPC_ERR_UNSUPPORTED;
        if (K % 64) return FHPC_ERR_SHAPE;
    }
    return FHPC_OK;
}

int qweight_quantize(const float* W, int qscheme, int block, void* Wq_out, void* scales_out,
                     int64_t K, int64_t N, void* hip_stream)
{
    if (!W || !Wq_out || !scales_out) return FHPC_ERR_NULL;
    int rc = check_qweight(qscheme, block, K, N, true);
    if (rc) return rc;
    // int8: the partial column maxima (ceil(K/64) * N floats, never more than the K * N code bytes)
    // are staged in the code buffer itself; they are consumed before the first code is written
    if (!aligned(W, 16) || !aligned(Wq_out, 16) || !aligned(scales_out, 2)) return FHPC_ERR_ALIGN;
    FHPC_HIP(launch_quantize(W, qscheme, block, Wq_out, scales_out, K, N, static_cast<float*>(Wq_out),
                             static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

int lowrank_merge(const void* W, const void* scales, int qscheme, int block, const void* A, const void* B,
                  float scaling, void* W_out, int out_dtype, int64_t K, int64_t r, int64_t N,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!A || !B || !W_out) return FHPC_ERR_NULL;
    if (out_dtype != FHPC_F32 && out_dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
    int rc = check_common(1, K, r, N);
    if (rc) return rc;
    int w_kind = 0;
    if (W) {
        if (qscheme == FHPC_W_BF16) {
            w_kind = 1;
        } else {
            rc = check_q(qscheme, block, K);
            if (rc) return rc;
            if (!scales) return FHPC_ERR_NULL;
            if (!aligned(scales, 2)) return FHPC_ERR_ALIGN;
            w_kind = (qscheme == FHPC_Q_INT8_PER_CHANNEL) ? 2 : 3;
        }
        if (!aligned(W, 16)) return FHPC_ERR_ALIGN;
    }
    if (K * N * 4 >= kMaxBytes) return FHPC_ERR_UNSUPPORTED;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(W_out, 16)) return FHPC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t rp = rank_pad(r);
    const void* Ap = A;
    const size_t need = merge_workspace(K, r, N);
    if (need) {
        if (!workspace || workspace_bytes < need) return FHPC_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return FHPC_ERR_ALIGN;
        void* const Apad = static_cast<unsigned char*>(workspace) + QSKINNY_HEADER_BYTES;
        FHPC_HIP(launch_pad2d_u16(A, r, K, r, Apad, rp, K, st));
        Ap = Apad;
    }
    FHPC_HIP(launch_merge(W, scales, w_kind, Ap, rp, B, 1.f, scaling, W_out, out_dtype == FHPC_F32, K, r, N, st, false, true));
    return FHPC_OK;
}

static int seq_decompose(Run& run, const DecompScratch& d, const void* W, const void* Omega, int power_iters,
                         void* A_out, void* B_out, int64_t K, int64_t r, int64_t N, int64_t batch)
{
    hipStream_t st = run.st;
    int rc;
    constexpr int kQuintic = 8, kCubic = 3;
    for (int64_t l = 0; l < batch; l++) {
        const void* Wl = static_cast<const uint16_t*>(W) + l * K * N;
        void* Al = static_cast<uint16_t*>(A_out) + l * K * r;
        void* Bl = static_cast<uint16_t*>(B_out) + l * r * N;
        const GemmOperand w = operand(Wl, N);
        // Y = W Omega, then `power_iters` rounds of  Z = W^T Y, orthonormalise, Y = W Z
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, w, operand(Omega, r), d.Yb, r, K, r, N, run));
        for (int it = 0; it < power_iters; it++) {
            rc = product_tn_bf16(w, operand(d.Yb, r), d.Zb, N, r, K, d, run);
            if (rc) return rc;
            rc = orthonormalise(d.Zb, d.Qt, N, r, kQuintic, kCubic, d, run);
            if (rc) return rc;
            FHPC_HIP(gemm_plain(OP_KC, OP_XC, w, operand(d.Qt, r), d.Yb, r, K, r, N, run));
        }
        rc = orthonormalise(d.Yb, Al, K, r, kQuintic, kCubic, d, run);                           // A = the basis, as it is used below
        if (rc) return rc;
        // B = (A^T A)^-1 A^T W, the least-squares fit given this very A.  G = A^T A = I + E with E small, so
        // G^-1 - I = -E + E^2 - E^3 (+ ...) and B = T + (G^-1 - I) T with T = A^T W.
        const GemmOperand a = operand(Al, r);
        FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, a, w, d.T, N, r, N, K, 1.f, d.part, run));
        FHPC_HIP(gemm_split_f32(OP_XC, OP_XC, a, a, d.G, r, r, r, K, 1.f, d.part, run));
        FHPC_LAUNCH(run, launch_gram_poly(d.G, nullptr, d.Gb, true, r, -1.f, 1.f, 0.f, 0, st));        // Gb = E = G - I
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(d.Gb, r), operand(d.Gb, r), d.G2b, r, r, r, r, run));   // E^2
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(d.G2b, r), operand(d.Gb, r), d.Sb, r, r, r, r, run));   // E^3
        FHPC_LAUNCH(run, launch_neumann(d.G, d.G2b, d.Sb, d.Gb, r, st));                               // Gb = -E + E^2 - E^3
        FHPC_LAUNCH(run, launch_compact_f32(d.T, N, d.Tb, N, r, N, 1.f, true, st));
        FHPC_HIP(gemm_plain(OP_KC, OP_XC, operand(d.Gb, r), operand(d.Tb, N), d.Cb, N, r, N, r, run));
        FHPC_LAUNCH(run, launch_add_f32_bf16(d.T, d.Cb, Bl, r * N, st));
    }
    return FHPC_OK;
}


int lowrank_decompose(const void* W, const void* Omega, int power_iters, void* A_out, void* B_out,
                      int64_t K, int64_t r, int64_t N, int64_t batch,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!W || !Omega || !A_out || !B_out) return FHPC_ERR_NULL;
    int rc = check_common(1, K, r, N);
    if (rc) return rc;
    if (batch < 1 || power_iters < 0 || power_iters > 16) return FHPC_ERR_SHAPE;
    if ((r % 8) || r > K || r > N) return FHPC_ERR_UNSUPPORTED;
    if (K * N * 2 >= kMaxBytes) return FHPC_ERR_UNSUPPORTED;
    if (!aligned(W, 16) || !aligned(Omega, 16) || !aligned(A_out, 16) || !aligned(B_out, 16)) return FHPC_ERR_ALIGN;
    Carver dry(nullptr);
    carve_decompose(dry, K, r, N);
    if (!workspace || workspace_bytes < dry.used) return FHPC_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return FHPC_ERR_ALIGN;
    Carver c(workspace);
    const DecompScratch d = carve_decompose(c, K, r, N);
    Run run;
    run.st = static_cast<hipStream_t>(hip_stream);
    run.part_cap = d.part_bytes;
    return seq_decompose(run, d, W, Omega, power_iters, A_out, B_out, K, r, N, batch);
}

int qweight_unpack(const void* Wq, int qscheme, int8_t* q_out, int64_t K, int64_t N, void* hip_stream)
{
    if (!Wq || !q_out) return FHPC_ERR_NULL;
    int rc = check_qweight(qscheme, 64, K, N, false);
    if (rc) return rc;
    FHPC_HIP(launch_unpack(Wq, qscheme, q_out, K, N, static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

int qweight_dequant(const void* Wq, const void* scales, int qscheme, int block, float* W_out,
                    int64_t K, int64_t N, void* hip_stream)
{
    if (!Wq || !scales || !W_out) return FHPC_ERR_NULL;
    int rc = check_qweight(qscheme, block, K, N, true);
    if (rc) return rc;
    FHPC_HIP(launch_dequant(Wq, scales, qscheme, block, W_out, K, N, static_cast<hipStream_t>(hip_stream)));
    return FHPC_OK;
}

int fhpc_gemm_bf16(const void* A, int64_t lda, int a_mode, const void* B, int64_t ldb, int b_mode,
                   void* C, int64_t ldc, int out_mode, int64_t M, int64_t N, int64_t K, float alpha,
                   int tile, int splits, int dbg, void* hip_stream)
{
    if (!A || !B || !C) return FHPC_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || (K % 8) || (N % 8) || splits < 1) return FHPC_ERR_SHAPE;
    if ((a_mode != OP_KC && a_mode != OP_XC) || (b_mode != OP_KC && b_mode != OP_XC)) return FHPC_ERR_DTYPE;
    if (a_mode == OP_XC && (M % 8)) return FHPC_ERR_SHAPE;
    if (M * K * 2 >= kMaxBytes || N * K * 2 >= kMaxBytes || tile < 0 || tile >= TILE_COUNT) return FHPC_ERR_UNSUPPORTED;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(C, 16)) return FHPC_ERR_ALIGN;
    GemmArgs g = {};
    g.a = operand(A, lda);
    g.b = operand(B, ldb);
    g.c = C; g.ldc = ldc;
    g.M = (int)M; g.N = (int)N; g.K = (int)K; g.K2 = 0;
    g.alpha = alpha; g.mid_scale = 1.f;
#ifdef FHPC_DIAG
    g.dbg = dbg;
#else
    g.dbg = dbg & 12;
#endif
    const int64_t ksteps = (K + 63) / 64;
    const int64_t per = (ksteps + splits - 1) / splits;
    g.k_chunk = (int)(per * 64);
    g.splits = (int)((ksteps + per - 1) / per);
    g.split_stride = M * ldc;
    hipError_t e = launch_gemm_bf16(a_mode, b_mode, OP_NONE, out_mode, tile, g, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return FHPC_ERR_UNSUPPORTED;
    FHPC_HIP(e);
    return FHPC_OK;
}

int fhpc_plan_slab_bytes(int call, int64_t M, int64_t K, int64_t r, int64_t N, int dtype, int qscheme, int g,
                         int outputs, float base_scale, int64_t* planned, int64_t* reserved)
{
    if (!planned || !reserved) return FHPC_ERR_NULL;
    // addresses that are never dereferenced: the dry pass launches nothing
    void* const fake = reinterpret_cast<void*>((uintptr_t)1 << 21);
    float* const ffake = static_cast<float*>(fake);
    void* const o0 = (outputs & 1) ? fake : nullptr;
    float* const o1 = (outputs & 2) ? ffake : nullptr;
    float* const o2 = (outputs & 4) ? ffake : nullptr;
    const void* const hs = (outputs & 8) ? fake : nullptr;
    Run run;
    run.dry = true;
    Carver c(nullptr);
    int rc = FHPC_ERR_SHAPE;
    if (call >= FHPC_OP_LOWRANK_FWD && call <= FHPC_OP_QLINEAR_BWD) {
        rc = check_common(M, K, r, N);
        if (rc) return rc;
        if (dtype != FHPC_F32 && dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
        const bool premerged = (qscheme == FHPC_W_MERGED), dense = premerged || (qscheme == FHPC_W_BF16);
        const bool q = (call == FHPC_OP_QLINEAR_FWD || call == FHPC_OP_QLINEAR_BWD);
        if (q) {
            if (dtype != FHPC_BF16) return FHPC_ERR_DTYPE;
            rc = dense ? FHPC_OK : check_q(qscheme, 64, K);
            if (rc) return rc;
        }
        const Scratch s = q ? carve(c, call, M, K, r, N, FHPC_BF16, !dense, premerged) : carve(c, call, M, K, r, N, dtype);
        *reserved = s.part_bytes;
        if (call == FHPC_OP_LOWRANK_FWD) rc = seq_lowrank_fwd(run, s, fake, fake, fake, fake, o0, M, K, r, N, dtype);
        else if (call == FHPC_OP_LOWRANK_BWD) rc = seq_lowrank_bwd(run, s, fake, fake, fake, fake, hs, o0, o1, o2, M, K, r, N, dtype);
        else if (call == FHPC_OP_QLINEAR_FWD)
            rc = seq_qlinear_fwd(run, s, fake, fake, fake, qscheme, fake, fake, base_scale, 1.f, fake, o0, M, K, r, N);
        else
            rc = seq_qlinear_bwd(run, s, fake, fake, fake, qscheme, fake, fake, base_scale, 1.f, fake, hs, o0, o1, o2, M, K, r, N);
    } else if (call == FHPC_OP_DECOMPOSE) {
        rc = check_common(1, K, r, N);
        if (rc) return rc;
        if ((r % 8) || r > K || r > N) return FHPC_ERR_UNSUPPORTED;
        const DecompScratch d = carve_decompose(c, K, r, N);
        *reserved = d.part_bytes;
        rc = seq_decompose(run, d, fake, fake, 1, fake, fake, K, r, N, 1);
    } else if (call == FHPC_PLAN_SHARED_FWD || call == FHPC_PLAN_SHARED_BWD) {
        rc = check_shared(M, K, r, N, g);
        if (rc) return rc;
        const bool bwd = (call == FHPC_PLAN_SHARED_BWD);
        const SharedScratch s = carve_shared(c, bwd, M, K, r, N, g);
        *reserved = s.part_bytes;
        const void* in[FHPC_MAX_SHARED];
        void* out[FHPC_MAX_SHARED];
        float* dB[FHPC_MAX_SHARED];
        for (int i = 0; i < g; i++) { in[i] = fake; out[i] = fake; dB[i] = o2; }
        rc = bwd ? seq_shared_bwd(run, s, fake, fake, in, in, hs, o0, o1, dB, o2 != nullptr, M, K, r, N, g)
                 : seq_shared_fwd(run, s, fake, fake, in, out, o0, M, K, r, N, g);
    } else if (call == FHPC_PLAN_FFN_GATE_UP) {
        rc = check_shared(M, K, r, N, 2);
        if (rc) return rc;
        const SharedScratch s = carve_shared(c, false, M, K, r, N, 2);
        *reserved = s.part_bytes;
        rc = seq_ffn_gate_up_fwd(run, s, fake, fake, fake, fake, fake, fake, fake, o0, M, K, r, N);
    } else if (call == FHPC_PLAN_FFN_DOWN_BWD) {
        rc = check_common(M, K, r, N);
        if (rc) return rc;
        const Scratch s = carve(c, FHPC_OP_LOWRANK_BWD, M, K, r, N, FHPC_BF16);
        *reserved = s.part_bytes;
        rc = seq_ffn_down_bwd(run, s, fake, fake, fake, fake, hs, fake, fake, fake, fake, o1, o2, M, K, r, N);
    }
    *planned = run.part_need;
    return rc;
}

const char* fhpc_status_string(int status)
{
    switch (status) {
        case FHPC_OK: return "ok";
        case FHPC_ERR_NULL: return "a required pointer is NULL";
        case FHPC_ERR_SHAPE: return "invalid shape (sizes must be positive; K and N multiples of 8; K a multiple of the block)";
        case FHPC_ERR_DTYPE: return "unknown dtype or quantisation scheme";
        case FHPC_ERR_ALIGN: return "pointer not sufficiently aligned (16 bytes; workspace 256)";
        case FHPC_ERR_WORKSPACE: return "workspace missing or smaller than fhpc_workspace_bytes (the entry point without a workspace argument: the sizes need more than its fixed scratch array)";
        case FHPC_ERR_UNSUPPORTED: return "unsupported configuration (block must be 64; matrices below 2 GiB)";
        case FHPC_ERR_HIP: return "a HIP call or kernel launch failed";
        default: return "unknown status";
    }
}

int fhpc_version(void) { return 100; }

}  // extern "C"
