// Adapted weight materialised for inference (Sec. 5.1, eq. new_linear_layer: W' = W + Delta W
// with Delta W the product of the factor pair):
//     W_out[K,N] = deq(W)[K,N] + scaling * A[K,r] * B[r,N]
//
// One pass over the weight: the kernel is bound by reading W once and writing W_out once; the
// rank-r product is a short matrix-core loop (reduction length r) per 64 x 128 tile of the
// output, on 32-deep slices of A and B double-buffered in LDS (global -> LDS requests,
// transposing LDS reads for B).
//
// The matrix instruction is oriented so that a lane ends up with columns of the output and groups
// of four consecutive rows k; one half-wave swap per register pair then gives every lane ONE
// column (lane = column, 64 columns per wave) and 32 consecutive rows.  That is exactly how a
// quantised base weight is stored (channel-major: the codes of one output channel are contiguous
// in k), so a lane loads the 32 codes of its channel once and adds them with no transposition
// anywhere; code * scale is exact in fp32 and the sum is rounded once.  Along a row the 64 lanes
// hold 64 consecutive columns: an fp32 store instruction writes 256 contiguous bytes.  bf16 output
// is packed into 32-bit words of two adjacent columns (neighbouring lanes trade one value each),
// turned round in a 4 KiB LDS patch per wave and stored 16 bytes per lane, eight rows of 128 bytes
// per instruction (as 32-bit stores, two rows per instruction, the kernel was bound by the number
// of stores: a bf16 output took as long as an fp32 one); a bf16 base weight is loaded as 32-bit
// column pairs.  The base weight of the tile is requested before the r-loop and stays in registers
// meanwhile.
#include "merge.h"
#include "gemm_ring.h"
#include "profile.h"

namespace fhpc {
namespace mrg {

using namespace ring;

constexpr int NT = 256;
constexpr int RB = 1;                         // 32-row blocks per wave (two: no faster for int4, slower for int8)
constexpr int TK = 64 * RB, TN = 128, BK = 32; // output tile (rows of W' x columns), rank slice
enum : int { W_NONE = 0, W_BF16 = 1, W_INT8 = 2, W_INT4 = 3 };

struct MergeArgs {
    const void* W;
    const uint16_t* scales;
    GemmOperand a, b;      // A[K][ld] (rank index contiguous), B[r][N]
    void* out;
    float scaling;
    float base_scale;      // factor on the base weight (1 for the merged weight of Sec. 5.1; alpha for the blend layer)
    int K, N, r;           // r: rank rounded up to a multiple of 8 (the copy of A is zero-padded)
    int r_rows;            // rows of B that exist
    int ldo;               // row stride of out in elements: N, or N + MERGE_EXT_PAD with `ext`
    int ext;               // out is [(K + r)][(N + MERGE_EXT_PAD)] bf16: W' in its K x N corner, A in columns N .. N + r - 1 of those
                           // rows, B in rows K .. K + r - 1 of those columns (the r x r corner zero): one buffer whose
                           // products with X and with dY also give H = X A and dH = dY B^T as r extra output columns
};

// value of the lane with the other parity in the same pair (lanes 2 m and 2 m + 1)
__device__ __forceinline__ uint32_t swap_with_neighbour(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1 /* quad_perm 1 0 3 2 */, 0xf, 0xf, true);
}

// Buffer descriptors of the output and of a bf16 base weight: stores and loads then take a 32-bit lane
// offset plus a scalar row offset, a lane whose column does not exist is parked at an offset the range
// check drops, and rows past the end are skipped by a scalar branch (they come in whole pairs), so the
// epilogue spends no vector instructions on addresses or bounds.
constexpr uint32_t MRG_OOB = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t matrix_rsrc(const void* ptr, int K, int N, int elt)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(ptr), 0, K * N * elt, 0x00020000);
}

// The base weight of a wave's 32 x 64 block in the layout the epilogue works in: lane = column n,
// 32 rows kw .. kw + 31.
template <int WMODE>
struct BaseRegs {
    uint32_t wb[WMODE == W_BF16 ? 16 : 1];     // bf16 pairs, one word per two rows (even lanes: row 2 q, odd lanes: row 2 q + 1)
    u32x2 q8[WMODE == W_INT8 ? 4 : 1];         // codes k = kw + 8 i .. + 7 of the lane's channel
    u32x4 q4;                                  // codes k = kw .. kw + 31
    float wscale;                              // base_scale * fp16 scale of the lane's channel (and block)
};

template <int WMODE>
__device__ __forceinline__ void load_base(BaseRegs<WMODE>& b, const MergeArgs& p, int kw, int n, int lane)
{
    b.q4 = (u32x4){0u, 0u, 0u, 0u};
    b.wscale = 0.f;
    if constexpr (WMODE == W_BF16) {
        // the column pair (n & ~1, + 1) of row 2 q (even lanes) or 2 q + 1 (odd lanes); rows past the end
        // and parked lanes read as zero
        const __amdgpu_buffer_rsrc_t rw = matrix_rsrc(p.W, p.K, p.N, 2);
        const uint32_t lane_off = (n < p.N) ? (uint32_t)((kw + (lane & 1)) * p.N + (n & ~1)) * 2u : MRG_OOB;
#pragma unroll
        for (int q = 0; q < 16; q++) {
            b.wb[q] = 0u;
            if (kw + 2 * q < p.K) b.wb[q] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane_off, 2 * q * p.N * 2, 0);     // uniform
        }
    } else if constexpr (WMODE == W_INT8) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            b.q8[i] = (u32x2){0u, 0u};
            if (n < p.N && kw + 8 * i < p.K)
                b.q8[i] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(p.W) + (size_t)n * (size_t)p.K + (size_t)(kw + 8 * i));
        }
        if (n < p.N) b.wscale = p.base_scale * (float)__builtin_bit_cast(_Float16, p.scales[n]);
    } else if constexpr (WMODE == W_INT4) {
        if (n < p.N && kw < p.K) {
            b.q4 = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(p.W) + ((size_t)n * (size_t)p.K + (size_t)kw) / 2);
            b.wscale = p.base_scale * (float)__builtin_bit_cast(_Float16, p.scales[(size_t)n * (size_t)(p.K / 64) + (size_t)(kw / 64)]);
        }
    }
}

// out = base_scale * base + scaling * acc for the wave's 32 x 64 block, straight from the accumulators
// (acc[j]: register v holds row kw + 8 (v / 4) + 4 (lane / 32) + v % 4, column n_block + 32 j + lane % 32).
template <int WMODE, bool OUT_F32, bool NT>
__device__ __forceinline__ void store_block(const f32x16 (&acc)[2], const BaseRegs<WMODE>& b, const MergeArgs& p, int kw, int n, int lane,
                                            unsigned char* patch)
{
    // rows[q]: row kw + q, lane = column.  One half-wave swap per register pair turns
    // (block 0 | block 1) x (rows of the lower | upper lanes) into (row | row + 4) x 64 columns.
    float rows[32];
#pragma unroll
    for (int v = 0; v < 16; v++) {
        // (the products are fresh registers for the swap, which exchanges in place; accumulators passed to it
        // directly came back wrong)
        const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, acc[0][v] * p.scaling),
                                                         __builtin_bit_cast(uint32_t, acc[1][v] * p.scaling), false, false);
        rows[8 * (v / 4) + (v % 4)] = __builtin_bit_cast(float, (uint32_t)sw[0]);
        rows[8 * (v / 4) + 4 + (v % 4)] = __builtin_bit_cast(float, (uint32_t)sw[1]);
    }
    const __amdgpu_buffer_rsrc_t ro = matrix_rsrc(p.out, p.K, p.ldo, OUT_F32 ? 4 : 2);
    const int rows_valid = p.K - kw;               // rows of this block that exist (scalar)
    const int rowbytes = p.ldo * (OUT_F32 ? 4 : 2);
    const bool odd = lane & 1;
    // fp32: the lane's own column, rows q and q + 1 in turn.  bf16: the column pair (n & ~1, + 1) of row
    // q (even lanes) or q + 1 (odd lanes), see below.
    const uint32_t lane_off = (n < p.N) ? (OUT_F32 ? (uint32_t)(kw * p.ldo + n) * 4u
                                                    : (uint32_t)((kw + (odd ? 1 : 0)) * p.ldo + (n & ~1)) * 2u) : MRG_OOB;
    // bf16 halves of (own, neighbour) words recombined by one byte permute: even lanes keep their low
    // half and take the neighbour's low half on top, odd lanes take the neighbour's high half below their own
    const uint32_t pick = odd ? 0x03020706u : 0x05040100u;
    // bf16 output: the 32 x 64 block is turned round in a 4 KiB LDS patch of the wave's own ([32 rows][128 bytes],
    // 16-byte pieces XOR-swizzled by the row) and leaves as 16-byte stores, eight columns per lane and eight rows
    // per instruction: a quarter of the store instructions the 32-bit pairs took.  (With those the kernel moved a
    // bf16 output in the time of an fp32 one, twice the bytes: it was bound by the number of stores, not by bytes.)
    const int prow = odd ? 1 : 0, pword = lane >> 1;             // this lane's word: row q + prow, columns 2 pword, + 1
#pragma unroll
    for (int q = 0; q < 32; q += 2) {
        float base0 = 0.f, base1 = 0.f;
        if constexpr (WMODE == W_BF16) {
            // the word holds this lane's column and its neighbour's for one of the two rows; the
            // neighbour holds the other row: swap the halves that belong to each other
            const uint32_t dw = b.wb[q / 2];
            const uint32_t got = swap_with_neighbour(odd ? (dw & 0xffffu) : (dw >> 16));
            base0 = p.base_scale * __builtin_bit_cast(float, (odd ? got : (dw & 0xffffu)) << 16);
            base1 = p.base_scale * __builtin_bit_cast(float, (odd ? (dw >> 16) : got) << 16);
        } else if constexpr (WMODE == W_INT8) {
            const uint32_t w = (q & 4) ? b.q8[q / 8].y : b.q8[q / 8].x;
            base0 = (float)(int)__builtin_amdgcn_sbfe((int)w, 8 * (q % 4), 8) * b.wscale;      // (the builtin's result type is unsigned)
            base1 = (float)(int)__builtin_amdgcn_sbfe((int)w, 8 * (q % 4) + 8, 8) * b.wscale;
        } else if constexpr (WMODE == W_INT4) {
            const uint32_t d = (q / 8 == 0) ? b.q4.x : (q / 8 == 1) ? b.q4.y : (q / 8 == 2) ? b.q4.z : b.q4.w;
            base0 = (float)(int)__builtin_amdgcn_sbfe((int)d, 4 * (q % 8), 4) * b.wscale;
            base1 = (float)(int)__builtin_amdgcn_sbfe((int)d, 4 * (q % 8) + 4, 4) * b.wscale;
        }
        const float o0 = rows[q] + base0;
        const float o1 = rows[q + 1] + base1;
        if constexpr (OUT_F32) {
            if (q >= rows_valid) continue;         // uniform: K is a multiple of 8, a row pair is in or out as one
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, o0), ro, lane_off, q * rowbytes, NT ? 2 : 0);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, o1), ro, lane_off, (q + 1) * rowbytes, NT ? 2 : 0);
        } else {
            // An even lane ends up with columns (n, n + 1) of row q, its odd neighbour with (n - 1, n) of row q + 1.
            const uint32_t own = pack_bf16(o0, o1);                          // (row q, row q + 1) of this column
            const uint32_t nb = swap_with_neighbour(own);                    // the same of the neighbour's column
            const uint32_t word = __builtin_amdgcn_perm(nb, own, pick);
            const int row = q + prow;
            *reinterpret_cast<uint32_t*>(patch + row * 128 + ((((pword >> 2) ^ row) & 7) << 4) + (pword & 3) * 4) = word;
        }
    }
    if constexpr (!OUT_F32) {
        // lane -> row lane / 8 (+ 8 per instruction), columns 8 (lane % 8) .. + 7 of the wave's 64
        const int rr = lane >> 3, rc = lane & 7;
        const int n8 = n - lane + rc * 8;                                   // first of the lane's eight columns
        const uint32_t off16 = (n8 < p.N) ? (uint32_t)((kw + rr) * p.ldo + n8) * 2u : MRG_OOB;   // (N is a multiple of 8)
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if (8 * k >= rows_valid) break;        // uniform: rows come in groups of eight
            const int row = rr + 8 * k;
            const u32x4 v = *reinterpret_cast<const u32x4*>(patch + row * 128 + (((rc ^ row) & 7) << 4));
            __builtin_amdgcn_raw_buffer_store_b128(v, ro, off16, 8 * k * rowbytes, NT ? 2 : 0);
        }
    }
}

template <int WMODE, bool OUT_F32, bool STREAM>
__global__ __launch_bounds__(NT) void merge_kernel(MergeArgs p)
{
    using FA = Feeder<OP_KC, TK, BK, 4>;
    using FB = Feeder<OP_XC, TN, BK, 4>;
    using TA = typename FA::Tile;
    using TB = typename FB::Tile;
    constexpr int TILE_A_BYTES = FA::TILE_BYTES, STAGE_BYTES = FA::TILE_BYTES + FB::TILE_BYTES;
    constexpr int L = FA::PER + FB::PER;

    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_k0 = (wave >> 1) * (32 * RB);               // the wave's RB blocks of 32 rows ...
    const int wave_n0 = (wave & 1) * 64;                       // ... by two blocks of 32 columns
    const int tiles_n = (p.N + TN - 1) / TN;
    int tk = blockIdx.x / tiles_n, tn = blockIdx.x - tk * tiles_n;
    if constexpr (STREAM) {
        // A quantised channel's codes are contiguous along k and a 64-row tile takes 32 (int4) or 64 (int8) bytes of
        // each 128-byte line: the four tiles that follow one another along k share their lines.  Workgroups go to
        // the eight XCDs in turn (id % 8), each with an L2 of its own, so the four tiles of a line take four
        // consecutive slots of one XCD and the line comes from memory once (row-major tile order fetched 78 MB for
        // a 37.6 MB int4 weight).  With streamed output the kernel is bound by bytes and this pays (40 -> 36 us);
        // with cached output it is not and it costs 3 % (measured both ways).
        const int tiles_k = (p.K + TK - 1) / TK;
        const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3;
        const int t = (slot >> 2) * 8 + xcd;                  // (column tile, group of four row tiles)
        tn = t % tiles_n;
        tk = 4 * (t / tiles_n) + (slot & 3);
        if (tk >= tiles_k) return;                             // (the whole workgroup: padding of the last group or block)
    }
    const int k0 = tk * TK, n0 = tn * TN;
    const int kw = k0 + wave_k0;                               // first row of the wave
    // accumulator register v of block (b, j): row kw + 32 b + 8 (v / 4) + 4 (lane / 32) + v % 4, column n0 + wave_n0 + 32 j + lane % 32

    // ---- base weight of the wave's RB blocks of 32 x 64, requested before anything else
    const int n = n0 + wave_n0 + lane;
    BaseRegs<WMODE> base[RB];
#pragma unroll
    for (int b = 0; b < RB; b++) load_base<WMODE>(base[b], p, kw + 32 * b, n, lane);

    // ---- acc[b][j] = (A B) block: rows from the A tile, columns from the B tile
    f32x16 acc[RB][2];
#pragma unroll
    for (int b = 0; b < RB; b++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[b][j][v] = 0.f;
    {
        FA fa;
        FB fb;
        fa.init(p.a, k0, p.K, p.r, wave, lane);
        fb.init(p.b, n0, p.N, p.r_rows, wave, lane);
        FragAddr aa[RB];
#pragma unroll
        for (int b = 0; b < RB; b++) aa[b] = TA::make(wave_k0 + 32 * b, lane);
        const FragAddr ab = TB::make(wave_n0, lane);
        fa.issue(lds, 0, p.r, wave);
        fb.issue(lds + TILE_A_BYTES, 0, p.r, wave);
        int stage = 0;
        for (int r0 = 0; r0 < p.r; r0 += BK) {
            unsigned char* cur = lds + stage * STAGE_BYTES;
            unsigned char* nxt = lds + (stage ^ 1) * STAGE_BYTES;
            // the other stage was released by the barrier that ended the previous trip
            fa.issue(nxt, r0 + BK, p.r, wave);
            fb.issue(nxt + TILE_A_BYTES, r0 + BK, p.r, wave);
            FHPC_WAIT_VM(L);
            wg_barrier();
#pragma unroll
            for (int s = 0; s < BK / 16; s++) {
                bf16x8 rb[2];
#pragma unroll
                for (int j = 0; j < 2; j++) rb[j] = TB::frag(cur + TILE_A_BYTES, ab, j, s);
#pragma unroll
                for (int b = 0; b < RB; b++) {
                    const bf16x8 ra = TA::frag(cur, aa[b], 0, s);
#pragma unroll
                    for (int j = 0; j < 2; j++) acc[b][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ra, rb[j], acc[b][j], 0, 0, 0);
                }
            }
            FHPC_WAIT_LGKM0();
            wg_barrier();
            stage ^= 1;
        }
        FHPC_WAIT_VM(0);        // the last trip's requests (past the end of the rank: zeros) still land in LDS
    }
    if constexpr (!OUT_F32) wg_barrier();     // ... every wave's: the stages now serve as the waves' output patches

#pragma unroll
    for (int b = 0; b < RB; b++) store_block<WMODE, OUT_F32, STREAM>(acc[b], base[b], p, kw + 32 * b, n, lane, lds + wave * 4096);

    if constexpr (!OUT_F32) {
        if (p.ext) {
            // the factor pair beside and below W' (16-byte pieces; rows of B beyond r_rows and the corner are zero)
            uint16_t* const out = static_cast<uint16_t*>(p.out);
            const u32x4 zero = {0u, 0u, 0u, 0u};
            const int pieces = p.r / 8;
            if (tn == 0) {
                const uint16_t* const A = static_cast<const uint16_t*>(p.a.ptr);
                for (int t = tid; t < TK * pieces; t += NT) {
                    const int k = k0 + t / pieces, c = (t % pieces) * 8;
                    if (k < p.K)
                        *reinterpret_cast<u32x4*>(out + (size_t)k * p.ldo + p.N + c) = *reinterpret_cast<const u32x4*>(A + (size_t)k * p.a.ld + c);
                }
            }
            if (tk == 0) {
                const uint16_t* const B = static_cast<const uint16_t*>(p.b.ptr);
                for (int t = tid; t < p.r * (TN / 8); t += NT) {
                    const int j = t / (TN / 8), c = n0 + (t % (TN / 8)) * 8;
                    if (c < p.N)
                        *reinterpret_cast<u32x4*>(out + (size_t)(p.K + j) * p.ldo + c) =
                            (j < p.r_rows) ? *reinterpret_cast<const u32x4*>(B + (size_t)j * p.b.ld + c) : zero;
                }
                if (tn == 0)
                    for (int t = tid; t < p.r * pieces; t += NT)
                        *reinterpret_cast<u32x4*>(out + (size_t)(p.K + t / pieces) * p.ldo + p.N + (t % pieces) * 8) = zero;
            }
        }
    }
}

template <int WMODE, bool OUT_F32, bool STREAM>
static hipError_t launch(const MergeArgs& a, double w_bytes, hipStream_t s)
{
    int tiles = ((a.K + TK - 1) / TK) * ((a.N + TN - 1) / TN);
    if (STREAM) {
        // (column tiles) x (groups of four row tiles), rounded up to whole blocks of 8 groups, four workgroups each
        const int groups = ((a.K + TK - 1) / TK + 3) / 4 * ((a.N + TN - 1) / TN);
        tiles = (groups + 7) / 8 * 32;
    }
    const double bytes = w_bytes + (double)a.K * a.N * (OUT_F32 ? 4.0 : 2.0) + 2.0 * a.r_rows * ((double)a.K + a.N);
    const char* names[4] = {"merge<none>", "merge<bf16>", "merge<int8>", "merge<int4>"};
    const int slot = prof_begin(names[WMODE], 2.0 * a.K * (double)a.N * a.r_rows, bytes, s);
    hipLaunchKernelGGL((merge_kernel<WMODE, OUT_F32, STREAM>), dim3((unsigned)tiles), dim3(NT), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

}  // namespace mrg

hipError_t launch_merge(const void* W, const void* scales, int w_kind, const void* A, int64_t lda, const void* B,
                        float base_scale, float scaling, void* out, bool out_f32, int64_t K, int64_t r, int64_t N, hipStream_t s,
                        bool ext, bool stream_out)
{
    using namespace mrg;
    MergeArgs a;
    a.W = W;
    a.scales = static_cast<const uint16_t*>(scales);
    a.a = GemmOperand{A, lda, nullptr, 0};
    a.b = GemmOperand{B, N, nullptr, 0};
    a.out = out;
    a.scaling = scaling;
    a.base_scale = base_scale;
    a.K = (int)K;
    a.N = (int)N;
    a.r = (int)lda;
    a.r_rows = (int)r;
    if (ext && out_f32) return hipErrorInvalidValue;
    a.ext = ext ? 1 : 0;
    a.ldo = (int)(ext ? N + MERGE_EXT_PAD : N);
    const double kn = (double)K * (double)N;
    const double wbytes[4] = {0.0, 2.0 * kn, kn + 2.0 * N, 0.5 * kn + kn / 32.0};
    if (w_kind < 0 || w_kind > 3) return hipErrorInvalidValue;
#define FHPC_MERGE_CASE(KIND, F32)                                                                               \
    if (w_kind == KIND && out_f32 == F32)                                                                        \
        return stream_out ? launch<KIND, F32, true>(a, wbytes[KIND], s) : launch<KIND, F32, false>(a, wbytes[KIND], s);
    FHPC_MERGE_CASE(W_NONE, true)
    FHPC_MERGE_CASE(W_NONE, false)
    FHPC_MERGE_CASE(W_BF16, true)
    FHPC_MERGE_CASE(W_BF16, false)
    FHPC_MERGE_CASE(W_INT8, true)
    FHPC_MERGE_CASE(W_INT8, false)
    FHPC_MERGE_CASE(W_INT4, true)
    FHPC_MERGE_CASE(W_INT4, false)
#undef FHPC_MERGE_CASE
    return hipErrorInvalidValue;
}

}  // namespace fhpc
