// bf16 MFMA GEMM core for gfx950 (CDNA4): v_mfma_f32_32x32x16_bf16, fp32 accumulation,
// 64-deep K steps double-buffered through LDS, operands staged through registers so
// that transposition and int8/int4 dequantisation happen on the way into LDS.
//
// LDS tile layout (both operands): [rows][64 bf16], 128 bytes per row, the eight
// 16-byte chunks of a row XOR-swizzled with (row ^ row>>3) & 7.  That keeps the
// fragment reads (32 consecutive rows, one chunk) and both kinds of staging writes
// (8 lanes along a row; 8 lanes down rows 8 apart) free of bank conflicts.
//
// Accumulator orientation: the B-side tile feeds the MFMA's row operand and the
// A-side tile its column operand, so a lane ends up holding 4 consecutive output
// columns n of one output row m (16-byte fp32 / 8-byte bf16 stores).
#include "gemm_bf16.h"
#include "profile.h"

#include <stdio.h>

namespace fhpc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

static constexpr int NTHREADS = 256;
static constexpr int BK = 64;
static constexpr uint32_t OOB = 0x80000000u;   // byte offset beyond any 2 GiB operand

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint32_t lds_off(int row, int chunk)
{
    return (uint32_t)row * 128u + (uint32_t)(((chunk ^ (row ^ (row >> 3))) & 7) << 4);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f;
    f.x = lo;
    f.y = hi;
    bf16x2 b = __builtin_convertvector(f, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}

// Sign-extended 4-bit field at bit `pos` (the bit-field-extract builtin returns unsigned).
__device__ __forceinline__ int nib(uint32_t word, int pos)
{
    return (int)__builtin_amdgcn_sbfe((int)word, (unsigned)pos, 4u);
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// 8x8 transposition of 16-bit elements held as 8 rows of 4 dwords: out[c] collects
// element c of every row (row 0 in the low half of dword 0).
__device__ __forceinline__ void transpose8x8(const u32x4 (&v)[8], u32x4 (&o)[8])
{
#pragma unroll
    for (int c = 0; c < 8; c++) {
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
        for (int w = 0; w < 4; w++)
            o[c][w] = __builtin_amdgcn_perm(v[2 * w + 1][c >> 1], v[2 * w][c >> 1], sel);
    }
}

// ---------------------------------------------------------------------------------
// Staging: global -> registers (issue) -> LDS tile (commit).  R = tile rows (BM or BN).
// row0 = first output index of the tile, dim = extent of the output index.
// ---------------------------------------------------------------------------------

template <int MODE, int R>
struct Stage;

// bf16, k contiguous.  Thread t: chunk t%8 of rows t/8 + 32 i.
template <int R>
struct Stage<OP_KC, R> {
    static constexpr int NL = R / 32;
    u32x4 raw[NL];
    uint32_t voff, rstep;
    int chunk;
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)op.ld * 2u);
        chunk = tid & 7;
        voff = ((uint32_t)(row0 + (tid >> 3)) * (uint32_t)op.ld + (uint32_t)chunk * 8u) * 2u;
        rstep = 32u * (uint32_t)op.ld * 2u;
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
        const uint32_t kofs = (k0 + chunk * 8 < kend) ? (uint32_t)k0 * 2u : OOB;
#pragma unroll
        for (int i = 0; i < NL; i++)
            raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + (uint32_t)i * rstep + kofs, 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int i = 0; i < NL; i++)
            *reinterpret_cast<u32x4*>(tile + lds_off((tid >> 3) + 32 * i, chunk)) = raw[i];
    }
};

// Geometry shared by the transposing stages: the [64 k][R rows] source tile is cut into
// 8x8 blocks; block b covers k-group b / (R/8) and row-chunk b % (R/8).
template <int R>
struct XcGeom {
    static constexpr int NBLK = R;                       // (64/8) * (R/8)
    static constexpr int PER_THREAD = (NBLK + NTHREADS - 1) / NTHREADS;
    static constexpr bool ALL_ACTIVE = (NBLK % NTHREADS) == 0;
};

template <int R>
__device__ __forceinline__ void commit_transposed(unsigned char* tile, const u32x4 (&v)[8], int cc, int kg)
{
    u32x4 o[8];
    transpose8x8(v, o);
#pragma unroll
    for (int c = 0; c < 8; c++)
        *reinterpret_cast<u32x4*>(tile + lds_off(cc * 8 + c, kg)) = o[c];
}

// bf16, output index contiguous: ptr[k*ld + row].
template <int R>
struct Stage<OP_XC, R> {
    using G = XcGeom<R>;
    u32x4 raw[G::PER_THREAD][8];
    uint32_t voff[G::PER_THREAD];
    uint32_t ldb;
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)op.ld * 2u);
        ldb = (uint32_t)op.ld * 2u;
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            const int cc = blk % (R / 8), kg = blk / (R / 8);
            const int row = row0 + cc * 8;
            const bool ok = (G::ALL_ACTIVE || blk < G::NBLK) && row < dim;
            voff[b] = ok ? ((uint32_t)(kg * 8) * (uint32_t)op.ld + (uint32_t)row) * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
        const uint32_t kofs = (uint32_t)k0 * ldb;
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++)
#pragma unroll
            for (int j = 0; j < 8; j++)
                raw[b][j] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[b] + kofs + (uint32_t)j * ldb, 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            if (G::ALL_ACTIVE || blk < G::NBLK)
                commit_transposed<R>(tile, raw[b], blk % (R / 8), blk / (R / 8));
        }
    }
};

// int8 codes, k contiguous, one fp16 scale per row.  Item = 16 codes (16 bytes).
template <int R>
struct Stage<OP_Q8_KC, R> {
    static constexpr int NITEM = R * 4;
    static constexpr int PER_THREAD = (NITEM + NTHREADS - 1) / NTHREADS;
    static constexpr bool ALL_ACTIVE = (NITEM % NTHREADS) == 0;
    u32x4 raw[PER_THREAD];
    float sc[PER_THREAD];
    uint32_t voff[PER_THREAD];
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)op.ld);
        __amdgpu_buffer_rsrc_t rsc = make_rsrc(op.scales, (uint32_t)dim * 2u);
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++) {
            const int item = tid + NTHREADS * i;
            const int row = row0 + (item >> 2);
            const bool ok = ALL_ACTIVE || item < NITEM;
            voff[i] = ok ? (uint32_t)row * (uint32_t)op.ld + (uint32_t)(item & 3) * 16u : OOB;
            sc[i] = half_bits_to_float(__builtin_amdgcn_raw_buffer_load_b16(rsc, ok ? (uint32_t)row * 2u : OOB, 0, 0));
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++)
            raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + (uint32_t)k0, 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++) {
            const int item = tid + NTHREADS * i;
            if (!(ALL_ACTIVE || item < NITEM)) continue;
            const int row = item >> 2, c16 = item & 3;
            const float s = sc[i];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    // dword (2h + w/2) of raw holds codes 4*(2h + w/2) .. +3; output dword w of
                    // this chunk holds codes 8h + 2w, 8h + 2w + 1
                    const uint32_t src = raw[i][2 * h + (w >> 1)];
                    const int sh = (w & 1) * 16;
                    const float f0 = (float)(int8_t)(src >> sh) * s;
                    const float f1 = (float)(int8_t)(src >> (sh + 8)) * s;
                    o[w] = pack_bf16(f0, f1);
                }
                *reinterpret_cast<u32x4*>(tile + lds_off(row, 2 * c16 + h)) = o;
            }
        }
    }
};

// 4-bit codes, k contiguous, one fp16 scale per row and 64-k block.  Item = 32 codes.
template <int R>
struct Stage<OP_Q4_KC, R> {
    static constexpr int NITEM = R * 2;
    static constexpr int PER_THREAD = (NITEM + NTHREADS - 1) / NTHREADS;
    static constexpr bool ALL_ACTIVE = (NITEM % NTHREADS) == 0;
    u32x4 raw[PER_THREAD];
    float sc[PER_THREAD];
    uint32_t voff[PER_THREAD], soff[PER_THREAD];
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)(op.ld >> 1));
        rsc = make_rsrc(op.scales, (uint32_t)dim * (uint32_t)op.scale_ld * 2u);
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++) {
            const int item = tid + NTHREADS * i;
            const int row = row0 + (item >> 1);
            const bool ok = ALL_ACTIVE || item < NITEM;
            voff[i] = ok ? (uint32_t)row * (uint32_t)(op.ld >> 1) + (uint32_t)(item & 1) * 16u : OOB;
            soff[i] = ok ? (uint32_t)row * (uint32_t)op.scale_ld * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++) {
            raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + (uint32_t)(k0 >> 1), 0, 0);
            sc[i] = half_bits_to_float(__builtin_amdgcn_raw_buffer_load_b16(rsc, soff[i] + (uint32_t)(k0 >> 6) * 2u, 0, 0));
        }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++) {
            const int item = tid + NTHREADS * i;
            if (!(ALL_ACTIVE || item < NITEM)) continue;
            const int row = item >> 1, half = item & 1;
            const float s = sc[i];
#pragma unroll
            for (int w = 0; w < 4; w++) {          // dword w = codes 8w .. 8w+7 = one 16-byte chunk
                const uint32_t src = raw[i][w];
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const float f0 = (float)nib(src, 8 * e) * s;
                    const float f1 = (float)nib(src, 8 * e + 4) * s;
                    o[e] = pack_bf16(f0, f1);
                }
                *reinterpret_cast<u32x4*>(tile + lds_off(row, 4 * half + w)) = o;
            }
        }
    }
};

// int8 codes stored [k][row] (the frozen weight seen from the backward pass), fp16 scale[k].
template <int R>
struct Stage<OP_Q8_XC, R> {
    using G = XcGeom<R>;
    u32x2 raw[G::PER_THREAD][8];
    u32x4 scr[G::PER_THREAD];                 // 8 fp16 scales of the block's 8 k rows
    uint32_t voff[G::PER_THREAD], soff[G::PER_THREAD];
    uint32_t ldb;
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)op.ld);
        rsc = make_rsrc(op.scales, (uint32_t)kdim * 2u);
        ldb = (uint32_t)op.ld;
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            const int cc = blk % (R / 8), kg = blk / (R / 8);
            const int row = row0 + cc * 8;
            const bool ok = (G::ALL_ACTIVE || blk < G::NBLK) && row < dim;
            voff[b] = ok ? (uint32_t)(kg * 8) * ldb + (uint32_t)row : OOB;
            soff[b] = ok ? (uint32_t)(kg * 8) * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
#pragma unroll
            for (int j = 0; j < 8; j++)
                raw[b][j] = __builtin_amdgcn_raw_buffer_load_b64(rs, voff[b] + (uint32_t)k0 * ldb + (uint32_t)j * ldb, 0, 0);
            scr[b] = __builtin_amdgcn_raw_buffer_load_b128(rsc, soff[b] + (uint32_t)k0 * 2u, 0, 0);
        }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            if (!(G::ALL_ACTIVE || blk < G::NBLK)) continue;
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const float s = half_bits_to_float((scr[b][j >> 1] >> ((j & 1) * 16)) & 0xFFFFu);
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    const uint32_t src = raw[b][j][w >> 1];
                    const int sh = (w & 1) * 16;
                    v[j][w] = pack_bf16((float)(int8_t)(src >> sh) * s, (float)(int8_t)(src >> (sh + 8)) * s);
                }
            }
            commit_transposed<R>(tile, v, blk % (R / 8), blk / (R / 8));
        }
    }
};

// 4-bit codes stored [k][row/2], fp16 scale[k][row/64].
template <int R>
struct Stage<OP_Q4_XC, R> {
    using G = XcGeom<R>;
    uint32_t raw[G::PER_THREAD][8];
    uint32_t scr[G::PER_THREAD][8];
    uint32_t voff[G::PER_THREAD], soff[G::PER_THREAD];
    uint32_t ldb, sldb;
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)(op.ld >> 1));
        rsc = make_rsrc(op.scales, (uint32_t)kdim * (uint32_t)op.scale_ld * 2u);
        ldb = (uint32_t)(op.ld >> 1);
        sldb = (uint32_t)op.scale_ld * 2u;
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            const int cc = blk % (R / 8), kg = blk / (R / 8);
            const int row = row0 + cc * 8;
            const bool ok = (G::ALL_ACTIVE || blk < G::NBLK) && row < dim;
            voff[b] = ok ? (uint32_t)(kg * 8) * ldb + (uint32_t)(row >> 1) : OOB;
            soff[b] = ok ? (uint32_t)(kg * 8) * sldb + (uint32_t)(row >> 6) * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend)
    {
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++)
#pragma unroll
            for (int j = 0; j < 8; j++) {
                raw[b][j] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff[b] + (uint32_t)(k0 + j) * ldb, 0, 0);
                scr[b][j] = __builtin_amdgcn_raw_buffer_load_b16(rsc, soff[b] + (uint32_t)(k0 + j) * sldb, 0, 0);
            }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, int tid)
    {
#pragma unroll
        for (int b = 0; b < G::PER_THREAD; b++) {
            const int blk = tid + NTHREADS * b;
            if (!(G::ALL_ACTIVE || blk < G::NBLK)) continue;
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const float s = half_bits_to_float(scr[b][j]);
                const uint32_t src = raw[b][j];
#pragma unroll
                for (int w = 0; w < 4; w++)
                    v[j][w] = pack_bf16((float)nib(src, 8 * w) * s,
                                        (float)nib(src, 8 * w + 4) * s);
            }
            commit_transposed<R>(tile, v, blk % (R / 8), blk / (R / 8));
        }
    }
};

// ---------------------------------------------------------------------------------
// One 64-deep K step on the matrix cores.  tileA: [BM][64], tileB: [BN][64].
// ---------------------------------------------------------------------------------
template <int TM, int TN>
__device__ __forceinline__ void mma_step(const unsigned char* tileA, const unsigned char* tileB,
                                         f32x16 (&acc)[TN][TM], int wave_m0, int wave_n0, int lane, int kslices)
{
    const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
        if (kk < kslices) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; i++)
                fa[i] = *reinterpret_cast<const bf16x8*>(tileA + lds_off(wave_m0 + i * 32 + l32, kk * 2 + hi));
#pragma unroll
            for (int j = 0; j < TN; j++)
                fb[j] = *reinterpret_cast<const bf16x8*>(tileB + lds_off(wave_n0 + j * 32 + l32, kk * 2 + hi));
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int i = 0; i < TM; i++)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[j][i], 0, 0, 0);
        }
    }
}

// Map the linear workgroup id to a tile so that (1) the eight XCDs, which receive
// consecutive workgroup ids round-robin and each own an L2, work on contiguous
// ranges of tiles and (2) within a range, tiles walk down GROUP_M row-tiles before
// moving to the next column-tile, so concurrently resident tiles share operands.
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    constexpr int NXCD = 8, GROUP_M = 8;
    const int total = tiles_m * tiles_n;
    const int per = (total + NXCD - 1) / NXCD;
    const int tall = (total % NXCD) ? (total % NXCD) : NXCD;
    const int xcd = pid % NXCD, local = pid / NXCD;
    int id = (xcd < tall) ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
    const int in_group = GROUP_M * tiles_n;
    const int group = id / in_group;
    const int first_m = group * GROUP_M;
    const int gsz = (tiles_m - first_m < GROUP_M) ? (tiles_m - first_m) : GROUP_M;
    const int rem = id % in_group;
    tm = first_m + rem % gsz;
    tn = rem / gsz;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int A_MODE, int B_MODE, int B2_MODE, int OUT_MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_bf16_kernel(GemmArgs p)
{
    static_assert(WAVES_M * WAVES_N == 4, "four waves");
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    constexpr int TILE_A_BYTES = BM * 128, TILE_B_BYTES = BN * 128;
    constexpr int BUF_BYTES = TILE_A_BYTES + TILE_B_BYTES;

    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m0 = (wave / WAVES_N) * WTM, wave_n0 = (wave % WAVES_N) * WTN;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    int tm, tn;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][i][v] = 0.f;

    // ---- optional leading low-rank sum (short: K2 is a rank); only split 0 adds it
    if constexpr (B2_MODE != OP_NONE) {
        if (blockIdx.z == 0) {
            Stage<OP_KC, BM> sa2;
            Stage<B2_MODE, BN> sb2;
            sa2.init(p.a2, m0, p.M, p.K2, tid);
            sb2.init(p.b2, n0, p.N, p.K2, tid);
            for (int k0 = 0; k0 < p.K2; k0 += BK) {
                sa2.issue(k0, p.K2);
                sb2.issue(k0, p.K2);
                sa2.commit(lds, tid);
                sb2.commit(lds + TILE_A_BYTES, tid);
                __syncthreads();
                const int left = (p.K2 - k0 + 15) >> 4;
                mma_step<TM, TN>(lds, lds + TILE_A_BYTES, acc, wave_m0, wave_n0, lane, left < 4 ? left : 4);
                __syncthreads();
            }
            const float ms = p.mid_scale;
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int i = 0; i < TM; i++)
#pragma unroll
                    for (int v = 0; v < 16; v++) acc[j][i][v] *= ms;
        }
    }

    // ---- main sum over this workgroup's k range
    const int kbeg = blockIdx.z * p.k_chunk;
    const int kend = (kbeg + p.k_chunk < p.K) ? kbeg + p.k_chunk : p.K;
    if (kbeg < kend) {
        Stage<A_MODE, BM> sa;
        Stage<B_MODE, BN> sb;
        sa.init(p.a, m0, p.M, p.K, tid);
        sb.init(p.b, n0, p.N, p.K, tid);
        sa.issue(kbeg, kend);
        sb.issue(kbeg, kend);
        sa.commit(lds, tid);
        sb.commit(lds + TILE_A_BYTES, tid);
        __syncthreads();
        int buf = 0;
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            const bool more = k0 + BK < kend;
            if (more) {
                sa.issue(k0 + BK, kend);
                sb.issue(k0 + BK, kend);
            }
            const unsigned char* cur = lds + buf * BUF_BYTES;
            mma_step<TM, TN>(cur, cur + TILE_A_BYTES, acc, wave_m0, wave_n0, lane, 4);
            if (more) {
                unsigned char* nxt = lds + (buf ^ 1) * BUF_BYTES;
                sa.commit(nxt, tid);
                sb.commit(nxt + TILE_A_BYTES, tid);
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32x32 block
    const float alpha = p.alpha;
    const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; j++) {
#pragma unroll
        for (int i = 0; i < TM; i++) {
            const int m = m0 + wave_m0 + i * 32 + l32;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int n = n0 + wave_n0 + j * 32 + g * 8 + hi * 4;
                if (m < p.M && n < p.N) {
                    const float c0 = acc[j][i][4 * g + 0] * alpha, c1 = acc[j][i][4 * g + 1] * alpha;
                    const float c2 = acc[j][i][4 * g + 2] * alpha, c3 = acc[j][i][4 * g + 3] * alpha;
                    const size_t idx = (size_t)m * (size_t)p.ldc + (size_t)n;
                    if constexpr (OUT_MODE == OUT_BF16) {
                        u32x2 o;
                        o.x = pack_bf16(c0, c1);
                        o.y = pack_bf16(c2, c3);
                        *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(p.c) + idx) = o;
                    } else if constexpr (OUT_MODE == OUT_F32) {
                        f32x4 o;
                        o.x = c0; o.y = c1; o.z = c2; o.w = c3;
                        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.c) + idx) = o;
                    } else {
                        float* dst = reinterpret_cast<float*>(p.c) + idx;
                        unsafeAtomicAdd(dst + 0, c0);
                        unsafeAtomicAdd(dst + 1, c1);
                        unsafeAtomicAdd(dst + 2, c2);
                        unsafeAtomicAdd(dst + 3, c3);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Host-side dispatch
// ---------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int AM, int BMODE, int B2, int OUT>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s)
{
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    dim3 grid((unsigned)tiles, 1, (unsigned)(a.splits > 1 ? a.splits : 1));
    char name[64];
    snprintf(name, sizeof(name), "gemm_bf16<%dx%d,a%d,b%d,l%d,o%d>", BM, BN, AM, BMODE, B2, OUT);
    const int slot = prof_begin(name, 2.0 * a.M * a.N * ((double)a.K + a.K2), 0.0, s);
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, AM, BMODE, B2, OUT>), grid, dim3(NTHREADS), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

template <int AM, int BMODE, int B2, int OUT>
static hipError_t launch_tile(int tile, const GemmArgs& a, hipStream_t s)
{
    switch (tile) {
        case TILE_256x256: return launch_one<256, 256, 2, 2, AM, BMODE, B2, OUT>(a, s);
        case TILE_128x256: return launch_one<128, 256, 2, 2, AM, BMODE, B2, OUT>(a, s);
        case TILE_256x128: return launch_one<256, 128, 2, 2, AM, BMODE, B2, OUT>(a, s);
        case TILE_128x128: return launch_one<128, 128, 2, 2, AM, BMODE, B2, OUT>(a, s);
        default: return hipErrorInvalidValue;
    }
}

template <int AM, int BMODE, int OUT>
static hipError_t launch_skinny(int tile, const GemmArgs& a, hipStream_t s)
{
    switch (tile) {
        case TILE_256x32: return launch_one<256, 32, 4, 1, AM, BMODE, OP_NONE, OUT>(a, s);
        case TILE_32x256: return launch_one<32, 256, 1, 4, AM, BMODE, OP_NONE, OUT>(a, s);
        default: return hipErrorInvalidValue;
    }
}

void gemm_tile_extent(int tile, int* bm, int* bn)
{
    static const int ext[TILE_COUNT][2] = {{256, 256}, {128, 256}, {256, 128}, {128, 128}, {256, 32}, {32, 256}};
    *bm = ext[tile][0];
    *bn = ext[tile][1];
}

hipError_t launch_gemm_bf16(int a_mode, int b_mode, int b2_mode, int out_mode, int tile,
                            const GemmArgs& args, hipStream_t stream)
{
    if (args.M <= 0 || args.N <= 0) return hipSuccess;
    if (args.splits > 1 && out_mode != OUT_F32_ATOMIC) return hipErrorInvalidValue;
    const bool skinny = (tile == TILE_256x32 || tile == TILE_32x256);
#define FHPC_CASE(AM, BMODE, B2, OUT)                                                         \
    if (a_mode == AM && b_mode == BMODE && b2_mode == B2 && out_mode == OUT && !skinny)       \
        return launch_tile<AM, BMODE, B2, OUT>(tile, args, stream);
#define FHPC_SKINNY(AM, BMODE, OUT)                                                           \
    if (a_mode == AM && b_mode == BMODE && b2_mode == OP_NONE && out_mode == OUT && skinny)   \
        return launch_skinny<AM, BMODE, OUT>(tile, args, stream);

    // factorised layer, rank in the hundreds
    FHPC_CASE(OP_KC, OP_XC, OP_NONE, OUT_BF16)          // H = X A ; Y = H B
    FHPC_CASE(OP_KC, OP_KC, OP_NONE, OUT_BF16)          // dH = dY B^T ; dX = dH A^T
    FHPC_CASE(OP_XC, OP_XC, OP_NONE, OUT_F32_ATOMIC)    // dB = H^T dY ; dA = X^T dH (split over tokens)
    FHPC_CASE(OP_XC, OP_XC, OP_NONE, OUT_F32)
    // finetuning layer: frozen quantised base + rank-r branch in the same accumulators
    FHPC_CASE(OP_KC, OP_Q8_KC, OP_XC, OUT_BF16)         // Y  = X deq(W) + s H B
    FHPC_CASE(OP_KC, OP_Q4_KC, OP_XC, OUT_BF16)
    FHPC_CASE(OP_KC, OP_Q8_XC, OP_KC, OUT_BF16)         // dX = dY deq(W)^T + s dH A^T
    FHPC_CASE(OP_KC, OP_Q4_XC, OP_KC, OUT_BF16)
    // rank-r (skinny) products of the finetuning layer
    FHPC_SKINNY(OP_KC, OP_XC, OUT_F32_ATOMIC)           // H  = X A      (split over K)
    FHPC_SKINNY(OP_KC, OP_KC, OUT_F32_ATOMIC)           // dH = dY B^T   (split over N)
    FHPC_SKINNY(OP_XC, OP_XC, OUT_F32_ATOMIC)           // dA, dB        (split over tokens)
#undef FHPC_CASE
#undef FHPC_SKINNY
    return hipErrorInvalidValue;
}

}  // namespace fhpc
