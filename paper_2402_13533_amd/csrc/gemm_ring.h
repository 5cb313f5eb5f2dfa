// Building blocks shared by the bf16 GEMM kernels that stream K tiles through a ring of LDS
// stages filled by global -> LDS requests (gfx950): LDS tile layouts and their MFMA fragment
// reads, the request feeders, the fence-free workgroup barrier and the workgroup -> tile map.
#pragma once
#include "gemm_bf16.h"

namespace fhpc {
namespace ring {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr uint32_t OOB = 0x80000000u;   // byte offset beyond any 2 GiB operand

// Raw buffer descriptor (base, stride 0, byte extent, 32-bit raw-buffer format word): offsets
// at or beyond the extent read as zero, which is how ragged edges and the tail of the k range
// are handled.
__device__ __forceinline__ u32x4 make_rsrc(const void* p, uint32_t bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    // the descriptor must sit in scalar registers; the values are wave-uniform by construction
    u32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
    r.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    r.z = __builtin_amdgcn_readfirstlane(bytes);
    r.w = 0x00020000u;
    return r;
}

// One global -> LDS request: lane l's 16 bytes at byte offset voff of the buffer land at
// lds_base + 16 l.  Written as an asm statement on purpose: the compiler's wait-count pass
// does not see it, so it inserts no vmcnt(0) ahead of later LDS reads (it does that before
// every transposing LDS read when it knows of a pending global -> LDS write, which would
// serialise the prefetch ring).  All waits for these requests are written by hand below.
__device__ __forceinline__ void dma_16B(const u32x4& rs, uint32_t lds_base, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rs)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p)
{
    return (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void*)p);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f;
    f.x = lo;
    f.y = hi;
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// Barrier without the fence that __syncthreads carries (the fence would wait for every
// outstanding global -> LDS request, i.e. drain the prefetch ring).  The waits that the
// data flow needs are written out where they belong; the empty asm statements keep the
// compiler from moving LDS accesses across the barrier.
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
#define FHPC_WAIT_LGKM0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")
#define FHPC_WAIT_VM(N) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory")

// ---------------------------------------------------------------------------------
// LDS tile layouts (BK = K depth of a stage) and their fragment reads
// ---------------------------------------------------------------------------------
struct FragAddr { uint32_t o[4]; };

// k contiguous: [rows][BK], 16-byte chunks of a row XOR-swizzled so that 16 consecutive
// rows reading the same logical chunk hit 16 different 16-byte bank groups.
template <int BK>
struct KTile {
    static constexpr int ROWB = BK * 2;
    static constexpr int CPR = BK / 8;
    static constexpr int SH = (BK == 64) ? 1 : 2;           // rows per 256 bytes: 2 or 4
    static __device__ __forceinline__ int swz(int row) { return (row >> SH) & (CPR - 1); }
    // o[s] for k slice s of the stage (s < BK/16): lane l holds row + l%32, chunk 2s + l/32
    static __device__ __forceinline__ FragAddr make(int wave_r0, int lane)
    {
        const int row = wave_r0 + (lane & 31);
        FragAddr a;
#pragma unroll
        for (int s = 0; s < 4; s++)
            a.o[s] = (uint32_t)row * ROWB + (uint32_t)((((2 * s + (lane >> 5)) ^ swz(row)) & (CPR - 1)) << 4);
        return a;
    }
    // fragment i (rows + 32 i; a multiple of 32 rows never changes the swizzle), k slice s
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* tile, const FragAddr& a, int i, int s)
    {
        return *reinterpret_cast<const bf16x8*>(tile + a.o[s] + i * (32 * ROWB));
    }
};

// output index contiguous: [BK k][R rows], read with ds_read_b64_tr_b16 (see gemm_bf16.hip
// for the lane semantics); chunks XOR-swizzled with (k & 3) << 2.
template <int R, int BK>
struct XTile {
    static constexpr int ROWB = R * 2;
    static constexpr int CPR = R / 8;
    static __device__ __forceinline__ int swz(int k) { return ((k & 3) << 2) & (CPR - 1); }
    static __device__ __forceinline__ FragAddr make(int wave_r0, int lane)
    {
        const int li = lane & 15, blk = lane >> 4;
        const int k = (blk >> 1) * 8 + (li >> 2);
        FragAddr a;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int row = wave_r0 + 32 * i + (blk & 1) * 16 + 4 * (li & 3);
            a.o[i] = (uint32_t)k * ROWB + (uint32_t)((((row >> 3) ^ swz(k)) & (CPR - 1)) << 4) + (uint32_t)(row & 4) * 2u;
        }
        return a;
    }
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* tile, const FragAddr& a, int i, int s)
    {
        union { s16x4 h[2]; bf16x8 v; } u;
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const unsigned char* p = tile + a.o[i] + (s * 16 + 4 * j) * ROWB;
            u.h[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(const_cast<unsigned char*>(p)));
        }
        return u.v;
    }
};

// ---------------------------------------------------------------------------------
// Global -> LDS requests.  One wave instruction fills 1 KiB of LDS (lane l writes bytes
// 16 l .. 16 l + 15 after the instruction's LDS base), so the swizzle is applied on the
// global side: each lane fetches the chunk that belongs at its LDS position.  Requests
// are bounds-checked buffer loads: anything outside the operand or past the end of the
// k range arrives as zeros.
// ---------------------------------------------------------------------------------
template <int MODE, int R, int BK, int NW = 8>
struct Feeder;

template <int R, int BK, int NW>
struct Feeder<OP_KC, R, BK, NW> {
    using Tile = KTile<BK>;
    static constexpr int TILE_BYTES = R * BK * 2;
    static constexpr int PER = TILE_BYTES / 1024 / NW;       // requests per wave per stage
    static constexpr int RPB = 1024 / Tile::ROWB;            // rows per request
    static_assert(PER >= 1, "tile too small for the wave count");
    uint32_t voff[PER];
    int logical[PER];                                        // the logical chunk this lane fetches in request j
    u32x4 rs;

    // descriptor of the whole operand (once per kernel), then the lane offsets of one output tile
    __device__ __forceinline__ void describe(const GemmOperand& op, int dim, int kdim)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)op.ld * 2u);
    }
    __device__ __forceinline__ void set_tile(const GemmOperand& op, int row0, int dim, int wave, int lane)
    {
        const int r_in_blk = lane / Tile::CPR, phys = lane % Tile::CPR;
#pragma unroll
        for (int j = 0; j < PER; j++) {
            const int row = (wave * PER + j) * RPB + r_in_blk;
            logical[j] = (phys ^ Tile::swz(row)) & (Tile::CPR - 1);
            voff[j] = ((uint32_t)(row0 + row) * (uint32_t)op.ld + (uint32_t)logical[j] * 8u) * 2u;
        }
    }
    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int wave, int lane)
    {
        describe(op, dim, kdim);
        set_tile(op, row0, dim, wave, lane);
    }
    // request j of the tile that starts at row `row0`, its lane offset formed on the spot (for the few
    // requests a kernel makes on behalf of another output tile than the one set_tile was called for)
    __device__ __forceinline__ void issue_one_for(const GemmOperand& op, int row0, int dim, unsigned char* tile, int k0,
                                                  int kend, int wave, int lane, int j)
    {
        const int r_in_blk = lane / Tile::CPR, phys = lane % Tile::CPR;
        const int row = (wave * PER + j) * RPB + r_in_blk;
        const int lg = (phys ^ Tile::swz(row)) & (Tile::CPR - 1);
        const uint32_t vo = ((uint32_t)(row0 + row) * (uint32_t)op.ld + (uint32_t)lg * 8u) * 2u;
        const uint32_t kofs = (k0 + lg * 8 < kend) ? (uint32_t)k0 * 2u : OOB;
        dma_16B(rs, lds_addr(tile) + (uint32_t)((wave * PER + j) * 1024), vo + kofs);
    }
    __device__ __forceinline__ void issue_one(unsigned char* tile, int k0, int kend, int wave, int j)
    {
        const uint32_t kofs = (k0 + logical[j] * 8 < kend) ? (uint32_t)k0 * 2u : OOB;
        dma_16B(rs, lds_addr(tile) + (uint32_t)((wave * PER + j) * 1024), voff[j] + kofs);
    }
    __device__ __forceinline__ void issue(unsigned char* tile, int k0, int kend, int wave)
    {
#pragma unroll
        for (int j = 0; j < PER; j++) issue_one(tile, k0, kend, wave, j);
    }
};

template <int R, int BK, int NW>
struct Feeder<OP_XC, R, BK, NW> {
    using Tile = XTile<R, BK>;
    static constexpr int TILE_BYTES = R * BK * 2;
    static constexpr int PER = TILE_BYTES / 1024 / NW;
    static constexpr int KPB = 1024 / Tile::ROWB;            // k rows per request
    static_assert(PER >= 1 && KPB >= 1, "tile shape");
    uint32_t voff[PER];
    uint32_t ldb;
    u32x4 rs;

    __device__ __forceinline__ void describe(const GemmOperand& op, int dim, int kdim)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)op.ld * 2u);
        ldb = (uint32_t)op.ld * 2u;
    }
    __device__ __forceinline__ void set_tile(const GemmOperand& op, int row0, int dim, int wave, int lane)
    {
        const int k_in_blk = lane / Tile::CPR, phys = lane % Tile::CPR;
#pragma unroll
        for (int j = 0; j < PER; j++) {
            const int k = (wave * PER + j) * KPB + k_in_blk;
            const int logical = (phys ^ Tile::swz(k)) & (Tile::CPR - 1);
            const int row = row0 + logical * 8;
            voff[j] = (row < dim) ? ((uint32_t)k * (uint32_t)op.ld + (uint32_t)row) * 2u : OOB;
        }
    }
    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int wave, int lane)
    {
        describe(op, dim, kdim);
        set_tile(op, row0, dim, wave, lane);
    }
    __device__ __forceinline__ void issue_one_for(const GemmOperand& op, int row0, int dim, unsigned char* tile, int k0,
                                                  int kend, int wave, int lane, int j)
    {
        const int k_in_blk = lane / Tile::CPR, phys = lane % Tile::CPR;
        const int k = (wave * PER + j) * KPB + k_in_blk;
        const int lg = (phys ^ Tile::swz(k)) & (Tile::CPR - 1);
        const int row = row0 + lg * 8;
        const uint32_t vo = (row < dim) ? ((uint32_t)k * (uint32_t)op.ld + (uint32_t)row) * 2u : OOB;
        const uint32_t kofs = (k0 < kend) ? (uint32_t)k0 * ldb : OOB;
        dma_16B(rs, lds_addr(tile) + (uint32_t)((wave * PER + j) * 1024), vo + kofs);
    }
    __device__ __forceinline__ void issue_one(unsigned char* tile, int k0, int kend, int wave, int j)
    {
        const uint32_t kofs = (k0 < kend) ? (uint32_t)k0 * ldb : OOB;
        dma_16B(rs, lds_addr(tile) + (uint32_t)((wave * PER + j) * 1024), voff[j] + kofs);
    }
    __device__ __forceinline__ void issue(unsigned char* tile, int k0, int kend, int wave)
    {
#pragma unroll
        for (int j = 0; j < PER; j++) issue_one(tile, k0, kend, wave, j);
    }
};

// Workgroup -> work item.  pid % 8 is the XCD a workgroup lands on (hardware round-robin), so every XCD gets a
// contiguous range of item numbers: the workgroups resident on an XCD then share operand tiles in its L2.
__device__ __forceinline__ int xcd_contiguous(int pid, int total)
{
    constexpr int NXCD = 8;
    const int per = (total + NXCD - 1) / NXCD;
    const int tall = (total % NXCD) ? (total % NXCD) : NXCD;
    const int xcd = pid % NXCD, local = pid / NXCD;
    return (xcd < tall) ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
}

// Item number within one product -> (slice of the reduction, tile row, tile column).
__device__ __forceinline__ void item_coords(int id, int tiles_m, int tiles_n, int splits, int& tm, int& tn, int& split)
{
    constexpr int GROUP_M = 8;
    const int tiles = tiles_m * tiles_n;
    if (splits > 1) {
        // Split-major, and within a slice the shorter tile dimension runs fastest: the tiles that read the same
        // panel of the larger operand (all row tiles of one column tile when there are more column tiles, and
        // the other way round) then sit in one XCD's contiguous range and the panel is fetched once.
        split = id / tiles;
        const int t = id - split * tiles;
        if (tiles_n > tiles_m) {
            tn = t / tiles_m;
            tm = t - tn * tiles_m;
        } else {
            tm = t / tiles_n;
            tn = t - tm * tiles_n;
        }
        return;
    }
    split = 0;
    const int in_group = GROUP_M * tiles_n;
    const int group = id / in_group;
    const int first_m = group * GROUP_M;
    const int gsz = (tiles_m - first_m < GROUP_M) ? (tiles_m - first_m) : GROUP_M;
    const int rem = id % in_group;
    tm = first_m + rem % gsz;
    tn = rem / gsz;
}

// Same workgroup -> tile mapping as the lockstep kernels (see gemm_bf16.hip).
__device__ __forceinline__ void work_coords(int pid, int tiles_m, int tiles_n, int splits, int& tm, int& tn, int& split)
{
    item_coords(xcd_contiguous(pid, tiles_m * tiles_n * splits), tiles_m, tiles_n, splits, tm, tn, split);
}

}  // namespace ring
}  // namespace fhpc
