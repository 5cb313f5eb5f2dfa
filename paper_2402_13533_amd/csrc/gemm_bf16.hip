// bf16 MFMA GEMM core for gfx950 (CDNA4): v_mfma_f32_32x32x16_bf16, fp32 accumulation,
// 64-deep K steps double-buffered through LDS, global loads prefetched one or two K steps
// ahead in registers, int8/int4 weights dequantised on the way into LDS.
//
// Two LDS tile layouts, chosen by how the operand is stored in memory, so that staging
// is always a plain copy of 16-byte chunks (no transposition in registers):
//   K layout  [rows][64 k]  (k contiguous, 128 B per row, chunks XOR-swizzled with
//             (row ^ row>>3) & 7): fragments are one ds_read_b128 per lane.
//   X layout  [64 k][R rows] (output index contiguous, chunks XOR-swizzled with
//             (k & 3) << 2): fragments are two ds_read_b64_tr_b16 per lane, the CDNA4
//             transposing LDS read, which hands each lane 4 consecutive k of one row.
//
// Accumulator orientation: the B-side tile feeds the MFMA's row operand and the A-side
// tile its column operand, so a lane ends up holding 4 consecutive output columns n of
// one output row m (16-byte fp32 / 8-byte bf16 stores).
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
typedef __attribute__((ext_vector_type(4))) short s16x4;

static constexpr int BK = 64;
static constexpr uint32_t OOB = 0x80000000u;   // byte offset beyond any 2 GiB operand

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
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

// 8 int8 codes (two dwords) -> 8 bf16 (one 16-byte chunk), each multiplied by s.
__device__ __forceinline__ u32x4 dequant8_i8(uint32_t lo, uint32_t hi, float s)
{
    u32x4 o;
    o[0] = pack_bf16((float)(int8_t)(lo) * s, (float)(int8_t)(lo >> 8) * s);
    o[1] = pack_bf16((float)(int8_t)(lo >> 16) * s, (float)(int8_t)(lo >> 24) * s);
    o[2] = pack_bf16((float)(int8_t)(hi) * s, (float)(int8_t)(hi >> 8) * s);
    o[3] = pack_bf16((float)(int8_t)(hi >> 16) * s, (float)(int8_t)(hi >> 24) * s);
    return o;
}

// 8 4-bit codes (one dword, element e in bits 4e..4e+3) -> 8 bf16, each multiplied by s.
__device__ __forceinline__ u32x4 dequant8_i4(uint32_t w, float s)
{
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; e++) o[e] = pack_bf16((float)nib(w, 8 * e) * s, (float)nib(w, 8 * e + 4) * s);
    return o;
}

// ---------------------------------------------------------------------------------
// LDS layouts
// ---------------------------------------------------------------------------------
// Per-lane byte offsets of a wave's fragments inside a tile, computed once: every fragment
// address is one of these plus a compile-time constant (the ds_read immediate offset).
struct FragAddr { uint32_t o[4]; };

struct KLayout {      // [rows][64 k]
    static __device__ __forceinline__ uint32_t off(int row, int chunk)
    {
        return (uint32_t)row * 128u + (uint32_t)(((chunk ^ (row ^ (row >> 3))) & 7) << 4);
    }
    // Fragment i (rows wave_r0 + 32 i .. +31), k slice kk: lane l holds row + l%32,
    // k = 16 kk + 8 (l/32) + 0..7, i.e. chunk 2 kk + l/32.  Its swizzled position is
    // base ^ (kk<<1) ^ ((i&1)<<2) with a lane constant `base`, so four offsets suffice.
    static __device__ __forceinline__ FragAddr make(int wave_r0, int lane)
    {
        const int row = wave_r0 + (lane & 31);
        const int base = (lane >> 5) ^ ((row ^ (row >> 3)) & 7);
        FragAddr a;
#pragma unroll
        for (int c2 = 0; c2 < 4; c2++) a.o[c2] = (uint32_t)row * 128u + (uint32_t)(((base ^ (c2 << 1)) & 7) << 4);
        return a;
    }
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* tile, const FragAddr& a, int i, int kk)
    {
        return *reinterpret_cast<const bf16x8*>(tile + a.o[(kk ^ ((i & 1) << 1)) & 3] + i * (32 * 128));
    }
};

template <int R>
struct XLayout {      // [64 k][R rows]
    static constexpr int CPR = R / 8;                 // 16-byte chunks per k row
    static __device__ __forceinline__ uint32_t off(int k, int chunk)
    {
        return (uint32_t)k * (uint32_t)(R * 2) + (uint32_t)(((chunk ^ ((k & 3) << 2)) & (CPR - 1)) << 4);
    }
    // ds_read_b64_tr_b16: within each block of 16 lanes, lane j supplies the address of 4
    // consecutive elements; the block's 64 elements, taken in lane order, form a 4 x 16 matrix
    // whose column i is returned to lane i.  Lanes 4e .. 4e+3 therefore point at k row e of the
    // patch and lane i receives 4 consecutive k of row (column of the patch) i.
    // One offset per fragment index i; the k slice and the two reads add constants (multiples
    // of 4 k rows, which leave the swizzle unchanged).
    static __device__ __forceinline__ FragAddr make(int wave_r0, int lane)
    {
        const int li = lane & 15, blk = lane >> 4;
        const int k = (blk >> 1) * 8 + (li >> 2);
        FragAddr a;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int row = wave_r0 + 32 * i + (blk & 1) * 16 + 4 * (li & 3);
            a.o[i] = off(k, row >> 3) + (uint32_t)(row & 4) * 2u;
        }
        return a;
    }
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* tile, const FragAddr& a, int i, int kk)
    {
        union { s16x4 h[2]; bf16x8 v; } u;
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const unsigned char* p = tile + a.o[i] + (kk * 16 + 4 * j) * (R * 2);
            u.h[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(const_cast<unsigned char*>(p)));
        }
        return u.v;
    }
};

// ---------------------------------------------------------------------------------
// Staging: global -> registers (issue) -> LDS tile (commit).  R = tile extent along the
// operand's output index (BM or BN), NT = threads in the workgroup.  row0 = first output
// index of the tile, dim = extent of the output index, kdim = reduction length.
// ---------------------------------------------------------------------------------
template <int MODE, int R, int NT>
struct Stage;

// bf16, k contiguous.
template <int R, int NT>
struct Stage<OP_KC, R, NT> {
    using Layout = KLayout;
    static constexpr int NCHUNK = R * 8;
    static constexpr int PER = (NCHUNK + NT - 1) / NT;
    static constexpr bool ALL = (NCHUNK % NT) == 0;
    struct Regs { u32x4 raw[PER]; };
    static_assert((NT / 8) % 32 == 0, "row step must be a multiple of 32");
    uint32_t voff, rstep, cbase;
    int chunk, row_in_tile;
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)op.ld * 2u);
        chunk = tid & 7;
        row_in_tile = tid >> 3;
        cbase = KLayout::off(row_in_tile, chunk);
        const bool ok = ALL || tid < NCHUNK;
        voff = ok ? ((uint32_t)(row0 + row_in_tile) * (uint32_t)op.ld + (uint32_t)chunk * 8u) * 2u : OOB;
        rstep = (uint32_t)(NT / 8) * (uint32_t)op.ld * 2u;
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
        const uint32_t kofs = (k0 + chunk * 8 < kend) ? (uint32_t)k0 * 2u : OOB;
#pragma unroll
        for (int i = 0; i < PER; i++)
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + (uint32_t)i * rstep + kofs, 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++)
            if (ALL || tid + NT * i < NCHUNK)
            {
                // rows advance by a multiple of 32: only bit 2 of the swizzle (from row >> 3) can flip
                const uint32_t flip = (uint32_t)((((NT / 8) * i) >> 3) & 4) << 4;
                *reinterpret_cast<u32x4*>(tile + (cbase ^ flip) + i * ((NT / 8) * 128)) = r.raw[i];
            }
    }
};

// bf16, output index contiguous: ptr[k*ld + row].
template <int R, int NT>
struct Stage<OP_XC, R, NT> {
    using Layout = XLayout<R>;
    static constexpr int CPR = R / 8;
    static constexpr int NCHUNK = 64 * CPR;
    static constexpr int PER = (NCHUNK + NT - 1) / NT;
    static constexpr bool ALL = (NCHUNK % NT) == 0;
    static constexpr int KSTEP = NT / CPR;            // k rows between a thread's successive chunks
    static_assert(ALL || PER == 1, "partial activity only in a single pass");
    static_assert(KSTEP % 4 == 0, "k step must keep the swizzle");
    struct Regs { u32x4 raw[PER]; };
    uint32_t voff, ldb, cbase;
    int chunk, k_in_tile;
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)op.ld * 2u);
        ldb = (uint32_t)op.ld * 2u;
        chunk = tid % CPR;
        k_in_tile = tid / CPR;
        cbase = Layout::off(k_in_tile, chunk);
        const int row = row0 + chunk * 8;
        const bool ok = (ALL || tid < NCHUNK) && row < dim;
        voff = ok ? ((uint32_t)k_in_tile * (uint32_t)op.ld + (uint32_t)row) * 2u : OOB;
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
        const uint32_t kofs = (k0 < kend) ? (uint32_t)k0 * ldb : OOB;
#pragma unroll
        for (int i = 0; i < PER; i++)
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + kofs + (uint32_t)(i * KSTEP) * ldb, 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++)
            if (ALL || tid + NT * i < NCHUNK)
                *reinterpret_cast<u32x4*>(tile + cbase + i * (KSTEP * R * 2)) = r.raw[i];
    }
};

// int8 codes, k contiguous, one fp16 scale per row.  Item = 16 codes (16 bytes) = 2 chunks.
template <int R, int NT>
struct Stage<OP_Q8_KC, R, NT> {
    using Layout = KLayout;
    static constexpr int NITEM = R * 4;
    static constexpr int PER = (NITEM + NT - 1) / NT;
    static constexpr bool ALL = (NITEM % NT) == 0;
    struct Regs { u32x4 raw[PER]; };
    float sc[PER];
    uint32_t voff[PER];
    __amdgpu_buffer_rsrc_t rs;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)op.ld);
        __amdgpu_buffer_rsrc_t rsc = make_rsrc(op.scales, (uint32_t)dim * 2u);
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            const int row = row0 + (item >> 2);
            const bool ok = ALL || item < NITEM;
            voff[i] = ok ? (uint32_t)row * (uint32_t)op.ld + (uint32_t)(item & 3) * 16u : OOB;
            sc[i] = half_bits_to_float(__builtin_amdgcn_raw_buffer_load_b16(rsc, ok ? (uint32_t)row * 2u : OOB, 0, 0));
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
#pragma unroll
        for (int i = 0; i < PER; i++)
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + ((k0 < kend) ? (uint32_t)k0 : OOB), 0, 0);
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            if (!(ALL || item < NITEM)) continue;
            const int row = item >> 2, c16 = item & 3;
#pragma unroll
            for (int h = 0; h < 2; h++)
                *reinterpret_cast<u32x4*>(tile + KLayout::off(row, 2 * c16 + h)) =
                    dequant8_i8(r.raw[i][2 * h], r.raw[i][2 * h + 1], sc[i]);
        }
    }
};

// 4-bit codes, k contiguous, one fp16 scale per row and 64-k block.  Item = 32 codes = 4 chunks.
template <int R, int NT>
struct Stage<OP_Q4_KC, R, NT> {
    using Layout = KLayout;
    static constexpr int NITEM = R * 2;
    static constexpr int PER = (NITEM + NT - 1) / NT;
    static constexpr bool ALL = (NITEM % NT) == 0;
    struct Regs { u32x4 raw[PER]; uint32_t sc[PER]; };
    uint32_t voff[PER], soff[PER];
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)dim * (uint32_t)(op.ld >> 1));
        rsc = make_rsrc(op.scales, (uint32_t)dim * (uint32_t)op.scale_ld * 2u);
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            const int row = row0 + (item >> 1);
            const bool ok = ALL || item < NITEM;
            voff[i] = ok ? (uint32_t)row * (uint32_t)(op.ld >> 1) + (uint32_t)(item & 1) * 16u : OOB;
            soff[i] = ok ? (uint32_t)row * (uint32_t)op.scale_ld * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + ((k0 < kend) ? (uint32_t)(k0 >> 1) : OOB), 0, 0);
            r.sc[i] = __builtin_amdgcn_raw_buffer_load_b16(rsc, soff[i] + ((k0 < kend) ? (uint32_t)(k0 >> 6) * 2u : OOB), 0, 0);
        }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            if (!(ALL || item < NITEM)) continue;
            const int row = item >> 1, half = item & 1;
            const float s = half_bits_to_float(r.sc[i]);
#pragma unroll
            for (int w = 0; w < 4; w++)          // dword w = codes 8w .. 8w+7 = one chunk
                *reinterpret_cast<u32x4*>(tile + KLayout::off(row, 4 * half + w)) = dequant8_i4(r.raw[i][w], s);
        }
    }
};

// int8 codes stored [k][row] (the frozen weight seen from the backward pass), fp16 scale[k].
// Item = 16 codes of one k row = 2 chunks.
template <int R, int NT>
struct Stage<OP_Q8_XC, R, NT> {
    using Layout = XLayout<R>;
    static constexpr int IPR = R / 16;                // items per k row
    static constexpr int NITEM = 64 * IPR;
    static constexpr int PER = (NITEM + NT - 1) / NT;
    static constexpr bool ALL = (NITEM % NT) == 0;
    struct Regs { u32x4 raw[PER]; uint32_t sc[PER]; };
    uint32_t voff[PER], soff[PER];
    uint32_t ldb;
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)op.ld);
        rsc = make_rsrc(op.scales, (uint32_t)kdim * 2u);
        ldb = (uint32_t)op.ld;
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            const int k = item / IPR, row = row0 + (item % IPR) * 16;
            const bool ok = (ALL || item < NITEM) && row < dim;
            voff[i] = ok ? (uint32_t)k * ldb + (uint32_t)row : OOB;
            soff[i] = ok ? (uint32_t)k * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + ((k0 < kend) ? (uint32_t)k0 * ldb : OOB), 0, 0);
            r.sc[i] = __builtin_amdgcn_raw_buffer_load_b16(rsc, soff[i] + ((k0 < kend) ? (uint32_t)k0 * 2u : OOB), 0, 0);
        }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            if (!(ALL || item < NITEM)) continue;
            const int k = item / IPR, c0 = (item % IPR) * 2;
            const float s = half_bits_to_float(r.sc[i]);
#pragma unroll
            for (int h = 0; h < 2; h++)
                *reinterpret_cast<u32x4*>(tile + Layout::off(k, c0 + h)) =
                    dequant8_i8(r.raw[i][2 * h], r.raw[i][2 * h + 1], s);
        }
    }
};

// 4-bit codes stored [k][row/2], fp16 scale[k][row/64].  Item = 32 codes of one k row = 4 chunks.
template <int R, int NT>
struct Stage<OP_Q4_XC, R, NT> {
    using Layout = XLayout<R>;
    static constexpr int IPR = R / 32;
    static constexpr int NITEM = 64 * IPR;
    static constexpr int PER = (NITEM + NT - 1) / NT;
    static constexpr bool ALL = (NITEM % NT) == 0;
    struct Regs { u32x4 raw[PER]; uint32_t sc[PER]; };
    uint32_t voff[PER], soff[PER];
    uint32_t ldb, sldb;
    __amdgpu_buffer_rsrc_t rs, rsc;

    __device__ __forceinline__ void init(const GemmOperand& op, int row0, int dim, int kdim, int tid)
    {
        rs = make_rsrc(op.ptr, (uint32_t)kdim * (uint32_t)(op.ld >> 1));
        rsc = make_rsrc(op.scales, (uint32_t)kdim * (uint32_t)op.scale_ld * 2u);
        ldb = (uint32_t)(op.ld >> 1);
        sldb = (uint32_t)op.scale_ld * 2u;
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            const int k = item / IPR, row = row0 + (item % IPR) * 32;
            const bool ok = (ALL || item < NITEM) && row < dim;
            voff[i] = ok ? (uint32_t)k * ldb + (uint32_t)(row >> 1) : OOB;
            soff[i] = ok ? (uint32_t)k * sldb + (uint32_t)(row >> 6) * 2u : OOB;
        }
    }
    __device__ __forceinline__ void issue(int k0, int kend, Regs& r)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            r.raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + ((k0 < kend) ? (uint32_t)k0 * ldb : OOB), 0, 0);
            r.sc[i] = __builtin_amdgcn_raw_buffer_load_b16(rsc, soff[i] + ((k0 < kend) ? (uint32_t)k0 * sldb : OOB), 0, 0);
        }
    }
    __device__ __forceinline__ void commit(unsigned char* tile, const Regs& r, int tid)
    {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int item = tid + NT * i;
            if (!(ALL || item < NITEM)) continue;
            const int k = item / IPR, c0 = (item % IPR) * 4;
            const float s = half_bits_to_float(r.sc[i]);
#pragma unroll
            for (int w = 0; w < 4; w++)
                *reinterpret_cast<u32x4*>(tile + Layout::off(k, c0 + w)) = dequant8_i4(r.raw[i][w], s);
        }
    }
};

// ---------------------------------------------------------------------------------
// One 64-deep K step on the matrix cores.
// ---------------------------------------------------------------------------------
// Fragments of k slice kk+1 are requested from LDS before the MFMAs of slice kk are issued,
// and scheduling barriers keep the compiler from hoisting every slice's reads to the top
// (which would need more registers than two resident waves per SIMD have).
template <class LA, class LB, int TM, int TN>
__device__ __forceinline__ void mma_step(const unsigned char* tileA, const unsigned char* tileB,
                                         f32x16 (&acc)[TN][TM], const FragAddr& fa_addr, const FragAddr& fb_addr,
                                         int kslices)
{
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; i++) fa[0][i] = LA::frag(tileA, fa_addr, i, 0);
#pragma unroll
    for (int j = 0; j < TN; j++) fb[0][j] = LB::frag(tileB, fb_addr, j, 0);
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
        if (kk < kslices) {
            if (kk + 1 < 4 && kk + 1 < kslices) {
#pragma unroll
                for (int i = 0; i < TM; i++) fa[(kk + 1) & 1][i] = LA::frag(tileA, fa_addr, i, kk + 1);
#pragma unroll
                for (int j = 0; j < TN; j++) fb[(kk + 1) & 1][j] = LB::frag(tileB, fb_addr, j, kk + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int i = 0; i < TM; i++)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[j][i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Map the linear workgroup id to a tile so that (1) the eight XCDs, which receive
// consecutive workgroup ids round-robin and each own an L2, work on contiguous
// ranges of tiles and (2) within a range, tiles walk down GROUP_M row-tiles before
// moving to the next column-tile, so concurrently resident tiles share operands.
//
// With a split reduction the work items are (split, tile) pairs in split-major order, and
// within a split the column-tiles of one row-tile are adjacent: the workgroups that stream
// the same slice of the long (token) dimension then run on the same XCD at the same time,
// so each slice comes from HBM once and is shared through that XCD's L2.
__device__ __forceinline__ void work_coords(int pid, int tiles_m, int tiles_n, int splits, int& tm, int& tn, int& split)
{
    constexpr int NXCD = 8, GROUP_M = 8;
    const int tiles = tiles_m * tiles_n;
    const int total = tiles * splits;
    const int per = (total + NXCD - 1) / NXCD;
    const int tall = (total % NXCD) ? (total % NXCD) : NXCD;
    const int xcd = pid % NXCD, local = pid / NXCD;
    int id = (xcd < tall) ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
    if (splits > 1) {
        split = id / tiles;
        const int t = id - split * tiles;
        tm = t / tiles_n;
        tn = t - tm * tiles_n;
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

template <int BM, int BN, int WAVES_M, int WAVES_N, int A_MODE, int B_MODE, int B2_MODE, int OUT_MODE, int PF, bool PP>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_bf16_kernel(GemmArgs p)
{
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    static_assert(PF == 1 || PF == 2, "prefetch distance");
    constexpr int TILE_A_BYTES = BM * 128, TILE_B_BYTES = BN * 128;
    constexpr int BUF_BYTES = TILE_A_BYTES + TILE_B_BYTES;
    using SA = Stage<A_MODE, BM, NT>;
    using SB = Stage<B_MODE, BN, NT>;

    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m0 = (wave / WAVES_N) * WTM, wave_n0 = (wave % WAVES_N) * WTN;

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

    // ---- optional leading low-rank sum (short: K2 is a rank); only split 0 adds it
    if constexpr (B2_MODE != OP_NONE) {
        if (split == 0) {
            using SA2 = Stage<OP_KC, BM, NT>;
            using SB2 = Stage<B2_MODE, BN, NT>;
            SA2 sa2;
            SB2 sb2;
            typename SA2::Regs ra2;
            typename SB2::Regs rb2;
            sa2.init(p.a2, m0, p.M, p.K2, tid);
            sb2.init(p.b2, n0, p.N, p.K2, tid);
            for (int k0 = 0; k0 < p.K2; k0 += BK) {
                sa2.issue(k0, p.K2, ra2);
                sb2.issue(k0, p.K2, rb2);
                sa2.commit(lds, ra2, tid);
                sb2.commit(lds + TILE_A_BYTES, rb2, tid);
                __syncthreads();
                const int left = (p.K2 - k0 + 15) >> 4;
                mma_step<typename SA2::Layout, typename SB2::Layout, TM, TN>(
                    lds, lds + TILE_A_BYTES, acc, SA2::Layout::make(wave_m0, lane), SB2::Layout::make(wave_n0, lane),
                    left < 4 ? left : 4);
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
    const int kbeg = split * p.k_chunk;
    const int kend = (kbeg + p.k_chunk < p.K) ? kbeg + p.k_chunk : p.K;
    if constexpr (PP) {
        // Ping-pong schedule for eight waves (two per SIMD).  Waves 0-3 and waves 4-7 run the
        // same steps half a step apart: in every phase (the stretch between two barriers) one
        // wave of each SIMD only issues matrix instructions on fragments it already holds in
        // registers, while the other wave of that SIMD does all the memory work of its own
        // step (LDS fragment reads, LDS writes of the next tile, global requests for the tile
        // after that).  The matrix pipe of a SIMD is therefore fed by one wave at a time and
        // never waits on LDS or memory latency, which the sibling wave absorbs.
        static_assert(NT == 512 && PF == 2, "ping-pong needs eight waves and two staging sets");
        if (kbeg < kend) {
            SA sa;
            SB sb;
            typename SA::Regs ra[2];
            typename SB::Regs rb[2];
            sa.init(p.a, m0, p.M, p.K, tid);
            sb.init(p.b, n0, p.N, p.K, tid);
            const int kld = FHPC_DBG_NO_LOADS(p) ? kbeg : kend;      // diagnostics: nothing is in range
            const bool do_mma = !FHPC_DBG_NO_MMA(p);
            const FragAddr fa_addr = SA::Layout::make(wave_m0, lane);
            const FragAddr fb_addr = SB::Layout::make(wave_n0, lane);
            const int group = __builtin_amdgcn_readfirstlane(wave >> 2);
            // tile u is staged in register set u % 2 and multiplied from LDS buffer u % 2
            sa.issue(kbeg, kld, ra[0]);
            sb.issue(kbeg, kld, rb[0]);
            sa.issue(kbeg + BK, kld, ra[1]);
            sb.issue(kbeg + BK, kld, rb[1]);
            sa.commit(lds, ra[0], tid);
            sb.commit(lds + TILE_A_BYTES, rb[0], tid);
            sa.issue(kbeg + 2 * BK, kld, ra[0]);
            sb.issue(kbeg + 2 * BK, kld, rb[0]);
            __syncthreads();
            if (group == 1) __syncthreads();                // the second group starts one phase later

            bf16x8 fa[4][TM], fb[4][TN];
#define FHPC_PP_STEP(S, KPOS)                                                                      \
    {                                                                                              \
        /* memory phase of tile t (buffer S): fragments -> registers, tile t+1 -> LDS, */          \
        /* request tile t+3 into the set that tile t+1 just left                        */          \
        const unsigned char* cur = lds + (S) * BUF_BYTES;                                          \
        _Pragma("unroll") for (int kk = 0; kk < 4; kk++) {                                         \
            _Pragma("unroll") for (int i = 0; i < TM; i++) fa[kk][i] = SA::Layout::frag(cur, fa_addr, i, kk); \
            _Pragma("unroll") for (int j = 0; j < TN; j++)                                         \
                fb[kk][j] = SB::Layout::frag(cur + TILE_A_BYTES, fb_addr, j, kk);                  \
        }                                                                                          \
        unsigned char* nxt = lds + ((S) ^ 1) * BUF_BYTES;                                          \
        sa.commit(nxt, ra[(S) ^ 1], tid);                                                          \
        sb.commit(nxt + TILE_A_BYTES, rb[(S) ^ 1], tid);                                           \
        sa.issue((KPOS) + 3 * BK, kld, ra[(S) ^ 1]);                                               \
        sb.issue((KPOS) + 3 * BK, kld, rb[(S) ^ 1]);                                               \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        __syncthreads();                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        /* compute phase */                                                                        \
        if (do_mma) {                                                                              \
            __builtin_amdgcn_s_setprio(1);                                                         \
            _Pragma("unroll") for (int kk = 0; kk < 4; kk++)                                       \
                _Pragma("unroll") for (int j = 0; j < TN; j++)                                     \
                    _Pragma("unroll") for (int i = 0; i < TM; i++)                                 \
                        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][j], fa[kk][i], acc[j][i], 0, 0, 0); \
            __builtin_amdgcn_s_setprio(0);                                                         \
        }                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        __syncthreads();                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
            for (int k0 = kbeg; k0 < kend; k0 += 2 * BK) {
                FHPC_PP_STEP(0, k0)
                FHPC_PP_STEP(1, k0 + BK)
            }
#undef FHPC_PP_STEP
            if (group == 0) __syncthreads();                // re-align the two groups
        }
    } else if (kbeg < kend) {
        SA sa;
        SB sb;
        typename SA::Regs ra[PF];
        typename SB::Regs rb[PF];
        sa.init(p.a, m0, p.M, p.K, tid);
        sb.init(p.b, n0, p.N, p.K, tid);
        const int kld = FHPC_DBG_NO_LOADS(p) ? kbeg : kend;      // diagnostics: nothing is in range
        const bool do_mma = !FHPC_DBG_NO_MMA(p);
        sa.issue(kbeg, kld, ra[0]);
        sb.issue(kbeg, kld, rb[0]);
        if constexpr (PF == 2) {
            sa.issue(kbeg + BK, kld, ra[1]);
            sb.issue(kbeg + BK, kld, rb[1]);
        }
        sa.commit(lds, ra[0], tid);
        sb.commit(lds + TILE_A_BYTES, rb[0], tid);
        __syncthreads();
        const FragAddr fa_addr = SA::Layout::make(wave_m0, lane);
        const FragAddr fb_addr = SB::Layout::make(wave_n0, lane);

        // Tile t lives in LDS buffer t % 2; with PF == 2 its staging registers are set t % 2.
        // While tile t is multiplied, tile t + PF is requested from memory and tile t + 1,
        // whose loads were issued PF - 1 steps earlier, is written to the other LDS buffer.
        // The body is branch-free: a request past the end of the k range returns zeros (the
        // loads are bounds-checked), so the one or two tiles staged after the last real one
        // are zero tiles; an odd tile count multiplies one of them, adding nothing.
#define FHPC_KSTEP(S, KPOS)                                                                        \
    {                                                                                              \
        constexpr int ISSUE_SET = (PF == 2) ? (S) : 0;                                             \
        constexpr int COMMIT_SET = (PF == 2) ? ((S) ^ 1) : 0;                                      \
        sa.issue((KPOS) + PF * BK, kld, ra[ISSUE_SET]);                                            \
        sb.issue((KPOS) + PF * BK, kld, rb[ISSUE_SET]);                                            \
        const unsigned char* cur = lds + (S) * BUF_BYTES;                                          \
        if (do_mma)                                                                                \
            mma_step<typename SA::Layout, typename SB::Layout, TM, TN>(cur, cur + TILE_A_BYTES,    \
                                                                       acc, fa_addr, fb_addr, 4);  \
        unsigned char* nxt = lds + ((S) ^ 1) * BUF_BYTES;                                          \
        sa.commit(nxt, ra[COMMIT_SET], tid);                                                       \
        sb.commit(nxt + TILE_A_BYTES, rb[COMMIT_SET], tid);                                        \
        __syncthreads();                                                                           \
    }
        for (int k0 = kbeg; k0 < kend; k0 += 2 * BK) {
            FHPC_KSTEP(0, k0)
            FHPC_KSTEP(1, k0 + BK)
        }
#undef FHPC_KSTEP
    }

    // ---- epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32x32 block
    const float alpha = p.alpha;
    const int l32 = lane & 31, hi = lane >> 5;
    if constexpr (OUT_MODE == OUT_BF16 && BM >= 128 && BN >= 128) {
        // bf16 output: the tile goes through LDS (free after the last barrier of the main loop)
        // as [BM][BN] with the 16-byte chunks of a row XOR-swizzled by the row, so that the
        // global stores are whole 16-byte chunks running along rows (full cache lines).
        constexpr int CPR = BN / 8;
        static_assert(BM * BN * 2 <= 2 * BUF_BYTES, "output tile must fit the operand buffers");
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
#pragma unroll
        for (int q = 0; q < PASSES; q++) {
            const int row = r0 + q * (NT / CPR);
            const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * (BN * 2) + (((c ^ row) & (CPR - 1)) << 4));
            const int m = m0 + row;
            if (m < p.M && col < p.N)
                *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.c) + (size_t)m * (size_t)p.ldc + (size_t)col) = v;
        }
    } else {
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
                        } else {
                            // fp32: this split's partial sum goes to its own slab
                            f32x4 o;
                            o.x = c0; o.y = c1; o.z = c2; o.w = c3;
                            float* dst = reinterpret_cast<float*>(p.c) + (size_t)split * (size_t)p.split_stride;
                            *reinterpret_cast<f32x4*>(dst + idx) = o;
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Host-side dispatch
// ---------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int AM, int BMODE, int B2, int OUT, int PF, bool PP>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s)
{
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    dim3 grid((unsigned)(tiles * (a.splits > 1 ? a.splits : 1)));
    int slot = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof(name), "gemm_bf16<%dx%d,w%d,a%d,b%d,l%d,o%d>", BM, BN, WM * WN, AM, BMODE, B2, OUT);
        slot = prof_begin(name, 2.0 * a.M * a.N * ((double)a.K + a.K2), 0.0, s);
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, AM, BMODE, B2, OUT, PF, PP>), grid, dim3(WM * WN * 64), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

// The 256x128 and 128x256 tiles run the eight-wave ping-pong schedule (two staging sets);
// 256x256 keeps all waves in lockstep with one set (its fragments for a whole K step do
// not fit beside the accumulators); 128x128 is the four-wave tile for small outputs.
template <int AM, int BMODE, int B2, int OUT>
static hipError_t launch_tile(int tile, const GemmArgs& a, hipStream_t s)
{
    constexpr int PF = (BMODE == OP_KC || BMODE == OP_XC) ? 2 : 1;
    switch (tile) {
        case TILE_256x256: return launch_one<256, 256, 2, 4, AM, BMODE, B2, OUT, 1, false>(a, s);
        case TILE_128x256: return launch_one<128, 256, 2, 4, AM, BMODE, B2, OUT, 2, true>(a, s);
        case TILE_256x128: return launch_one<256, 128, 4, 2, AM, BMODE, B2, OUT, 2, true>(a, s);
        case TILE_128x128: return launch_one<128, 128, 2, 2, AM, BMODE, B2, OUT, PF, false>(a, s);
        default: return hipErrorInvalidValue;
    }
}

template <int AM, int BMODE, int OUT>
static hipError_t launch_skinny(int tile, const GemmArgs& a, hipStream_t s)
{
    switch (tile) {
        case TILE_256x32: return launch_one<256, 32, 4, 1, AM, BMODE, OP_NONE, OUT, 1, false>(a, s);
        case TILE_32x256: return launch_one<32, 256, 1, 4, AM, BMODE, OP_NONE, OUT, 1, false>(a, s);
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
    if (args.splits > 1 && out_mode != OUT_F32) return hipErrorInvalidValue;
    if ((args.dbg & 8) && gemm_w4_supports(a_mode, b_mode, b2_mode, out_mode, tile))
        return launch_gemm_w4(a_mode, b_mode, out_mode, args, stream);
    if (!(args.dbg & 4) && gemm_pp_supports(a_mode, b_mode, b2_mode, out_mode, tile))
        return launch_gemm_pp(a_mode, b_mode, out_mode, tile, args, stream);
    if (args.groups > 1) return hipErrorInvalidValue;           // grouped products: the request-fed kernels only
    if (args.n_split > 0) return hipErrorInvalidValue;          // a second output: the request-fed kernels only
    if (args.gate != 0) return hipErrorInvalidValue;           // the gate epilogue: the request-fed kernels only
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
    FHPC_CASE(OP_XC, OP_XC, OP_NONE, OUT_F32)           // dB = H^T dY ; dA = X^T dH (split over tokens)
    // finetuning layer: frozen quantised base + rank-r branch in the same accumulators
    FHPC_CASE(OP_KC, OP_Q8_KC, OP_XC, OUT_BF16)         // Y  = X deq(W) + s H B
    FHPC_CASE(OP_KC, OP_Q4_KC, OP_XC, OUT_BF16)
    FHPC_CASE(OP_KC, OP_Q8_XC, OP_KC, OUT_BF16)         // dX = dY deq(W)^T + s dH A^T
    FHPC_CASE(OP_KC, OP_Q4_XC, OP_KC, OUT_BF16)
    // blend layer with a dense bf16 frozen weight W[K][N]
    FHPC_CASE(OP_KC, OP_XC, OP_XC, OUT_BF16)            // Y  = alpha X W + (1 - alpha) H B
    FHPC_CASE(OP_KC, OP_KC, OP_KC, OUT_BF16)            // dX = alpha dY W^T + (1 - alpha) dH A^T
    // the same four (and the dense pair) with the reduction split over workgroups: fp32 slabs
    FHPC_CASE(OP_KC, OP_Q8_KC, OP_XC, OUT_F32)
    FHPC_CASE(OP_KC, OP_Q4_KC, OP_XC, OUT_F32)
    FHPC_CASE(OP_KC, OP_Q8_XC, OP_KC, OUT_F32)
    FHPC_CASE(OP_KC, OP_Q4_XC, OP_KC, OUT_F32)
    FHPC_CASE(OP_KC, OP_XC, OP_XC, OUT_F32)
    FHPC_CASE(OP_KC, OP_KC, OP_KC, OUT_F32)
    // rank-r (skinny) products of the finetuning layer
    FHPC_SKINNY(OP_KC, OP_XC, OUT_F32)                  // H  = X A      (split over K)
    FHPC_SKINNY(OP_KC, OP_KC, OUT_F32)                  // dH = dY B^T   (split over N)
    FHPC_SKINNY(OP_XC, OP_XC, OUT_F32)                  // dA, dB        (split over tokens)
#undef FHPC_CASE
#undef FHPC_SKINNY
    return hipErrorInvalidValue;
}

}  // namespace fhpc
