// Weight-streaming forward of the quantised finetuning layer for a handful of tokens
// (M <= 64, in tiles of 16):  Y = base_scale * X * deq(Wq, scales) + scaling * (X * A) * B.
//
// At this size the layer is bound by reading the packed weight once from HBM, so the kernel
// is built around that stream: every lane loads 16-byte pieces of its own weight row straight
// into registers (no LDS hop for the weight), turns the codes into exact small bf16 integers
// with a few bit operations, and feeds them to v_mfma_f32_16x16x32_bf16 against the token
// fragments, which sit in LDS (they are the only operand that is reused).
//
// Code -> operand without per-element floating point:
//   int4: nibble n (two's complement) -> u = n ^ 8 = q + 8 in [0, 15]; the bf16 pattern
//         0x4300 | u is exactly 128 + u.
//   int8: byte b -> u = b ^ 0x80 = q + 128 in [0, 255]; float(u) is exact in bf16.
// The matrix instruction therefore accumulates sum_k X[m,k] * (q[n,k] + c) with c = 136 or
// 128.  The offset is taken out again on the matrix unit: for int4 a second instruction with a
// constant operand -136 adds sum_k X[m,k] * (-136) into the same accumulator; for int8 a
// second accumulator fed with an all-ones operand gives sum_k X[m,k], subtracted at the end.
// The fp16 scale is applied to the fp32 sums: per 64-wide block for int4 (Sec. 5.2: one scale
// per weight vector, here a block of 64 inputs of one output channel), once at the end for
// int8 (one scale per output channel).  The weight is thus used unrounded.
//
// Work split: a workgroup of four waves owns 64 output channels (16 per wave) and one slice
// of the reduction; slices write fp32 partial sums to slabs.  H = X * A is formed in 128-deep
// chunks by extra workgroups at the head of the same grid (the last of them to arrive adds the
// chunks up and raises a flag).  There is one launch: the slice that is the last to arrive at a
// 64-channel block (a ticket counter per block in the workspace header) adds the slabs and the
// rank-r branch and rounds to bf16.  It looks at H's flag a bounded number of times and
// otherwise forms H itself, in the same order of sums, so that no wave ever waits without an
// end and the result does not depend on which happened.  Every counter and flag is put back
// to zero by the launch itself: nothing has to be cleared between launches.
#include "qskinny.h"
#include "profile.h"

#include <hip/hip_fp16.h>
#include <type_traits>
#include <stdio.h>
#include <stdlib.h>

namespace fhpc {
namespace skinny {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int NT = 256;
#ifdef FHPC_TRACE
__device__ unsigned long long g_qtrace[2048 * 8];
#define QTS(slot) do { if (threadIdx.x == 0 && blockIdx.x < 2048) g_qtrace[blockIdx.x * 8 + (slot)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define QTS(slot) do { } while (0)
#endif
constexpr int ROWS_WG = 64;            // output channels per workgroup
constexpr int TOK = 16;                // token rows of the MFMA tile
// Reduction depth per pipeline step: 512, or 256 (template parameter SD).  The double-buffered token
// tile of a step takes tokens * depth * 4 bytes of LDS; with 64 tokens the shallower step lets two
// workgroups share a compute unit, which hides more of the weight stream's latency than the deeper
// step does.  The shallower step also serves reductions K that are a multiple of 256 but not of 512
// (a step never straddles the end of K, so the loop needs no guard along k).
constexpr int step_depth(int tt, int64_t K) { return (tt == 4 || (K % 512) != 0) ? 256 : 512; }
constexpr int HCHUNK = 128;            // reduction depth per workgroup of the H = X A kernel
constexpr uint32_t OOB = 0x80000000u;

// Up to four weights that share X (the q/k/v or the gate/up projections of a decoder layer) go through
// one launch: their 64-channel row blocks are numbered one after the other (rb0[j] = first block of
// weight j, rb0[count] = all), and a workgroup finds its weight from its block number.
struct SkinnyJobs {
    const void* Wq[QSKINNY_MAX_JOBS];
    const void* scales[QSKINNY_MAX_JOBS];
    const void* A[QSKINNY_MAX_JOBS];
    const void* B[QSKINNY_MAX_JOBS];
    void* Y[QSKINNY_MAX_JOBS];
    void* H_out[QSKINNY_MAX_JOBS];
    const void* X[QSKINNY_MAX_JOBS];        // token rows of the job and how many (at most the launch's M, which stays
    int M[QSKINNY_MAX_JOBS];                // the row count of every job's scratch areas)
    int N[QSKINNY_MAX_JOBS];
    int rb0[QSKINNY_MAX_JOBS + 1];
    float base_scale[QSKINNY_MAX_JOBS];
    float scaling[QSKINNY_MAX_JOBS];
    int count;
};

__device__ __forceinline__ int job_of_block(const SkinnyJobs& jb, int rb)
{
    int j = 0;
#pragma unroll
    for (int i = 1; i < QSKINNY_MAX_JOBS; i++) j += (i < jb.count && rb >= jb.rb0[i]) ? 1 : 0;
    return j;
}
__device__ __forceinline__ int pick_rb0(const SkinnyJobs& jb, int j)
{
    int v = jb.rb0[0];
#pragma unroll
    for (int i = 1; i < QSKINNY_MAX_JOBS; i++) v = (j == i) ? jb.rb0[i] : v;
    return v;
}
// element j of a small array in the kernel arguments, j uniform: a chain of selects, no indexed memory
template <typename T>
__device__ __forceinline__ T pick(const T (&a)[QSKINNY_MAX_JOBS], int j)
{
    T v = a[0];
#pragma unroll
    for (int i = 1; i < QSKINNY_MAX_JOBS; i++) v = (j == i) ? a[i] : v;
    return v;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* p, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Exchange between the two halves of a wave: lanes 0..31 keep w[0], w[1] and get the upper
// partner's (lane + 32) w[0], w[1] in w[2], w[3]; lanes 32..63 keep w[2], w[3] and get the lower
// partner's w[2], w[3] in w[0], w[1].
__device__ __forceinline__ void exchange_halves(uint32_t (&w)[4])
{
    // v_permlane32_swap a, b: lanes 32..63 of a <-> lanes 0..31 of b
    auto s0 = __builtin_amdgcn_permlane32_swap(w[0], w[2], false, false);
    auto s1 = __builtin_amdgcn_permlane32_swap(w[1], w[3], false, false);
    w[0] = s0[0]; w[2] = s0[1];
    w[1] = s1[0]; w[3] = s1[1];
}

// eight int4 codes (one 32-bit word, element 2j in the low nibble of byte j) -> eight bf16
// values 128 + (q + 8).  The even and the odd nibbles are isolated as bytes (u = n ^ 8), and one
// byte permute per result word interleaves two of them with the constant byte 0x43, so the
// operand's k order is 0 2 4 6 1 3 5 7; the token tile is stored in the same order
// (x_even_odd_order).
__device__ __forceinline__ bf16x8 int4_operand(uint32_t w)
{
    const uint32_t lo = (w & 0x0f0f0f0fu) ^ 0x08080808u;            // u of elements 0 2 4 6
    const uint32_t hi = ((w >> 4) & 0x0f0f0f0fu) ^ 0x08080808u;     // u of elements 1 3 5 7
    const uint32_t c43 = 0x43434343u;
    u32x4 r;
    r.x = __builtin_amdgcn_perm(c43, lo, 0x04010400u);
    r.y = __builtin_amdgcn_perm(c43, lo, 0x04030402u);
    r.z = __builtin_amdgcn_perm(c43, hi, 0x04010400u);
    r.w = __builtin_amdgcn_perm(c43, hi, 0x04030402u);
    return as_bf16x8(r);
}

// eight consecutive bf16 (four words) -> the order 0 2 4 6 1 3 5 7
__device__ __forceinline__ u32x4 x_even_odd_order(u32x4 v)
{
    u32x4 r;
    r.x = __builtin_amdgcn_perm(v.y, v.x, 0x05040100u);
    r.y = __builtin_amdgcn_perm(v.w, v.z, 0x05040100u);
    r.z = __builtin_amdgcn_perm(v.y, v.x, 0x07060302u);
    r.w = __builtin_amdgcn_perm(v.w, v.z, 0x07060302u);
    return r;
}

// eight int8 codes (two words) -> eight bf16 values q + 128
__device__ __forceinline__ bf16x8 int8_operand(uint32_t w0, uint32_t w1)
{
    const uint32_t a = w0 ^ 0x80808080u, b = w1 ^ 0x80808080u;
    const float f0 = (float)(a & 0xffu), f1 = (float)((a >> 8) & 0xffu), f2 = (float)((a >> 16) & 0xffu), f3 = (float)(a >> 24);
    const float f4 = (float)(b & 0xffu), f5 = (float)((b >> 8) & 0xffu), f6 = (float)((b >> 16) & 0xffu), f7 = (float)(b >> 24);
    // the values are integers below 256: the upper 16 bits of the fp32 pattern are the exact bf16
    u32x4 r;
    r.x = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
    r.z = __builtin_amdgcn_perm(__float_as_uint(f5), __float_as_uint(f4), 0x07060302u);
    r.w = __builtin_amdgcn_perm(__float_as_uint(f7), __float_as_uint(f6), 0x07060302u);
    return as_bf16x8(r);
}

// LDS tile of the token rows for one step: [tokens][DEPTH k] bf16, 16-byte chunks XOR-swizzled
// by the token so that the 16 lanes of a group (16 tokens, same chunk) hit 16 different banks.
template <int DEPTH>
__device__ __forceinline__ uint32_t x_off(int tok, int chunk)
{
    return (uint32_t)tok * (DEPTH * 2) + (uint32_t)(((chunk ^ tok) & (DEPTH / 8 - 1)) << 4);
}

// Data that one workgroup writes and another reads within the launch (slabs, chunk sums of H, H) moves with
// device-scope accesses: a store goes through to the level all compute units share and a load comes from there,
// instruction by instruction.  (Ordinary accesses would need a device-scope fence on either side, which writes
// back and invalidates a whole L2 on this chip: measured, that made a launch 8 to 50 times slower.)
__device__ __forceinline__ void shared_store(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float shared_load(const float* p)
{
    return __hip_atomic_load(const_cast<float*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// hpart[kc][m][j] = sum over the 128-deep chunk kc of X[m][k] A[k][j]   (fp32, m < M, j < r).
// Run by the extra workgroups at the end of the streaming kernel's grid, so that H = X A costs no
// launch of its own.  The chunk of X ([M][128]) and of A ([128][r]) is copied to LDS with
// coalesced loads; thread (m, j16) then forms the sums for the columns j = j16, j16 + 16, ...
constexpr int H_XLD = HCHUNK + 8;                    // padded token row (bank spread)
constexpr int h_lds_bytes(int toks) { return (toks * H_XLD + HCHUNK * 64) * 2; }
template <int TOKS>
__device__ __forceinline__ void hpart_body(unsigned char* smem, int kc, const uint16_t* __restrict__ X,
                                           const uint16_t* __restrict__ A, float* __restrict__ hpart, int M, int K, int r)
{
    uint16_t* Xs = reinterpret_cast<uint16_t*>(smem);
    uint16_t* As = Xs + TOKS * H_XLD;
    const int k0 = kc * HCHUNK;
    const int kn = (K - k0 < HCHUNK) ? K - k0 : HCHUNK;          // K is a multiple of 8
    for (int c = threadIdx.x; c < M * (HCHUNK / 8); c += NT) {
        const int m = c / (HCHUNK / 8), kk = (c % (HCHUNK / 8)) * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (kk < kn) v = *reinterpret_cast<const u32x4*>(X + (int64_t)m * K + k0 + kk);
        *reinterpret_cast<u32x4*>(Xs + m * H_XLD + kk) = v;
    }
    // A chunk: kn * r contiguous elements starting at A[k0][0]
    const int64_t abase = (int64_t)k0 * r;
    const int an = kn * r;
    if ((r & 7) == 0) {
        for (int c = threadIdx.x * 8; c < an; c += NT * 8)
            *reinterpret_cast<u32x4*>(As + c) = *reinterpret_cast<const u32x4*>(A + abase + c);
    } else {
        for (int c = threadIdx.x; c < an; c += NT) As[c] = A[abase + c];
    }
    __syncthreads();
    const int j16 = threadIdx.x & 15;
    for (int m = threadIdx.x >> 4; m < M; m += 16) {
        for (int j = j16; j < r; j += 16) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll 8
            for (int k = 0; k + 1 < kn; k += 2) {
                s0 = fmaf(__uint_as_float((uint32_t)Xs[m * H_XLD + k] << 16), __uint_as_float((uint32_t)As[k * r + j] << 16), s0);
                s1 = fmaf(__uint_as_float((uint32_t)Xs[m * H_XLD + k + 1] << 16), __uint_as_float((uint32_t)As[(k + 1) * r + j] << 16), s1);
            }
            shared_store(hpart + ((int64_t)kc * M + m) * r + j, s0 + s1);
        }
    }
}

// Arrival at a counter in the workspace header.  Every thread waits until its own shared_stores have been
// acknowledged, the workgroup meets, and one thread draws the ticket (the number of earlier arrivals).  The
// workgroup that draws the last ticket may shared_load what all earlier arrivals stored.
__device__ __forceinline__ uint32_t arrive(uint32_t* counter, uint32_t* s_ticket)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) *s_ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t t = *s_ticket;
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return t;
}

// The 64-channel block rb is complete (all slices' slabs and H are in memory): Y = bf16(base_scale * sum of the slabs
// + scaling * H B) for its channels and every token.  One workgroup; thread (c = tid % 64, tg = tid / 64) takes
// channel c and the tokens tg, tg + 4, ...  H (fp32, [M][r]) is staged in LDS.  The rank-r sums come first, sixteen
// ranks of the thread's column of B in registers at a time, and wait in LDS ([M][64]) for the slab sums: few
// registers, so that this tail does not lower the occupancy the streaming loop was planned for.
__device__ __forceinline__ void finish_block(unsigned char* smem, int rb, const SkinnyJobs& jb, const float* __restrict__ part,
                                             int splits, const float* __restrict__ hsum_all, const uint32_t* hready, int poll_limit,
                                             const uint16_t* __restrict__ X, int K, int M, int Mstride, int r)
{
    float* Hs = reinterpret_cast<float*>(smem);                 // [M][r], at most 64 x 64 floats
    const int job = job_of_block(jb, rb);
    const int N = pick(jb.N, job);
    const uint16_t* const B = static_cast<const uint16_t*>(pick(jb.B, job));
    uint16_t* const Y = static_cast<uint16_t*>(pick(jb.Y, job));
    const float base_scale = pick(jb.base_scale, job), scaling = pick(jb.scaling, job);
    const float* const hsum = hsum_all + (int64_t)job * Mstride * r;
    const int ld_part = jb.rb0[jb.count] * ROWS_WG;
    const int c = threadIdx.x & 63, tg = threadIdx.x >> 6;
    const int ncomb = rb * ROWS_WG + c;
    const int n = (rb - pick_rb0(jb, job)) * ROWS_WG + c;
    const int nc = n < N ? n : N - 1;
    const __amdgpu_buffer_rsrc_t rB = rsrc(B, (int64_t)r * N * 2);
    auto slab_batch = [&](float (&v)[8], int m, int sp0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 8; q++) {
            const int sp = sp0 + q;
            const float x = shared_load(part + ((int64_t)(sp < splits ? sp : sp0) * M + m) * ld_part + ncomb);
            v[q] = (sp < splits) ? x : 0.f;
        }
    };
    auto sum8 = [](const float (&v)[8]) __attribute__((always_inline)) {
        return ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    };
    // the first tokens' slab values and the first sixteen ranks of B's column are requested before anything waits
    float v[4][8];
    // (always a row that exists: with fewer than four tokens some threads have no token of their own, and a row
    // index beyond M would read past the slabs, for one token and a wide weight past the workspace)
    const int tg_row = tg < M ? tg : 0;
#pragma unroll
    for (int u = 0; u < 4; u++) slab_batch(v[u], (tg + 4 * u < M) ? tg + 4 * u : tg_row, 0);
    float b0[16];
#pragma unroll
    for (int j = 0; j < 16; j++) {                               // (a row beyond r reads as zero)
        const uint32_t off = (j < r) ? (uint32_t)(j * N + nc) * 2u : OOB;
        b0[j] = __uint_as_float((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rB, off, 0, 0) << 16);
    }
    // H is formed by the workgroups at the head of the grid, which wait for nobody, so it is normally complete
    // long before a block's last slice arrives; one thread looks at the weight's flag, a bounded number of times.
    __shared__ uint32_t s_ready;
    if (threadIdx.x == 0) {
        uint32_t ok = 0;
        for (int polls = 0; polls <= poll_limit && !ok; polls++) {
            ok = __hip_atomic_load(const_cast<uint32_t*>(hready + job), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!ok) __builtin_amdgcn_s_sleep(8);
        }
        s_ready = ok;
    }
    __syncthreads();
    if (s_ready) {
        for (int i = threadIdx.x; i < M * r; i += NT) Hs[i] = shared_load(hsum + i);
    } else {
        // Not complete within the bound (never seen; it is what lets every wave end whatever the order in which
        // the hardware starts workgroups): this workgroup forms H itself, with the very sums and the very
        // order of the chunk workgroups, so the result is the same bits.
        const uint16_t* const A = static_cast<const uint16_t*>(pick(jb.A, job));
        for (int i = threadIdx.x; i < M * r; i += NT) {
            const int m = i / r, j = i - m * r;
            float t = 0.f;
            for (int k0 = 0; k0 < K; k0 += HCHUNK) {
                const int kn = (K - k0 < HCHUNK) ? K - k0 : HCHUNK;
                float s0 = 0.f, s1 = 0.f;
                for (int k = 0; k + 1 < kn; k += 2) {
                    s0 = fmaf(__uint_as_float((uint32_t)X[(int64_t)m * K + k0 + k] << 16), __uint_as_float((uint32_t)A[(int64_t)(k0 + k) * r + j] << 16), s0);
                    s1 = fmaf(__uint_as_float((uint32_t)X[(int64_t)m * K + k0 + k + 1] << 16), __uint_as_float((uint32_t)A[(int64_t)(k0 + k + 1) * r + j] << 16), s1);
                }
                t += s0 + s1;
            }
            Hs[i] = t;
        }
    }
    __syncthreads();
    // Four of the thread's tokens at a time, so that their slab values are all in flight together (the work is a
    // chain of memory round trips and little else).
    for (int mb = tg; mb < M; mb += 16) {
        if (mb != tg) {
#pragma unroll
            for (int u = 0; u < 4; u++) slab_batch(v[u], (mb + 4 * u < M) ? mb + 4 * u : mb, 0);
        }
        float l[4] = {0.f, 0.f, 0.f, 0.f};
        for (int j0 = 0; j0 < r; j0 += 16) {
            float b[16];
#pragma unroll
            for (int j = 0; j < 16; j++) {
                if (j0 == 0) {
                    b[j] = b0[j];
                } else {
                    const uint32_t off = (j0 + j < r) ? (uint32_t)((j0 + j) * N + nc) * 2u : OOB;
                    b[j] = __uint_as_float((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rB, off, 0, 0) << 16);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int m = (mb + 4 * u < M) ? mb + 4 * u : mb;
#pragma unroll
                for (int j = 0; j < 16; j++) l[u] = fmaf(Hs[m * r + (j0 + j < r ? j0 + j : 0)], b[j], l[u]);
            }
        }
        float base[4];
#pragma unroll
        for (int u = 0; u < 4; u++) base[u] = sum8(v[u]);
        for (int sp0 = 8; sp0 < splits; sp0 += 8) {
#pragma unroll
            for (int u = 0; u < 4; u++) slab_batch(v[u], (mb + 4 * u < M) ? mb + 4 * u : mb, sp0);
#pragma unroll
            for (int u = 0; u < 4; u++) base[u] += sum8(v[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int m = mb + 4 * u;
            if (n < N && m < M) {
                const __bf16 yb = (__bf16)(base_scale * base[u] + scaling * l[u]);
                Y[(int64_t)m * N + n] = __builtin_bit_cast(uint16_t, yb);
            }
        }
    }
    __syncthreads();                                            // Hs is reused if this workgroup finishes another block
}

// Header words: one ticket per 64-channel block; then, per weight, an arrival counter for the chunks of H = X A and
// a flag that H is complete; then the number of finished blocks of the launch.
constexpr int TICKETS = 4080;
constexpr int HCOUNT = TICKETS, HREADY = TICKETS + QSKINNY_MAX_JOBS, DONE = TICKETS + 2 * QSKINNY_MAX_JOBS;
static_assert((DONE + 1) * 4 <= QSKINNY_HEADER_BYTES, "header words");

template <int SCHEME, int TT, int SD>
__global__ __launch_bounds__(NT) void qskinny_fwd_kernel(SkinnyJobs jb, float* __restrict__ part,
                                                         int M, int K, int k_chunk, float* __restrict__ hpart, int r,
                                                         int kchunks, int head_grid, int splits, uint32_t* __restrict__ tickets,
                                                         float* __restrict__ hsum, int poll_limit)
{
    constexpr bool I4 = (SCHEME == 4);
    constexpr int WLOADS = I4 ? SD / 128 : SD / 64;  // 16-byte weight loads per lane per step
    constexpr int TOKS = TOK * TT;                   // token rows this instantiation covers
    constexpr int XS_BYTES = TOKS * SD * 2;
    constexpr int XCH = SD / 8;                      // 16-byte pieces per token row per step
    constexpr int XL = TOKS * XCH / NT;              // ... per thread per step
    // (the H = X A workgroups reuse the token tiles' LDS)
    constexpr int LDS_BYTES = (2 * XS_BYTES > h_lds_bytes(TOKS)) ? 2 * XS_BYTES : h_lds_bytes(TOKS);
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    static_assert(LDS_BYTES >= 64 * 64 * 4, "the finish stages H ([M][r] fp32) in the same LDS");
    unsigned char* const xs[2] = {smem, smem + XS_BYTES};
    __shared__ uint32_t s_ticket;
    const int row_blocks = jb.rb0[jb.count];                   // of all weights together
    // a 64-channel block counts its `splits` slices
    const uint32_t last_ticket = (uint32_t)(splits - 1);
    // One thread, after a block is finished or a weight's flag is set: the last of these events of the launch
    // (row_blocks + count of them) puts the remaining header words back to zero.  By then every block has been
    // finished, so every workgroup has arrived and nobody reads the flags any more.
    auto done = [&]() __attribute__((always_inline)) {
        if (__hip_atomic_fetch_add(tickets + DONE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(row_blocks + jb.count - 1)) {
            __hip_atomic_store(tickets + DONE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int j = 0; j < QSKINNY_MAX_JOBS; j++)
                __hip_atomic_store(tickets + HREADY + j, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    auto finish = [&](int rb) __attribute__((always_inline)) {
        const int fj = job_of_block(jb, rb);
        finish_block(smem, rb, jb, part, splits, hsum, tickets + HREADY, poll_limit, static_cast<const uint16_t*>(pick(jb.X, fj)), K,
                     pick(jb.M, fj), M, r);
        if (threadIdx.x == 0) {
            __hip_atomic_store(tickets + rb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            done();
        }
    };
    QTS(0);
    if ((int)blockIdx.x < head_grid) {
        // the H = X A chunks: kchunks workgroups per weight, at the head of the grid so that they start first
        const int idx = (int)blockIdx.x, hj = idx / kchunks, kc = idx - hj * kchunks;
        float* const hp = hpart + (int64_t)hj * kchunks * M * r;
        const int Mj = pick(jb.M, hj);                              // the job's own token count (scratch strides: M)
        hpart_body<TOKS>(smem, kc, static_cast<const uint16_t*>(pick(jb.X, hj)), static_cast<const uint16_t*>(pick(jb.A, hj)), hp, Mj, K, r);
        QTS(1);
        if (arrive(tickets + HCOUNT + hj, &s_ticket) != (uint32_t)(kchunks - 1)) return;
        QTS(2);
        // the last chunk of this weight: H = the sum of the chunks, in chunk order (the same order every run)
        uint16_t* const H_out = static_cast<uint16_t*>(pick(jb.H_out, hj));
        float* const hs = hsum + (int64_t)hj * M * r;
        for (int i = threadIdx.x; i < Mj * r; i += NT) {
            float t = 0.f;
            for (int c0 = 0; c0 < kchunks; c0 += 48) {         // 48 loads in flight, added in chunk order
                float v[48];
#pragma unroll
                for (int q = 0; q < 48; q++) {
                    const int c = c0 + q;
                    const float x = shared_load(hp + (int64_t)(c < kchunks ? c : c0) * Mj * r + i);
                    v[q] = (c < kchunks) ? x : 0.f;
                }
#pragma unroll
                for (int q = 0; q < 48; q++) t += v[q];
            }
            shared_store(hs + i, t);
            if (H_out) {
                const __bf16 hb = (__bf16)t;
                H_out[i] = __builtin_bit_cast(uint16_t, hb);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) __hip_atomic_store(tickets + HCOUNT + hj, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        QTS(3);
        // H is in memory: the flag the blocks' finishers look at
        if (threadIdx.x == 0) {
            __hip_atomic_store(tickets + HREADY + hj, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            done();
        }
        QTS(4);
        return;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = (int)blockIdx.x - head_grid;
    const int rb = wg % row_blocks, split = wg / row_blocks;
    const int job = job_of_block(jb, rb);
    const int N = pick(jb.N, job);
    const int Mj = pick(jb.M, job);                                // this job's token rows
    const void* const Xj = pick(jb.X, job);
    const void* const Wq = pick(jb.Wq, job);
    const void* const scales = pick(jb.scales, job);
    const int n0 = (rb - pick_rb0(jb, job)) * ROWS_WG + wave * 16;      // channel within its weight
    const int ncomb0 = rb * ROWS_WG + wave * 16;                       // column in the combined slabs
    const int ld_part = row_blocks * ROWS_WG;
    const int kbeg = split * k_chunk;
    const int kend = (kbeg + k_chunk < K) ? kbeg + k_chunk : K;
    const int steps = (kend - kbeg + SD - 1) / SD;
    const int lr = lane & 15, g = lane >> 4;         // operand view: row / token lr, k group g

    const int64_t row_bytes = I4 ? K / 2 : K;
    const __amdgpu_buffer_rsrc_t rw = rsrc(Wq, (int64_t)N * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = rsrc(Xj, (int64_t)Mj * K * 2);
    const __amdgpu_buffer_rsrc_t rsc = rsrc(scales, I4 ? (int64_t)N * (K / 64) * 2 : (int64_t)N * 2);
    const bool row_ok = (n0 + lr) < N;
    const uint32_t wrow = row_ok ? (uint32_t)((int64_t)(n0 + lr) * row_bytes) : OOB;

    // A step never straddles the end of the slice (K and the slice depth are multiples of 512, the
    // step depth divides 512), so only rows and tokens need a bounds guard; it sits in the
    // loop-invariant vector offset (an offset beyond the buffer reads as zero), and the position
    // along k travels in the scalar offset, so the loop spends no vector instructions on addresses.
    // weight pieces of one step for this lane.  int4: load u covers k = 128 u + 32 g .. + 31
    // (16 bytes); int8: load u covers k = 64 u + 16 g .. + 15: byte 64 u + 16 g of the step either way.
    const uint32_t wlane = row_ok ? wrow + 16u * (uint32_t)g : OOB;
    auto load_w = [&](u32x4 (&w)[WLOADS], int k0) __attribute__((always_inline)) {
        const int sk = I4 ? k0 >> 1 : k0;
#pragma unroll
        for (int u = 0; u < WLOADS; u++) w[u] = __builtin_amdgcn_raw_buffer_load_b128(rw, wlane + 64u * u, sk, 0);
    };
    // int4 scales of one step: the SD / 64 consecutive blocks of each of the four output channels
    // this lane owns in the accumulator view (channel n0 + 4 g + v)
    uint32_t srow[4];
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const int n = n0 + 4 * g + v;
        srow[v] = (I4 && n < N) ? (uint32_t)((int64_t)n * (K / 64) * 2) : OOB;
    }
    auto load_s = [&](u32x4 (&s)[4], int k0) __attribute__((always_inline)) {
        const int sk = k0 >> 5;                      // block k0 / 64, two bytes each
#pragma unroll
        for (int v = 0; v < 4; v++) {
            if constexpr (SD == 512) {
                s[v] = __builtin_amdgcn_raw_buffer_load_b128(rsc, srow[v], sk, 0);
            } else {
                const auto h = __builtin_amdgcn_raw_buffer_load_b64(rsc, srow[v], sk, 0);
                s[v].x = h[0]; s[v].y = h[1];
            }
        }
    };
    // token tile of one step: XCH chunks of 16 bytes per token, XL per thread
    uint32_t xlane[XL];
#pragma unroll
    for (int j = 0; j < XL; j++) {
        const int c = tid + NT * j, tok = c / XCH, chunk = c % XCH;
        xlane[j] = (tok < Mj) ? (uint32_t)(((int64_t)tok * K + chunk * 8) * 2) : OOB;
    }
    auto load_x = [&](u32x4 (&x)[XL], int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < XL; j++) x[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, xlane[j], k0 * 2, 0);
    };
    auto store_x = [&](const u32x4 (&x)[XL], unsigned char* dst) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < XL; j++) {
            const int c = tid + NT * j, tok = c / XCH, chunk = c % XCH;
            *reinterpret_cast<u32x4*>(dst + x_off<SD>(tok, chunk)) = I4 ? x_even_odd_order(x[j]) : x[j];
        }
    };

    u32x4 wreg[3][WLOADS];                           // weights of the steps t, t + 1, t + 2
    u32x4 sreg[3][4];
    u32x4 xreg[XL];
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    f32x4 acc[TT];                                   // scaled sums (int4) / raw code sums (int8), per token tile
    f32x4 ones_acc[TT];                              // int8: sum of X over the whole slice
#pragma unroll
    for (int tt = 0; tt < TT; tt++) acc[tt] = ones_acc[tt] = zero4;
    u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bf16x8 ones = as_bf16x8(ones_bits);
    u32x4 moff_bits = {0xc308c308u, 0xc308c308u, 0xc308c308u, 0xc308c308u};     // bf16(-136) x 8
    const bf16x8 minus_offset = as_bf16x8(moff_bits);

    const int gchunk = 4 * (g & 1) + 2 * (g >> 1);  // int4: 16-byte chunk of this lane group's codes within a block
    auto xfrag = [&](const unsigned char* tile, int tt, int chunk) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8*>(tile + x_off<SD>(TOK * tt + lr, chunk));
    };
    // one step of the reduction from registers w (and s) against the token tile
    auto compute = [&](u32x4 (&w)[WLOADS], u32x4 (&s)[4], const unsigned char* tile) __attribute__((always_inline)) {
        if constexpr (I4) {
#pragma unroll
            for (int u = 0; u < WLOADS; u++) {       // 128 k: two scale blocks
                // t[2 b + h] = codes k = 128 u + 64 b + gk + 8 h .. + 7,  gk = 32 (g & 1) + 16 (g >> 1):
                // the four lane groups of one matrix instruction stay inside one scale block
                uint32_t t[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
                exchange_halves(t);
#pragma unroll
                for (int b = 0; b < 2; b++) {
                    // sum over the block of X (q + 136) and of X (-136), in one accumulator
                    f32x4 cw[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; tt++) cw[tt] = zero4;
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        const int c = 2 * b + h;
                        const bf16x8 wf = int4_operand(t[c]);
#pragma unroll
                        for (int tt = 0; tt < TT; tt++) {
                            const bf16x8 xf = xfrag(tile, tt, 16 * u + 8 * b + h + gchunk);
                            cw[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, cw[tt], 0, 0, 0);
                            cw[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(minus_offset, xf, cw[tt], 0, 0, 0);
                        }
                    }
                    // block 2 u + b of this step: fp16 scale of channel n0 + 4 g + v
                    const int blk = 2 * u + b;
#pragma unroll
                    for (int v = 0; v < 4; v++) {
                        const uint32_t word = s[v][blk >> 1];
                        const __half hs = __ushort_as_half((unsigned short)((blk & 1) ? (word >> 16) : (word & 0xffffu)));
                        const float sc = __half2float(hs);
#pragma unroll
                        for (int tt = 0; tt < TT; tt++) acc[tt][v] += sc * cw[tt][v];
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < WLOADS; u++) {       // 64 k: lane holds k = 64 u + 16 g .. + 15
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const bf16x8 wf = h ? int8_operand(w[u].z, w[u].w) : int8_operand(w[u].x, w[u].y);
#pragma unroll
                    for (int tt = 0; tt < TT; tt++) {
                        const bf16x8 xf = xfrag(tile, tt, (64 * u + 16 * g + 8 * h) / 8);
                        acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc[tt], 0, 0, 0);
                        ones_acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, xf, ones_acc[tt], 0, 0, 0);
                    }
                }
            }
        }
    };

    // Step t computes from weight registers t % (DEPTH + 1) and token tile t % 2.  Its requests: the token
    // rows of step t + 1 first, then the weights of step t + DEPTH, so that the wait for the token
    // rows at the top of the next step leaves the weight requests in flight (loads return in
    // order).  (Measured: DEPTH 2 costs a third of the resident waves and is slower.)
    constexpr int DEPTH = 1;
    auto step = [&](auto WB, auto XB, int t) __attribute__((always_inline)) {
        constexpr int wb = decltype(WB)::value, xb = decltype(XB)::value, wn = (wb + DEPTH) % (DEPTH + 1);
        store_x(xreg, xs[xb]);
        if (t + 1 < steps) load_x(xreg, kbeg + (t + 1) * SD);
        if (t + DEPTH < steps) {
            load_w(wreg[wn], kbeg + (t + DEPTH) * SD);
            if constexpr (I4) load_s(sreg[wn], kbeg + (t + DEPTH) * SD);
        }
        __syncthreads();
        compute(wreg[wb], sreg[wb], xs[xb]);
    };
    if (steps > 0) {
        load_x(xreg, kbeg);
        load_w(wreg[0], kbeg);
        if constexpr (I4) load_s(sreg[0], kbeg);
        if (DEPTH == 2 && steps > 1) {
            load_w(wreg[1], kbeg + SD);
            if constexpr (I4) load_s(sreg[1], kbeg + SD);
        }
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        if constexpr (DEPTH == 1) {
            for (int t = 0; t < steps; t += 2) {
                step(I0{}, I0{}, t);
                if (t + 1 >= steps) break;
                step(I1{}, I1{}, t + 1);
            }
        } else
        for (int t = 0; t < steps; t += 6) {
            step(I0{}, I0{}, t);
            if (t + 1 >= steps) break;
            step(I1{}, I1{}, t + 1);
            if (t + 2 >= steps) break;
            step(I2{}, I0{}, t + 2);
            if (t + 3 >= steps) break;
            step(I0{}, I1{}, t + 3);
            if (t + 4 >= steps) break;
            step(I1{}, I0{}, t + 4);
            if (t + 5 >= steps) break;
            step(I2{}, I1{}, t + 5);
        }
    }

    QTS(1);
    // accumulator view: lane holds token 16 tt + lr, channels n0 + 4 g + v
    const int n = n0 + 4 * g;
    if (n < N) {
        float ch_scale[4] = {1.f, 1.f, 1.f, 1.f};
        if constexpr (!I4) {
            // one fp16 scale per output channel, applied once
            const unsigned short* sc = reinterpret_cast<const unsigned short*>(scales);
#pragma unroll
            for (int v = 0; v < 4; v++) ch_scale[v] = __half2float(__ushort_as_half(sc[n + v]));
        }
#pragma unroll
        for (int tt = 0; tt < TT; tt++) {
            const int m = TOK * tt + lr;
            if (m >= Mj) continue;
            f32x4 o = acc[tt];
            if constexpr (!I4) {
#pragma unroll
                for (int v = 0; v < 4; v++) o[v] = ch_scale[v] * (acc[tt][v] - 128.f * ones_acc[tt][v]);
            }
            float* const dst = part + ((int64_t)split * Mj + m) * ld_part + ncomb0 + 4 * g;
#pragma unroll
            for (int v = 0; v < 4; v++) shared_store(dst + v, o[v]);
        }
    }
    // the last of this block's slices to arrive finishes it
    QTS(3);
    const bool last = arrive(tickets + rb, &s_ticket) == last_ticket;
    QTS(4);
    if (last) finish(rb);
    QTS(5);
}

}  // namespace skinny

#ifdef FHPC_TRACE
extern "C" int fhpc_debug_read_qts(unsigned long long* out, int n)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(skinny::g_qtrace), sizeof(unsigned long long) * (size_t)n);
}
#endif

bool qskinny_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme)
{
    if (scheme != 4 && scheme != 8) return false;
    // the kernels address each operand with 32-bit byte offsets below 2^31
    const int64_t lim = (int64_t)1 << 31;
    if (N < 1 || K < 1 || N * K >= lim || 2 * r * N >= lim) return false;
    if ((N + skinny::ROWS_WG - 1) / skinny::ROWS_WG > skinny::TICKETS / QSKINNY_MAX_JOBS) return false;   // tickets in the header
    return M >= 1 && M <= 4 * skinny::TOK && r >= 1 && r <= 64 && (K % 256) == 0;
}

QskinnyPlan qskinny_plan(int64_t M, int64_t K, int64_t r, const int64_t* N, int count, int num_cu)
{
    QskinnyPlan p;
    int64_t row_blocks = 0;
    for (int j = 0; j < count; j++) row_blocks += (N[j] + skinny::ROWS_WG - 1) / skinny::ROWS_WG;
    const int tt = (M <= 16) ? 1 : (M <= 32) ? 2 : 4;
    const int64_t sd = skinny::step_depth(tt, K);
    const int64_t ksteps = K / sd;
    // One round of workgroups: as many as are resident at once (registers and the token tiles' LDS
    // allow three per compute unit with 16 tokens, two with more) and no more, so that
    // no second, partly filled round follows; at least one step each.
    const int64_t per_cu = (M <= 16) ? 3 : 2;
    // (the chunks of H = X A run at the head of the same grid and hold slots of that round meanwhile)
    const int64_t hchunks = (int64_t)count * ((K + skinny::HCHUNK - 1) / skinny::HCHUNK);
    int64_t s = (per_cu * (int64_t)num_cu - hchunks) / row_blocks;
    if (s > ksteps) s = ksteps;
    if (s < 1) s = 1;
    const int64_t per = (ksteps + s - 1) / s;
    p.k_chunk = (int)(per * sd);
    p.splits = (int)((ksteps + per - 1) / per);
    p.kchunks = (int)((K + skinny::HCHUNK - 1) / skinny::HCHUNK);
    p.row_blocks = (int)row_blocks;
    p.part_bytes = (int64_t)p.splits * M * row_blocks * skinny::ROWS_WG * 4;
    p.hpart_bytes = (int64_t)count * (p.kchunks + 1) * M * r * 4;          // the chunks, then H itself ([count][M][r])
    return p;
}

hipError_t launch_qskinny_fwd(const void* X, const QskinnyJob* jobs, int count, int scheme, int64_t M, int64_t K, int64_t r,
                              const QskinnyPlan& p, float* part, float* hpart, uint32_t* tickets, hipStream_t st)
{
    using namespace skinny;
    if (count < 1 || count > QSKINNY_MAX_JOBS) return hipErrorInvalidValue;
    SkinnyJobs jb = {};
    jb.count = count;
    double wbytes = 0.0, nsum = 0.0;
    int rb = 0;
    for (int j = 0; j < QSKINNY_MAX_JOBS; j++) {
        const QskinnyJob& q = jobs[j < count ? j : 0];          // unused slots repeat the first weight
        jb.Wq[j] = q.Wq; jb.scales[j] = q.scales; jb.A[j] = q.A; jb.B[j] = q.B; jb.Y[j] = q.Y; jb.H_out[j] = q.H_out;
        jb.N[j] = (int)q.N; jb.base_scale[j] = q.base_scale; jb.scaling[j] = q.scaling;
        jb.X[j] = q.X_own ? q.X_own : X;
        jb.M[j] = q.X_own ? (int)q.M_own : (int)M;
        if (jb.M[j] < 1 || jb.M[j] > (int)M) return hipErrorInvalidValue;
        jb.rb0[j] = rb;
        if (j < count) {
            rb += (int)((q.N + ROWS_WG - 1) / ROWS_WG);
            bool seen = false;                                  // (token blocks of one weight: its bytes count once)
            for (int i = 0; i < j; i++) seen = seen || jobs[i].Wq == q.Wq;
            if (!seen) wbytes += (scheme == 4) ? (double)q.N * K / 2 + (double)q.N * (K / 64) * 2 : (double)q.N * K + (double)q.N * 2;
            nsum += (double)q.N;
        }
    }
    for (int j = count; j <= QSKINNY_MAX_JOBS; j++) jb.rb0[j] = rb;
    if (rb > TICKETS) return hipErrorInvalidValue;
    const int head_grid = count * p.kchunks;                       // the H = X A chunks first, then the streaming workgroups
    const dim3 grid((unsigned)(head_grid + rb * p.splits));
    float* const hsum = hpart + (int64_t)count * p.kchunks * M * r;
    // how often a finisher looks at H's flag before it forms H itself (about a microsecond a look); the
    // environment variable is for the test that forces that path (a negative value: never look)
    int poll_limit = 8192;
    if (const char* e = getenv("FHPC_H_POLLS")) poll_limit = atoi(e);
    const int slot = prof_begin(scheme == 4 ? "qskinny_fwd<int4>" : "qskinny_fwd<int8>", 2.0 * M * K * nsum,
                                wbytes + 2.0 * M * K + 4.0 * p.splits * M * nsum + 2.0 * M * nsum, st);
#define FHPC_MAIN(SCHEME, TT, SD)                                                                                   \
    hipLaunchKernelGGL((qskinny_fwd_kernel<SCHEME, TT, SD>), grid, dim3(NT), 0, st, jb, part, (int)M, (int)K,       \
                       p.k_chunk, hpart, (int)r, p.kchunks, head_grid, p.splits, tickets, hsum, poll_limit)
    const int tt = (M <= 16) ? 1 : (M <= 32) ? 2 : 4;
    const bool deep = step_depth(tt, K) == 512;
    if (scheme == 4) {
        if (tt == 1) { if (deep) FHPC_MAIN(4, 1, 512); else FHPC_MAIN(4, 1, 256); }
        else if (tt == 2) { if (deep) FHPC_MAIN(4, 2, 512); else FHPC_MAIN(4, 2, 256); }
        else FHPC_MAIN(4, 4, 256);
    } else {
        if (tt == 1) { if (deep) FHPC_MAIN(8, 1, 512); else FHPC_MAIN(8, 1, 256); }
        else if (tt == 2) { if (deep) FHPC_MAIN(8, 2, 512); else FHPC_MAIN(8, 2, 256); }
        else FHPC_MAIN(8, 4, 256);
    }
#undef FHPC_MAIN
    prof_end(slot, st);
    return hipGetLastError();
}

}  // namespace fhpc
