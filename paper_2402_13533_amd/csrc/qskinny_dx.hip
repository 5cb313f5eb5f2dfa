// Weight-streaming input gradient of the quantised finetuning layer for a handful of tokens
// (M <= 64, in blocks of 16):
//   dX[m][k] = base_scale * sum_n dY[m][n] q[n][k] scale(n, k) + scaling * sum_j dH[m][j] A[k][j],
// the backward of Y = X deq(W) + s (X A) B with respect to X (Sec. 5.1; W is frozen, so there is no dW).
//
// The reduction runs over the rows n of the stored weight ([N][K] codes, k contiguous), so the
// contraction index of the matrix instruction is the one index along which nothing is contiguous
// in memory.  Lane (i, g) therefore loads eight bytes - eight int8 or sixteen int4 codes along k -
// from each of the eight rows n = n0 + 8 g + s, and builds, for every code position c, the operand
// of v_mfma_f32_16x16x32_bf16 from code c of its eight rows: the instruction's 16 operand rows are
// the inputs k = k0 + CODES * i + c, its 32 contraction slots the 32 rows n of the step.  The other
// operand is the 16-byte piece dY[m][n0 + 8 g .. + 7] as it lies in memory.  Each code position has
// its own 16 x 16 accumulator (CODES * 4 registers).  A code becomes an operand element with
// v_cvt_f32_ubyte (after an XOR that makes it unsigned), one fma with the fp16 scale,
// (u - offset) * scale, which is exact in fp32, and the rounding to bf16 that every product with
// this weight applies to deq(W).  Both schemes have the scale of a lane's codes of one row in one
// scalar: int8 scales belong to the row n, int4 scales to (row n, block k / 64), and a lane's
// sixteen codes lie in one block.
//
// Work split: a workgroup of eight waves owns a column strip of 16 * CODES inputs k and a slice
// of the rows n; its waves take the 32-row steps of the slice in turn and add their accumulators
// through LDS; slices write fp32 slabs [slice][M][K]; dx_finish_kernel adds the slabs and the
// rank-r branch and rounds to bf16.  Two blocks of 16 tokens can share one pass over the codes
// (template parameter TT: every operand built from the codes feeds TT matrix instructions); more
// than 32 tokens are further workgroups that stream the same weight again (from the caches).  dH = dY B^T (M x r), which the rank-r branch
// and dA need, is formed on the way when r <= 16: the workgroups of the first strip also multiply
// their dY pieces with the matching pieces of B (one more 16-byte load and one more matrix
// instruction per step) and write dH's sums over their slices; the finish kernel adds them (and
// stores dH as bf16 for dA).
#include "qskinny.h"
#include "few_token_grads.h"
#include "profile.h"

#include <hip/hip_fp16.h>
#include <stdio.h>
#include <type_traits>

namespace fhpc {
namespace skinny_dx {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int NT = 512, WAVES = 8;
constexpr int TOK = 16;                // tokens per workgroup (the matrix instruction's columns)
constexpr int STEP_ROWS = 32;          // rows n per step of a wave: four lane groups x eight loads
constexpr uint32_t OOB = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* p, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f;
    f.x = lo;
    f.y = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__device__ __forceinline__ float half_bits_to_float(uint32_t h) { return __half2float(__ushort_as_half((unsigned short)h)); }

// Column of the LDS reduction buffer for strip-local input k: within each run of 64 columns the
// index is XORed with 16 * (run number), which spreads the four lane groups of a wave (whose
// columns differ by the run) over different banks; rows are padded to an odd length for the
// sixteen tokens.
__device__ __forceinline__ int red_col(int kl)
{
    const int run = kl >> 6;
    return (run << 6) | ((kl & 63) ^ ((run & 3) << 4));
}

// TT: blocks of 16 tokens that share one pass over the codes (each operand built from the codes feeds TT
// matrix instructions), 1 or 2.  A lane takes 16 int4 codes per row with one token block, 8 codes per row
// otherwise (4 * TT accumulator registers per code position have to fit).
constexpr int dx_codes(int scheme, int tt) { return (scheme == 4 && tt == 1) ? 16 : 8; }

template <int SCHEME, int TT>
__global__ __launch_bounds__(NT) void qskinny_dx_kernel(const void* __restrict__ dY, const void* __restrict__ Wq,
                                                        const void* __restrict__ scales, float* __restrict__ part,
                                                        int M, int K, int N, int steps_per_slice, int steps_total,
                                                        int strips, int slices, int token_blocks,
                                                        const void* __restrict__ Bf, float* __restrict__ dhpart, int rp)
{
    constexpr bool I4 = (SCHEME == 4);
    constexpr int CODES = dx_codes(SCHEME, TT);      // codes of a lane per row
    constexpr int WORDS = (I4 ? CODES / 2 : CODES) / 4;          // 32-bit words they take
    constexpr int CPW = I4 ? 8 : 4;                  // codes per word
    constexpr int KC = 16 * CODES;                   // inputs k per workgroup
    constexpr int RS = KC + 1;                       // padded row of the reduction buffer
    __shared__ float red[WAVES * TOK * RS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    // Workgroup -> work item.  Consecutive workgroup numbers go to the eight XCDs in turn, each with
    // its own L2, so item w = (number % 8) * (items / 8) + number / 8 gives every XCD a contiguous
    // run of the list (token block fastest, then strip, then slice): the token blocks of one strip read
    // the same codes, and neighbouring strips of one slice share the lines of int4 scales (64 blocks
    // per 128-byte line) and the dY rows.
    const int per_xcd = (int)gridDim.x >> 3;
    const int w = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (w >= strips * slices * token_blocks) return;             // the grid is rounded up to a multiple of 8
    const int tb = w % token_blocks, strip = (w / token_blocks) % strips, slice = w / (token_blocks * strips);
    const int k0 = strip * KC + CODES * i;           // first input of this lane's codes
    const int step_beg = slice * steps_per_slice;
    const int step_end = (step_beg + steps_per_slice < steps_total) ? step_beg + steps_per_slice : steps_total;

    const int64_t row_bytes = I4 ? K / 2 : K;
    const __amdgpu_buffer_rsrc_t rw = rsrc(Wq, (int64_t)N * row_bytes);
    const __amdgpu_buffer_rsrc_t rs = rsrc(scales, I4 ? (int64_t)N * (K / 64) * 2 : (int64_t)N * 2);
    const __amdgpu_buffer_rsrc_t rd = rsrc(dY, (int64_t)M * N * 2);
    const uint32_t wcol = (uint32_t)(I4 ? k0 / 2 : k0);          // byte of the lane's codes within a row
    const uint32_t scol = I4 ? (uint32_t)(k0 / 64) * 2u : 0u;    // byte of the lane's block scale within a row of scales
    const int m0 = tb * (TOK * TT);                              // first token of this workgroup
    uint32_t dyrow[TT];                                          // this lane's token of every block (dY operand, accumulator column)
#pragma unroll
    for (int t = 0; t < TT; t++) dyrow[t] = (m0 + TOK * t + i < M) ? (uint32_t)((int64_t)(m0 + TOK * t + i) * N * 2) : OOB;

    // first strip: dH[m][j] = sum_n dY[m][n] B[j][n] over this slice beside the main sums (lane i is row j of B)
    const bool with_dh = (strip == 0) && (dhpart != nullptr);
    const __amdgpu_buffer_rsrc_t rb = rsrc(Bf, with_dh ? (int64_t)rp * N * 2 : 0);
    const uint32_t brow = (with_dh && i < rp) ? (uint32_t)((int64_t)i * N * 2) : OOB;
    f32x4 acc_dh[TT];
    u32x4 bq[2];

    f32x4 acc[TT][CODES];
#pragma unroll
    for (int t = 0; t < TT; t++) {
        acc_dh[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < CODES; c++) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // What a lane reads for one step: rows n = 32 step + 8 g + s, s < 8.  N is a multiple of 8, so the
    // eight rows are inside the weight together or not at all; what lies outside reads as zero
    // (an offset beyond the buffer), and so do the dY pieces, which makes those rows contribute 0.
    uint32_t wq[2][8][WORDS];
    uint32_t sc4[2][8];                              // int4: one fp16 scale per row (this lane's block)
    u32x4 sc8[2];                                    // int8: the eight rows' fp16 scales
    u32x4 dyq[2][TT];                                // dY[m][n .. n + 7] bf16
    auto load = [&](auto BUF, int step) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value;
        const int n0 = step * STEP_ROWS + 8 * g;
        const bool inside = n0 < N;
        const uint32_t guard = inside ? 0u : OOB;    // ORed into every offset: outside rows read as zero
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const uint32_t off = ((uint32_t)(n0 + s) * (uint32_t)row_bytes + wcol) | guard;
            if constexpr (WORDS == 2) {
                const auto v = __builtin_amdgcn_raw_buffer_load_b64(rw, off, 0, 0);
                wq[b][s][0] = v[0]; wq[b][s][1] = v[1];
            } else {
                wq[b][s][0] = __builtin_amdgcn_raw_buffer_load_b32(rw, off, 0, 0);
            }
        }
        if constexpr (I4) {
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const uint32_t off = ((uint32_t)(n0 + s) * (uint32_t)(K / 64) * 2u + scol) | guard;
                sc4[b][s] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
            }
        } else {
            sc8[b] = __builtin_amdgcn_raw_buffer_load_b128(rs, ((uint32_t)n0 * 2u) | guard, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < TT; t++) dyq[b][t] = __builtin_amdgcn_raw_buffer_load_b128(rd, (dyrow[t] + (uint32_t)n0 * 2u) | guard, 0, 0);
        if (with_dh) bq[b] = __builtin_amdgcn_raw_buffer_load_b128(rb, (brow + (uint32_t)n0 * 2u) | guard, 0, 0);
    };
    auto compute = [&](auto BUF) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value;
        // per row s: the lane's scale and the term that takes the unsigned code's offset out again
        float sc[8], off[8];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            if constexpr (I4) {
                sc[s] = half_bits_to_float(sc4[b][s]);
            } else {
                const uint32_t sword = sc8[b][s >> 1];
                sc[s] = half_bits_to_float((s & 1) ? (sword >> 16) : (sword & 0xffffu));
            }
            off[s] = (I4 ? -8.f : -128.f) * sc[s];
        }
        bf16x8 dy[TT];                                             // dY[m][n0 + 8 g + 0 .. 7] of every token block
#pragma unroll
        for (int t = 0; t < TT; t++) dy[t] = __builtin_bit_cast(bf16x8, dyq[b][t]);
        if (with_dh) {
#pragma unroll
            for (int t = 0; t < TT; t++)
                acc_dh[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bq[b]), dy[t], acc_dh[t], 0, 0, 0);
        }
        // one word of the eight rows at a time (keeps the unpacked codes of one word live, not of all)
#pragma unroll
        for (int h = 0; h < WORDS; h++) {
            // unsigned codes as bytes: int4 -> lo (codes 0 2 4 6 of the word) and hi (codes 1 3 5 7)
            uint32_t ub[8][I4 ? 2 : 1];
#pragma unroll
            for (int s = 0; s < 8; s++) {
                if constexpr (I4) {
                    const uint32_t u = wq[b][s][h] ^ 0x88888888u;      // nibble ^ 8 = q + 8
                    ub[s][0] = u & 0x0f0f0f0fu;
                    ub[s][1] = (u >> 4) & 0x0f0f0f0fu;
                    // (opaque to the optimiser: a byte of a masked word converts with one
                    // v_cvt_f32_ubyteN; seen through, it becomes a 4-bit field extract plus a convert)
                    asm volatile("" : "+v"(ub[s][0]), "+v"(ub[s][1]));
                } else {
                    ub[s][0] = wq[b][s][h] ^ 0x80808080u;              // byte ^ 0x80 = q + 128
                }
            }
#pragma unroll
            for (int cc = 0; cc < CPW; cc++) {
                // code c of the lane's eight rows -> one operand: element s = bf16((u - offset) * scale of row s)
                const int c = h * CPW + cc;
                const int j = I4 ? cc >> 1 : cc;                       // byte within the word
                const int par = I4 ? cc & 1 : 0;                       // int4: even / odd code of the byte
                float f[8];
#pragma unroll
                for (int s = 0; s < 8; s++) f[s] = fmaf((float)((ub[s][par] >> (8 * j)) & 0xffu), sc[s], off[s]);
                u32x4 wv;
                wv.x = pack_bf16(f[0], f[1]);
                wv.y = pack_bf16(f[2], f[3]);
                wv.z = pack_bf16(f[4], f[5]);
                wv.w = pack_bf16(f[6], f[7]);
#pragma unroll
                for (int t = 0; t < TT; t++)
                    acc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv), dy[t], acc[t][c], 0, 0, 0);
            }
        }
    };

    // the waves of the workgroup take the steps of the slice in turn; two register sets, the
    // loads of a wave's next step are out before it computes the current one
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    int step = step_beg + wave;
    if (step < step_end) load(B0{}, step);
    while (step < step_end) {
        if (step + WAVES < step_end) load(B1{}, step + WAVES);
        compute(B0{});
        step += WAVES;
        if (step >= step_end) break;
        if (step + WAVES < step_end) load(B0{}, step + WAVES);
        compute(B1{});
        step += WAVES;
    }

    // accumulator view: lane holds token i (column) of each block and the operand rows 4 g + v, i.e. the
    // strip-local inputs CODES * (4 g + v) + c.  One token block at a time through the reduction buffer.
#pragma unroll
    for (int t = 0; t < TT; t++) {
        if (t > 0) __syncthreads();
#pragma unroll
        for (int c = 0; c < CODES; c++)
#pragma unroll
            for (int v = 0; v < 4; v++) red[(wave * TOK + i) * RS + red_col(CODES * (4 * g + v) + c)] = acc[t][c][v];
        __syncthreads();
        for (int o = tid; o < TOK * KC; o += NT) {
            const int mm = o / KC, kl = o - mm * KC;
            float sum = 0.f;
#pragma unroll
            for (int w8 = 0; w8 < WAVES; w8++) sum += red[(w8 * TOK + mm) * RS + red_col(kl)];
            const int mg = m0 + TOK * t + mm;
            if (mg < M) part[((int64_t)slice * M + mg) * K + strip * KC + kl] = sum;
        }
    }
    if (with_dh) {
        // dH of this slice: lane holds token i and the rows j = 4 g + v; added over the waves like the main sums
        constexpr int DS = TOK + 1;
#pragma unroll
        for (int t = 0; t < TT; t++) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 4; v++) red[(wave * TOK + i) * DS + 4 * g + v] = acc_dh[t][v];
            __syncthreads();
            if (tid < TOK * TOK) {
                const int mm = tid >> 4, j = tid & 15;
                float sum = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < WAVES; w8++) sum += red[(w8 * TOK + mm) * DS + j];
                const int mg = m0 + TOK * t + mm;
                if (mg < M && j < rp) dhpart[((int64_t)slice * M + mg) * rp + j] = sum;
            }
        }
    }
}

// dX[m][k] = bf16( base_scale * sum_s part[s][m][k] + scaling * sum_j dH[m][j] A[k][j] ),  dH = sum_c dhpart[c].
// One output per thread (grid: 256 inputs k x one token).  A is bf16 [K][rp], rp a multiple of 8 and at
// most 64.  All loads are requested before the first wait: the pieces of the row of A beyond rp get an
// offset outside the buffer and read as zero; the chunk sums of dH are read as 16-byte pieces, thread
// (p, g) taking piece p of the chunks g, g + G, ..., eight in flight; the workgroups of the first 256
// inputs then also store dH[m] as bf16 (dA is formed from it afterwards).  Without dhpart, dH is an
// input (bf16 [M][rp]).
constexpr int FIN_NT = 256, FIN_DEPTH = 8, FIN_RMAX = 64;
constexpr int FIN_LDS = FIN_NT * 4 + FIN_RMAX;                             // floats: group sums, then dH[m]
struct FinishArgs {
    const float* part;
    int slices;
    const float* dhpart;
    int dh_chunks;
    uint16_t* dH;
    const uint16_t* A;
    int rp;
    float base_scale, scaling;
    uint16_t* dX;
    int M, K;
};
// workgroup (bx, m): the 256 inputs k from 256 bx of token m
__device__ __forceinline__ void dx_finish_body(float* smem, int bx, int m, const FinishArgs& fa)
{
    float* const dg = smem;
    float* const dh = smem + FIN_NT * 4;
    const float* __restrict__ part = fa.part;
    const float* __restrict__ dhpart = fa.dhpart;
    uint16_t* __restrict__ dH = fa.dH;
    const uint16_t* __restrict__ A = fa.A;
    uint16_t* __restrict__ dX = fa.dX;
    const int slices = fa.slices, dh_chunks = fa.dh_chunks, rp = fa.rp, M = fa.M, K = fa.K;
    const float base_scale = fa.base_scale, scaling = fa.scaling;
    const int k = bx * FIN_NT + threadIdx.x;                               // K is a multiple of 256
    const bool branch = (scaling != 0.f) && A;
    const __amdgpu_buffer_rsrc_t rA = rsrc(A, branch ? (int64_t)K * rp * 2 : 0);
    u32x4 a[FIN_RMAX / 8];
#pragma unroll
    for (int q = 0; q < FIN_RMAX / 8; q++) {
        const uint32_t off = (branch && 8 * q < rp) ? (uint32_t)((int64_t)k * rp + 8 * q) * 2u : OOB;
        a[q] = __builtin_amdgcn_raw_buffer_load_b128(rA, off, 0, 0);
    }
    auto sum8 = [](const auto (&v)[FIN_DEPTH]) __attribute__((always_inline)) {
        return ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    };
    auto part_batch = [&](float (&v)[FIN_DEPTH], int s0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < FIN_DEPTH; q++) {
            const int s = s0 + q;
            const float x = part[((int64_t)(s < slices ? s : s0) * M + m) * K + k];
            v[q] = (s < slices) ? x : 0.f;
        }
    };
    float pv[FIN_DEPTH];
    part_batch(pv, 0);
    // dH[m][.]: chunk c holds it at dhpart[(c M + m) rp ..]
    const int P = rp >> 2;                                      // 16-byte pieces per chunk
    const int G = (FIN_NT / P < dh_chunks) ? FIN_NT / P : dh_chunks;   // groups that have a chunk to start from
    {
        const int p = threadIdx.x % P, g = threadIdx.x / P;
        const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
        f32x4 sv = zero4;
        if (dhpart && g < G) {
            const float* src = dhpart + (int64_t)m * rp + 4 * p;
            const int64_t stride = (int64_t)M * rp;
            for (int c0 = g; c0 < dh_chunks; c0 += FIN_DEPTH * G) {
                f32x4 v[FIN_DEPTH];
#pragma unroll
                for (int q = 0; q < FIN_DEPTH; q++) {
                    const int c = c0 + q * G;
                    const f32x4 x = *reinterpret_cast<const f32x4*>(src + (int64_t)(c < dh_chunks ? c : c0) * stride);
                    v[q] = (c < dh_chunks) ? x : zero4;
                }
                sv += sum8(v);
            }
            *reinterpret_cast<f32x4*>(dg + (g * P + p) * 4) = sv;          // dg[g][4 p ..] of [G][rp]
        }
    }
    float base = sum8(pv);
    for (int s0 = FIN_DEPTH; s0 < slices; s0 += FIN_DEPTH) {
        part_batch(pv, s0);
        base += sum8(pv);
    }
    __syncthreads();
    if (threadIdx.x < FIN_RMAX) {
        float t = 0.f;
        if (dhpart && (int)threadIdx.x < rp) {
            for (int g = 0; g < G; g++) t += dg[g * rp + threadIdx.x];     // group order: the same sum every run
            if (bx == 0 && dH) {
                const __bf16 hb = (__bf16)t;
                dH[(int64_t)m * rp + threadIdx.x] = __builtin_bit_cast(uint16_t, hb);
            }
        } else if (!dhpart && dH && branch && (int)threadIdx.x < rp) {
            t = __uint_as_float((uint32_t)dH[(int64_t)m * rp + threadIdx.x] << 16);   // formed by the caller
        }
        dh[threadIdx.x] = t;
    }
    __syncthreads();
    float l = 0.f;
#pragma unroll
    for (int q = 0; q < FIN_RMAX / 8; q++) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const uint32_t word = a[q][e];
            l = fmaf(__uint_as_float(word << 16), dh[8 * q + 2 * e], l);
            l = fmaf(__uint_as_float(word & 0xffff0000u), dh[8 * q + 2 * e + 1], l);
        }
    }
    const __bf16 o = (__bf16)(base_scale * base + scaling * l);
    dX[(int64_t)m * K + k] = __builtin_bit_cast(uint16_t, o);
}

__global__ __launch_bounds__(FIN_NT) void dx_finish_kernel(FinishArgs fa)
{
    __shared__ __attribute__((aligned(16))) float smem[FIN_LDS];
    dx_finish_body(smem, blockIdx.x, blockIdx.y, fa);
}

// The finish of dX and the rank-r weight gradients in one launch (they are independent of each other
// once the streaming launch has written its slabs): workgroups [0, fin_blocks) finish dX, the next
// blocks_a form dA = alpha X^T dH with dH summed in fp32 from the per-slice sums, the rest
// dB = alpha H^T dY.  rp <= 16.
struct GradArgs {
    const uint16_t* X;
    const uint16_t* H;
    const uint16_t* dY;
    float* dA;
    float* dB;
    int r, N, fin_blocks, blocks_a;
    float alpha;
};
template <int MT>
__global__ __launch_bounds__(FIN_NT) void dx_tail_kernel(FinishArgs fa, GradArgs ga)
{
    constexpr int RP = 16;
    static_assert(FTG_NT == FIN_NT && MT * RP <= FIN_LDS, "shared workgroup shape and LDS");
    __shared__ __attribute__((aligned(16))) float smem[FIN_LDS];
    const int b = blockIdx.x;
    if (b < ga.fin_blocks) {
        const int per_token = fa.K / FIN_NT;
        dx_finish_body(smem, b % per_token, b / per_token, fa);
    } else if (b < ga.fin_blocks + ga.blocks_a) {
        const int c = (b - ga.fin_blocks) * FIN_NT + (int)threadIdx.x;
        few_token_grads_body<MT, RP, false>(smem, ga.X, fa.K, c, fa.M, ga.r, ga.alpha, ga.dA, [&](float* v) {
            // v[m][j] = sum over the slices of dhpart[(s M + m) rp + j], eight loads in flight (a slice
            // index past the end repeats an earlier, valid address and is dropped by the select)
            for (int e = threadIdx.x; e < MT * RP; e += FIN_NT) {
                const int m = e / RP, j = e - m * RP;
                float t = 0.f;
                if (m < fa.M && j < fa.rp) {
                    const float* src = fa.dhpart + (int64_t)m * fa.rp + j;
                    const int64_t stride = (int64_t)fa.M * fa.rp;
                    for (int s0 = 0; s0 < fa.dh_chunks; s0 += FIN_DEPTH) {
                        float x[FIN_DEPTH];
#pragma unroll
                        for (int q = 0; q < FIN_DEPTH; q++) {
                            const int sl = s0 + q;
                            const float y = src[(int64_t)(sl < fa.dh_chunks ? sl : s0) * stride];
                            x[q] = (sl < fa.dh_chunks) ? y : 0.f;
                        }
                        t += ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
                    }
                }
                v[e] = t;
            }
        });
    } else {
        const int c = (b - ga.fin_blocks - ga.blocks_a) * FIN_NT + (int)threadIdx.x;
        few_token_grads_body<MT, RP, true>(smem, ga.dY, ga.N, c, fa.M, ga.r, ga.alpha, ga.dB,
                                           [&](float* v) { fill_from_bf16<MT, RP>(v, ga.H, fa.M, fa.rp); });
    }
}

}  // namespace skinny_dx

bool qskinny_dx_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme)
{
    if (scheme != 4 && scheme != 8) return false;
    // the kernels address each operand with 32-bit byte offsets below 2^31
    const int64_t lim = (int64_t)1 << 31;
    if (N < 8 || K < 256 || (N % 8) || (K % 256)) return false;
    if (N * K >= lim || M * N * 2 >= lim || K * 64 * 2 >= lim) return false;
    return M >= 1 && M <= 4 * skinny_dx::TOK && r >= 1 && r <= skinny_dx::FIN_RMAX;
}

QskinnyDxPlan qskinny_dx_plan(int64_t M, int64_t K, int64_t N, int scheme, int num_cu)
{
    using namespace skinny_dx;
    QskinnyDxPlan p;
    p.tt = (M <= TOK) ? 1 : 2;            // (four blocks per pass do not fit the registers: 600 bytes of spills per lane)
    const int64_t kc = 16 * dx_codes(scheme, p.tt);
    // one workgroup per compute unit (registers: two waves per SIMD; the reduction buffer is 65 or 129 KB)
    const int64_t per_cu = 1;
    p.strips = (int)(K / kc);
    p.token_blocks = (int)((M + TOK * p.tt - 1) / (TOK * p.tt));
    p.steps_total = (int)((N + STEP_ROWS - 1) / STEP_ROWS);
    // one round of resident workgroups; a slice is at least one step for each of the eight waves
    int64_t s = per_cu * (int64_t)num_cu / ((int64_t)p.strips * p.token_blocks);
    const int64_t most = (p.steps_total + WAVES - 1) / WAVES;
    if (s > most) s = most;
    if (s < 1) s = 1;
    p.steps_per_slice = (int)((p.steps_total + s - 1) / s);
    p.slices = (int)((p.steps_total + p.steps_per_slice - 1) / p.steps_per_slice);
    p.part_bytes = (int64_t)p.slices * M * K * 4;
    return p;
}

hipError_t launch_qskinny_dx(const void* dY, const void* Wq, const void* scales, int scheme, const void* B, const void* A,
                             int64_t rp, float base_scale, float scaling, void* dX, void* dH, int64_t M, int64_t K, int64_t N,
                             const QskinnyDxPlan& p, float* part, float* dhpart, const QskinnyDxGrads* grads, hipStream_t st)
{
    using namespace skinny_dx;
    if (rp > FIN_RMAX || rp < 8 || (rp % 8)) return hipErrorInvalidValue;
    if (dhpart && (rp > TOK || !B)) return hipErrorInvalidValue;
    if (grads && !dhpart) return hipErrorInvalidValue;
    const int64_t items = (int64_t)p.strips * p.slices * p.token_blocks;
    const dim3 grid((unsigned)((items + 7) / 8 * 8));
    const double wbytes = (scheme == 4) ? (double)N * K / 2 + (double)N * (K / 64) * 2 : (double)N * K + (double)N * 2;
    const int slot = prof_begin(scheme == 4 ? "qskinny_dx<int4>" : "qskinny_dx<int8>", 2.0 * M * K * (double)N,
                                wbytes + 2.0 * M * N + 4.0 * p.slices * M * K, st);
#define FHPC_DX(SCHEME, TT)                                                                                                  \
    hipLaunchKernelGGL((qskinny_dx_kernel<SCHEME, TT>), grid, dim3(NT), 0, st, dY, Wq, scales, part, (int)M, (int)K, (int)N, \
                       p.steps_per_slice, p.steps_total, p.strips, p.slices, p.token_blocks, B, dhpart, (int)rp)
    if (scheme == 4) {
        if (p.tt == 1) FHPC_DX(4, 1); else FHPC_DX(4, 2);
    } else {
        if (p.tt == 1) FHPC_DX(8, 1); else FHPC_DX(8, 2);
    }
#undef FHPC_DX
    prof_end(slot, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    FinishArgs fa;
    fa.part = part; fa.slices = p.slices; fa.dhpart = dhpart; fa.dh_chunks = p.slices;
    fa.dH = static_cast<uint16_t*>(dH); fa.A = static_cast<const uint16_t*>(A); fa.rp = (int)rp;
    fa.base_scale = base_scale; fa.scaling = scaling; fa.dX = static_cast<uint16_t*>(dX); fa.M = (int)M; fa.K = (int)K;
    if (grads && (grads->dA || grads->dB)) {
        GradArgs ga;
        ga.X = static_cast<const uint16_t*>(grads->X); ga.H = static_cast<const uint16_t*>(grads->H);
        ga.dY = static_cast<const uint16_t*>(dY); ga.dA = grads->dA; ga.dB = grads->dB;
        ga.r = (int)grads->r; ga.N = (int)N; ga.alpha = grads->alpha;
        ga.fin_blocks = (int)(K / FIN_NT * M);
        ga.blocks_a = grads->dA ? (int)(K / FIN_NT) : 0;
        const int blocks_b = grads->dB ? (int)((N + FIN_NT - 1) / FIN_NT) : 0;
        const dim3 tgrid((unsigned)(ga.fin_blocks + ga.blocks_a + blocks_b));
        const int tslot = prof_begin("qskinny_dx_finish+grads", 0.0, 0.0, st);
        if (M <= 16) hipLaunchKernelGGL((dx_tail_kernel<16>), tgrid, dim3(FIN_NT), 0, st, fa, ga);
        else hipLaunchKernelGGL((dx_tail_kernel<64>), tgrid, dim3(FIN_NT), 0, st, fa, ga);
        prof_end(tslot, st);
        return hipGetLastError();
    }
    const int fslot = prof_begin("qskinny_dx_finish", 0.0, 0.0, st);
    hipLaunchKernelGGL(dx_finish_kernel, dim3((unsigned)(K / FIN_NT), (unsigned)M), dim3(FIN_NT), 0, st, fa);
    prof_end(fslot, st);
    return hipGetLastError();
}

}  // namespace fhpc
