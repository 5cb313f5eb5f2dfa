// Device-side body of the rank-r weight gradients from a handful of tokens, shared by the kernel
// that computes them alone (kernels_misc.hip) and by the one that runs them beside the finish of
// the input gradient (qskinny_dx.hip).  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

constexpr int FTG_NT = 256, FTG_MMAX = 64, FTG_RMAX = 64;

// out[c][j] (TRANSPOSED = false, row length r) or out[j][c] (TRANSPOSED = true, row length ld)
//   = alpha * sum_m U[m][c] V[m][j],   c = column of the bf16 matrix U ([M][ld]), j < r.
// The thread owns column c and reads it a few tokens at a time (tokens past M and columns past
// the end get an offset outside the buffer and read as zero); `fill` puts V as fp32 [MT][RP]
// (zero beyond M and rp) into Vs (16-byte aligned), where every lane reads the same words; r running
// sums per thread.
template <int MT, int RP, bool TRANSPOSED, class Fill>
__device__ __forceinline__ void few_token_grads_body(float* Vs, const uint16_t* __restrict__ U, int ld, int c, int M, int r,
                                                     float alpha, float* __restrict__ out, Fill fill)
{
    const __amdgpu_buffer_rsrc_t ru =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(U), 0, (int)((int64_t)M * ld * 2), 0x00020000);
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    constexpr int MB = (RP <= 16) ? 16 : (RP <= 32) ? 8 : 4;   // tokens per trip to memory: MB * RP values of V at a time
    static_assert(MT % MB == 0, "token tile");
    auto load_block = [&](float (&u)[MB], int m0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < MB; q++) {
            const int m = m0 + q;
            const uint32_t off = (m < M && c < ld) ? (uint32_t)(((int64_t)m * ld + c) * 2) : 0x80000000u;
            u[q] = __uint_as_float((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(ru, off, 0, 0) << 16);
        }
    };
    float u[MB];
    load_block(u, 0);
    fill(Vs);
    __syncthreads();
    float acc[RP];
#pragma unroll
    for (int j = 0; j < RP; j++) acc[j] = 0.f;
    // MB tokens at a time; the loop is kept rolled (unrolled over all tokens the compiler starts
    // every load and every LDS read first and spills)
#pragma unroll 1
    for (int m0 = 0; m0 < MT; m0 += MB) {
        float un[MB];
        if (m0 + MB < MT) load_block(un, m0 + MB);   // the next tokens are on their way meanwhile
#pragma unroll
        for (int q = 0; q < MB; q++) {
#pragma unroll
            for (int j = 0; j < RP; j += 4) {
                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(Vs + (m0 + q) * RP + j);
                acc[j] = fmaf(u[q], v.x, acc[j]);
                acc[j + 1] = fmaf(u[q], v.y, acc[j + 1]);
                acc[j + 2] = fmaf(u[q], v.z, acc[j + 2]);
                acc[j + 3] = fmaf(u[q], v.w, acc[j + 3]);
            }
            // (the instruction scheduler would otherwise start every LDS read of the block first:
            // MB * RP values, more than a lane has registers for)
            __builtin_amdgcn_sched_barrier(0);
        }
        if (m0 + MB < MT) {
#pragma unroll
            for (int q = 0; q < MB; q++) u[q] = un[q];
        }
    }
    if (c >= ld) return;
#pragma unroll
    for (int j = 0; j < RP; j++) {
        if (j < r) {
            if constexpr (TRANSPOSED) out[(int64_t)j * ld + c] = alpha * acc[j];
            else out[(int64_t)c * r + j] = alpha * acc[j];
        }
    }
}

// Vs[m][j] = V[m][j] (bf16 [M][rp]) for m < M, j < rp, else 0
template <int MT, int RP>
__device__ __forceinline__ void fill_from_bf16(float* Vs, const uint16_t* __restrict__ V, int M, int rp)
{
    for (int e = threadIdx.x; e < MT * RP; e += FTG_NT) {
        const int m = e / RP, j = e - m * RP;
        Vs[e] = (m < M && j < rp) ? __uint_as_float((uint32_t)V[(int64_t)m * rp + j] << 16) : 0.f;
    }
}

}  // namespace fhpc
