// The SiLU gate of the FFN (Sec. 3.1, eq. FFN): Z = SiLU(G) * U elementwise, and its backward
//   dU = dZ * SiLU(G),   dG = dZ * U * sigma(G) * (1 + G * (1 - sigma(G))),
// in fp32 on bf16 data, two elements (one 32-bit word) at a time.  One definition for the streaming kernels
// and for the GEMM epilogue that applies the gate to a tile it has just produced: both give the same bits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {
namespace gate {

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// sigma(g) with the hardware's exponential and reciprocal (each within one ulp or so of fp32, far below the bf16
// rounding of the results; a correctly rounded division costs as much as the rest of the gate together, and in a
// GEMM epilogue that is time the matrix cores stand idle)
__device__ __forceinline__ float sigmoid_f(float g) { return __builtin_amdgcn_rcpf(1.f + __expf(-g)); }
__device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack(float a, float b)
{
    f32x2_t v;
    v.x = a;
    v.y = b;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float fwd(float g, float u) { return u * g * sigmoid_f(g); }
__device__ __forceinline__ void bwd(float g, float u, float dz, float& dg, float& du)
{
    const float s = sigmoid_f(g);
    du = dz * g * s;
    dg = dz * u * s * (1.f + g * (1.f - s));
}

// two bf16 elements per word
__device__ __forceinline__ uint32_t fwd_pair(uint32_t g, uint32_t u)
{
    return pack(fwd(lo(g), lo(u)), fwd(hi(g), hi(u)));
}
__device__ __forceinline__ void bwd_pair(uint32_t g, uint32_t u, uint32_t dz, uint32_t& og, uint32_t& ou)
{
    float dg0, du0, dg1, du1;
    bwd(lo(g), lo(u), lo(dz), dg0, du0);
    bwd(hi(g), hi(u), hi(dz), dg1, du1);
    og = pack(dg0, dg1);
    ou = pack(du0, du1);
}

}  // namespace gate
}  // namespace fhpc
