// Two probes of what this GPU delivers with no kernel design in the way, so that a benchmark can quote its
// kernels against measured ceilings beside the published ones:
//   fhpc_probe_mfma : every SIMD issues v_mfma_f32_32x32x16_bf16 back to back from registers (no memory
//                     traffic at all), on operand data the caller chooses (zeros, or random values);
//   fhpc_probe_copy : a plain streaming copy, 16 bytes per lane per access.
#include "../../include/fingpt_hpc.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kMfmaPerIter = 8;     // independent accumulators, so that no instruction waits for the previous one

// seed[lane + 64 * j], j < 4: the lane's operand words.  Results are stored only when `sink` asks for them
// (it never does on a timed run; the store keeps the loop from being optimised away).
__global__ __launch_bounds__(256) void mfma_probe_kernel(const uint32_t* __restrict__ seed, int iters, float* sink)
{
    const int lane = threadIdx.x & 63;
    union { u32x4 w; bf16x8 v; } a, b;
    for (int j = 0; j < 4; j++) {
        a.w[j] = seed[lane + 64 * j];
        b.w[j] = seed[lane + 64 * ((j + 1) & 3)] ^ 0x00010001u * (uint32_t)(threadIdx.x >> 6);
    }
    f32x16 acc[kMfmaPerIter];
    for (int u = 0; u < kMfmaPerIter; u++)
        for (int v = 0; v < 16; v++) acc[u][v] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int u = 0; u < kMfmaPerIter; u++) acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc[u], 0, 0, 0);
    }
    if (sink) {
        float s = 0.f;
        for (int u = 0; u < kMfmaPerIter; u++)
            for (int v = 0; v < 16; v++) s += acc[u][v];
        sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(256) void copy_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = __builtin_nontemporal_load(src + i);
}

}  // namespace

extern "C" {

int fhpc_probe_mfma(const void* seed, int workgroups, int iters, float* sink, double* flops, void* hip_stream)
{
    if (!seed || !flops) return FHPC_ERR_NULL;
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1) return FHPC_ERR_SHAPE;
    *flops = (double)workgroups * 4.0 * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint32_t*>(seed), iters, sink);
    if (hipGetLastError() != hipSuccess) return FHPC_ERR_HIP;
    return FHPC_OK;
}

int fhpc_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream)
{
    if (!src || !dst) return FHPC_ERR_NULL;
    if (bytes < 16 || (bytes % 16)) return FHPC_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) % 16) return FHPC_ERR_ALIGN;
    const int64_t n16 = bytes / 16;
    int64_t wg = (n16 + 255) / 256;
    if (wg > 256 * 32) wg = 256 * 32;
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)wg), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n16);
    if (hipGetLastError() != hipSuccess) return FHPC_ERR_HIP;
    return FHPC_OK;
}

}  // extern "C"
