// Probes of what this GPU delivers with no kernel design in the way, so that a benchmark can quote its
// kernels against measured ceilings beside the published ones:
//   fhpc_probe_mfma : every SIMD issues v_mfma_f32_32x32x16_bf16 back to back from registers (no memory
//                     traffic at all), on operand data the caller chooses (zeros, or random values);
//   fhpc_probe_copy : a plain streaming copy, 16 bytes per lane per access;
//   fhpc_probe_read_rows : one pass over a row-major matrix of bytes in the access pattern of the few-token
//                     weight-streaming kernels (64 rows x 256 bytes per workgroup and step, the next step requested
//                     before the current one is used, one round of resident workgroups) and nothing else: no
//                     decode, no matrix work, no reduction across workgroups, no output.
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

// Workgroup (row block rb, slice) reads rows 64 rb .. 64 rb + 63, bytes [slice * chunk, (slice + 1) * chunk) of each,
// 256 bytes per row and step: wave w takes sixteen rows, lane (lr, g) the 16 bytes at 64 u + 16 g of row 16 w + lr,
// u < 4.  The words are folded together; the fold is stored only if it equals a value it practically never takes
// (the store keeps the loads alive).
__global__ __launch_bounds__(256) void read_rows_probe_kernel(const unsigned char* __restrict__ W, int N, int row_bytes, int row_blocks,
                                                              int chunk, uint32_t* sink)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 15, g = lane >> 4;
    const int rb = (int)blockIdx.x % row_blocks, slice = (int)blockIdx.x / row_blocks;
    const int b0 = slice * chunk;
    const int b1 = (b0 + chunk < row_bytes) ? b0 + chunk : row_bytes;
    const int steps = (b1 - b0) / 256;
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(W), 0, N * row_bytes, 0x00020000);
    const int row = rb * 64 + wave * 16 + lr;
    const uint32_t off = (row < N) ? (uint32_t)(row * row_bytes + 16 * g) : 0x80000000u;      // beyond the buffer: reads as zero
    u32x4 w[2][4];
    u32x4 acc = {0u, 0u, 0u, 0u};
    auto load = [&](u32x4 (&x)[4], int s) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; u++) x[u] = __builtin_amdgcn_raw_buffer_load_b128(r, off + 64u * u, b0 + s * 256, 0);
    };
    if (steps > 0) load(w[0], 0);
    for (int t = 0; t < steps; t += 2) {
        if (t + 1 < steps) load(w[1], t + 1);
#pragma unroll
        for (int u = 0; u < 4; u++) acc ^= w[0][u];
        if (t + 1 >= steps) break;
        if (t + 2 < steps) load(w[0], t + 2);
#pragma unroll
        for (int u = 0; u < 4; u++) acc ^= w[1][u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5ca1ab1eu) sink[tid] = 1u;
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

int fhpc_probe_read_rows(const void* W, int64_t N, int64_t row_bytes, int workgroups, void* sink, void* hip_stream)
{
    if (!W || !sink) return FHPC_ERR_NULL;
    if (N < 1 || row_bytes < 256 || (row_bytes % 256) || N * row_bytes >= ((int64_t)1 << 31) || workgroups < 1) return FHPC_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(W) % 16) return FHPC_ERR_ALIGN;
    // as the streaming kernels plan it: as many slices of the rows as give one round of `workgroups` workgroups
    const int64_t row_blocks = (N + 63) / 64, ksteps = row_bytes / 256;
    int64_t s = workgroups / row_blocks;
    if (s < 1) s = 1;
    if (s > ksteps) s = ksteps;
    const int64_t per = (ksteps + s - 1) / s, slices = (ksteps + per - 1) / per;
    hipLaunchKernelGGL(read_rows_probe_kernel, dim3((unsigned)(row_blocks * slices)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const unsigned char*>(W), (int)N, (int)row_bytes, (int)row_blocks, (int)(per * 256),
                       static_cast<uint32_t*>(sink));
    if (hipGetLastError() != hipSuccess) return FHPC_ERR_HIP;
    return FHPC_OK;
}

}  // extern "C"
