// fp32 GEMM (true fp32 arithmetic), SiLU gate, weight quantise / unpack / dequantise,
// and the small copy / convert kernels the entry points use around the GEMM core.
#include "kernels_misc.h"
#include "gate_math.h"
#include "profile.h"

#include <type_traits>

namespace fhpc {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b << 16); }

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    f32x2 v;
    v.x = f;
    v.y = 0.f;
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return (uint16_t)(__builtin_bit_cast(uint32_t, b) & 0xFFFFu);
}

// ---------------------------------------------------------------------------------
// fp32 GEMM with arbitrary strides: C[m,n] = alpha * sum_k A(m,k) B(k,n),
// A(m,k) = A[m*ars + k*acs], B(k,n) = B[k*brs + n*bcs].  64x64 tile, 16-deep steps,
// 256 threads, each a 4x4 block of C, plain v_fma_f32 (no reduced-precision path).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t ars, int64_t acs,
                                                       const float* __restrict__ B, int64_t brs, int64_t bcs,
                                                       float* __restrict__ C, int64_t ldc, int M, int N, int K, float alpha)
{
    __shared__ float sA[16][64 + 4];
    __shared__ float sB[16][64 + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    // element i of this thread in the A and B tiles: the faster-varying thread index follows the contiguous stride
    int amm[4], akk[4], bnn[4], bkk[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int e = tid + 256 * i;
        if (acs == 1) { akk[i] = e & 15; amm[i] = e >> 4; } else { amm[i] = e & 63; akk[i] = e >> 6; }
        if (brs == 1) { bkk[i] = e & 15; bnn[i] = e >> 4; } else { bnn[i] = e & 63; bkk[i] = e >> 6; }
    }
    // the next 16-deep step's operands are requested before the current step's sums, so that a step does not wait
    // out a round trip to memory (the products of the fp32 configuration are small: the latency was all they took)
    float ra[4], rb[4];
    auto fetch = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int m = m0 + amm[i], k = k0 + akk[i];
            ra[i] = (m < M && k < K) ? A[(int64_t)m * ars + (int64_t)k * acs] : 0.f;
            const int n = n0 + bnn[i], k2 = k0 + bkk[i];
            rb[i] = (n < N && k2 < K) ? B[(int64_t)k2 * brs + (int64_t)n * bcs] : 0.f;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            sA[akk[i]][amm[i]] = ra[i];
            sB[bkk[i]][bnn[i]] = rb[i];
        }
        __syncthreads();
        if (k0 + 16 < K) fetch(k0 + 16);
#pragma unroll
        for (int kk = 0; kk < 16; kk++) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; j++) b[j] = sB[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int m = m0 + ty * 4 + i;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int n = n0 + tx * 4 + j;
            if (m < M && n < N) C[(int64_t)m * ldc + n] = alpha * acc[i][j];
        }
    }
}

hipError_t launch_gemm_f32(const float* A, int64_t ars, int64_t acs, const float* B, int64_t brs, int64_t bcs,
                           float* C, int64_t ldc, int M, int N, int K, float alpha, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, A, ars, acs, B, brs, bcs, C, ldc, M, N, K, alpha);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Two chained fp32 products through a rank that fits a workgroup's LDS (r <= 64):
//     P[m][j]   = sum_t L[m][t] R(t, j)          R(t, j) = R[t * rrs + j * rcs]
//     Out[m][c] = sum_j P[m][j] S(j, c)          S(j, c) = S[j * srs + c * scs]
// for 16 rows m per workgroup.  Forward of the factorised layer (Sec. 3.2 eq. low_rank_layer): L = X, R = A,
// S = B gives H = X A and Y = H B; its input gradient: L = dY, R = B (transposed through the strides),
// S = A gives dH = dY B^T and dX = dH A^T.  The rank-r intermediate stays in LDS between the two
// products (it is also stored to P_out when the caller wants it: H for the backward pass, dH for dA); each
// sum runs in index order, in fp32.
// ---------------------------------------------------------------------------------
constexpr int CHAIN_ROWS = 16, CHAIN_TC = 64, CHAIN_RMAX = 64;

__global__ __launch_bounds__(256) void lowrank_chain_f32_kernel(const float* __restrict__ L, int64_t ldl,
                                                                const float* __restrict__ R, int64_t rrs, int64_t rcs,
                                                                const float* __restrict__ S, int64_t srs, int64_t scs,
                                                                float* __restrict__ Out, int64_t ldo, float* __restrict__ P_out,
                                                                int M, int T, int r, int C)
{
    __shared__ float sL[CHAIN_ROWS][CHAIN_TC + 1];
    __shared__ float sR[CHAIN_TC][CHAIN_RMAX + 1];
    __shared__ float sP[CHAIN_ROWS][CHAIN_RMAX + 1];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.x * CHAIN_ROWS;
    const int row = tid >> 4, jg = tid & 15;          // thread: one row, the ranks jg, jg + 16, jg + 32, jg + 48
    float h[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < T; t0 += CHAIN_TC) {
        // the rows' next 64 elements (contiguous along t) ...
#pragma unroll
        for (int i = 0; i < CHAIN_ROWS * CHAIN_TC / 256; i++) {
            const int e = tid + 256 * i, rr = e / CHAIN_TC, tt = e % CHAIN_TC;
            const int m = m0 + rr, t = t0 + tt;
            sL[rr][tt] = (m < M && t < T) ? L[(int64_t)m * ldl + t] : 0.f;
        }
        // ... and the 64 x r piece of R, read along whichever of its indices is contiguous
        for (int e = tid; e < CHAIN_TC * r; e += 256) {
            int tt, j;
            if (rcs == 1) { tt = e / r; j = e - tt * r; } else { j = e / CHAIN_TC; tt = e - j * CHAIN_TC; }
            const int t = t0 + tt;
            sR[tt][j] = (t < T) ? R[(int64_t)t * rrs + (int64_t)j * rcs] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int tt = 0; tt < CHAIN_TC; tt++) {
            const float x = sL[row][tt];
#pragma unroll
            for (int c = 0; c < 4; c++) h[c] = __builtin_fmaf(x, sR[tt][jg + 16 * c], h[c]);     // (ranks beyond r: zero columns of sR are never read back)
        }
        __syncthreads();
    }
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const int j = jg + 16 * c;
        if (j < r) {
            sP[row][j] = h[c];
            if (P_out && m0 + row < M) P_out[(int64_t)(m0 + row) * r + j] = h[c];
        }
    }
    __syncthreads();
    // second product: a thread owns output columns c = tid, tid + 256, ... for all 16 rows
    for (int c = tid; c < C; c += 256) {
        float acc[CHAIN_ROWS];
#pragma unroll
        for (int rr = 0; rr < CHAIN_ROWS; rr++) acc[rr] = 0.f;
        for (int j = 0; j < r; j++) {
            const float b = S[(int64_t)j * srs + (int64_t)c * scs];
#pragma unroll
            for (int rr = 0; rr < CHAIN_ROWS; rr++) acc[rr] = __builtin_fmaf(sP[rr][j], b, acc[rr]);
        }
#pragma unroll
        for (int rr = 0; rr < CHAIN_ROWS; rr++)
            if (m0 + rr < M) Out[(int64_t)(m0 + rr) * ldo + c] = acc[rr];
    }
}

bool lowrank_chain_f32_supports(int64_t r) { return r >= 1 && r <= CHAIN_RMAX; }

hipError_t launch_lowrank_chain_f32(const float* L, int64_t ldl, const float* R, int64_t rrs, int64_t rcs,
                                    const float* S, int64_t srs, int64_t scs, float* Out, int64_t ldo, float* P_out,
                                    int M, int T, int r, int C, hipStream_t s)
{
    if (M <= 0 || C <= 0) return hipSuccess;
    if (!lowrank_chain_f32_supports(r)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lowrank_chain_f32_kernel, dim3((unsigned)((M + CHAIN_ROWS - 1) / CHAIN_ROWS)), dim3(256), 0, s,
                       L, ldl, R, rrs, rcs, S, srs, scs, Out, ldo, P_out, M, T, r, C);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// SiLU gate (Sec. 3.1 eq. FFN): fp32 arithmetic on bf16 or fp32 storage.
// ---------------------------------------------------------------------------------

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, int64_t i)
{
    if constexpr (BF16) return bf16_bits_to_float(reinterpret_cast<const uint16_t*>(p)[i]);
    else return reinterpret_cast<const float*>(p)[i];
}
template <bool BF16>
__device__ __forceinline__ void store_elem(void* p, int64_t i, float v)
{
    if constexpr (BF16) reinterpret_cast<uint16_t*>(p)[i] = float_to_bf16_bits(v);
    else reinterpret_cast<float*>(p)[i] = v;
}

// bf16 storage moves 16 bytes (8 elements) per lane per access; the last n % 8 elements are
// handled one by one.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi)
{
    f32x2 v;
    v.x = lo;
    v.y = hi;
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

template <bool BF16>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const void* G, const void* U, void* Z, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t done = 0;
    if constexpr (BF16) {
        const int64_t n8 = n / 8;
        for (int64_t i = tid; i < n8; i += stride) {
            const u32x4_t g = reinterpret_cast<const u32x4_t*>(G)[i], u = reinterpret_cast<const u32x4_t*>(U)[i];
            u32x4_t z;
#pragma unroll
            for (int e = 0; e < 4; e++) z[e] = gate::fwd_pair(g[e], u[e]);
            reinterpret_cast<u32x4_t*>(Z)[i] = z;
        }
        done = n8 * 8;
    }
    for (int64_t i = done + tid; i < n; i += stride) {
        store_elem<BF16>(Z, i, gate::fwd(load_elem<BF16>(G, i), load_elem<BF16>(U, i)));
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const void* G, const void* U, const void* dZ,
                                                         void* dG, void* dU, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t done = 0;
    if constexpr (BF16) {
        const int64_t n8 = n / 8;
        for (int64_t i = tid; i < n8; i += stride) {
            const u32x4_t g = reinterpret_cast<const u32x4_t*>(G)[i], u = reinterpret_cast<const u32x4_t*>(U)[i];
            const u32x4_t dz = reinterpret_cast<const u32x4_t*>(dZ)[i];
            u32x4_t og, ou;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                uint32_t a, b;
                gate::bwd_pair(g[e], u[e], dz[e], a, b);
                og[e] = a;
                ou[e] = b;
            }
            reinterpret_cast<u32x4_t*>(dU)[i] = ou;
            reinterpret_cast<u32x4_t*>(dG)[i] = og;
        }
        done = n8 * 8;
    }
    for (int64_t i = done + tid; i < n; i += stride) {
        float dg, du;
        gate::bwd(load_elem<BF16>(G, i), load_elem<BF16>(U, i), load_elem<BF16>(dZ, i), dg, du);
        store_elem<BF16>(dU, i, du);
        store_elem<BF16>(dG, i, dg);
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void add_kernel(const void* a, const void* b, void* out, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t done = 0;
    if constexpr (BF16) {
        const int64_t n8 = n / 8;
        for (int64_t i = tid; i < n8; i += stride) {
            const u32x4_t x = reinterpret_cast<const u32x4_t*>(a)[i], y = reinterpret_cast<const u32x4_t*>(b)[i];
            u32x4_t o;
#pragma unroll
            for (int e = 0; e < 4; e++) o[e] = bf16_pack(bf16_lo(x[e]) + bf16_lo(y[e]), bf16_hi(x[e]) + bf16_hi(y[e]));
            reinterpret_cast<u32x4_t*>(out)[i] = o;
        }
        done = n8 * 8;
    }
    for (int64_t i = done + tid; i < n; i += stride)
        store_elem<BF16>(out, i, load_elem<BF16>(a, i) + load_elem<BF16>(b, i));
}

static unsigned grid_for(int64_t n)
{
    int64_t b = (n + 255) / 256;            // one element per thread and trip
    return (unsigned)(b < 1 ? 1 : (b > 8192 ? 8192 : b));
}

// for the kernels that move 8 bf16 elements (16 bytes) per thread and trip
static unsigned grid_for8(int64_t n, bool bf16)
{
    return grid_for(bf16 ? (n + 7) / 8 : n);
}

hipError_t launch_swiglu_fwd(const void* G, const void* U, void* Z, int64_t n, bool bf16, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int slot = prof_begin("swiglu_fwd", 0.0, 3.0 * n * (bf16 ? 2 : 4), s);
    if (bf16) hipLaunchKernelGGL(swiglu_fwd_kernel<true>, dim3(grid_for8(n, true)), dim3(256), 0, s, G, U, Z, n);
    else hipLaunchKernelGGL(swiglu_fwd_kernel<false>, dim3(grid_for(n)), dim3(256), 0, s, G, U, Z, n);
    prof_end(slot, s);
    return hipGetLastError();
}

hipError_t launch_add(const void* a, const void* b, void* out, int64_t n, bool bf16, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(add_kernel<true>, dim3(grid_for8(n, true)), dim3(256), 0, s, a, b, out, n);
    else hipLaunchKernelGGL(add_kernel<false>, dim3(grid_for(n)), dim3(256), 0, s, a, b, out, n);
    return hipGetLastError();
}

hipError_t launch_swiglu_bwd(const void* G, const void* U, const void* dZ, void* dG, void* dU, int64_t n,
                             bool bf16, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int slot = prof_begin("swiglu_bwd", 0.0, 5.0 * n * (bf16 ? 2 : 4), s);
    if (bf16) hipLaunchKernelGGL(swiglu_bwd_kernel<true>, dim3(grid_for8(n, true)), dim3(256), 0, s, G, U, dZ, dG, dU, n);
    else hipLaunchKernelGGL(swiglu_bwd_kernel<false>, dim3(grid_for(n)), dim3(256), 0, s, G, U, dZ, dG, dU, n);
    prof_end(slot, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Weight codes: unpack, dequantise, quantise (Sec. 5.2).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpack_int4_kernel(const uint8_t* __restrict__ p, int8_t* __restrict__ q, int64_t nbytes)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nbytes; i += stride) {
        const int b = p[i];
        q[2 * i] = (int8_t)__builtin_amdgcn_sbfe(b, 0, 4);
        q[2 * i + 1] = (int8_t)__builtin_amdgcn_sbfe(b, 4, 4);
    }
}

__global__ __launch_bounds__(256) void copy_bytes_kernel(const uint8_t* __restrict__ p, uint8_t* __restrict__ q, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) q[i] = p[i];
}

hipError_t launch_unpack(const void* Wq, int scheme, int8_t* q, int64_t K, int64_t N, hipStream_t s)
{
    if (scheme == 8) {
        const int64_t n = K * N;
        hipLaunchKernelGGL(copy_bytes_kernel, dim3(grid_for(n)), dim3(256), 0, s, (const uint8_t*)Wq, (uint8_t*)q, n);
    } else {
        const int64_t n = K * N / 2;
        hipLaunchKernelGGL(unpack_int4_kernel, dim3(grid_for(n)), dim3(256), 0, s, (const uint8_t*)Wq, q, n);
    }
    return hipGetLastError();
}

// W_out[n][k] = code * scale, exact in fp32 (at most 8 + 11 significant bits).  A thread takes eight
// consecutive k of one row (K is a multiple of 8, and of the block for the 4-bit scheme, so the
// eight share one scale): 4 or 8 bytes of codes in, 32 bytes out.
template <int SCHEME>
__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* __restrict__ Wq, const uint16_t* __restrict__ scales,
                                                      int64_t block, float* __restrict__ out, int64_t K, int64_t N)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    const int64_t per_row = K / 8, total = per_row * N;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int64_t n = i / per_row, k = (i - n * per_row) * 8;
        int q[8];
        float sc;
        if (SCHEME == 8) {
            const u32x2_t w = *reinterpret_cast<const u32x2_t*>(Wq + n * K + k);
#pragma unroll
            for (int e = 0; e < 4; e++) {
                q[e] = (int)__builtin_amdgcn_sbfe(w.x, 8 * e, 8);
                q[4 + e] = (int)__builtin_amdgcn_sbfe(w.y, 8 * e, 8);
            }
            sc = (float)__builtin_bit_cast(_Float16, scales[n]);
        } else {
            const uint32_t w = *reinterpret_cast<const uint32_t*>(Wq + n * (K / 2) + k / 2);
#pragma unroll
            for (int e = 0; e < 8; e++) q[e] = (int)__builtin_amdgcn_sbfe(w, 4 * e, 4);     // element k even in the low nibble
            sc = (float)__builtin_bit_cast(_Float16, scales[n * (K / block) + k / block]);
        }
        f32x4_t lo = {(float)q[0] * sc, (float)q[1] * sc, (float)q[2] * sc, (float)q[3] * sc};
        f32x4_t hi = {(float)q[4] * sc, (float)q[5] * sc, (float)q[6] * sc, (float)q[7] * sc};
        float* dst = out + n * K + k;
        *reinterpret_cast<f32x4_t*>(dst) = lo;
        *reinterpret_cast<f32x4_t*>(dst + 4) = hi;
    }
}

hipError_t launch_dequant(const void* Wq, const void* scales, int scheme, int64_t block, float* out,
                          int64_t K, int64_t N, hipStream_t s)
{
    // algorithmic bytes: the packed codes and scales in, fp32 out
    const double in_bytes = (scheme == 4) ? K * N * 0.5 + 2.0 * N * (K / block) : (double)K * N + 2.0 * N;
    const int slot = prof_begin(scheme == 4 ? "qweight_dequant<int4>" : "qweight_dequant<int8>", 0.0, in_bytes + 4.0 * K * N, s);
    if (scheme == 4)
        hipLaunchKernelGGL(dequant_kernel<4>, dim3(grid_for(K * N / 8)), dim3(256), 0, s, (const uint8_t*)Wq,
                           (const uint16_t*)scales, block, out, K, N);
    else
        hipLaunchKernelGGL(dequant_kernel<8>, dim3(grid_for(K * N / 8)), dim3(256), 0, s, (const uint8_t*)Wq,
                           (const uint16_t*)scales, block, out, K, N);
    prof_end(slot, s);
    return hipGetLastError();
}

// Quantiser (Sec. 5.2: one scale per weight vector; here symmetric absmax).  W is [K][N] fp32 with n
// contiguous, the codes are [N][K] with k contiguous, so this is a transposing pass.  The work is cut
// into tiles of 64 k x 64 output channels so that thousands of workgroups stream W at once:
// 256 threads = 64 columns x 4 k-lanes, rows of W read 256 bytes at a time, each thread keeps its 16
// values in registers; the codes pass through LDS and leave as 8-byte stores, 16 codes of one channel
// per thread (with byte stores the same kernels ran at two thirds of the speed).  Small tiles on
// purpose: a thread cannot produce a code before the whole weight vector's absmax is known, so loads and
// arithmetic overlap only across waves, and 64-deep blocks per thread (fewer, fatter waves with wider
// loads) measured 149-157 us against 87 us on a 5120 x 13824 weight.
//   4-bit, block 64: a tile is exactly one weight vector per column: absmax, scale, codes.
//   int8 per channel: the vector is the whole column, so the column maxima come first
//   (absmax_rows_kernel -> partial maxima, column_scale_kernel -> fp16 scales) and the code
//   kernel then reads the finished scale: two passes over W.
// Arithmetic per element, identical in both: scale = fp16_rne(absmax / qmax) with an fp32
// divide; q = clamp(rint(w / float(scale)), -qmax, qmax), 0 when the scale is 0.
constexpr int QT = 64;

template <int QMAX>
__device__ __forceinline__ int quantize_code(float w, float sf)
{
    if (sf == 0.f) return 0;
    float t = rintf(w / sf);
    t = fminf(fmaxf(t, -(float)QMAX), (float)QMAX);
    return (int)t;
}

__device__ __forceinline__ void load_tile_column(const float* __restrict__ W, int64_t K, int64_t N, int64_t k0, int64_t n,
                                                 int kl, float (&w)[16])
{
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const int64_t k = k0 + kl + 4 * i;
        w[i] = (n < N && k < K) ? W[k * N + n] : 0.f;
    }
}

// codes of one tile: thread (col, kl) holds k = kl + 4 i; they pass through LDS so that thread
// (channel r, piece) then owns 16 consecutive codes of one channel: 8 bytes packed (4-bit), or two
// 8-byte halves (int8; K is a multiple of 8, so a half is inside the row or not at all)
template <int QMAX, bool PACK4>
__device__ __forceinline__ void store_tile_codes(const float (&w)[16], float sf, uint8_t* __restrict__ Wq, int64_t K, int64_t N,
                                                 int64_t k0, int64_t n0, uint8_t (&s_code)[QT][QT + 8])
{
    const int col = threadIdx.x & 63, kl = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 16; i++) s_code[col][kl + 4 * i] = (uint8_t)quantize_code<QMAX>(w[i], sf);
    __syncthreads();
    const int r = threadIdx.x >> 2, piece = threadIdx.x & 3;     // 16 codes of channel n0 + r
    const int64_t nn = n0 + r, kbase = k0 + piece * 16;
    if (nn >= N) return;
    const uint64_t lo = *reinterpret_cast<const uint64_t*>(&s_code[r][piece * 16]);
    const uint64_t hi = *reinterpret_cast<const uint64_t*>(&s_code[r][piece * 16 + 8]);
    if (PACK4) {
        // element k even in the low nibble of byte k / 2
        auto pack8 = [](uint64_t v) {                            // eight code bytes -> four packed bytes
            uint32_t out = 0;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const uint32_t b0 = (uint32_t)(v >> (16 * e)) & 0xFu, b1 = (uint32_t)(v >> (16 * e + 8)) & 0xFu;
                out |= (b0 | (b1 << 4)) << (8 * e);
            }
            return out;
        };
        if (kbase < K)                                           // K is a multiple of 64: all 16 codes or none
            *reinterpret_cast<uint64_t*>(Wq + nn * (K / 2) + kbase / 2) = (uint64_t)pack8(lo) | ((uint64_t)pack8(hi) << 32);
    } else {
        uint8_t* dst = Wq + nn * K + kbase;
        if (kbase < K) *reinterpret_cast<uint64_t*>(dst) = lo;
        if (kbase + 8 < K) *reinterpret_cast<uint64_t*>(dst + 8) = hi;
    }
}

// 4-bit, block 64: grid (N / 64, K / 64)
__global__ __launch_bounds__(256) void quantize_int4_kernel(const float* __restrict__ W, uint8_t* __restrict__ Wq,
                                                            uint16_t* __restrict__ scales, int64_t K, int64_t N)
{
    __shared__ float s_max[4][QT];
    __shared__ __attribute__((aligned(8))) uint8_t s_code[QT][QT + 8];
    const int col = threadIdx.x & 63, kl = threadIdx.x >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * QT, k0 = (int64_t)blockIdx.y * QT;
    const int64_t n = n0 + col;
    float w[16];
    load_tile_column(W, K, N, k0, n, kl, w);
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) a = fmaxf(a, fabsf(w[i]));
    s_max[kl][col] = a;
    __syncthreads();
    a = fmaxf(fmaxf(s_max[0][col], s_max[1][col]), fmaxf(s_max[2][col], s_max[3][col]));
    const _Float16 hs = (_Float16)(a / 7.f);                // round to nearest even
    if (n < N && kl == 0) scales[n * (K / QT) + blockIdx.y] = __builtin_bit_cast(uint16_t, hs);
    store_tile_codes<7, true>(w, (float)hs, Wq, K, N, k0, n0, s_code);
}

// int8 per channel, step 1: pmax[slice][n] = max |W| over the slice's 64 rows k.  Nothing is transposed
// here, so the pass reads W the way it lies: a thread owns four neighbouring columns, a workgroup
// 4 KB of every row of its slice (the tiled pattern of the code kernels reads cold data at about half
// the rate of this one).  grid (ceil(N / 1024), ceil(K / 64)); N is a multiple of 8.
__global__ __launch_bounds__(256) void absmax_rows_kernel(const float* __restrict__ W, float* __restrict__ pmax, int64_t K, int64_t N)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    const int64_t n = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4, k0 = (int64_t)blockIdx.y * QT;
    if (n >= N) return;
    f32x4_t a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 16
    for (int t = 0; t < QT; t++) {
        const int64_t k = k0 + t;
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(W + (k < K ? k : K - 1) * N + n);   // (a repeated row changes no maximum)
        a.x = fmaxf(a.x, fabsf(v.x));
        a.y = fmaxf(a.y, fabsf(v.y));
        a.z = fmaxf(a.z, fabsf(v.z));
        a.w = fmaxf(a.w, fabsf(v.w));
    }
    *reinterpret_cast<f32x4_t*>(pmax + (int64_t)blockIdx.y * N + n) = a;
}

// step 2: scale[n] = fp16(max over tile rows / 127)
__global__ __launch_bounds__(256) void column_scale_kernel(const float* __restrict__ pmax, int64_t rows, int64_t N, uint16_t* __restrict__ scales)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float a = 0.f;
    for (int64_t r0 = 0; r0 < rows; r0 += 8) {           // eight loads in flight (a row past the end repeats row r0)
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; q++) v[q] = pmax[(r0 + q < rows ? r0 + q : r0) * N + n];
#pragma unroll
        for (int q = 0; q < 8; q++) a = fmaxf(a, v[q]);
    }
    const _Float16 hs = (_Float16)(a / 127.f);
    scales[n] = __builtin_bit_cast(uint16_t, hs);
}

// step 3: codes with the finished scales; grid (N / 64, K / 64)
__global__ __launch_bounds__(256) void quantize_int8_kernel(const float* __restrict__ W, const uint16_t* __restrict__ scales,
                                                            uint8_t* __restrict__ Wq, int64_t K, int64_t N)
{
    __shared__ __attribute__((aligned(8))) uint8_t s_code[QT][QT + 8];
    const int col = threadIdx.x & 63, kl = threadIdx.x >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * QT, k0 = (int64_t)blockIdx.y * QT;
    const int64_t n = n0 + col;
    float w[16];
    load_tile_column(W, K, N, k0, n, kl, w);
    const float sf = (n < N) ? (float)__builtin_bit_cast(_Float16, scales[n]) : 0.f;
    store_tile_codes<127, false>(w, sf, Wq, K, N, k0, n0, s_code);
}

// `scratch` (int8 only): (K / 64 rounded up) * N floats for the partial maxima.
hipError_t launch_quantize(const float* W, int scheme, int64_t block, void* Wq, void* scales,
                           int64_t K, int64_t N, float* scratch, hipStream_t s)
{
    (void)block;
    const dim3 grid((unsigned)((N + QT - 1) / QT), (unsigned)((K + QT - 1) / QT));
    // algorithmic bytes: W once in, codes and scales out (the int8 path reads W a second time for the
    // codes, after the column maxima; that second pass is not credited)
    if (scheme == 4) {
        const int slot = prof_begin("qweight_quantize<int4>", 0.0, 4.0 * K * N + 0.5 * K * N + 2.0 * N * (K / 64), s);
        hipLaunchKernelGGL(quantize_int4_kernel, grid, dim3(256), 0, s, W, (uint8_t*)Wq, (uint16_t*)scales, K, N);
        prof_end(slot, s);
        return hipGetLastError();
    }
    const int slot = prof_begin("qweight_quantize<int8>", 0.0, 4.0 * K * N + 1.0 * K * N + 2.0 * N, s);
    hipLaunchKernelGGL(absmax_rows_kernel, dim3((unsigned)((N + 1023) / 1024), grid.y), dim3(256), 0, s, W, scratch, K, N);
    hipLaunchKernelGGL(column_scale_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, scratch, (int64_t)grid.y, N, (uint16_t*)scales);
    hipLaunchKernelGGL(quantize_int8_kernel, grid, dim3(256), 0, s, W, (const uint16_t*)scales, (uint8_t*)Wq, K, N);
    prof_end(slot, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Copies around the GEMM core
// ---------------------------------------------------------------------------------
// dst[rows_dst][ld_dst] (16-bit elements) = src[rows_src][cols_src] zero-extended.
__global__ __launch_bounds__(256) void pad2d_u16_kernel(const uint16_t* __restrict__ src, int64_t ld_src, int64_t rows_src, int64_t cols_src,
                                                        uint16_t* __restrict__ dst, int64_t ld_dst, int64_t rows_dst)
{
    const int64_t total = rows_dst * ld_dst;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int64_t r = i / ld_dst, c = i % ld_dst;
        dst[i] = (r < rows_src && c < cols_src) ? src[r * ld_src + c] : (uint16_t)0;
    }
}

hipError_t launch_pad2d_u16(const void* src, int64_t ld_src, int64_t rows_src, int64_t cols_src,
                            void* dst, int64_t ld_dst, int64_t rows_dst, hipStream_t s)
{
    const int64_t total = rows_dst * ld_dst;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(pad2d_u16_kernel, dim3(grid_for(total)), dim3(256), 0, s, (const uint16_t*)src, ld_src, rows_src, cols_src,
                       (uint16_t*)dst, ld_dst, rows_dst);
    return hipGetLastError();
}

// dst[rows][cols] (dense) = scale * src[rows][ld_src] (first cols columns); fp32 -> fp32 or bf16.
template <bool TO_BF16>
__global__ __launch_bounds__(256) void compact_f32_kernel(const float* __restrict__ src, int64_t ld_src, void* __restrict__ dst,
                                                          int64_t ld_dst, int64_t rows, int64_t cols, float scale)
{
    const int64_t total = rows * cols;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int64_t r = i / cols, c = i % cols;
        const float v = src[r * ld_src + c] * scale;
        if constexpr (TO_BF16) reinterpret_cast<uint16_t*>(dst)[r * ld_dst + c] = float_to_bf16_bits(v);
        else reinterpret_cast<float*>(dst)[r * ld_dst + c] = v;
    }
}

hipError_t launch_compact_f32(const float* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int64_t cols,
                              float scale, bool to_bf16, hipStream_t s)
{
    const int64_t total = rows * cols;
    if (total <= 0) return hipSuccess;
    if (to_bf16) hipLaunchKernelGGL(compact_f32_kernel<true>, dim3(grid_for(total)), dim3(256), 0, s, src, ld_src, dst, ld_dst, rows, cols, scale);
    else hipLaunchKernelGGL(compact_f32_kernel<false>, dim3(grid_for(total)), dim3(256), 0, s, src, ld_src, dst, ld_dst, rows, cols, scale);
    return hipGetLastError();
}

// out[i] = sum over s of slabs[s * slab + i]: the second half of a split reduction.  A workgroup
// covers 64 float4 outputs with four groups of threads, group g adding the slabs g, g+4, ...; the
// four partial sums are then added in group order through LDS, so the result is the same from run
// to run.  Output fp32, or bf16 for the rank-r intermediates that feed the next product.
template <bool TO_BF16>
__global__ __launch_bounds__(256) void sum_slabs_kernel(const float* __restrict__ slabs, int64_t slab, int nslab,
                                                        void* __restrict__ out, int64_t n4)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    __shared__ f32x4 red[3][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    for (int64_t base = (int64_t)blockIdx.x * 64; base < n4; base += (int64_t)gridDim.x * 64) {
        const int64_t i = base + lane;
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
        if (i < n4)
            for (int s = g; s < nslab; s += 4) a += reinterpret_cast<const f32x4*>(slabs + (int64_t)s * slab)[i];
        if (g > 0) red[g - 1][lane] = a;
        __syncthreads();
        if (g == 0 && i < n4) {
            a = ((a + red[0][lane]) + red[1][lane]) + red[2][lane];
            if constexpr (TO_BF16) {
                u32x2_t o;
                o.x = bf16_pack(a.x, a.y);
                o.y = bf16_pack(a.z, a.w);
                reinterpret_cast<u32x2_t*>(out)[i] = o;
            } else {
                reinterpret_cast<f32x4*>(out)[i] = a;
            }
        }
        __syncthreads();
    }
}

// Two small slab sums in one launch (the two rank-r weight gradients of a layer: a launch each would cost more in
// launch latency than in work).  Block b < blocks[0] belongs to the first sum, the others to the second; within a sum
// the arithmetic and its order are those of sum_slabs_kernel<false>.
struct SlabSumPair {
    const float* slabs[2];
    float* out[2];
    int64_t slab[2], n4[2];
    int nslab[2];
    int blocks[2];
};
__global__ __launch_bounds__(256) void sum_slabs_pair_kernel(SlabSumPair p)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    __shared__ f32x4 red[3][64];
    const int which = ((int)blockIdx.x < p.blocks[0]) ? 0 : 1;
    const float* const slabs = which ? p.slabs[1] : p.slabs[0];
    float* const out = which ? p.out[1] : p.out[0];
    const int64_t slab = which ? p.slab[1] : p.slab[0], n4 = which ? p.n4[1] : p.n4[0];
    const int nslab = which ? p.nslab[1] : p.nslab[0];
    const int nblocks = which ? p.blocks[1] : p.blocks[0];
    const int block = (int)blockIdx.x - (which ? p.blocks[0] : 0);
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    for (int64_t base = (int64_t)block * 64; base < n4; base += (int64_t)nblocks * 64) {
        const int64_t i = base + lane;
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
        if (i < n4)
            for (int s = g; s < nslab; s += 4) a += reinterpret_cast<const f32x4*>(slabs + (int64_t)s * slab)[i];
        if (g > 0) red[g - 1][lane] = a;
        __syncthreads();
        if (g == 0 && i < n4) {
            a = ((a + red[0][lane]) + red[1][lane]) + red[2][lane];
            reinterpret_cast<f32x4*>(out)[i] = a;
        }
        __syncthreads();
    }
}

// P[M][rp] (bf16) = L[M][Kred] * R[rp][Kred]^T for a rank-r output of many rows (rp <= 32, both operands with the
// reduction index contiguous: dH = dY B^T).  The output is too narrow for the GEMM tiles, which have to cut the
// reduction into slices and add slabs afterwards; here a workgroup owns 16 rows and the whole reduction: its eight
// waves take an eighth of it each, both operands of v_mfma_f32_16x16x32_bf16 come straight from memory as the 16
// bytes a lane needs (eight consecutive k of its row), and the partial tiles meet in LDS.  One launch, no slabs.
typedef __attribute__((ext_vector_type(8))) __bf16 ts_bf16x8;
typedef __attribute__((ext_vector_type(4))) float ts_f32x4;
constexpr int TS_UNROLL = 8, TS_WAVES = 8;
__global__ __launch_bounds__(64 * TS_WAVES) void tall_skinny_kc_kernel(const uint16_t* __restrict__ L, int64_t ldl, const uint16_t* __restrict__ R,
                                                             int64_t ldr, uint16_t* __restrict__ P, int M, int rp, int Kred)
{
    __shared__ ts_f32x4 red[TS_WAVES - 1][2][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 15, g = lane >> 4;
    const int row0 = (int)blockIdx.x * 16;
    const int steps = Kred / 32;                         // 32-deep steps of the whole reduction (Kred is a multiple of 32)
    const int per = (steps + TS_WAVES - 1) / TS_WAVES;
    const int s0 = wave * per, s1 = (s0 + per < steps) ? s0 + per : steps;
    const bool row_ok = row0 + lr < M;
    const bool r0_ok = lr < rp, r1_ok = 16 + lr < rp;
    const bool two = rp > 16;
    // Rows that do not exist read as zero through the buffer bounds; the position along k travels in the scalar
    // offset.  (A select behind every load would make the compiler wait for each load in turn.)
    constexpr uint32_t OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(L), 0, (int)((int64_t)M * ldl * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(R), 0, (int)((int64_t)rp * ldr * 2), 0x00020000);
    const uint32_t la = row_ok ? (uint32_t)((int64_t)(row0 + lr) * ldl * 2) + 16u * g : OOB;
    const uint32_t lb0 = r0_ok ? (uint32_t)((int64_t)lr * ldr * 2) + 16u * g : OOB;
    const uint32_t lb1 = r1_ok ? (uint32_t)((int64_t)(16 + lr) * ldr * 2) + 16u * g : OOB;
    ts_f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    auto batch = [&](int sb, auto NU) __attribute__((always_inline)) {
        constexpr int nu = decltype(NU)::value;
        u32x4_t a[nu], b0[nu], b1[nu];
#pragma unroll
        for (int u = 0; u < nu; u++) {
            const int kb = (sb + u) * 64;                // byte position of the 32-deep step in a row
            a[u] = __builtin_amdgcn_raw_buffer_load_b128(rl, la, kb, 0);
            b0[u] = __builtin_amdgcn_raw_buffer_load_b128(rr, lb0, kb, 0);
            if (two) b1[u] = __builtin_amdgcn_raw_buffer_load_b128(rr, lb1, kb, 0);
        }
#pragma unroll
        for (int u = 0; u < nu; u++) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(ts_bf16x8, a[u]), __builtin_bit_cast(ts_bf16x8, b0[u]), acc0, 0, 0, 0);
            if (two) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(ts_bf16x8, a[u]), __builtin_bit_cast(ts_bf16x8, b1[u]), acc1, 0, 0, 0);
        }
    };
    int sb = s0;
    for (; sb + TS_UNROLL <= s1; sb += TS_UNROLL) batch(sb, std::integral_constant<int, TS_UNROLL>{});
    for (; sb < s1; sb++) batch(sb, std::integral_constant<int, 1>{});
    if (wave > 0) {
        red[wave - 1][0][lane] = acc0;
        red[wave - 1][1][lane] = acc1;
    }
    __syncthreads();
    if (wave == 0) {
        // lane holds rows row0 + 4 g + v (from the row operand), rank lr (+ 16): the waves' shares added in wave order
#pragma unroll
        for (int w = 0; w < TS_WAVES - 1; w++) {
            acc0 += red[w][0][lane];
            acc1 += red[w][1][lane];
        }
#pragma unroll
        for (int v = 0; v < 4; v++) {
            const int m = row0 + 4 * g + v;
            if (m < M) {
                if (r0_ok) P[(int64_t)m * rp + lr] = float_to_bf16_bits(acc0[v]);
                if (r1_ok) P[(int64_t)m * rp + 16 + lr] = float_to_bf16_bits(acc1[v]);
            }
        }
    }
}

// Large outputs with few slabs: one thread per float4 output adds its slabs in order.
__global__ __launch_bounds__(256) void sum_slabs_wide_kernel(const float* __restrict__ slabs, int64_t slab, int nslab,
                                                             float* __restrict__ out, int64_t n4)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f32x4 a = reinterpret_cast<const f32x4*>(slabs)[i];
        for (int s = 1; s < nslab; s++) a += reinterpret_cast<const f32x4*>(slabs + (int64_t)s * slab)[i];
        reinterpret_cast<f32x4*>(out)[i] = a;
    }
}

// n = elements per slab, a multiple of 4 (every output here has a leading dimension that is one).
hipError_t launch_sum_slabs(const float* slabs, int64_t n, int nslab, void* out, bool to_bf16, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t n4 = n / 4;
    if (!to_bf16 && nslab <= 8 && n4 >= 65536) {
        // enough independent outputs to fill the chip with one thread each
        hipLaunchKernelGGL(sum_slabs_wide_kernel, dim3(grid_for(n4)), dim3(256), 0, s, slabs, n, nslab, (float*)out, n4);
        return hipGetLastError();
    }
    int64_t blocks = (n4 + 63) / 64;
    if (blocks > 16384) blocks = 16384;
    if (to_bf16) hipLaunchKernelGGL(sum_slabs_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, slabs, n, nslab, out, n4);
    else hipLaunchKernelGGL(sum_slabs_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, slabs, n, nslab, out, n4);
    return hipGetLastError();
}

hipError_t launch_tall_skinny_kc(const void* L, int64_t ldl, const void* R, int64_t ldr, void* P, int64_t M, int64_t rp,
                                 int64_t Kred, hipStream_t s)
{
    if (M <= 0) return hipSuccess;
    if (rp < 1 || rp > 32 || (Kred % 32) != 0 || (ldl % 8) != 0 || (ldr % 8) != 0 || M * ldl * 2 >= ((int64_t)1 << 31))
        return hipErrorInvalidValue;
    const int slot = prof_begin("tall_skinny<kc>", 2.0 * M * rp * (double)Kred, 0.0, s);
    hipLaunchKernelGGL(tall_skinny_kc_kernel, dim3((unsigned)((M + 15) / 16)), dim3(64 * TS_WAVES), 0, s, static_cast<const uint16_t*>(L), ldl,
                       static_cast<const uint16_t*>(R), ldr, static_cast<uint16_t*>(P), (int)M, (int)rp, (int)Kred);
    prof_end(slot, s);
    return hipGetLastError();
}

bool sum_slabs_is_small(int64_t n, int nslab)
{
    return !(nslab <= 8 && n / 4 >= 65536);
}

hipError_t launch_sum_slabs_pair(const float* slabs0, int64_t n0, int nslab0, float* out0,
                                 const float* slabs1, int64_t n1, int nslab1, float* out1, hipStream_t s)
{
    SlabSumPair p;
    const float* sl[2] = {slabs0, slabs1};
    float* o[2] = {out0, out1};
    const int64_t n[2] = {n0, n1};
    const int ns[2] = {nslab0, nslab1};
    for (int i = 0; i < 2; i++) {
        p.slabs[i] = sl[i]; p.out[i] = o[i]; p.slab[i] = n[i]; p.n4[i] = n[i] / 4; p.nslab[i] = ns[i];
        int64_t blocks = (p.n4[i] + 63) / 64;
        if (blocks > 8192) blocks = 8192;
        if (blocks < 1) blocks = 1;
        p.blocks[i] = (int)blocks;
    }
    hipLaunchKernelGGL(sum_slabs_pair_kernel, dim3((unsigned)(p.blocks[0] + p.blocks[1])), dim3(256), 0, s, p);
    return hipGetLastError();
}

// Zero fill with a kernel (usable inside a captured graph, unlike a memset node).
__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* __restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

// ---------------------------------------------------------------------------------
// Small r x r helpers of the rank-r factorisation (iterations that orthonormalise a tall matrix
// with matrix products only: every step is "Gram matrix -> polynomial of it -> product").
// ---------------------------------------------------------------------------------

// C[M][N] = A' B in fp32 on the matrix cores (v_mfma_f32_16x16x4_f32: fp32 operands, fp32 accumulation),
// A' = A (M x K, row-major) or A^T (A is K x M), B is K x N; all dimensions multiples of 4, rows 16-byte
// aligned.  The matrices here are a few hundred rows, so the tile is small on purpose: a workgroup covers
// 32 x 32 of the output with one 16 x 16 block per wave (a 512 x 512 product is then 1024 waves, one per
// SIMD of the chip, instead of 256 that each work four times as long).  32-deep steps are staged in LDS
// with the reduction index outermost, so that the 16 lanes of an operand read are consecutive floats; the
// row stride of 48 floats keeps the four k rows of one read on different banks.
constexpr int MMF_T = 32, MMF_K = 32, MMF_LD = 48;
template <bool TRANSPOSE_A>
__global__ __launch_bounds__(256) void mm_f32_kernel(const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb,
                                                     float* __restrict__ C, int ldc, int M, int N, int K)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    __shared__ __attribute__((aligned(16))) float As[MMF_K][MMF_LD];
    __shared__ __attribute__((aligned(16))) float Bs[MMF_K][MMF_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * MMF_T, n0 = blockIdx.x * MMF_T;
    const int wm = (wave >> 1) * 16, wn = (wave & 1) * 16;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += MMF_K) {
        // 32 x 32 floats of each operand: 256 pieces of four, one per thread
        f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
        if constexpr (TRANSPOSE_A) {
            const int k = tid >> 3, m = (tid & 7) * 4;                      // A[k][m .. m+3]
            if (k0 + k < K && m0 + m < M) a = *reinterpret_cast<const f32x4*>(A + (int64_t)(k0 + k) * lda + m0 + m);
            *reinterpret_cast<f32x4*>(&As[k][m]) = a;
        } else {
            const int m = tid >> 3, k = (tid & 7) * 4;                      // A[m][k .. k+3]
            if (m0 + m < M && k0 + k < K) a = *reinterpret_cast<const f32x4*>(A + (int64_t)(m0 + m) * lda + k0 + k);
            As[k][m] = a.x; As[k + 1][m] = a.y; As[k + 2][m] = a.z; As[k + 3][m] = a.w;
        }
        const int kb = tid >> 3, n = (tid & 7) * 4;                         // B[k][n .. n+3]
        if (k0 + kb < K && n0 + n < N) b = *reinterpret_cast<const f32x4*>(B + (int64_t)(k0 + kb) * ldb + n0 + n);
        *reinterpret_cast<f32x4*>(&Bs[kb][n]) = b;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < MMF_K; kk += 4) {
            const float av = As[kk + (lane >> 4)][wm + (lane & 15)];
            const float bv = Bs[kk + (lane >> 4)][wn + (lane & 15)];
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // lane holds column wn + lane % 16, rows wm + 4 (lane / 16) .. + 3
    const int n = n0 + wn + (lane & 15);
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const int m = m0 + wm + 4 * (lane >> 4) + v;
        if (m < M && n < N) C[(int64_t)m * ldc + n] = acc[v];
    }
}

hipError_t launch_mm_f32(const float* A, bool transpose_a, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                         int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    const dim3 grid((unsigned)((N + MMF_T - 1) / MMF_T), (unsigned)((M + MMF_T - 1) / MMF_T));
    if (transpose_a) hipLaunchKernelGGL(mm_f32_kernel<true>, grid, dim3(256), 0, s, A, (int)lda, B, (int)ldb, C, (int)ldc, (int)M, (int)N, (int)K);
    else hipLaunchKernelGGL(mm_f32_kernel<false>, grid, dim3(256), 0, s, A, (int)lda, B, (int)ldb, C, (int)ldc, (int)M, (int)N, (int)K);
    return hipGetLastError();
}

// trace of an r x r fp32 matrix, summed by one workgroup in a fixed order
__device__ __forceinline__ float block_trace(const float* __restrict__ G, int r)
{
    __shared__ float red[256];
    float t = 0.f;
    for (int i = threadIdx.x; i < r; i += 256) t += G[(int64_t)i * r + i];
    red[threadIdx.x] = t;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    return red[0];
}

// out = post * (a I + b * pre * G + c * G2), fp32 or bf16.  mode 0: pre = post = 1.  mode 1: pre = 1 / trace(G),
// post = 1.  mode 2: pre = 1 / trace(G), post = sqrt(pre) (the first step of an iteration on a matrix
// Q that has not been scaled: Q / |Q|_F has the Gram matrix G / trace(G)).  G2 (fp32) may be NULL.
template <bool TO_BF16>
__global__ __launch_bounds__(256) void gram_poly_kernel(const float* __restrict__ G, const float* __restrict__ G2,
                                                        void* __restrict__ out, int r, float a, float b, float c, int mode)
{
    float pre = 1.f, post = 1.f;
    if (mode) {
        const float t = block_trace(G, r);
        pre = (t > 0.f) ? 1.f / t : 0.f;
        if (mode == 2) post = sqrtf(pre);
    }
    const int64_t total = (int64_t)r * r;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        float v = b * pre * G[i];
        if (G2) v += c * G2[i];
        if (i / r == i % r) v += a;
        if constexpr (TO_BF16) reinterpret_cast<uint16_t*>(out)[i] = float_to_bf16_bits(post * v);
        else reinterpret_cast<float*>(out)[i] = post * v;
    }
}

hipError_t launch_gram_poly(const float* G, const float* G2, void* out, bool to_bf16, int64_t r, float a, float b, float c, int mode, hipStream_t s)
{
    if (to_bf16) hipLaunchKernelGGL(gram_poly_kernel<true>, dim3(grid_for(r * r)), dim3(256), 0, s, G, G2, out, (int)r, a, b, c, mode);
    else hipLaunchKernelGGL(gram_poly_kernel<false>, dim3(grid_for(r * r)), dim3(256), 0, s, G, G2, out, (int)r, a, b, c, mode);
    return hipGetLastError();
}

// out (bf16) = -(G - I) + E2 - E3: the first terms of the inverse of G = I + E around the identity, minus I
__global__ __launch_bounds__(256) void neumann_kernel(const float* __restrict__ G, const uint16_t* __restrict__ E2,
                                                      const uint16_t* __restrict__ E3, uint16_t* __restrict__ out, int r)
{
    const int64_t total = (int64_t)r * r;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const float e = G[i] - ((i / r == i % r) ? 1.f : 0.f);
        out[i] = float_to_bf16_bits(-e + bf16_bits_to_float(E2[i]) - bf16_bits_to_float(E3[i]));
    }
}

hipError_t launch_neumann(const float* G, const void* E2, const void* E3, void* out, int64_t r, hipStream_t s)
{
    hipLaunchKernelGGL(neumann_kernel, dim3(grid_for(r * r)), dim3(256), 0, s, G, (const uint16_t*)E2, (const uint16_t*)E3, (uint16_t*)out, (int)r);
    return hipGetLastError();
}

// out (bf16) = a (fp32) + b (bf16)
__global__ __launch_bounds__(256) void add_f32_bf16_kernel(const float* __restrict__ a, const uint16_t* __restrict__ b,
                                                           uint16_t* __restrict__ out, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        out[i] = float_to_bf16_bits(a[i] + bf16_bits_to_float(b[i]));
}

hipError_t launch_add_f32_bf16(const float* a, const void* b, void* out, int64_t n, hipStream_t s)
{
    hipLaunchKernelGGL(add_f32_bf16_kernel, dim3(grid_for(n)), dim3(256), 0, s, a, (const uint16_t*)b, (uint16_t*)out, n);
    return hipGetLastError();
}

hipError_t launch_zero(void* p, int64_t bytes, hipStream_t s)
{
    const int64_t n = bytes / 4;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_u32_kernel, dim3(grid_for(n)), dim3(256), 0, s, (uint32_t*)p, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Rank-r weight gradients from at most 64 tokens:
//   out[a][b] = alpha * sum_m U[m][a] V[m][b]      (dA: U = X, V = dH;  dB: U = H, V = dY)
// are M-deep sums, far too shallow for the matrix-core tiles, over fp32 outputs that are written once
// (and at a large rank bound by that).  A workgroup owns a 32 x 128 tile of the output,
// stages the tokens' 32 + 128 operand values as fp32 in LDS and every thread sums a 4 x 4 patch over
// the tokens; rows leave as 16-byte stores, 512 contiguous bytes per 32 lanes.  The tiles of both
// products share a launch.
// ---------------------------------------------------------------------------------
constexpr int TOG_NT = 256, TOG_A = 32, TOG_B = 128, TOG_M = 64;

struct TokenOuterJob {
    const uint16_t* U;   // bf16 [M][ldu]
    const uint16_t* V;   // bf16 [M][ldv]
    float* out;          // fp32 [na][ldo], columns < nb written
    int ldu, ldv, ldo, na, nb, tiles_b, tiles;
};

__global__ __launch_bounds__(TOG_NT) void token_outer_kernel(TokenOuterJob j0, TokenOuterJob j1, int M, float alpha)
{
    __shared__ __attribute__((aligned(16))) float Us[TOG_M][TOG_A];
    __shared__ __attribute__((aligned(16))) float Vs[TOG_M][TOG_B];
    const bool first = (int)blockIdx.x < j0.tiles;
    const TokenOuterJob j = first ? j0 : j1;
    const int t = first ? (int)blockIdx.x : (int)blockIdx.x - j0.tiles;
    const int a0 = (t / j.tiles_b) * TOG_A, b0 = (t % j.tiles_b) * TOG_B;
    const int tid = threadIdx.x;
    // stage: 4 bf16 (8 bytes) per request; leading dimensions and tile origins are multiples of 8
    for (int e = tid; e < TOG_M * (TOG_A / 4); e += TOG_NT) {
        const int m = e / (TOG_A / 4), q = (e % (TOG_A / 4)) * 4;
        uint2 w = make_uint2(0u, 0u);
        if (m < M && a0 + q < j.ldu) w = *reinterpret_cast<const uint2*>(j.U + (int64_t)m * j.ldu + a0 + q);
        Us[m][q + 0] = __uint_as_float(w.x << 16); Us[m][q + 1] = __uint_as_float(w.x & 0xFFFF0000u);
        Us[m][q + 2] = __uint_as_float(w.y << 16); Us[m][q + 3] = __uint_as_float(w.y & 0xFFFF0000u);
    }
    for (int e = tid; e < TOG_M * (TOG_B / 4); e += TOG_NT) {
        const int m = e / (TOG_B / 4), q = (e % (TOG_B / 4)) * 4;
        uint2 w = make_uint2(0u, 0u);
        if (m < M && b0 + q < j.ldv) w = *reinterpret_cast<const uint2*>(j.V + (int64_t)m * j.ldv + b0 + q);
        Vs[m][q + 0] = __uint_as_float(w.x << 16); Vs[m][q + 1] = __uint_as_float(w.x & 0xFFFF0000u);
        Vs[m][q + 2] = __uint_as_float(w.y << 16); Vs[m][q + 3] = __uint_as_float(w.y & 0xFFFF0000u);
    }
    __syncthreads();
    const int tx = tid & 31, ty = tid >> 5;      // 4 columns from tx, 4 rows from ty
    float acc[4][4] = {};
    const int mt = (M + 3) & ~3;                 // (rows past M hold zeros)
#pragma unroll 4
    for (int m = 0; m < mt; m++) {
        const float4 u = *reinterpret_cast<const float4*>(&Us[m][ty * 4]);
        const float4 v = *reinterpret_cast<const float4*>(&Vs[m][tx * 4]);
        const float uu[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            acc[i][0] = fmaf(uu[i], v.x, acc[i][0]);
            acc[i][1] = fmaf(uu[i], v.y, acc[i][1]);
            acc[i][2] = fmaf(uu[i], v.z, acc[i][2]);
            acc[i][3] = fmaf(uu[i], v.w, acc[i][3]);
        }
    }
    const int b = b0 + tx * 4;
    const bool vec = (j.ldo % 4) == 0 && b + 4 <= j.nb;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int a = a0 + ty * 4 + i;
        if (a >= j.na) continue;
        float* dst = j.out + (int64_t)a * j.ldo + b;
        if (vec) {
            *reinterpret_cast<float4*>(dst) = make_float4(alpha * acc[i][0], alpha * acc[i][1], alpha * acc[i][2], alpha * acc[i][3]);
        } else {
#pragma unroll
            for (int c = 0; c < 4; c++)
                if (b + c < j.nb) dst[c] = alpha * acc[i][c];
        }
    }
}

bool token_outer_supports(int64_t M) { return M >= 1 && M <= TOG_M; }

hipError_t launch_token_outer_grads(const void* X, const void* dH, float* dA, const void* H, const void* dY, float* dB,
                                    int64_t M, int64_t K, int64_t r, int64_t rp, int64_t N, float alpha, hipStream_t s)
{
    if (!token_outer_supports(M)) return hipErrorInvalidValue;
    auto job = [](const void* U, int64_t ldu, const void* V, int64_t ldv, float* out, int64_t ldo, int64_t na, int64_t nb) {
        TokenOuterJob j = {};
        if (!out) return j;
        j.U = static_cast<const uint16_t*>(U); j.V = static_cast<const uint16_t*>(V); j.out = out;
        j.ldu = (int)ldu; j.ldv = (int)ldv; j.ldo = (int)ldo; j.na = (int)na; j.nb = (int)nb;
        j.tiles_b = (int)((nb + TOG_B - 1) / TOG_B);
        j.tiles = (int)((na + TOG_A - 1) / TOG_A) * j.tiles_b;
        return j;
    };
    const TokenOuterJob ja = job(X, K, dH, rp, dA, r, K, r);      // dA[k][j] = sum_m X[m][k] dH[m][j]
    const TokenOuterJob jb = job(H, rp, dY, N, dB, N, r, N);      // dB[j][n] = sum_m H[m][j] dY[m][n]
    if (ja.tiles + jb.tiles == 0) return hipSuccess;
    const int slot = prof_begin("token_outer_grads", 2.0 * M * r * (double)((dA ? K : 0) + (dB ? N : 0)),
                                4.0 * r * (double)((dA ? K : 0) + (dB ? N : 0)), s);
    hipLaunchKernelGGL(token_outer_kernel, dim3((unsigned)(ja.tiles + jb.tiles)), dim3(TOG_NT), 0, s, ja, jb, (int)M, alpha);
    prof_end(slot, s);
    return hipGetLastError();
}

}  // namespace fhpc
