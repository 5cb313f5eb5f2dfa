// Internal launchers for the non-MFMA kernels.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

hipError_t launch_gemm_f32(const float* A, int64_t ars, int64_t acs, const float* B, int64_t brs, int64_t bcs,
                           float* C, int64_t ldc, int M, int N, int K, float alpha, hipStream_t s);
// Two chained fp32 products with the rank-r intermediate kept in LDS (r <= 64), see kernels_misc.hip:
// P = L R (M x r, also stored to P_out when given), Out = P S (M x C).
bool lowrank_chain_f32_supports(int64_t r);
hipError_t launch_lowrank_chain_f32(const float* L, int64_t ldl, const float* R, int64_t rrs, int64_t rcs,
                                    const float* S, int64_t srs, int64_t scs, float* Out, int64_t ldo, float* P_out,
                                    int M, int T, int r, int C, hipStream_t s);
hipError_t launch_swiglu_fwd(const void* G, const void* U, void* Z, int64_t n, bool bf16, hipStream_t s);
hipError_t launch_swiglu_bwd(const void* G, const void* U, const void* dZ, void* dG, void* dU, int64_t n,
                             bool bf16, hipStream_t s);
hipError_t launch_add(const void* a, const void* b, void* out, int64_t n, bool bf16, hipStream_t s);
hipError_t launch_unpack(const void* Wq, int scheme, int8_t* q, int64_t K, int64_t N, hipStream_t s);
hipError_t launch_dequant(const void* Wq, const void* scales, int scheme, int64_t block, float* out,
                          int64_t K, int64_t N, hipStream_t s);
// int8: `scratch` holds ceil(K / 64) * N floats (partial column maxima); unused for the 4-bit scheme.
hipError_t launch_quantize(const float* W, int scheme, int64_t block, void* Wq, void* scales,
                           int64_t K, int64_t N, float* scratch, hipStream_t s);
hipError_t launch_pad2d_u16(const void* src, int64_t ld_src, int64_t rows_src, int64_t cols_src,
                            void* dst, int64_t ld_dst, int64_t rows_dst, hipStream_t s);
hipError_t launch_compact_f32(const float* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int64_t cols,
                              float scale, bool to_bf16, hipStream_t s);
// out: fp32, or bf16 when to_bf16 (n a multiple of 4)
hipError_t launch_sum_slabs(const float* slabs, int64_t n, int nslab, void* out, bool to_bf16, hipStream_t s);
// Two fp32 slab sums in one launch, bit for bit the sums launch_sum_slabs forms; for sums launch_sum_slabs would not
// hand to its wide kernel (sum_slabs_is_small).
// P[M][rp] bf16 = L[M][Kred] (row stride ldl) * R[rp][Kred]^T (row stride ldr), rp <= 32, Kred a multiple of 32, the strides multiples of 8,
// 16-byte aligned rows: one launch without partial-sum slabs, for outputs of many rows.
hipError_t launch_tall_skinny_kc(const void* L, int64_t ldl, const void* R, int64_t ldr, void* P, int64_t M, int64_t rp,
                                 int64_t Kred, hipStream_t s);
bool sum_slabs_is_small(int64_t n, int nslab);
hipError_t launch_sum_slabs_pair(const float* slabs0, int64_t n0, int nslab0, float* out0,
                                 const float* slabs1, int64_t n1, int nslab1, float* out1, hipStream_t s);
// C = A' B in fp32 on the matrix cores, A' = A or A^T; dimensions multiples of 4, rows 16-byte aligned
hipError_t launch_mm_f32(const float* A, bool transpose_a, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                         int64_t M, int64_t N, int64_t K, hipStream_t s);
// r x r helpers of the rank-r factorisation (see kernels_misc.hip)
hipError_t launch_gram_poly(const float* G, const float* G2, void* out, bool to_bf16, int64_t r, float a, float b, float c, int mode, hipStream_t s);
hipError_t launch_neumann(const float* G, const void* E2, const void* E3, void* out, int64_t r, hipStream_t s);
hipError_t launch_add_f32_bf16(const float* a, const void* b, void* out, int64_t n, hipStream_t s);
hipError_t launch_zero(void* p, int64_t bytes, hipStream_t s);
// Rank-r weight gradients from at most 64 tokens, both in one launch (either output may be NULL):
//   dA[k][j] = alpha sum_m X[m][k] dH[m][j]  (fp32 [K][r]),   dB[j][n] = alpha sum_m H[m][j] dY[m][n]  (fp32 [r][N]).
// X [M][K], dY [M][N], dH and H [M][rp] are bf16; any rank; tiles of the outputs, a 4 x 4 patch per thread.
bool token_outer_supports(int64_t M);
hipError_t launch_token_outer_grads(const void* X, const void* dH, float* dA, const void* H, const void* dY, float* dB,
                                    int64_t M, int64_t K, int64_t r, int64_t rp, int64_t N, float alpha, hipStream_t s);

}  // namespace fhpc
