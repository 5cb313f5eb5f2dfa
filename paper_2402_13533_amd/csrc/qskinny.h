// Internal interface of the weight-streaming forward for a handful of tokens.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

struct QskinnyPlan {
    int splits;            // slices of the reduction (each writes its own fp32 slab of M x N)
    int k_chunk;           // reduction depth per slice, a multiple of 512
    int kchunks;           // partial sums of H = X A
    int64_t part_bytes;    // splits * M * N * 4
    int64_t hpart_bytes;   // kchunks * M * r * 4
};

// M <= 64 tokens, r <= 64, K a multiple of 512, scheme 4 (block 64) or 8.
bool qskinny_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme);
QskinnyPlan qskinny_plan(int64_t M, int64_t K, int64_t r, int64_t N, int num_cu);

// Y[M,N] bf16 = base_scale X deq(Wq) + scaling (X A) B;  H_out (M x r bf16) optional.  A is [K][r], B is [r][N]
// (unpadded).  part and hpart are scratch of the plan's sizes.
hipError_t launch_qskinny_fwd(const void* X, const void* Wq, const void* scales, int scheme, const void* A, const void* B,
                              float base_scale, float scaling, void* Y, void* H_out, int64_t M, int64_t K, int64_t r, int64_t N,
                              const QskinnyPlan& p, float* part, float* hpart, hipStream_t st);

}  // namespace fhpc
