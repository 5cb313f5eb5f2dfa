// Internal interface of the weight-streaming forward for a handful of tokens.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

constexpr int QSKINNY_MAX_JOBS = 4;

struct QskinnyPlan {
    int splits;            // slices of the reduction (each writes its own fp32 slab of M x (64 * row_blocks))
    int k_chunk;           // reduction depth per slice, a multiple of 512
    int kchunks;           // partial sums of H = X A, per weight
    int row_blocks;        // 64-channel blocks of all weights together
    int64_t part_bytes;    // splits * M * 64 * row_blocks * 4
    int64_t hpart_bytes;   // count * kchunks * M * r * 4
};

// One weight of a launch: Y[M,N] bf16 = base_scale X deq(Wq) + scaling (X A) B;  H_out (M x r bf16) optional.
// A is [K][r], B is [r][N] (unpadded).
struct QskinnyJob {
    const void* Wq;
    const void* scales;
    const void* A;
    const void* B;
    void* Y;
    void* H_out;
    int64_t N;
    float base_scale, scaling;
};

// M <= 64 tokens, r <= 64, K a multiple of 512, scheme 4 (block 64) or 8.
bool qskinny_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme);
// `count` weights (at most QSKINNY_MAX_JOBS) with output widths N[0..count) that share X, K and r
QskinnyPlan qskinny_plan(int64_t M, int64_t K, int64_t r, const int64_t* N, int count, int num_cu);

// All weights in one launch pair.  part and hpart are scratch of the plan's sizes.
hipError_t launch_qskinny_fwd(const void* X, const QskinnyJob* jobs, int count, int scheme, int64_t M, int64_t K, int64_t r,
                              const QskinnyPlan& p, float* part, float* hpart, hipStream_t st);

}  // namespace fhpc
