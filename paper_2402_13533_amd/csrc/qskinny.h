// Internal interface of the weight-streaming forward for a handful of tokens.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

constexpr int QSKINNY_MAX_JOBS = 4;

struct QskinnyPlan {
    int splits;            // slices of the reduction (each writes its own fp32 slab of M x (64 * row_blocks))
    int k_chunk;           // reduction depth per slice, a multiple of the step depth (512, or 256)
    int kchunks;           // partial sums of H = X A, per weight
    int row_blocks;        // 64-channel blocks of all weights together
    int64_t part_bytes;    // splits * M * 64 * row_blocks * 4
    int64_t hpart_bytes;   // count * (kchunks + 1) * M * r * 4: the chunk sums, then H
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
    // A job may have token rows of its own (a block of the rows of a larger X goes through the launch as a job of the
    // same weight): X_own [M_own][K], M_own <= the launch's M.  NULL: the launch's X and M.
    const void* X_own = nullptr;
    int64_t M_own = 0;
};

// M <= 64 tokens, r <= 64, K a multiple of 256, scheme 4 (block 64) or 8.
bool qskinny_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme);
// `count` weights (at most QSKINNY_MAX_JOBS) with output widths N[0..count) that share X, K and r
QskinnyPlan qskinny_plan(int64_t M, int64_t K, int64_t r, const int64_t* N, int count, int num_cu);

// Words of the workspace header (QSKINNY_HEADER_BYTES at the start of every workspace) that the weight-streaming
// launches use as arrival counters.  They must be zero when a launch starts and are zero again when it ends.
constexpr int QSKINNY_HEADER_BYTES = 16384;

// All weights in one launch.  part and hpart are scratch of the plan's sizes; tickets is the workspace header.
hipError_t launch_qskinny_fwd(const void* X, const QskinnyJob* jobs, int count, int scheme, int64_t M, int64_t K, int64_t r,
                              const QskinnyPlan& p, float* part, float* hpart, uint32_t* tickets, hipStream_t st);

// ---- input gradient dX for a handful of tokens (csrc/qskinny_dx.hip)
struct QskinnyDxPlan {
    int tt;                // blocks of 16 tokens that share a pass over the codes: 1 or 2
    int strips;            // column strips of dX: K / 256 (int4 with tt = 1) or K / 128
    int token_blocks;      // workgroups along the tokens: ceil(M / (16 tt))
    int steps_total;       // 32-row steps of the weight: ceil(N / 32)
    int steps_per_slice;   // steps of one slice of the reduction
    int slices;            // slices; each writes its own fp32 slab of M x K
    int64_t part_bytes;    // slices * M * K * 4
};

// M <= 64 tokens, r <= 64, K a multiple of 256, N a multiple of 8, scheme 4 (block 64) or 8.
bool qskinny_dx_supports(int64_t M, int64_t K, int64_t r, int64_t N, int scheme);
QskinnyDxPlan qskinny_dx_plan(int64_t M, int64_t K, int64_t N, int scheme, int num_cu);

// The rank-r weight gradients that may ride in the finish launch (only with dhpart, i.e. rp <= 16):
// dA[K][r] = alpha X^T dH, dB[r][N] = alpha H^T dY (fp32; either may be NULL).  X: bf16 [M][K], H: bf16 [M][rp].
struct QskinnyDxGrads {
    const void* X;
    const void* H;
    float* dA;
    float* dB;
    int64_t r;
    float alpha;
};

// dX[M,K] bf16 = base_scale dY deq(Wq)^T + scaling dH A^T,  dH = dY B^T (bf16 [M][rp]).
// With dhpart (scratch of slices * M * rp floats; rp <= 16, B: bf16 [rp][N]) dH is formed by the launch
// itself and stored to dH (may be NULL); without it dH is an input.  A: bf16 [K][rp]; rp a multiple of 8,
// at most 64.  part is scratch of the plan's size.  grads may be NULL.
hipError_t launch_qskinny_dx(const void* dY, const void* Wq, const void* scales, int scheme, const void* B, const void* A,
                             int64_t rp, float base_scale, float scaling, void* dX, void* dH, int64_t M, int64_t K, int64_t N,
                             const QskinnyDxPlan& p, float* part, float* dhpart, const QskinnyDxGrads* grads, hipStream_t st);

}  // namespace fhpc
