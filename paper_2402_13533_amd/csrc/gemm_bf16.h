// Internal interface of the bf16 MFMA GEMM core (gfx950).  Not part of the C ABI.
//
// One kernel family computes
//     C[M,N] (=|+=) alpha * ( mid_scale * sum_{k<K2} A2(m,k) B2(n,k)  +  sum_{k<K} A(m,k) B(n,k) )
// with fp32 accumulation on the matrix cores.  The optional first sum is the
// rank-r branch of the finetuning layer riding in the same accumulators as the
// frozen base weight's product.  Operands are described by how the element
// (row, k) is stored, so that every product of the layer's forward and backward
// (X*A, H*B, dY*B^T, dH*A^T, H^T*dY, X^T*dH, X*deq(W), dY*deq(W)^T) is one call.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

// Storage of an operand whose logical element is (row, k), row = output index
// (m for the A side, n for the B side), k = reduction index.
enum : int {
    OP_KC = 0,     // bf16, k contiguous:   ptr[row*ld + k]
    OP_XC = 1,     // bf16, row contiguous: ptr[k*ld + row]  (transposed while staging)
    OP_Q8_KC = 2,  // int8 codes ptr[row*ld + k], fp16 scale[row]
    OP_Q4_KC = 3,  // 4-bit codes, byte ptr[row*ld/2 + k/2], fp16 scale[row*scale_ld + k/64]
    OP_Q8_XC = 4,  // int8 codes ptr[k*ld + row], fp16 scale[k]
    OP_Q4_XC = 5,  // 4-bit codes, byte ptr[k*ld/2 + row/2], fp16 scale[k*scale_ld + row/64]
    OP_NONE = 6
};

// OUT_F32: fp32 C.  With a split reduction, split s writes its partial sum to
// c + s * split_stride (plain stores, no atomics); the caller adds the slabs afterwards.
enum : int { OUT_BF16 = 0, OUT_F32 = 1 };

// Tile shapes (BM x BN) and the wave grid that covers them.
enum : int {
    TILE_256x256 = 0,  // 2 x 4 waves of 128 x 64
    TILE_128x256 = 1,  // 2 x 4 waves of 64 x 64, ping-pong schedule
    TILE_256x128 = 2,  // 4 x 2 waves of 64 x 64, ping-pong schedule
    TILE_128x128 = 3,  // 2 x 2 waves of 64 x 64
    TILE_256x32 = 4,   // 4 x 1 waves of 64 x 32   (rank-r outputs: H, dH, dA)
    TILE_32x256 = 5,   // 1 x 4 waves of 32 x 64   (dB)
    TILE_COUNT = 6
};

constexpr int GEMM_MAX_GROUPS = 8;

struct GemmOperand {
    const void* ptr;
    int64_t ld;            // leading dimension in elements (codes for quantised operands)
    const void* scales;    // fp16 scales for quantised operands
    int64_t scale_ld;      // scales per row of the scale array (int4 only)
};

struct GemmArgs {
    GemmOperand a, b;      // main sum, reduction length K
    GemmOperand a2, b2;    // optional leading sum, reduction length K2 (a rank; short)
    void* c;
    int64_t ldc;
    int M, N, K, K2;
    float alpha;
    float mid_scale;
    int splits;            // >1: the reduction is cut into slices of k_chunk (multiple of 64); needs OUT_F32
    int k_chunk;
    int64_t split_stride;  // elements between the partial-sum slabs of consecutive splits
    // groups > 1 (request-fed kernels only): that many independent products of the same shape, layout and
    // leading dimensions in one launch; product i takes its operand and output addresses from ga[i], gb[i],
    // gc[i] (a.ptr, b.ptr and c are then unused).  With a split reduction, gc[i] is product i's slab area.
    int groups;
    const void* ga[GEMM_MAX_GROUPS];
    const void* gb[GEMM_MAX_GROUPS];
    void* gc[GEMM_MAX_GROUPS];
    // n_split > 0 (request-fed kernels, bf16 output, no groups): a second output of the same launch.  Columns
    // [0, n_split) go to c (ldc) as usual, columns [n_split, N) to c2 (leading dimension ldc2) as its columns
    // 0 .. N - n_split - 1.  n_split must be a multiple of the tile's width and N - n_split of 8.
    void* c2;
    int64_t ldc2;
    int n_split;
    // gate != 0 (request-fed kernels, 256 x 256 tile, bf16 output, no groups, no second output): the SiLU gate of the
    // FFN applied to the tile in the epilogue, on C rounded to bf16, with the arithmetic of the streaming gate kernels.
    // gate == 1: C (the up projection) is stored as usual and gate_out1 = SiLU(gate_g) * C as well.
    // gate == 2: C (the gradient of the gate's output) is not stored: gate_out1 = d gate_g and gate_out2 = d gate_u.
    // All four are [M][N] bf16 with C's leading dimension ldc.
    int gate;
    const void* gate_g;
    const void* gate_u;
    void* gate_out1;
    void* gate_out2;
    int dbg;               // kernel choice for tests, 0 in normal use: bit 2 = lockstep kernels only, bit 3 =
                           // four-wave kernel where it exists.  A build with -DFHPC_DIAG also honours bit 0
                           // (request no operand data) and bit 1 (skip the matrix instructions, lockstep only).
};

// The diagnostic bits cost a scalar compare per K tile in the hot loops, so the product build folds them away.
#ifdef FHPC_DIAG
#define FHPC_DBG_NO_LOADS(p) (((p).dbg & 1) != 0)
#define FHPC_DBG_NO_MMA(p) (((p).dbg & 2) != 0)
#else
#define FHPC_DBG_NO_LOADS(p) false
#define FHPC_DBG_NO_MMA(p) false
#endif

// Launches the instantiation (a_mode, b_mode, b2_mode, out_mode, tile).  a2 is always OP_KC.
// Returns hipErrorInvalidValue when that combination is not instantiated.
hipError_t launch_gemm_bf16(int a_mode, int b_mode, int b2_mode, int out_mode, int tile,
                            const GemmArgs& args, hipStream_t stream);

// The eight-wave ping-pong kernels (gemm_pp.hip) cover the plain bf16 products on the
// 256x256 and 256x128 tiles; launch_gemm_bf16 routes to them unless args.dbg bit 2 is set.
bool gemm_pp_supports(int a_mode, int b_mode, int b2_mode, int out_mode, int tile);
hipError_t launch_gemm_pp(int a_mode, int b_mode, int out_mode, int tile, const GemmArgs& args, hipStream_t stream);

// The four-wave kernel (gemm_w4.hip) covers the same products on the 256x256 tile.  It matches
// the ping-pong kernels when the reduction is long and the output has at least one 256x256 tile
// per compute unit, and loses to them otherwise, so it is selected only by args.dbg bit 3.
bool gemm_w4_supports(int a_mode, int b_mode, int b2_mode, int out_mode, int tile);
hipError_t launch_gemm_w4(int a_mode, int b_mode, int out_mode, const GemmArgs& args, hipStream_t stream);

// Compute units of the current device in whole multiples of 8 (256 if no device answers): what the
// planner and the persistent launches size themselves for.
int compute_units();

// Tile extents, for planning on the host.
void gemm_tile_extent(int tile, int* bm, int* bn);

}  // namespace fhpc
