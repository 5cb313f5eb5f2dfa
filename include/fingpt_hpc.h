/*
 * fingpt_hpc.h -- C ABI of the MI355X (gfx950) library for the factorised linear
 * layer of FinGPT-HPC and its quantised finetuning form.
 *
 * Notation (row form): tokens are the M rows of X[M,K]; the factor pair is
 * A[K,r], B[r,N] with r << K,N; H = X*A is the rank-r intermediate.  The paper
 * writes the same layer with column vectors, y = B A x (Sec. 3.2, eq.
 * "low_rank_layer"; Sec. 4.1 item 1 gives the row-form shapes A: n x r, B: r x n).
 *
 * Conventions for every entry point
 *  - All matrices are row-major and contiguous.  Every data pointer is a DEVICE
 *    pointer owned by the caller; the library never allocates, frees or retains
 *    device memory.  Scratch comes from `workspace` (device pointer, 256-byte
 *    aligned, size from fhpc_workspace_bytes); too small => FHPC_ERR_WORKSPACE
 *    and nothing is launched.  Every workspace layout begins with a header of
 *    FHPC_WORKSPACE_HEADER_BYTES that holds arrival counters of the weight-streaming
 *    launches (a launch's last workgroup to reach a block of outputs finishes it).  The
 *    header must be ZERO when a buffer is first handed to the library (clear the buffer
 *    once after allocating it); every call leaves the header zero again, so a buffer
 *    can be reused from call to call, by any entry point, without clearing, also under
 *    HIP graph replay.  The rest of a workspace may hold anything.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued asynchronously; no call synchronises.  Inputs, outputs and
 *    workspace must stay alive and untouched until the stream has passed the
 *    call.  Outputs must not alias inputs.  Two calls that share a workspace
 *    must be ordered on one stream.
 *  - Shapes: M >= 1, r >= 1 arbitrary; K and N multiples of 8; data pointers
 *    16-byte aligned; every matrix smaller than 2 GiB.  Violations return an
 *    error code before anything is launched.
 *  - Return value: FHPC_OK or an FHPC_ERR_* code.  Nothing throws, exits or
 *    prints.  HIP launch failures map to FHPC_ERR_HIP.
 *  - dA and dB are produced in fp32.  Reductions over tokens are cut into slices
 *    whose partial sums go to separate slabs of the workspace and are added in a
 *    fixed order: no floating-point atomics, results are bit-reproducible from run to run.
 */
#ifndef FINGPT_HPC_H
#define FINGPT_HPC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FHPC_WORKSPACE_HEADER_BYTES 16384

/* dtype of X, A, B, Y, dY, dX, H (dA/dB are always fp32) */
enum { FHPC_F32 = 0, FHPC_BF16 = 1 };

/* storage scheme of the frozen base weight (Sec. 5.2 "Quantization": one scale
 * per weight vector; here symmetric absmax, no zero point):
 *  FHPC_Q_INT8_PER_CHANNEL: Wq int8 [N][K], scales fp16 [N] (vector = one output channel)
 *  FHPC_Q_INT4_BLOCK:       Wq bytes [N][K/2], element k (even) in the low nibble and
 *                           k+1 in the high nibble, two's complement 4-bit;
 *                           scales fp16 [N][K/block] (vector = `block` consecutive k
 *                           of one output channel); block must be 64. */
enum { FHPC_Q_INT8_PER_CHANNEL = 8, FHPC_Q_INT4_BLOCK = 4 };

/* blend and merge entry points only: the frozen weight is not quantised: W bf16 [K][N] row-major in the
 * `Wq` argument, `scales` and `block` ignored (scales may be NULL) */
enum { FHPC_W_BF16 = 16 };

/* qlinear_lowrank_fwd / _bwd only: `Wq` is not the stored weight but the merged weight W' = deq(W) + scaling * A * B
 * as bf16 [K][N], written by lowrank_merge (bf16 output) for the SAME A, B and scaling that the call receives;
 * `scales` and `block` are ignored.  The calls then skip their own merge: Y = X W', dX = dY W'^T, while H, dA and
 * dB are formed from A and B as always.  A training step merges once (A and B change once per step) and passes
 * the result to both calls; the caller answers for W' matching A, B and scaling. */
enum { FHPC_W_MERGED = 17 };

enum {
    FHPC_OK = 0,
    FHPC_ERR_NULL = 1,        /* a required pointer is NULL */
    FHPC_ERR_SHAPE = 2,       /* non-positive size, K or N not a multiple of 8, K % block != 0 */
    FHPC_ERR_DTYPE = 3,       /* unknown dtype / qscheme */
    FHPC_ERR_ALIGN = 4,       /* a data pointer is not 16-byte aligned (workspace: 256) */
    FHPC_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than fhpc_workspace_bytes */
    FHPC_ERR_UNSUPPORTED = 6, /* block != 64, matrix >= 2 GiB, ... */
    FHPC_ERR_HIP = 7          /* a HIP call or kernel launch failed */
};

/* which entry point a workspace is sized for */
enum { FHPC_OP_LOWRANK_FWD = 0, FHPC_OP_LOWRANK_BWD = 1, FHPC_OP_QLINEAR_FWD = 2, FHPC_OP_QLINEAR_BWD = 3,
       FHPC_OP_MERGE = 4, FHPC_OP_DECOMPOSE = 5 };

/* Factorised linear layer, forward (Sec. 3.2 eq. low_rank_layer; Sec. 4.1 "Method 1"):
 *   Y[M,N] = (X[M,K] * A[K,r]) * B[r,N].
 * X, A, B, Y have `dtype`.  H_out (M x r, `dtype`), if not NULL, receives H = X*A for
 * the backward pass.  bf16: fp32 accumulation, H rounded to bf16 between the two
 * products.  f32: plain fp32 arithmetic throughout. */
int lowrank_linear_fwd(const void* X, const void* A, const void* B, void* Y, void* H_out,
                       int64_t M, int64_t K, int64_t r, int64_t N, int dtype,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Factorised linear layer, backward (the gradients of the layer above; the paper's
 * forward/backward flow figure in Sec. 4.2 shows the data flow):
 *   dH = dY * B^T;  dX[M,K] = dH * A^T (`dtype`);  dA[K,r] = X^T * dH (fp32);
 *   dB[r,N] = H^T * dY (fp32).
 * H_saved (M x r, `dtype`) may be NULL: H is then recomputed from X and A (the
 * layer-local form of the recomputation of Sec. 4.2).  Any of dX, dA, dB may be NULL
 * and is then skipped.  Outputs are overwritten. */
int lowrank_linear_bwd(const void* X, const void* A, const void* B, const void* dY,
                       const void* H_saved, void* dX, float* dA, float* dB,
                       int64_t M, int64_t K, int64_t r, int64_t N, int dtype,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* g factorised layers that read the same activations: the query, key and value projections of an
 * attention block, or the gate and up projections of the FFN (Sec. 3.1 eqs. attention and FFN; each
 * of them replaced by a factor pair, Sec. 4.1 "Method 1").  bf16 only.
 *   Y_i[M,N] = (X[M,K] * A_i[K,r]) * B_i[r,N],   i = 0 .. g-1,   1 <= g <= FHPC_MAX_SHARED
 * A_all is one bf16 matrix [K][g*r], row-major, with A_i in columns i*r .. (i+1)*r-1, so that X*A_all
 * is a single product.  B and Y are HOST arrays of g device pointers (B_i [r][N], Y_i [M][N], bf16).
 * H_all_out ([M][g*r] bf16, H_i = X*A_i in columns i*r ..), if not NULL, receives the intermediate for
 * the backward pass.  r must be a multiple of 8 (FHPC_ERR_UNSUPPORTED otherwise); every other rule
 * of lowrank_linear_fwd applies with g*r as the rank.  Results are those of g calls of lowrank_linear_fwd up
 * to the rounding of H (the wide product may sum its reduction in another order).  The pointer arrays are
 * read during the call only.
 * Workspace: fhpc_workspace_bytes_lowrank_shared_x (host-only; 0 for invalid arguments). */
#define FHPC_MAX_SHARED 8
int lowrank_linear_fwd_shared_x(const void* X, const void* A_all, const void* const* B, void* const* Y, void* H_all_out,
                                int64_t M, int64_t K, int64_t r, int64_t N, int g,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward of the g layers above:
 *   dH_i = dY_i * B_i^T;   dX[M,K] = sum_i dH_i * A_i^T  (bf16; one product over the g*r columns of
 *   [dH_0 | ... | dH_g-1], the per-layer input gradients are never formed);
 *   dA_all[K][g*r] = X^T * [dH_0 | ...] (fp32, dA_i in columns i*r ..);   dB_i[r,N] = H_i^T * dY_i (fp32).
 * dY and dB are HOST arrays of g device pointers.  H_all_saved may be NULL (H is recomputed).  dX,
 * dA_all, dB (the array) and any dB[i] may be NULL and are then skipped.  Outputs are overwritten. */
int lowrank_linear_bwd_shared_x(const void* X, const void* A_all, const void* const* B, const void* const* dY,
                                const void* H_all_saved, void* dX, float* dA_all, float* const* dB,
                                int64_t M, int64_t K, int64_t r, int64_t N, int g,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
size_t fhpc_workspace_bytes_lowrank_shared_x(int backward, int64_t M, int64_t K, int64_t r, int64_t N, int g);

/* The FFN's gate and up projections with the gate itself (Sec. 3.1 eq. FFN, every projection a factor pair,
 * Sec. 4.1 "Method 1"), bf16:
 *   H_all = X * A_all,   G = H_gate * B_gate,   U = H_up * B_up,   Z = SiLU(G) (.) U   (elementwise)
 * X [M][K]; A_all [K][2r] = [A_gate | A_up]; B_gate, B_up [r][N]; G_out, U_out, Z_out [M][N] (all three are
 * written: the backward pass needs G and U); H_all_out [M][2r] or NULL.  All device pointers, 16-byte aligned.
 * Exactly the results of lowrank_linear_fwd_shared_x with g = 2 followed by swiglu_fwd, bit for bit; when N's
 * tiles go through the large matrix-core kernel, U's tiles pass the gate in that kernel's epilogue and Z costs
 * no pass of its own over G and U.  Rules and status codes of lowrank_linear_fwd_shared_x with g = 2.
 * Workspace: fhpc_workspace_bytes_lowrank_shared_x(0, M, K, r, N, 2). */
int lowrank_ffn_gate_up_fwd(const void* X, const void* A_all, const void* B_gate, const void* B_up,
                            void* G_out, void* U_out, void* Z_out, void* H_all_out,
                            int64_t M, int64_t K, int64_t r, int64_t N,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward of the FFN's down projection Y = (Z * A) * B (Sec. 3.1 eq. FFN; Sec. 3.2 eq. low_rank_layer) with
 * its input gradient taken through the gate, bf16:
 *   dH = dY * B^T,   dZ = dH * A^T (never stored),   dU = dZ (.) SiLU(G),   dG = dZ (.) U (.) SiLU'(G),
 *   dA[K,r] = Z^T * dH (fp32),   dB[r,N] = H^T * dY (fp32).
 * Z [M][K] (the gate's output, this layer's input; K is the FFN's inner width); A [K][r]; B [r][N]; dY [M][N];
 * H_saved [M][r] or NULL (recomputed); G, U [M][K] as the forward call wrote them; dG_out, dU_out [M][K] bf16;
 * dA, dB may be NULL.  dZ is rounded to bf16 before the gate, so the results are exactly those of
 * lowrank_linear_bwd followed by swiglu_bwd.  dU_out may not overlap G or U.  Rules and status codes of
 * lowrank_linear_bwd.  Workspace: fhpc_workspace_bytes(FHPC_OP_LOWRANK_BWD, M, K, r, N, FHPC_BF16, 0). */
int lowrank_ffn_down_bwd(const void* Z, const void* A, const void* B, const void* dY, const void* H_saved,
                         const void* G, const void* U, void* dG_out, void* dU_out, float* dA, float* dB,
                         int64_t M, int64_t K, int64_t r, int64_t N,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Finetuning layer, forward (Sec. 5.1 eq. new_linear_layer with the frozen weight
 * stored quantised, Sec. 5.2):
 *   Y[M,N] = X[M,K] * deq(Wq, scales)[K,N] + scaling * (X * A[K,r]) * B[r,N].
 * X, A, B, Y, H_out are bf16.  deq(.)[k,n] = code[n][k] * scale(n, k); the product is
 * rounded to bf16 when it enters the matrix unit.  H_out as above (unscaled X*A). */
int qlinear_lowrank_fwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                        const void* A, const void* B, float scaling, void* Y, void* H_out,
                        int64_t M, int64_t K, int64_t r, int64_t N,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* qlinear_lowrank_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, layouts, results (bit
 * for bit) and status codes as qlinear_lowrank_fwd, without the workspace pair: scratch comes from a fixed
 * array of FHPC_NOALLOC_SCRATCH_BYTES in device memory that belongs to the library (one per GPU, held until the
 * process ends).  The call allocates nothing and frees nothing.  Sizes whose workspace need
 * (fhpc_workspace_bytes(FHPC_OP_QLINEAR_FWD, ...)) exceeds the array return FHPC_ERR_WORKSPACE before anything
 * is launched; every token count up to 64 on the weights of a 13B decoder layer needs 8 MiB or less.
 * All calls on one GPU share the array: two calls that overlap in time on one GPU (different streams, different
 * threads) race on it; calls ordered on one stream do not.  The first call on a device looks the array's
 * address up, which is not a capturable operation: make one call on the device before capturing. */
#define FHPC_NOALLOC_SCRATCH_BYTES (16u << 20)
int qlinear_lowrank_fwd_noalloc(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                                const void* A, const void* B, float scaling, void* Y, void* H_out,
                                int64_t M, int64_t K, int64_t r, int64_t N, void* hip_stream);

/* Finetuning layer, backward; W is frozen (Sec. 5.1), so there is no dW:
 *   dH = dY * B^T;  dX = dY * deq(W)^T + scaling * dH * A^T  (bf16);
 *   dA = scaling * X^T * dH (fp32);  dB = scaling * (X*A)^T * dY (fp32).
 * H_saved may be NULL (recompute).  Any of dX, dA, dB may be NULL. */
int qlinear_lowrank_bwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                        const void* A, const void* B, float scaling, const void* dY,
                        const void* H_saved, void* dX, float* dA, float* dB,
                        int64_t M, int64_t K, int64_t r, int64_t N,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* Finetuning layer, forward, for several weights that read the same X: the q, k, v projections of a
 * decoder layer, or its gate and up projections (Sec. 3.1 lists them; Sec. 4.2 batches same-shape work).
 * `weights` is a HOST array of `count` descriptors whose pointers are device pointers laid out as for
 * qlinear_lowrank_fwd; K, r, the storage scheme and M are shared, N and scaling are per weight.  Each
 * Y is its own dense [M][N] matrix.  Result: exactly what `count` calls of qlinear_lowrank_fwd give up
 * to summation order.  With at most 64 tokens (and up to four weights, r <= 64, K a multiple of 256)
 * all weights go through one launch, which is the point: such a call is bound by launch
 * latency, not by the weight stream.  Otherwise the weights are processed one after another.
 * Workspace: fhpc_workspace_bytes_shared_x (host-only; 0 for invalid arguments). */
typedef struct {
    const void* Wq;        /* quantised weight, device */
    const void* scales;    /* fp16 scales, device */
    const void* A;         /* bf16 [K][r], device */
    const void* B;         /* bf16 [r][N], device */
    void* Y;               /* bf16 [M][N], device */
    void* H_out;           /* bf16 [M][r], device, or NULL */
    int64_t N;
    float scaling;
} fhpc_qlinear_weight;
int qlinear_lowrank_fwd_shared_x(const void* X, const fhpc_qlinear_weight* weights, int count, int qscheme, int block,
                                 int64_t M, int64_t K, int64_t r, void* workspace, size_t workspace_bytes, void* hip_stream);
size_t fhpc_workspace_bytes_shared_x(const int64_t* N, int count, int64_t M, int64_t K, int64_t r, int qscheme);

/* Blend of a frozen pretrained weight with the factor pair (Sec. 4.1 item 3:
 * y = alpha W x + (1 - alpha) B A x, 0 <= alpha <= 1, W frozen), with W stored quantised as above:
 *   Y = alpha * X * deq(Wq, scales) + (1 - alpha) * (X * A) * B
 * Arguments, layouts, workspace (FHPC_OP_QLINEAR_FWD / _BWD sizes) and error behaviour are those of
 * qlinear_lowrank_fwd / _bwd with `alpha` in place of `scaling`; alpha outside [0, 1] (or NaN)
 * returns FHPC_ERR_SHAPE.  alpha = 0 gives the factorised layer alone; with more than 64 tokens Wq is then
 * never read, with at most 64 the forward still streams Wq and its scales and multiplies them by 0, so the
 * scales must be finite there.
 * qscheme may also be FHPC_W_BF16: the pretrained weight kept in bf16, W[K,N] row-major. */
int qlinear_blend_fwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                      const void* A, const void* B, float alpha, void* Y, void* H_out,
                      int64_t M, int64_t K, int64_t r, int64_t N,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*   dX = alpha * dY * deq(W)^T + (1 - alpha) * (dY * B^T) * A^T;
 *   dA = (1 - alpha) * X^T * (dY * B^T);   dB = (1 - alpha) * (X * A)^T * dY;   no dW. */
int qlinear_blend_bwd(const void* X, const void* Wq, const void* scales, int qscheme, int block,
                      const void* A, const void* B, float alpha, const void* dY,
                      const void* H_saved, void* dX, float* dA, float* dB,
                      int64_t M, int64_t K, int64_t r, int64_t N,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace the entry point `op` (FHPC_OP_*) needs for these sizes.
 * Host-only; returns 0 for invalid arguments (and for FHPC_OP_MERGE when it needs none).  qscheme is
 * ignored for op 0/1/4/5; M and dtype are ignored for op 4/5. */
size_t fhpc_workspace_bytes(int op, int64_t M, int64_t K, int64_t r, int64_t N, int dtype, int qscheme);

/* SiLU-gated product between the FFN's linears (Sec. 3.1 eq. FFN):
 *   Z = U .* G .* sigmoid(G)            (n_elems elements of `dtype`, fp32 arithmetic)
 *   dU = dZ .* G .* sigmoid(G);  dG = dZ .* U .* sigmoid(G) .* (1 + G .* (1 - sigmoid(G))). */
int swiglu_fwd(const void* G, const void* U, void* Z, int64_t n_elems, int dtype, void* hip_stream);
int swiglu_bwd(const void* G, const void* U, const void* dZ, void* dG, void* dU,
               int64_t n_elems, int dtype, void* hip_stream);

/* out = a + b elementwise (n_elems of `dtype`, fp32 add).  The FFN feeds one input to
 * both the gate and the up projection (Sec. 3.1 eq. FFN), so its input gradient is
 * the sum of the two projections' dX.  `out` may alias `a` or `b`. */
int fhpc_add(const void* a, const void* b, void* out, int64_t n_elems, int dtype, void* hip_stream);

/* Per-vector quantisation of a weight (Sec. 5.2: one scaling factor per vector, the
 * vector's elements multiplied through, stored in low precision).  W is fp32 [K,N];
 * outputs use the canonical layout above.  scale = fp16_rne(absmax / qmax) with
 * qmax = 127 (scheme 8) or 7 (scheme 4); code = clamp(rint(w / scale), -qmax, qmax)
 * with an fp32 divide and ties to even; a zero scale gives zero codes.  Results are
 * bit-exact functions of W. */
int qweight_quantize(const float* W, int qscheme, int block, void* Wq_out, void* scales_out,
                     int64_t K, int64_t N, void* hip_stream);

/* Adapted weight materialised once for inference (Sec. 5.1, eq. new_linear_layer: W' = W + Delta W,
 * Delta W the product of the factor pair):
 *   W_out[K,N] = deq(W)[K,N] + scaling * A[K,r] * B[r,N]          (the paper's case: scaling = 1)
 * W is the frozen weight in the storage `qscheme` names: FHPC_W_BF16 (bf16 [K][N], scales ignored) or one
 * of the quantised layouts above with its fp16 `scales`.  W == NULL means no base weight: W_out is then
 * the dense weight the factor pair stands for.  A, B are bf16; W_out is row-major [K][N] of `out_dtype`
 * (FHPC_F32 or FHPC_BF16) and must not alias W.  The product is accumulated in fp32, the base weight
 * (exact in fp32) is added in fp32 and the sum is rounded once.  To keep the merged weight quantised,
 * write fp32 and pass it to qweight_quantize.  Workspace: FHPC_OP_MERGE (zero bytes, and workspace may
 * be NULL, when r is a multiple of 8). */
int lowrank_merge(const void* W, const void* scales, int qscheme, int block, const void* A, const void* B,
                  float scaling, void* W_out, int out_dtype, int64_t K, int64_t r, int64_t N,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Factor pair from a pretrained weight (Sec. 4.1 item 2: W is decomposed into A[K,r] and B[r,N], which
 * initialise the factorised layer; Sec. 4.2 "weight decomposition in parallel": the same-shape weights of
 * different decoder layers are handled by one call, `batch` of them stored back to back).  The paper
 * names no algorithm.  Here: randomised subspace iteration on the matrix cores,
 *   Y = W Omega;  repeat power_iters times { Z = W^T Y, orthonormalise Z, Y = W Z };  A = orthonormalised Y;
 *   B = (A^T A)^-1 A^T W   (the least-squares fit for this A, so that A B is the projection of W on span A),
 * with the orthonormalisation done by matrix products only (polynomial iterations on the Gram matrix).
 * W: bf16 [batch][K][N];  Omega: bf16 [N][r], a random test matrix from the caller (standard normal
 * entries; the same one serves every weight of the batch);  A_out: bf16 [batch][K][r], columns orthonormal
 * up to bf16 rounding;  B_out: bf16 [batch][r][N].  With power_iters around 2 the error |W - A B|_F is
 * within a few per cent of the best rank-r approximation's for spectra that decay, and equal to it up to
 * rounding when W has rank r.  r must be a multiple of 8 and at most min(K, N) (else FHPC_ERR_UNSUPPORTED);
 * 0 <= power_iters <= 16.  Workspace: FHPC_OP_DECOMPOSE (M, dtype, qscheme ignored). */
int lowrank_decompose(const void* W, const void* Omega, int power_iters, void* A_out, void* B_out,
                      int64_t K, int64_t r, int64_t N, int64_t batch,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Integer codes of a stored weight, q_out int8 [N][K] (scheme 8: a copy; scheme 4:
 * sign-extended nibbles, including the code -8).  Bit-exact. */
int qweight_unpack(const void* Wq, int qscheme, int8_t* q_out, int64_t K, int64_t N, void* hip_stream);

/* Dequantised weight W_out fp32 [N][K] = code * scale (exact in fp32).  Bit-exact. */
int qweight_dequant(const void* Wq, const void* scales, int qscheme, int block, float* W_out,
                    int64_t K, int64_t N, void* hip_stream);

/* Static, NUL-terminated description of a status code. */
const char* fhpc_status_string(int status);

/* Diagnostic: one launch of the bf16 matrix-core GEMM that the entry points above are
 * built from,  C[M,N] = alpha * sum_k A(m,k) B(n,k)  with fp32 accumulation.
 * a_mode / b_mode say how element (row, k) of an operand is stored: 0 = bf16 ptr[row*ld + k],
 * 1 = bf16 ptr[k*ld + row].  out_mode: 0 = bf16 C, 1 = fp32 C (required when splits > 1:
 * slice s of the reduction then stores its partial sums to C + s*M*ldc, so C must hold
 * `splits` slabs of M*ldc floats and the caller adds them).  tile: 0 = 256x256,
 * 1 = 128x256, 2 = 256x128, 3 = 128x128, 4 = 256x32, 5 = 32x256 (the last two with out_mode 1
 * only).  splits cuts the reduction into that many slices.  dbg chooses among the kernels that
 * cover a tile, for their parity tests: 0 = the one the entry points use, 4 = the register-staged
 * lockstep kernel, 8 = the four-wave kernel (256x256 only); other bits are ignored.
 * Returns FHPC_ERR_UNSUPPORTED for a combination that is not instantiated. */
int fhpc_gemm_bf16(const void* A, int64_t lda, int a_mode, const void* B, int64_t ldb, int b_mode,
                   void* C, int64_t ldc, int out_mode, int64_t M, int64_t N, int64_t K, float alpha,
                   int tile, int splits, int dbg, void* hip_stream);

/* Diagnostic per-launch timing (off by default; not thread-safe; host-side state only).
 * fhpc_profile_start arms a pool of `max_records` HIP event pairs; while armed, every
 * matrix-core GEMM launch records an event before and after itself on its stream, which
 * costs a few microseconds per launch.  fhpc_profile_stop disarms and returns the number
 * of launches recorded.  fhpc_profile_get waits for record `index` and returns the
 * kernel's name (NUL-terminated, truncated to name_len), its duration in milliseconds and
 * the algorithmic flop count of that launch; `bytes` is the algorithmic byte count for the
 * weight-streaming kernels and 0 elsewhere. */
int fhpc_profile_start(int max_records);
int fhpc_profile_stop(void);
int fhpc_profile_get(int index, char* name, int name_len, float* ms, double* flops, double* bytes);

/* Measurement probes: what this GPU delivers with no kernel design in the way, for a benchmark that quotes its
 * kernels against measured ceilings beside the published ones.
 * fhpc_probe_mfma: `workgroups` x 4 waves each issue iters * 8 v_mfma_f32_32x32x16_bf16 back to back from
 * registers, with no memory traffic; seed (device, 256 x uint32) holds the operand words of a wave (all zero, or
 * random bf16 pairs: the matrix pipes' clock under load depends on the data).  *flops (host) receives the
 * flop count of the launch.  sink (device, workgroups * 256 floats) may be NULL.
 * fhpc_probe_copy: dst[0 .. bytes) = src[0 .. bytes), 16 bytes per lane; bytes a multiple of 16.
 * fhpc_probe_read_rows: one pass over W (device, [N][row_bytes] bytes, 16-byte aligned, row_bytes a multiple of 256,
 * N * row_bytes < 2^31) in the access pattern of the few-token weight-streaming kernels of Sec. 5.3's inference
 * path (64 rows x 256 bytes per workgroup and step, the rows cut into as many slices as give one round of
 * `workgroups` workgroups) with nothing else in the kernel: the time below which no such kernel can get on this
 * chip at that size.  sink (device, 1 KiB) is never written in practice.  All three return a status code and
 * only enqueue work on hip_stream. */
int fhpc_probe_mfma(const void* seed, int workgroups, int iters, float* sink, double* flops, void* hip_stream);
int fhpc_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream);
int fhpc_probe_read_rows(const void* W, int64_t N, int64_t row_bytes, int workgroups, void* sink, void* hip_stream);

/* Host-only test hook (needs no GPU, touches no memory): walks the launch sequence of an entry point for
 * these sizes without launching anything and reports, in bytes, the largest partial-sum area any of its
 * split reductions would use (*planned) and what the workspace layout reserves for them (*reserved).
 * The calls themselves refuse, with FHPC_ERR_WORKSPACE, a launch whose slabs would not fit; this hook lets
 * a test show on the CPU that planned <= reserved over a grid of shapes.
 * call: FHPC_OP_LOWRANK_FWD .. FHPC_OP_QLINEAR_BWD, FHPC_OP_DECOMPOSE, FHPC_PLAN_SHARED_FWD / _BWD (the
 * shared-X calls of the factorised layer, g layers), FHPC_PLAN_FFN_GATE_UP / _DOWN_BWD (lowrank_ffn_gate_up_fwd,
 * lowrank_ffn_down_bwd).  outputs: bit 0 = dX wanted (forward calls: H_out given),
 * bit 1 = dA, bit 2 = dB, bit 3 = H_saved given.  base_scale: 1 for the finetuning layer, alpha for the blend
 * layer.  dtype, qscheme, g are ignored where the call has no such argument.  Returns a status code. */
enum { FHPC_PLAN_SHARED_FWD = 16, FHPC_PLAN_SHARED_BWD = 17, FHPC_PLAN_FFN_GATE_UP = 18, FHPC_PLAN_FFN_DOWN_BWD = 19 };
int fhpc_plan_slab_bytes(int call, int64_t M, int64_t K, int64_t r, int64_t N, int dtype, int qscheme, int g,
                         int outputs, float base_scale, int64_t* planned, int64_t* reserved);

/* Library version (major * 100 + minor). */
int fhpc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FINGPT_HPC_H */
