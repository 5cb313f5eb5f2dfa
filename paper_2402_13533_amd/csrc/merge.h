// Internal launcher of the weight-merge kernel.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fhpc {

constexpr int MERGE_EXT_PAD = 128;

// out[K][N] (fp32 or bf16) = base_scale * base + scaling * A B.  w_kind: 0 = no base weight, 1 = bf16 W[K][N],
// 2 = int8 codes [N][K] + fp16 scale per channel, 3 = 4-bit codes [N][K/2] + fp16 scale per 64 k.
// A is bf16 [K][lda] with lda a multiple of 8 (columns r .. lda-1 zero), B bf16 [r][N].
// With `ext` (bf16 output only; lda <= MERGE_EXT_PAD) out is [(K + lda)][(N + MERGE_EXT_PAD)]: the merged weight in
// its K x N corner, A in columns N .. N + lda - 1 of those rows, B in rows K .. K + r - 1 of the first N columns
// (further rows and the lda x lda corner zero; the remaining pad columns are never read).  The pad keeps the rows
// 256-byte aligned: with a row stride of N + 16 every 256-byte request of the products straddled three cache lines
// and the products ran 8 % slower.  X times that buffer's first K rows is [Y | H]; dY times its first N columns,
// transposed, is [dX | dH].
// `stream_out`: the output leaves with non-temporal stores.  Right when nothing reads it soon (the merged weight
// handed to the caller: the kernel alone is a third faster); wrong inside the layer's own calls, whose product reads
// the merged weight straight back and wants it in the Infinity Cache (measured: the step gets 3 % slower).
hipError_t launch_merge(const void* W, const void* scales, int w_kind, const void* A, int64_t lda, const void* B,
                        float base_scale, float scaling, void* out, bool out_f32, int64_t K, int64_t r, int64_t N, hipStream_t s,
                        bool ext = false, bool stream_out = false);

}  // namespace fhpc
