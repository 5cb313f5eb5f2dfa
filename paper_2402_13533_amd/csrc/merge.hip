// Adapted weight materialised for inference (Sec. 5.1, eq. new_linear_layer: W' = W + Delta W
// with Delta W the product of the factor pair):
//     W_out[K,N] = deq(W)[K,N] + scaling * A[K,r] * B[r,N]
//
// One pass over the weight: the kernel is bound by reading W once and writing W_out once; the
// rank-r product is a short matrix-core loop (reduction length r) per 128 x 128 tile of the
// output.  Per tile: (1) the thread's share of the base weight is requested first and stays in
// registers while (2) the r-loop runs on 32-deep slices of A and B double-buffered in LDS
// (global -> LDS requests, transposing LDS reads for B); (3) scaling * A B goes to LDS as an
// fp32 tile (over the operand buffers); a quantised base weight, stored channel-major, is
// dequantised and added there, which transposes it on the way; (4) rows of the tile are
// streamed out 16 or 32 bytes per lane, adding a bf16 base weight on the way.
#include "merge.h"
#include "gemm_ring.h"
#include "profile.h"

namespace fhpc {
namespace mrg {

using namespace ring;

constexpr int NT = 256;
constexpr int TK = 128, TN = 128, BK = 32;
enum : int { W_NONE = 0, W_BF16 = 1, W_INT8 = 2, W_INT4 = 3 };

struct MergeArgs {
    const void* W;
    const uint16_t* scales;
    GemmOperand a, b;      // A[K][ld] (rank index contiguous), B[r][N]
    void* out;
    float scaling;
    int K, N, r;           // r: rank rounded up to a multiple of 8 (the copy of A is zero-padded)
    int r_rows;            // rows of B that exist
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// fp32 tile in LDS, [TK][TN], 16-byte chunks of a row XOR-swizzled with the row so that the 32
// rows a wave writes at one column land in 32 different chunks
__device__ __forceinline__ uint32_t t_off(int row, int col)
{
    return (uint32_t)row * (TN * 4) + (uint32_t)((((col >> 2) ^ row) & 31) << 4) + (uint32_t)(col & 3) * 4u;
}

template <int WMODE, bool OUT_F32>
__global__ __launch_bounds__(NT) void merge_kernel(MergeArgs p)
{
    using FA = Feeder<OP_KC, TK, BK, 4>;
    using FB = Feeder<OP_XC, TN, BK, 4>;
    using TA = typename FA::Tile;
    using TB = typename FB::Tile;
    constexpr int TILE_A_BYTES = FA::TILE_BYTES, STAGE_BYTES = FA::TILE_BYTES + FB::TILE_BYTES;
    constexpr int L = FA::PER + FB::PER;
    constexpr int LDS_BYTES = TK * TN * 4;
    static_assert(2 * STAGE_BYTES <= LDS_BYTES, "operand stages live under the output tile");

    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_k0 = (wave >> 1) * 64;
    const int wave_n0 = (wave & 1) * 64;
    const int tiles_n = (p.N + TN - 1) / TN;
    const int tk = blockIdx.x / tiles_n, tn = blockIdx.x - tk * tiles_n;
    const int k0 = tk * TK, n0 = tn * TN;

    // ---- (1) base weight of this tile, requested before anything else
    // bf16: row-major, the same 8-column pieces the thread streams out in (4)
    // quantised: channel n0 + tid/2, k half tid%2 (64 codes)
    constexpr int PASSES = TK * (TN / 8) / NT;                 // 8 rows of 16 per thread
    const int oc = tid & 15, orow = tid >> 4;                   // output piece: cols 8 oc.., rows orow + 16 q
    u32x4 wreg[WMODE == W_BF16 ? PASSES : 1];
    u32x2 q8[WMODE == W_INT8 ? 8 : 1];
    u32x4 q4[WMODE == W_INT4 ? 2 : 1];
    float wscale = 0.f;
    const int qn = n0 + (tid >> 1), qk = k0 + (tid & 1) * 64;
    if constexpr (WMODE == W_BF16) {
#pragma unroll
        for (int q = 0; q < PASSES; q++) {
            const int k = k0 + orow + 16 * q, n = n0 + oc * 8;
            wreg[q] = (u32x4){0u, 0u, 0u, 0u};
            if (k < p.K && n < p.N)
                wreg[q] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(p.W) + (size_t)k * (size_t)p.N + (size_t)n);
        }
    } else if constexpr (WMODE == W_INT8) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            q8[j] = (u32x2){0u, 0u};
            if (qn < p.N && qk + 8 * j < p.K)
                q8[j] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(p.W) + (size_t)qn * (size_t)p.K + (size_t)(qk + 8 * j));
        }
        if (qn < p.N) wscale = (float)__builtin_bit_cast(_Float16, p.scales[qn]);
    } else if constexpr (WMODE == W_INT4) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
            q4[j] = (u32x4){0u, 0u, 0u, 0u};
            if (qn < p.N && qk + 32 * j < p.K)
                q4[j] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(p.W) + ((size_t)qn * (size_t)p.K + (size_t)(qk + 32 * j)) / 2);
        }
        if (qn < p.N && qk < p.K) wscale = (float)__builtin_bit_cast(_Float16, p.scales[(size_t)qn * (size_t)(p.K / 64) + (size_t)(qk / 64)]);
    }

    // ---- (2) acc[j][i]: lane holds (A B)[k][n .. n+3] for k = wave_k0 + 32 i + lane % 32
    f32x16 acc[2][2];
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][i][v] = 0.f;
    {
        FA fa;
        FB fb;
        fa.init(p.a, k0, p.K, p.r, wave, lane);
        fb.init(p.b, n0, p.N, p.r_rows, wave, lane);
        const FragAddr aa = TA::make(wave_k0, lane);
        const FragAddr ab = TB::make(wave_n0, lane);
        fa.issue(lds, 0, p.r, wave);
        fb.issue(lds + TILE_A_BYTES, 0, p.r, wave);
        int stage = 0;
        for (int r0 = 0; r0 < p.r; r0 += BK) {
            unsigned char* cur = lds + stage * STAGE_BYTES;
            unsigned char* nxt = lds + (stage ^ 1) * STAGE_BYTES;
            // the other stage was released by the barrier that ended the previous trip
            fa.issue(nxt, r0 + BK, p.r, wave);
            fb.issue(nxt + TILE_A_BYTES, r0 + BK, p.r, wave);
            FHPC_WAIT_VM(L);
            wg_barrier();
#pragma unroll
            for (int s = 0; s < BK / 16; s++) {
                bf16x8 ra[2], rb[2];
#pragma unroll
                for (int i = 0; i < 2; i++) ra[i] = TA::frag(cur, aa, i, s);
#pragma unroll
                for (int j = 0; j < 2; j++) rb[j] = TB::frag(cur + TILE_A_BYTES, ab, j, s);
#pragma unroll
                for (int j = 0; j < 2; j++)
#pragma unroll
                    for (int i = 0; i < 2; i++)
                        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rb[j], ra[i], acc[j][i], 0, 0, 0);
            }
            FHPC_WAIT_LGKM0();
            wg_barrier();
            stage ^= 1;
        }
        FHPC_WAIT_VM(0);        // the last trip's requests (past the end of the rank: zeros) still land in LDS
        wg_barrier();
    }

    // ---- (3) scaling * A B -> fp32 tile
    const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int row = wave_k0 + 32 * i + l32;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4 o;
                o.x = acc[j][i][4 * g + 0] * p.scaling;
                o.y = acc[j][i][4 * g + 1] * p.scaling;
                o.z = acc[j][i][4 * g + 2] * p.scaling;
                o.w = acc[j][i][4 * g + 3] * p.scaling;
                *reinterpret_cast<f32x4*>(lds + t_off(row, wave_n0 + 32 * j + 8 * g + 4 * hi)) = o;
            }
        }
    __syncthreads();
    if constexpr (WMODE == W_INT8 || WMODE == W_INT4) {
        // element (k, n) of the tile belongs to exactly one thread here: code * scale is exact in
        // fp32, the sum is rounded once
        const int col = tid >> 1, rbase = (tid & 1) * 64;
#pragma unroll
        for (int e = 0; e < 64; e++) {
            int code;
            if constexpr (WMODE == W_INT8) {
                const uint32_t w = (e & 4) ? q8[e >> 3].y : q8[e >> 3].x;
                code = __builtin_amdgcn_sbfe((int)w, 8 * (e & 3), 8);
            } else {
                const u32x4 v = q4[e >> 5];
                const uint32_t w = ((e >> 3) & 3) == 0 ? v.x : ((e >> 3) & 3) == 1 ? v.y : ((e >> 3) & 3) == 2 ? v.z : v.w;
                code = __builtin_amdgcn_sbfe((int)w, 4 * (e & 7), 4);
            }
            float* t = reinterpret_cast<float*>(lds + t_off(rbase + e, col));
            *t += (float)code * wscale;
        }
        __syncthreads();
    }

    // ---- (4) rows out
#pragma unroll
    for (int q = 0; q < PASSES; q++) {
        const int row = orow + 16 * q;
        const int k = k0 + row, n = n0 + oc * 8;
        f32x4 lo = *reinterpret_cast<const f32x4*>(lds + t_off(row, oc * 8));
        f32x4 hi4 = *reinterpret_cast<const f32x4*>(lds + t_off(row, oc * 8 + 4));
        if constexpr (WMODE == W_BF16) {
            const u32x4 w = wreg[q];
            lo.x += bf16_lo(w.x); lo.y += bf16_hi(w.x); lo.z += bf16_lo(w.y); lo.w += bf16_hi(w.y);
            hi4.x += bf16_lo(w.z); hi4.y += bf16_hi(w.z); hi4.z += bf16_lo(w.w); hi4.w += bf16_hi(w.w);
        }
        if (k < p.K && n < p.N) {
            if constexpr (OUT_F32) {
                float* dst = reinterpret_cast<float*>(p.out) + (size_t)k * (size_t)p.N + (size_t)n;
                *reinterpret_cast<f32x4*>(dst) = lo;
                *reinterpret_cast<f32x4*>(dst + 4) = hi4;
            } else {
                u32x4 o;
                o.x = pack_bf16(lo.x, lo.y);
                o.y = pack_bf16(lo.z, lo.w);
                o.z = pack_bf16(hi4.x, hi4.y);
                o.w = pack_bf16(hi4.z, hi4.w);
                *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.out) + (size_t)k * (size_t)p.N + (size_t)n) = o;
            }
        }
    }
}

template <int WMODE, bool OUT_F32>
static hipError_t launch(const MergeArgs& a, double w_bytes, hipStream_t s)
{
    const int tiles = ((a.K + TK - 1) / TK) * ((a.N + TN - 1) / TN);
    const double bytes = w_bytes + (double)a.K * a.N * (OUT_F32 ? 4.0 : 2.0) + 2.0 * a.r_rows * ((double)a.K + a.N);
    const char* names[4] = {"merge<none>", "merge<bf16>", "merge<int8>", "merge<int4>"};
    const int slot = prof_begin(names[WMODE], 2.0 * a.K * (double)a.N * a.r_rows, bytes, s);
    hipLaunchKernelGGL((merge_kernel<WMODE, OUT_F32>), dim3((unsigned)tiles), dim3(NT), 0, s, a);
    prof_end(slot, s);
    return hipGetLastError();
}

}  // namespace mrg

hipError_t launch_merge(const void* W, const void* scales, int w_kind, const void* A, int64_t lda, const void* B,
                        float scaling, void* out, bool out_f32, int64_t K, int64_t r, int64_t N, hipStream_t s)
{
    using namespace mrg;
    MergeArgs a;
    a.W = W;
    a.scales = static_cast<const uint16_t*>(scales);
    a.a = GemmOperand{A, lda, nullptr, 0};
    a.b = GemmOperand{B, N, nullptr, 0};
    a.out = out;
    a.scaling = scaling;
    a.K = (int)K;
    a.N = (int)N;
    a.r = (int)lda;
    a.r_rows = (int)r;
    const double kn = (double)K * (double)N;
    switch (w_kind) {
    case W_NONE: return out_f32 ? launch<W_NONE, true>(a, 0.0, s) : launch<W_NONE, false>(a, 0.0, s);
    case W_BF16: return out_f32 ? launch<W_BF16, true>(a, 2.0 * kn, s) : launch<W_BF16, false>(a, 2.0 * kn, s);
    case W_INT8: return out_f32 ? launch<W_INT8, true>(a, kn + 2.0 * N, s) : launch<W_INT8, false>(a, kn + 2.0 * N, s);
    case W_INT4: return out_f32 ? launch<W_INT4, true>(a, 0.5 * kn + kn / 32.0, s) : launch<W_INT4, false>(a, 0.5 * kn + kn / 32.0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace fhpc
