/*
 * CPU oracle for the factorised linear layer and its quantised finetuning form.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file; it
 * exists so that tests, the smoke check and the benchmark's cpu_baseline leg can
 * compare the HIP library against an independent, obviously-correct reference.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Everything is the plain definition evaluated in fp64 with triple loops
 * (i-k-j order, OpenMP over independent output rows only, no blocking, no BLAS).
 * Inputs arrive already up-cast exactly to double by the Python wrapper, except
 * the quantised weight bytes and the fp16 scale bit patterns, which are decoded
 * here.
 *
 * Notation (row form of the paper's layer, Sec. 3.2 eq. "low_rank_layer" and
 * Sec. 4.1 item 1): tokens are rows of X[M,K]; A[K,r], B[r,N]; H = X A; Y = H B.
 * The paper writes y = B A x with column vectors, i.e. A_paper = A^T,
 * B_paper = B^T.
 *
 * Pins: every function below is pinned by tests/test_oracle_*.py (association
 * identity, gradient identities, finite differences, adjoint test, numpy fp64
 * cross-check, hand-built exact quantisation cases, exhaustive nibble table).
 * No function here is "parity unpinned".  (The rank-r factorisation of a pretrained weight, which
 * needs a singular value decomposition, lives in the Python wrapper and uses numpy's.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* fp16 <-> fp32 bit conversions (IEEE binary16, round to nearest even) */
/* ------------------------------------------------------------------ */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* binary16 bit pattern -> double, exact. */
double orc_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)        v = ldexp((double)m, -24);            /* zero / subnormal */
    else if (e == 31)  v = m ? NAN : INFINITY;
    else               v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

/* float -> binary16 bit pattern, round to nearest, ties to even. */
uint16_t orc_f32_to_f16(float f)
{
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u)                       /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((a > 0x7F800000u) ? 0x200u : 0u));
    if (a >= 0x477FF000u)                       /* rounds to >= 65520 -> inf */
        return (uint16_t)(sign | 0x7C00u);
    int e = (int)(a >> 23) - 127;               /* unbiased exponent */
    if (e >= -14) {                             /* normal half */
        uint32_t mant = a & 0x7FFFFFu;
        uint32_t half = ((uint32_t)(e + 15) << 10) | (mant >> 13);
        uint32_t rem = mant & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) half++;
        return (uint16_t)(sign | half);         /* carry into exponent is correct */
    }
    if (e < -25) return sign;                   /* below half of the smallest subnormal */
    /* subnormal half: value = mant24 * 2^(e-23); unit is 2^-24 */
    uint32_t mant24 = (a & 0x7FFFFFu) | 0x800000u;
    int shift = -e - 1;                         /* 14..24 : mant24 >> shift gives units of 2^-24 */
    uint32_t q = mant24 >> shift;
    uint32_t rem = mant24 & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1);
    if (rem > halfway || (rem == halfway && (q & 1u))) q++;
    return (uint16_t)(sign | q);
}

/* ------------------------------------------------------------------ */
/* Factorised linear layer, Sec. 3.2 eq. low_rank_layer (row form)      */
/* ------------------------------------------------------------------ */

/* C[M,N] = A[M,K] * B[K,N], all row-major doubles; i-k-j. */
static void mm_nn(const double *A, const double *B, double *C,
                  int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; i++) {
        double *c = C + i * N;
        for (int64_t j = 0; j < N; j++) c[j] = 0.0;
        for (int64_t k = 0; k < K; k++) {
            double a = A[i * K + k];
            const double *b = B + k * N;
            for (int64_t j = 0; j < N; j++) c[j] += a * b[j];
        }
    }
}

/* C[M,N] = A[M,K] * B[N,K]^T. */
static void mm_nt(const double *A, const double *B, double *C,
                  int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; i++) {
        for (int64_t j = 0; j < N; j++) {
            double s = 0.0;
            for (int64_t k = 0; k < K; k++) s += A[i * K + k] * B[j * K + k];
            C[i * N + j] = s;
        }
    }
}

/* C[K,N] = A[M,K]^T * B[M,N]  (sum over the M rows). */
static void mm_tn(const double *A, const double *B, double *C,
                  int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; k++) {
        double *c = C + k * N;
        for (int64_t j = 0; j < N; j++) c[j] = 0.0;
        for (int64_t i = 0; i < M; i++) {
            double a = A[i * K + k];
            const double *b = B + i * N;
            for (int64_t j = 0; j < N; j++) c[j] += a * b[j];
        }
    }
}

/* H = X A ; Y = H B.  H is never rounded between the two sums.
 * H (M*r doubles) is an output too so that tests can inspect it. */
void orc_lowrank_fwd(const double *X, const double *A, const double *B,
                     double *H, double *Y,
                     int64_t M, int64_t K, int64_t r, int64_t N)
{
    mm_nn(X, A, H, M, K, r);
    mm_nn(H, B, Y, M, r, N);
}

/* Matrix calculus on Y = (X A) B with upstream gradient dY:
 *   dH = dY B^T ; dB = H^T dY ; dA = X^T dH ; dX = dH A^T.
 * (The paper's forward/backward flow figure in Sec. 4.2 shows this data flow;
 * it prints no formulas.) */
void orc_lowrank_bwd(const double *X, const double *A, const double *B,
                     const double *dY, double *dX, double *dA, double *dB,
                     int64_t M, int64_t K, int64_t r, int64_t N)
{
    double *H  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    double *dH = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    mm_nn(X, A, H, M, K, r);
    mm_nt(dY, B, dH, M, N, r);
    mm_tn(H, dY, dB, M, r, N);
    mm_tn(X, dH, dA, M, K, r);
    mm_nt(dH, A, dX, M, r, K);
    free(H);
    free(dH);
}

/* ------------------------------------------------------------------ */
/* Per-vector weight quantisation, Sec. 5.2 "Quantization"              */
/* ------------------------------------------------------------------ */

/* Signed 4-bit codes, two per byte: element k (even) in the low nibble,
 * element k+1 in the high nibble, two's complement. */
void orc_unpack_int4(const uint8_t *packed, int8_t *q, int64_t n_bytes)
{
    for (int64_t i = 0; i < n_bytes; i++) {
        uint8_t b = packed[i];
        int lo = b & 0xF, hi = (b >> 4) & 0xF;
        q[2 * i]     = (int8_t)(lo >= 8 ? lo - 16 : lo);
        q[2 * i + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
    }
}

void orc_pack_int4(const int8_t *q, uint8_t *packed, int64_t n_bytes)
{
    for (int64_t i = 0; i < n_bytes; i++)
        packed[i] = (uint8_t)((q[2 * i] & 0xF) | ((q[2 * i + 1] & 0xF) << 4));
}

/* Symmetric absmax quantiser of one vector of `len` fp32 values with stride
 * `stride`: scale = fp16_rne(absmax / qmax) computed in fp32; codes are
 * rint(w / (float)scale) (ties to even, fp32 divide) clamped to [-qmax, qmax].
 * A zero scale (all-zero vector, or absmax/qmax underflowing fp16) gives
 * all-zero codes. */
static uint16_t quantize_vector(const float *w, int64_t stride, int64_t len,
                                int qmax, int8_t *q)
{
    float a = 0.0f;
    for (int64_t i = 0; i < len; i++) {
        float v = fabsf(w[i * stride]);
        if (v > a) a = v;
    }
    float sc32 = a / (float)qmax;
    uint16_t hs = orc_f32_to_f16(sc32);
    float sf = (float)orc_f16_to_f64(hs);
    for (int64_t i = 0; i < len; i++) {
        int c = 0;
        if (sf != 0.0f) {
            float t = w[i * stride] / sf;       /* fp32 divide */
            float rr = rintf(t);                /* default rounding mode: nearest even */
            if (rr > (float)qmax) rr = (float)qmax;
            if (rr < -(float)qmax) rr = -(float)qmax;
            c = (int)rr;
        }
        q[i] = (int8_t)c;
    }
    return hs;
}

/* W fp32 [K,N] row-major -> q int8 [N][K], scales fp16 bits [N]:
 * one vector per output channel n (column of W). */
void orc_quantize_int8_perchannel(const float *W, int8_t *q, uint16_t *scales,
                                  int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++)
        scales[n] = quantize_vector(W + n, N, K, 127, q + n * K);
}

/* W fp32 [K,N] -> packed [N][K/2], scales fp16 bits [N][K/block]:
 * one vector per output channel n and per block of `block` consecutive k. */
void orc_quantize_int4_block(const float *W, uint8_t *packed, uint16_t *scales,
                             int64_t K, int64_t N, int64_t block)
{
    int64_t nb = K / block;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        int8_t *tmp = (int8_t *)malloc((size_t)K);
        for (int64_t b = 0; b < nb; b++)
            scales[n * nb + b] =
                quantize_vector(W + (b * block) * N + n, N, block, 7, tmp + b * block);
        orc_pack_int4(tmp, packed + n * (K / 2), K / 2);
        free(tmp);
    }
}

/* Dequantise to Wd[K,N] (double, exact product of integer code and fp16 scale).
 * scheme 8: q int8 [N][K], scales [N].  scheme 4: packed [N][K/2], scales [N][K/block]. */
void orc_dequant(const void *Wq, const uint16_t *scales, int scheme, int64_t block,
                 double *Wd, int64_t K, int64_t N)
{
    if (scheme == 8) {
        const int8_t *q = (const int8_t *)Wq;
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            double s = orc_f16_to_f64(scales[n]);
            for (int64_t k = 0; k < K; k++)
                Wd[k * N + n] = (double)q[n * K + k] * s;
        }
    } else {
        const uint8_t *p = (const uint8_t *)Wq;
        int64_t nb = K / block;
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            int8_t *tmp = (int8_t *)malloc((size_t)K);
            orc_unpack_int4(p + n * (K / 2), tmp, K / 2);
            for (int64_t k = 0; k < K; k++) {
                double s = orc_f16_to_f64(scales[n * nb + k / block]);
                Wd[k * N + n] = (double)tmp[k] * s;
            }
            free(tmp);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Finetuning layer, Sec. 5.1 eq. new_linear_layer, frozen quantised W  */
/* ------------------------------------------------------------------ */

/* Y = X Wd + s (X A) B, with Wd[K,N] the dequantised frozen weight. */
void orc_qlinear_lowrank_fwd(const double *X, const double *Wd,
                             const double *A, const double *B, double s,
                             double *H, double *Y,
                             int64_t M, int64_t K, int64_t r, int64_t N)
{
    double *L = (double *)malloc(sizeof(double) * (size_t)M * (size_t)N);
    mm_nn(X, Wd, Y, M, K, N);
    mm_nn(X, A, H, M, K, r);
    mm_nn(H, B, L, M, r, N);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M * N; i++) Y[i] += s * L[i];
    free(L);
}

/* dH = dY B^T ; dX = dY Wd^T + s dH A^T ; dA = s X^T dH ; dB = s (X A)^T dY.
 * W is frozen (Sec. 5.1): no dW. */
void orc_qlinear_lowrank_bwd(const double *X, const double *Wd,
                             const double *A, const double *B, double s,
                             const double *dY, double *dX, double *dA, double *dB,
                             int64_t M, int64_t K, int64_t r, int64_t N)
{
    double *H  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    double *dH = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    double *T  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
    mm_nn(X, A, H, M, K, r);
    mm_nt(dY, B, dH, M, N, r);
    mm_nt(dY, Wd, dX, M, N, K);            /* dY[M,N] * Wd[K,N]^T */
    mm_nt(dH, A, T, M, r, K);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M * K; i++) dX[i] += s * T[i];
    mm_tn(X, dH, dA, M, K, r);
    mm_tn(H, dY, dB, M, r, N);
    for (int64_t i = 0; i < K * r; i++) dA[i] *= s;
    for (int64_t i = 0; i < r * N; i++) dB[i] *= s;
    free(H);
    free(dH);
    free(T);
}

/* ------------------------------------------------------------------ */
/* Blend of a frozen pretrained weight with the factor pair, Sec. 4.1    */
/* item 3:  y = alpha W x + (1 - alpha) B A x,  0 <= alpha <= 1          */
/* ------------------------------------------------------------------ */

/* Row form: Y = alpha X W + (1 - alpha) (X A) B, with W[K,N] frozen. */
void orc_blend_fwd(const double *X, const double *W,
                   const double *A, const double *B, double alpha,
                   double *H, double *Y,
                   int64_t M, int64_t K, int64_t r, int64_t N)
{
    double *P = (double *)malloc(sizeof(double) * (size_t)M * (size_t)N);   /* X W */
    double *L = (double *)malloc(sizeof(double) * (size_t)M * (size_t)N);   /* (X A) B */
    mm_nn(X, W, P, M, K, N);
    mm_nn(X, A, H, M, K, r);
    mm_nn(H, B, L, M, r, N);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M * N; i++) Y[i] = alpha * P[i] + (1.0 - alpha) * L[i];
    free(P);
    free(L);
}

/* dH = dY B^T ; dX = alpha dY W^T + (1 - alpha) dH A^T ;
 * dA = (1 - alpha) X^T dH ; dB = (1 - alpha) (X A)^T dY.  W is frozen: no dW. */
void orc_blend_bwd(const double *X, const double *W,
                   const double *A, const double *B, double alpha,
                   const double *dY, double *dX, double *dA, double *dB,
                   int64_t M, int64_t K, int64_t r, int64_t N)
{
    double *H  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    double *dH = (double *)malloc(sizeof(double) * (size_t)M * (size_t)r);
    double *P  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);   /* dY W^T */
    double *T  = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);   /* dH A^T */
    const double beta = 1.0 - alpha;
    mm_nn(X, A, H, M, K, r);
    mm_nt(dY, B, dH, M, N, r);
    mm_nt(dY, W, P, M, N, K);
    mm_nt(dH, A, T, M, r, K);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M * K; i++) dX[i] = alpha * P[i] + beta * T[i];
    mm_tn(X, dH, dA, M, K, r);
    mm_tn(H, dY, dB, M, r, N);
    for (int64_t i = 0; i < K * r; i++) dA[i] *= beta;
    for (int64_t i = 0; i < r * N; i++) dB[i] *= beta;
    free(H);
    free(dH);
    free(P);
    free(T);
}

/* ------------------------------------------------------------------ */
/* Adapted weight materialised for inference, Sec. 5.1 (eq.             */
/* new_linear_layer: W' = W + Delta W, Delta W the product of the pair) */
/* ------------------------------------------------------------------ */

/* Row form: Wp[K,N] = W[K,N] + s * A[K,r] B[r,N]; the paper's case is s = 1.
 * W may be NULL (then Wp = s A B: the dense weight a factor pair stands for). */
void orc_merge(const double *W, const double *A, const double *B, double s,
               double *Wp, int64_t K, int64_t r, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; k++) {
        for (int64_t n = 0; n < N; n++) {
            double d = 0.0;
            for (int64_t j = 0; j < r; j++) d += A[k * r + j] * B[j * N + n];
            Wp[k * N + n] = (W ? W[k * N + n] : 0.0) + s * d;
        }
    }
}

/* ------------------------------------------------------------------ */
/* SiLU-gated product between the FFN's linears, Sec. 3.1 eq. FFN       */
/* ------------------------------------------------------------------ */

static double sigmoid_stable(double g)
{
    if (g >= 0.0) return 1.0 / (1.0 + exp(-g));
    double e = exp(g);
    return e / (1.0 + e);
}

/* Z = U * SiLU(G),  SiLU(g) = g * sigmoid(g). */
void orc_swiglu_fwd(const double *G, const double *U, double *Z, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) Z[i] = U[i] * G[i] * sigmoid_stable(G[i]);
}

/* dU = dZ * SiLU(G);  dG = dZ * U * sigmoid(G) * (1 + G (1 - sigmoid(G))). */
void orc_swiglu_bwd(const double *G, const double *U, const double *dZ,
                    double *dG, double *dU, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) {
        double sg = sigmoid_stable(G[i]);
        dU[i] = dZ[i] * G[i] * sg;
        dG[i] = dZ[i] * U[i] * sg * (1.0 + G[i] * (1.0 - sg));
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
