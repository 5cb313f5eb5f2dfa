/* Drives every function of oracle/oracle.c on small, odd-sized inputs held in exactly sized
 * heap blocks.  Built with -fsanitize=address,undefined by tests/test_oracle_sanitized.py: an
 * out-of-bounds index, a use of freed memory, a signed overflow or a misaligned access in the
 * oracle aborts the run.  Prints a checksum so that the work cannot be optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double orc_f16_to_f64(uint16_t h);
uint16_t orc_f32_to_f16(float f);
void orc_lowrank_fwd(const double *, const double *, const double *, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_lowrank_bwd(const double *, const double *, const double *, const double *, double *, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_unpack_int4(const uint8_t *, int8_t *, int64_t);
void orc_pack_int4(const int8_t *, uint8_t *, int64_t);
void orc_quantize_int8_perchannel(const float *, int8_t *, uint16_t *, int64_t, int64_t);
void orc_quantize_int4_block(const float *, uint8_t *, uint16_t *, int64_t, int64_t, int64_t);
void orc_dequant(const void *, const uint16_t *, int, int64_t, double *, int64_t, int64_t);
void orc_qlinear_lowrank_fwd(const double *, const double *, const double *, const double *, double, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_qlinear_lowrank_bwd(const double *, const double *, const double *, const double *, double, const double *, double *, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_blend_fwd(const double *, const double *, const double *, const double *, double, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_blend_bwd(const double *, const double *, const double *, const double *, double, const double *, double *, double *, double *, int64_t, int64_t, int64_t, int64_t);
void orc_merge(const double *, const double *, const double *, double, double *, int64_t, int64_t, int64_t);
void orc_swiglu_fwd(const double *, const double *, double *, int64_t);
void orc_swiglu_bwd(const double *, const double *, const double *, double *, double *, int64_t);
int orc_num_threads(void);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static double *dvec(size_t n) { double *p = malloc(sizeof(double) * n); for (size_t i = 0; i < n; i++) p[i] = rnd(); return p; }
static double sum(const double *p, size_t n) { double s = 0; for (size_t i = 0; i < n; i++) s += p[i]; return s; }

int main(void)
{
    const int64_t M = 7, K = 128, r = 3, N = 5;      /* K a multiple of 64 for the 4-bit blocks */
    double acc = 0;
    double *X = dvec(M * K), *A = dvec(K * r), *B = dvec(r * N), *dY = dvec(M * N);
    double *H = dvec(M * r), *Y = dvec(M * N), *dX = dvec(M * K), *dA = dvec(K * r), *dB = dvec(r * N);
    orc_lowrank_fwd(X, A, B, H, Y, M, K, r, N);
    orc_lowrank_bwd(X, A, B, dY, dX, dA, dB, M, K, r, N);
    acc += sum(Y, M * N) + sum(dX, M * K) + sum(dA, K * r) + sum(dB, r * N);

    float *W = malloc(sizeof(float) * K * N);
    for (int64_t i = 0; i < K * N; i++) W[i] = (float)(0.04 * rnd());
    for (int64_t k = 0; k < K; k++) W[k * N + 2] = 0.f;                 /* an all-zero channel */
    int8_t *q8 = malloc(N * K);
    uint16_t *s8 = malloc(sizeof(uint16_t) * N);
    uint8_t *q4 = malloc(N * K / 2);
    uint16_t *s4 = malloc(sizeof(uint16_t) * N * (K / 64));
    double *Wd = dvec(K * N);
    orc_quantize_int8_perchannel(W, q8, s8, K, N);
    orc_dequant(q8, s8, 8, 64, Wd, K, N);
    acc += sum(Wd, K * N);
    orc_qlinear_lowrank_fwd(X, Wd, A, B, 2.0, H, Y, M, K, r, N);
    orc_qlinear_lowrank_bwd(X, Wd, A, B, 2.0, dY, dX, dA, dB, M, K, r, N);
    acc += sum(Y, M * N) + sum(dX, M * K);
    orc_quantize_int4_block(W, q4, s4, K, N, 64);
    orc_dequant(q4, s4, 4, 64, Wd, K, N);
    acc += sum(Wd, K * N);
    orc_blend_fwd(X, Wd, A, B, 0.3, H, Y, M, K, r, N);
    orc_blend_bwd(X, Wd, A, B, 0.3, dY, dX, dA, dB, M, K, r, N);
    acc += sum(Y, M * N) + sum(dA, K * r);
    double *Wp = dvec(K * N);
    orc_merge(Wd, A, B, 0.5, Wp, K, r, N);
    acc += sum(Wp, K * N);
    orc_merge(NULL, A, B, 1.0, Wp, K, r, N);
    acc += sum(Wp, K * N);

    uint8_t bytes[256];
    int8_t codes[512];
    for (int i = 0; i < 256; i++) bytes[i] = (uint8_t)i;
    orc_unpack_int4(bytes, codes, 256);
    orc_pack_int4(codes, bytes, 256);
    for (int i = 0; i < 256; i++) acc += bytes[i] == (uint8_t)i ? 0 : 1e9;

    double *G = dvec(33), *U = dvec(33), *dZ = dvec(33), *Z = dvec(33), *dG = dvec(33), *dU = dvec(33);
    G[0] = 800.0; G[1] = -800.0;                                          /* saturating gates */
    orc_swiglu_fwd(G, U, Z, 33);
    orc_swiglu_bwd(G, U, dZ, dG, dU, 33);
    acc += sum(Z, 33) + sum(dG, 33) + sum(dU, 33);
    for (int i = 0; i < 65536; i += 257) acc += orc_f16_to_f64((uint16_t)i) == orc_f16_to_f64((uint16_t)i) ? 0 : 0;   /* NaNs pass through */
    acc += orc_f32_to_f16(65504.0f) + orc_f32_to_f16(1e-8f) + orc_f32_to_f16(-0.0f);

    free(X); free(A); free(B); free(dY); free(H); free(Y); free(dX); free(dA); free(dB);
    free(W); free(q8); free(s8); free(q4); free(s4); free(Wd); free(Wp);
    free(G); free(U); free(dZ); free(Z); free(dG); free(dU);
    printf("threads %d checksum %.6f\n", orc_num_threads(), acc);
    return 0;
}
