/* Drives every entry point of the CPU oracle on small, ragged, strided inputs.  Built together with
 * oracle/brq_oracle.c under -fsanitize=address,undefined by tests/test_sanitizers.py: an out-of-bounds access,
 * a misaligned or overflowing operation anywhere in the oracle ends the run with a non-zero status.  It checks
 * memory behaviour, not values (the pins do that). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_hadamard_sylvester(int B, int *out);
int oracle_rotate_dense_f64(const double *x, int64_t M, int64_t K, int64_t B, double *y);
int oracle_block_rotate_signed(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B, const int8_t *signs,
                               void *y, int ydt, int64_t ldy);
int oracle_mxfp4_quantize(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, uint8_t *codes, uint8_t *scales);
int oracle_rotate_quantize_fused_signed(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                                        const int8_t *signs, uint8_t *codes, uint8_t *scales);
int oracle_swiglu(const void *gate, const void *up, int dt, int64_t M, int64_t K, int64_t ldg, int64_t ldu, void *h, int hdt,
                  int64_t ldh);
int oracle_swiglu_rotate_quantize_fused(const void *gate, const void *up, int dt, int64_t M, int64_t K, int64_t ldg,
                                        int64_t ldu, int hdt, int64_t B, const int8_t *signs, uint8_t *codes, uint8_t *scales);
int oracle_matrix_rotate_quantize_fused(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, const float *R, int64_t nR,
                                        uint8_t *codes, uint8_t *scales);
int oracle_block_stats(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B, const int8_t *signs,
                       const float *thresholds, int nt, float *amax, uint64_t *count, double *sqerr, double *sqerr_bfp4);
int oracle_block_stats_summary(const float *amax, const float *sqerr, const float *ref, int64_t n, float outlier,
                               const float *edges, int nedges, uint64_t *hist, uint64_t *counts, double *sums);
int oracle_mxfp4_gemm(const uint8_t *aq, const uint8_t *as, const uint8_t *wq, const uint8_t *ws, int64_t M, int64_t N,
                      int64_t K, const int64_t *rows, int64_t nrows, double *y, double *bound);
uint16_t oracle_f32_to_bf16(float f);
uint16_t oracle_f64_to_bf16(double x);
float oracle_round_to_f16(float f);

static uint32_t rng_state = 12345u;
static float rnd(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) / 8388608.0f - 1.0f) * 8.0f;
}

#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s -> %d\n", #call, rc_); return 1; } } while (0)

int main(void) {
    enum { M = 5, K = 256, LD = K + 24, N = 7 };
    /* every buffer is exactly as large as the call may touch: the sanitizer sees any step outside */
    float *x = malloc(sizeof(float) * M * LD), *y = malloc(sizeof(float) * M * LD);
    uint16_t *xb = malloc(sizeof(uint16_t) * M * LD), *hb = malloc(sizeof(uint16_t) * M * K);
    int8_t *signs = malloc(K);
    uint8_t *codes = malloc(M * K / 2), *scales = malloc(M * K / 32), *wq = malloc(N * K / 2), *ws = malloc(N * K / 32);
    float *R = malloc(sizeof(float) * (K / 32) * 1024), *amax = malloc(sizeof(float) * M * K / 32), *sq32 = malloc(sizeof(float) * M * K / 32);
    double *sqerr = malloc(sizeof(double) * M * K / 32), *bf = malloc(sizeof(double) * M * K / 32), *yy = malloc(sizeof(double) * 2 * N),
           *bound = malloc(sizeof(double) * 2 * N), *xd = malloc(sizeof(double) * M * K), *yd = malloc(sizeof(double) * M * K);
    int *H = malloc(sizeof(int) * 64 * 64);
    if (!x || !y || !xb || !hb || !signs || !codes || !scales || !wq || !ws || !R || !amax || !sq32 || !sqerr || !bf || !yy || !bound || !xd || !yd || !H) return 2;
    for (int i = 0; i < M * LD; ++i) { x[i] = rnd(); xb[i] = oracle_f32_to_bf16(rnd()); }
    for (int i = 0; i < M * K; ++i) xd[i] = rnd();
    for (int i = 0; i < K; ++i) signs[i] = (i * 7 % 3) ? 1 : -1;
    for (int i = 0; i < (K / 32) * 1024; ++i) R[i] = rnd() * 0.1f;
    for (int i = 0; i < N * K / 2; ++i) wq[i] = (uint8_t)(rng_state = rng_state * 1664525u + 1013904223u, rng_state >> 24);
    for (int i = 0; i < N * K / 32; ++i) ws[i] = (uint8_t)(120 + i % 12);
    CHECK(oracle_hadamard_sylvester(64, H));
    CHECK(oracle_rotate_dense_f64(xd, M, K, 64, yd));
    for (int B = 2; B <= K; B *= 2) {
        CHECK(oracle_block_rotate_signed(x, 0, M, K, LD, B, signs, y, 0, LD));
        CHECK(oracle_block_rotate_signed(xb, 1, M, K, LD, B, NULL, hb, 1, K));
        CHECK(oracle_rotate_quantize_fused_signed(xb, 1, M, K, LD, B, signs, codes, scales));
    }
    CHECK(oracle_mxfp4_quantize(x, 0, M, K, LD, codes, scales));
    CHECK(oracle_swiglu(xb, xb + K / 2 - 8 + 24, 1, M, K / 2 - 8 + 0, LD, LD, hb, 1, K));     /* two halves of one buffer, ragged K */
    CHECK(oracle_swiglu_rotate_quantize_fused(x, x + 128, 0, M, 128, LD, LD, 1, 32, signs, codes, scales));
    CHECK(oracle_swiglu_rotate_quantize_fused(x, x + 128, 0, M, 128, LD, LD, 0, 1, NULL, codes, scales));
    CHECK(oracle_matrix_rotate_quantize_fused(xb, 1, M, K, LD, R, K / 32, codes, scales));
    CHECK(oracle_matrix_rotate_quantize_fused(x, 0, M, K, LD, R, 1, codes, scales));
    {
        const float th[3] = {0.5f, 1.5f, 3.0f}, edges[4] = {0.5f, 1.0f, 2.0f, 4.0f};
        uint64_t cnt[3] = {0, 0, 0}, hist[5] = {0}, c4[4] = {0};
        double s4[4] = {0};
        CHECK(oracle_block_stats(xb, 1, M, K, LD, 32, signs, th, 3, amax, cnt, sqerr, bf));
        CHECK(oracle_block_stats(x, 0, M, K, LD, 1, NULL, NULL, 0, amax, NULL, sqerr, NULL));
        for (int i = 0; i < M * K / 32; ++i) sq32[i] = (float)sqerr[i];
        CHECK(oracle_block_stats_summary(amax, sq32, amax, M * K / 32, 2.0f, edges, 4, hist, c4, s4));
        CHECK(oracle_block_stats_summary(amax, NULL, NULL, M * K / 32, 2.0f, NULL, 0, hist, c4, s4));
    }
    {
        const int64_t rows[2] = {4, 0};
        CHECK(oracle_mxfp4_quantize(x, 0, M, K, LD, codes, scales));
        CHECK(oracle_mxfp4_gemm(codes, scales, wq, ws, M, N, K, rows, 2, yy, bound));
    }
    /* the scalar conversions at the ends of their ranges */
    volatile uint16_t sink = 0;
    const double edge[] = {0.0, -0.0, 1e-45, 1e-40, 3.0e38, -3.0e38, 65504.0, 65520.0, 1e-8, 2.938735877e-39};
    for (unsigned i = 0; i < sizeof(edge) / sizeof(edge[0]); ++i) {
        sink ^= oracle_f64_to_bf16(edge[i]);
        sink ^= oracle_f32_to_bf16((float)edge[i]);
        sink ^= (uint16_t)oracle_round_to_f16((float)edge[i]);
    }
    free(x); free(y); free(xb); free(hb); free(signs); free(codes); free(scales); free(wq); free(ws); free(R); free(amax);
    free(sq32); free(sqerr); free(bf); free(yy); free(bound); free(xd); free(yd); free(H);
    printf("oracle sanitizer driver ok\n");
    return 0;
}
