/*
 * brq_oracle.c -- plain, slow, CPU-only reference for the block-rotation MXFP4 path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists so that the HIP library can be checked
 * against something that was written from the paper alone.  It shares no code, table,
 * header or helper with the HIP path and must never be linked into, imported by or
 * called from the product library or its Python binding.  Only the tests, the smoke
 * entry and the benchmark's cpu_baseline leg may load it.
 *
 * What it implements ("Block Rotation is All You Need for MXFP4 Quantization"):
 *   - Sec. 4.1: MXFP4 = E2M1 elements (1 sign / 2 exponent / 1 mantissa bit), symmetric,
 *     groups of 32 along the reduction axis, one power-of-two E8M0 scale per group.
 *     The encoding rule itself is the OCP Microscaling v1.0 convention the paper cites:
 *     shared exponent = floor(log2(amax)) - emax_elem, elements rounded to nearest
 *     (ties to the even code) and saturated at +-6, shared exponent clamped to E8M0.
 *   - Sec. 4.3, Eq. (1): R_block = diag(R_1..R_B), R_i orthogonal g x g.  R_i is the
 *     normalised Sylvester Hadamard H_g / sqrt(g) (Sec. 5.1 / Appendix: block-wise
 *     Hadamard, no learned rotation).  This file follows the benchmark's naming and
 *     calls the block SIZE "B" (the paper's g).
 *   - Sec. 4.3 ("reduced online computing"): the online rotation sits in front of down_proj,
 *     whose input in the evaluated LLaMA models is silu(gate) * up; oracle_swiglu* are that
 *     definition in fp64, rounded once, fed to the same rotation and quantizer.
 *   - Eq. (1) with arbitrary orthogonal 32 x 32 blocks (oracle_matrix_rotate*): the dense
 *     per-block product in fp64.
 *   - Sec. 4.1 / 4.2 / Appendix "Rotation Comparison": the block statistics behind the paper's
 *     analysis (block-wise scale, share of data above a threshold, per-block MXFP4 loss),
 *     oracle_block_stats.
 *   - Sec. 2 ("equivalent transformations"): Y = (X R)(W R)^T = X W^T, evaluated on the
 *     quantized operands: Y[m][n] = sum_k deq(A)[m][k] * deq(W)[n][k].
 *
 * Arithmetic: the rotation that feeds the quantizer is an fp32 computation whose
 * operation order is fixed here (oracle_block_rotate), because codes and scales are
 * compared bit for bit; everything else is done in fp64.
 *
 * Pins (tests/test_oracle_pins.py): H H^T = B I; popcount closed form; exact integer
 * products; one-hot rows; norm preservation; involution; block independence; the E2M1
 * value table from the 1/2/1 bit split; hand-worked rounding / tie / saturation /
 * scale cases; round trip of representable blocks; (XH)(WH)^T = XW^T; brute-force GEMM;
 * the SwiGLU producer against torch's float64 silu, the identity silu(g) - silu(-g) = g,
 * known values and limits, the single rounding to bf16 against a hand-worked double-rounding
 * case, and the fused call against the composition of the pinned parts.
 * parity unpinned: the paper prints no quantized block, code, scale or kernel output,
 * so the whole pipeline has no paper-printed value to be compared with.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no -ffast-math, no FTZ/DAZ).
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1

/* Row loops are split over OpenMP threads; rows are independent, so the thread count
 * changes nothing but the wall time. */
void oracle_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
int oracle_get_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------------------------
 * scalar helpers
 * ---------------------------------------------------------------------------------- */

/* bf16 is the upper half of an IEEE fp32: widening is exact. */
float oracle_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even (finite inputs). */
uint16_t oracle_f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

void oracle_bf16_to_f32_array(const uint16_t *in, int64_t n, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_bf16_to_f32(in[i]);
}

static int popcount_u32(uint32_t v) {
    int c = 0;
    while (v) {
        c += (int)(v & 1u);
        v >>= 1;
    }
    return c;
}

static int is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

static float load_elem(const void *x, int dt, int64_t idx) {
    if (dt == ORACLE_BF16) return oracle_bf16_to_f32(((const uint16_t *)x)[idx]);
    return ((const float *)x)[idx];
}

/* ------------------------------------------------------------------------------------
 * Sylvester Hadamard (Sec. 4.3: the orthogonal block R_i, before normalisation)
 *   H_1 = [1],  H_2n = [[H_n, H_n], [H_n, -H_n]]   <=>   H[i][j] = (-1)^popcount(i & j)
 * ---------------------------------------------------------------------------------- */
int oracle_hadamard_entry(int B, int i, int j) {
    (void)B;
    return (popcount_u32((uint32_t)i & (uint32_t)j) & 1) ? -1 : 1;
}

/* H built by the recursive doubling definition (kept separate from the closed form
 * above so that a test can check one against the other). out is B*B ints. */
int oracle_hadamard_sylvester(int B, int *out) {
    if (!is_pow2(B) || !out) return ORACLE_ERR_ARG;
    out[0] = 1;
    for (int n = 1; n < B; n *= 2) {
        /* grow the n x n matrix held in the top-left corner (row pitch B) to 2n x 2n */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                int h = out[i * B + j];
                out[i * B + (j + n)] = h;
                out[(i + n) * B + j] = h;
                out[(i + n) * B + (j + n)] = -h;
            }
    }
    return ORACLE_OK;
}

/* Mathematical rotation, Eq. (1) with R_i = H_B / sqrt(B), in fp64:
 *   y[r][b*B + j] = (1/sqrt(B)) * sum_i x[r][b*B + i] * H[i][j]                        */
int oracle_rotate_dense_f64(const double *x, int64_t M, int64_t K, int64_t B, double *y) {
    if (!x || !y || !is_pow2(B) || K % B) return ORACLE_ERR_ARG;
    const double c = 1.0 / sqrt((double)B);
    for (int64_t r = 0; r < M; ++r)
        for (int64_t b = 0; b < K / B; ++b)
            for (int64_t j = 0; j < B; ++j) {
                double acc = 0.0;
                for (int64_t i = 0; i < B; ++i)
                    acc += x[r * K + b * B + i] * (double)oracle_hadamard_entry((int)B, (int)i, (int)j);
                y[r * K + b * B + j] = acc * c;
            }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * The rotation as it is computed online: fp32, fixed operation order.
 *
 * In exact arithmetic the in-place butterfly below equals x * H_B (natural order, no
 * bit reversal).  In fp32 the order of the additions decides the last bit, and the
 * quantizer downstream turns last bits into codes, so the order is part of the
 * definition:  stages h = 1, 2, 4, ..., B/2 in ascending order; within a stage the pair
 * (i, i+h) becomes (a+b, a-b); every add/sub is one IEEE round-to-nearest-even fp32
 * operation (no FMA contraction, no reassociation, subnormals kept); then one multiply
 * by fl32(1/sqrt(B)).
 * ---------------------------------------------------------------------------------- */
static void butterfly_f32(float *v, int64_t B) {
    for (int64_t h = 1; h < B; h *= 2)
        for (int64_t i = 0; i < B; ++i)
            if ((i & h) == 0) {
                float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
}

float oracle_rotation_norm(int64_t B) { return (float)(1.0 / sqrt((double)B)); }

/* x: [M][ldx] of xdt, y: [M][ldy] of ydt (fp32, or bf16 = RNE of the fp32 value). */
int oracle_block_rotate_signed(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                               const int8_t *signs, void *y, int ydt, int64_t ldy) {
    if (!x || !y || !is_pow2(B) || B < 2 || K % B || ldx < K || ldy < K) return ORACLE_ERR_ARG;
    const float c = oracle_rotation_norm(B);
    int rc = ORACLE_OK;
#pragma omp parallel
    {
        float *v = (float *)malloc((size_t)B * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < M; ++r) {
            if (!v) { rc = ORACLE_ERR_ARG; continue; }
            for (int64_t b = 0; b < K / B; ++b) {
                for (int64_t i = 0; i < B; ++i) {
                    float e = load_elem(x, xdt, r * ldx + b * B + i);
                    /* randomized Hadamard (Sec. 5.1): x D H with D = diag(s), s_k = +-1; the
                       flip is exact and comes before the butterfly */
                    if (signs && signs[b * B + i] < 0) e = -e;
                    v[i] = e;
                }
                butterfly_f32(v, B);
                for (int64_t i = 0; i < B; ++i) {
                    float out = v[i] * c;
                    if (ydt == ORACLE_BF16)
                        ((uint16_t *)y)[r * ldy + b * B + i] = oracle_f32_to_bf16(out);
                    else
                        ((float *)y)[r * ldy + b * B + i] = out;
                }
            }
        }
        free(v);
    }
    return rc;
}

int oracle_block_rotate(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B,
                        void *y, int ydt, int64_t ldy) {
    return oracle_block_rotate_signed(x, xdt, M, K, ldx, B, NULL, y, ydt, ldy);
}

/* ------------------------------------------------------------------------------------
 * MXFP4 (Sec. 4.1)
 * ---------------------------------------------------------------------------------- */

/* E2M1: code = s<<3 | E<<1 | m, exponent bias 1, IEEE-style subnormal, no Inf/NaN:
 *   E > 0: (-1)^s * 2^(E-1) * (1 + m/2);   E = 0: (-1)^s * m/2                        */
double oracle_e2m1_value(int code) {
    int s = (code >> 3) & 1, E = (code >> 1) & 3, m = code & 1;
    double mag = (E > 0) ? ldexp(1.0 + 0.5 * m, E - 1) : 0.5 * m;
    return s ? -mag : mag;
}

/* Shared scale of one group: e = floor(log2(amax)) - 2 (2 = exponent of the largest E2M1
 * normal, 6 = 1.5 * 2^2), clamped to the E8M0 range; byte = e + 127.  amax = 0 gives the
 * smallest scale.  Finite input never produces 0xFF (the E8M0 NaN). */
uint8_t oracle_e8m0_from_amax(float amax) {
    int e;
    if (amax == 0.0f) {
        e = -127;
    } else {
        int ex;
        (void)frexp((double)amax, &ex); /* amax = m * 2^ex, m in [0.5, 1) */
        e = (ex - 1) - 2;
    }
    if (e < -127) e = -127;
    if (e > 127) e = 127;
    return (uint8_t)(e + 127);
}

double oracle_e8m0_value(uint8_t byte) { return ldexp(1.0, (int)byte - 127); }

/* Element code for value y under scale byte sb: r = y / 2^e exactly (fp64 holds it),
 * magnitude = nearest of the eight E2M1 magnitudes, a tie goes to the code whose mantissa
 * bit is 0, anything above 6 saturates to 6.  A result of magnitude zero is emitted as
 * code 0 whatever the sign of y (no negative zero is produced). */
uint8_t oracle_e2m1_encode(float y, uint8_t sb) {
    double r = fabs(ldexp((double)y, 127 - (int)sb));
    int best = 0;
    double bestd = fabs(r - oracle_e2m1_value(0));
    for (int c = 1; c < 8; ++c) {
        double d = fabs(r - oracle_e2m1_value(c));
        if (d < bestd || (d == bestd && (c & 1) == 0)) {
            best = c;
            bestd = d;
        }
    }
    if (best == 0) return 0;
    return (uint8_t)(best | (signbit(y) ? 8 : 0));
}

/* Quantize one group of 32 fp32 values: scale byte + 16 packed bytes
 * (element 2j in the low nibble of byte j, element 2j+1 in the high nibble). */
static void quantize_group(const float *y, uint8_t *codes16, uint8_t *scale) {
    float amax = 0.0f;
    for (int i = 0; i < 32; ++i) {
        float a = fabsf(y[i]);
        if (a > amax) amax = a;
    }
    uint8_t sb = oracle_e8m0_from_amax(amax);
    *scale = sb;
    for (int j = 0; j < 16; ++j) {
        uint8_t lo = oracle_e2m1_encode(y[2 * j], sb);
        uint8_t hi = oracle_e2m1_encode(y[2 * j + 1], sb);
        codes16[j] = (uint8_t)(lo | (hi << 4));
    }
}

/* x [M][ldx] -> codes [M][K/2], scales [M][K/32] (row-major). */
int oracle_mxfp4_quantize(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx,
                          uint8_t *codes, uint8_t *scales) {
    if (!x || !codes || !scales || K % 32 || ldx < K) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        float g[32];
        for (int64_t b = 0; b < K / 32; ++b) {
            for (int i = 0; i < 32; ++i) g[i] = load_elem(x, xdt, r * ldx + b * 32 + i);
            quantize_group(g, codes + r * (K / 2) + b * 16, scales + r * (K / 32) + b);
        }
    }
    return ORACLE_OK;
}

/* Fused call = quantize(block_rotate(x) kept in fp32): the composition, nothing else. */
int oracle_rotate_quantize_fused_signed(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx,
                                        int64_t B, const int8_t *signs, uint8_t *codes, uint8_t *scales) {
    /* B may be smaller than the quantization group (rotation-dimension sweep, Sec. 5.2): the
       rotation block and the 32-element group are independent */
    if (!x || !codes || !scales || K % 32 || B < 2) return ORACLE_ERR_ARG;
    float *y = (float *)malloc((size_t)M * (size_t)K * sizeof(float));
    if (!y) return ORACLE_ERR_ARG;
    int rc = oracle_block_rotate_signed(x, xdt, M, K, ldx, B, signs, y, ORACLE_F32, K);
    if (rc == ORACLE_OK) rc = oracle_mxfp4_quantize(y, ORACLE_F32, M, K, K, codes, scales);
    free(y);
    return rc;
}

int oracle_rotate_quantize_fused(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx,
                                 int64_t B, uint8_t *codes, uint8_t *scales) {
    return oracle_rotate_quantize_fused_signed(x, xdt, M, K, ldx, B, NULL, codes, scales);
}

/* ------------------------------------------------------------------------------------
 * The producer of the rotated layer's input (Sec. 4.3, "reduced online computing": the
 * online rotation R_4 sits in front of down_proj).  In the LLaMA models the paper evaluates,
 * down_proj reads the gated activation
 *
 *     h = silu(gate) * up,      silu(g) = g * sigmoid(g) = g / (1 + exp(-g)).
 *
 * The paper says nothing about how h is computed, so the oracle is the definition itself,
 * written out in fp64 (libm's exp) and rounded ONCE to the type h is kept in: fp32, or bf16
 * when a separate activation kernel would have stored bf16.  An implementation that works in
 * fp32 (hardware exp and reciprocal, say) lands within a few ulp of this value; it is judged
 * by an error bound on h and, for the codes and scales behind it, by the interval that bound
 * leaves open -- not by bit equality with one particular fp32 operation sequence.
 * ---------------------------------------------------------------------------------- */
double oracle_swiglu_f64(double g, double u) { return g / (1.0 + exp(-g)) * u; }

float oracle_swiglu_elem(float g, float u) { return (float)oracle_swiglu_f64((double)g, (double)u); }

/* fp64 -> bf16, one rounding to nearest, ties to even (finite values inside the bf16 range).
 * bf16 keeps 8 significant bits down to 2^-126 and a fixed quantum of 2^-133 below. */
uint16_t oracle_f64_to_bf16(double x) {
    double a = fabs(x), q;
    int ex;
    (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5, 1) */
    int quantum = ex - 8; /* exponent of the last kept bit */
    if (quantum < -133) quantum = -133;
    q = ldexp(rint(ldexp(a, -quantum)), quantum); /* rint: to nearest, ties to even */
    float f = (float)q; /* exact: q has at most 8 significant bits */
    uint32_t bits;
    memcpy(&bits, &f, 4);
    return (uint16_t)((bits >> 16) | (signbit(x) ? 0x8000u : 0u));
}

/* h[r][k] = silu(gate[r][k]) * up[r][k]; gate, up: [M][ldg], [M][ldu] of dt; h: [M][ldh] of
 * hdt: the fp64 value rounded once to fp32, or once to bf16. */
int oracle_swiglu(const void *gate, const void *up, int dt, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                  void *h, int hdt, int64_t ldh) {
    if (!gate || !up || !h || ldg < K || ldu < K || ldh < K) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        for (int64_t k = 0; k < K; ++k) {
            double v = oracle_swiglu_f64((double)load_elem(gate, dt, r * ldg + k), (double)load_elem(up, dt, r * ldu + k));
            if (hdt == ORACLE_BF16)
                ((uint16_t *)h)[r * ldh + k] = oracle_f64_to_bf16(v);
            else
                ((float *)h)[r * ldh + k] = (float)v;
        }
    }
    return ORACLE_OK;
}

/* The same in fp64, unrounded (the value an error bound is stated against). */
int oracle_swiglu_f64_array(const void *gate, const void *up, int dt, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                            double *h) {
    if (!gate || !up || !h || ldg < K || ldu < K) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r)
        for (int64_t k = 0; k < K; ++k)
            h[r * K + k] = oracle_swiglu_f64((double)load_elem(gate, dt, r * ldg + k), (double)load_elem(up, dt, r * ldu + k));
    return ORACLE_OK;
}

/* Producer fused with the online step: quantize(block_rotate(h)) with h as above (rounded once
 * to hdt, then widened exactly), the composition and nothing else.  B = 1 means no rotation
 * (H_1 = [1]). */
int oracle_swiglu_rotate_quantize_fused(const void *gate, const void *up, int dt, int64_t M, int64_t K,
                                        int64_t ldg, int64_t ldu, int hdt, int64_t B, const int8_t *signs,
                                        uint8_t *codes, uint8_t *scales) {
    if (!codes || !scales || K % 32 || B < 1) return ORACLE_ERR_ARG;
    size_t n = (size_t)(M > 0 ? M : 1) * (size_t)K;
    float *h = (float *)malloc(n * sizeof(float));
    uint16_t *hb = (hdt == ORACLE_BF16) ? (uint16_t *)malloc(n * sizeof(uint16_t)) : NULL;
    int rc = (h && (hdt != ORACLE_BF16 || hb)) ? ORACLE_OK : ORACLE_ERR_ARG;
    if (rc == ORACLE_OK) {
        if (hdt == ORACLE_BF16) {
            rc = oracle_swiglu(gate, up, dt, M, K, ldg, ldu, hb, ORACLE_BF16, K);
            if (rc == ORACLE_OK) oracle_bf16_to_f32_array(hb, M * K, h);
        } else {
            rc = oracle_swiglu(gate, up, dt, M, K, ldg, ldu, h, ORACLE_F32, K);
        }
    }
    if (rc == ORACLE_OK) {
        if (B == 1)
            rc = signs ? ORACLE_ERR_ARG : oracle_mxfp4_quantize(h, ORACLE_F32, M, K, K, codes, scales);
        else
            rc = oracle_rotate_quantize_fused_signed(h, ORACLE_F32, M, K, K, B, signs, codes, scales);
    }
    free(h);
    free(hb);
    return rc;
}

/* ------------------------------------------------------------------------------------
 * Block rotation with arbitrary orthogonal blocks (Eq. (1): R_block = diag(R_1, ..., R_n) with
 * every R_i an orthogonal 32 x 32 matrix; the conclusion names learned block rotations for the
 * online step as the next thing to try).  The definition written out, in fp64:
 *     y[r][32 b + j] = sum_i x[r][32 b + i] * R[b][i][j]
 * R: [nR][32][32] fp32, nR = K/32 (one matrix per block) or 1 (the same matrix for every block).
 * bound (optional): sum_i |x_i| |R_ij|, the scale of the rounding error of any evaluation.
 * ---------------------------------------------------------------------------------- */
int oracle_matrix_rotate_f64(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, const float *R,
                             int64_t nR, double *y, double *bound) {
    if (!x || !R || !y || K % 32 || ldx < K || (nR != 1 && nR != K / 32)) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        for (int64_t b = 0; b < K / 32; ++b) {
            const float *Rb = R + (nR == 1 ? 0 : b) * 1024;
            for (int j = 0; j < 32; ++j) {
                double acc = 0.0, mag = 0.0;
                for (int i = 0; i < 32; ++i) {
                    double xv = (double)load_elem(x, xdt, r * ldx + b * 32 + i);
                    double rv = (double)Rb[i * 32 + j];
                    acc += xv * rv;
                    mag += fabs(xv) * fabs(rv);
                }
                y[r * K + b * 32 + j] = acc;
                if (bound) bound[r * K + b * 32 + j] = mag;
            }
        }
    }
    return ORACLE_OK;
}

/* The online step with such blocks: quantize(fl32(y)), y as above.  The rotated value is the
 * exact one rounded once to fp32; an implementation that sums in fp32 lands within a few ulp
 * of it, and the parity tests allow for exactly that (codes are checked against the interval
 * that the error bound leaves open, not for equality). */
int oracle_matrix_rotate_quantize_fused(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx,
                                        const float *R, int64_t nR, uint8_t *codes, uint8_t *scales) {
    if (!codes || !scales) return ORACLE_ERR_ARG;
    size_t n = (size_t)(M > 0 ? M : 1) * (size_t)K;
    double *y = (double *)malloc(n * sizeof(double));
    float *yf = (float *)malloc(n * sizeof(float));
    int rc = (y && yf) ? oracle_matrix_rotate_f64(x, xdt, M, K, ldx, R, nR, y, NULL) : ORACLE_ERR_ARG;
    if (rc == ORACLE_OK) {
        for (int64_t i = 0; i < M * K; ++i) yf[i] = (float)y[i];
        rc = oracle_mxfp4_quantize(yf, ORACLE_F32, M, K, K, codes, scales);
    }
    free(y);
    free(yf);
    return rc;
}

/* Codes of y [M][K] fp32 under GIVEN scale bytes [M][K/32] (the element rule alone; used to ask
 * which codes a value interval allows under the scale an implementation chose). */
int oracle_mxfp4_encode_with_scales(const float *y, const uint8_t *scales, int64_t M, int64_t K, uint8_t *codes) {
    if (!y || !scales || !codes || K % 32) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t sb = scales[r * (K / 32) + j / 16];
            uint8_t lo = oracle_e2m1_encode(y[r * K + 2 * j], sb), hi = oracle_e2m1_encode(y[r * K + 2 * j + 1], sb);
            codes[r * (K / 2) + j] = (uint8_t)((hi << 4) | lo); /* element 2j in the low nibble */
        }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Block statistics of the paper's analysis (Sec. 4.1, 4.2 and the Appendix "Rotation
 * Comparison"), on y = the activation after a transformation: none (B = 1), block rotation
 * (B = 32 ...), global rotation (B = K):
 *   amax[r][g]  = max_j |y[r][32 g + j]|        the "block-wise scale" whose distribution the
 *                                               Appendix compares across transformations
 *   count[t]   += #{ (r, k) : |y[r][k]| > thresholds[t] }    the share of data above a threshold
 *                                               (Sec. 4.2: above 1.5 and above 3, before/after)
 *   sqerr[r][g] = sum_j (y_j - deq(q(y))_j)^2   the block's MXFP4 quantization loss (Sec. 4.1,
 *                                               4.2: loss of regular vs outlier blocks)
 * y is the canonical fp32 rotation (oracle_block_rotate_signed); amax and the comparisons are
 * fp32, the loss is summed in fp64.  Which blocks are "outlier blocks" is the caller's choice
 * of a threshold on amax (the paper: the top 0.1 % of magnitudes).
 * Any of amax, count, sqerr may be NULL.  count is accumulated into (the caller zeroes it).
 * ---------------------------------------------------------------------------------- */
/* fp32 -> IEEE binary16 value (returned as fp32), round to nearest even, finite results only: values
 * beyond the largest half (65504) saturate to it.  Written out on the bit pattern. */
float oracle_round_to_f16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = u & 0x80000000u, mag = u & 0x7FFFFFFFu;
    float a;
    memcpy(&a, &mag, 4);
    if (a >= 65520.0f) a = 65504.0f; /* 65520 is the midpoint to 2^16: it and everything above saturate */
    else if (a < 6.103515625e-05f) {
        /* below the smallest normal half (2^-14): multiples of 2^-24, nearest even */
        a = (float)(rint((double)a * 16777216.0) / 16777216.0);
    } else {
        uint32_t b;
        memcpy(&b, &a, 4);
        uint32_t lsb = (b >> 13) & 1u;
        b += 0xFFFu + lsb; /* keep 10 mantissa bits */
        b &= ~0x1FFFu;
        memcpy(&a, &b, 4);
    }
    uint32_t r;
    memcpy(&r, &a, 4);
    r |= sign;
    memcpy(&a, &r, 4);
    return a;
}

/* sqerr_bfp4 (optional): the same loss under the FP16-scale counterpart of MXFP4 that Sec. 3 and 4.1
 * compare it with ("BFP4": E2M1 elements, one FP16 scale per block).  The paper does not spell the
 * format out; taken: blocks of 32, scale s = half(fl32(amax / 6)) so that the block maximum maps onto
 * the largest E2M1 value, element code = E2M1 rounding (ties to the even code, saturation) of
 * fl32(y / s), dequantized value = code value * s.  s = 0 (an all-zero or vanishing block) encodes
 * every element as 0. */
int oracle_block_stats(const void *x, int xdt, int64_t M, int64_t K, int64_t ldx, int64_t B, const int8_t *signs,
                       const float *thresholds, int nt, float *amax, uint64_t *count, double *sqerr,
                       double *sqerr_bfp4) {
    if (!x || K % 32 || ldx < K || B < 1 || nt < 0 || (nt > 0 && count && !thresholds)) return ORACLE_ERR_ARG;
    if (B == 1 && signs) return ORACLE_ERR_ARG;
    size_t n = (size_t)(M > 0 ? M : 1) * (size_t)K;
    float *y = (float *)malloc(n * sizeof(float));
    if (!y) return ORACLE_ERR_ARG;
    int rc = ORACLE_OK;
    if (B == 1) {
        for (int64_t r = 0; r < M; ++r)
            for (int64_t k = 0; k < K; ++k) y[r * K + k] = load_elem(x, xdt, r * ldx + k);
    } else {
        rc = oracle_block_rotate_signed(x, xdt, M, K, ldx, B, signs, y, ORACLE_F32, K);
    }
    if (rc == ORACLE_OK) {
        for (int64_t r = 0; r < M; ++r) {
            for (int64_t g = 0; g < K / 32; ++g) {
                const float *v = y + r * K + g * 32;
                uint8_t codes16[16], sb;
                quantize_group(v, codes16, &sb);
                float am = 0.0f;
                double loss = 0.0;
                for (int j = 0; j < 32; ++j) {
                    float a = fabsf(v[j]);
                    if (a > am) am = a;
                    for (int t = 0; t < nt && count; ++t)
                        if (a > thresholds[t]) count[t] += 1;
                    int code = (j & 1) ? (codes16[j / 2] >> 4) : (codes16[j / 2] & 0xF);
                    double d = (double)v[j] - oracle_e2m1_value(code) * oracle_e8m0_value(sb);
                    loss += d * d;
                }
                if (amax) amax[r * (K / 32) + g] = am;
                if (sqerr) sqerr[r * (K / 32) + g] = loss;
                if (sqerr_bfp4) {
                    const float s = oracle_round_to_f16(am / 6.0f);
                    double lb = 0.0;
                    for (int j = 0; j < 32; ++j) {
                        int code = 0;
                        if (s > 0.0f) code = oracle_e2m1_encode(v[j] / s, 127); /* scale byte 127 = 2^0 */
                        double d = (double)v[j] - oracle_e2m1_value(code) * (double)s;
                        lb += d * d;
                    }
                    sqerr_bfp4[r * (K / 32) + g] = lb;
                }
            }
        }
    }
    free(y);
    return rc;
}

/* What the paper's analysis reports from the per-block statistics (Sec. 4.1: loss of regular against
 * outlier blocks; Sec. 4.2 and Appendix "Rotation Comparison": distribution of the block-wise scales,
 * share of regular blocks whose scale a rotation inflates).  amax / sqerr: per-block outputs for the
 * transformation under study; ref (optional): block-wise scales of the reference (the untransformed
 * activations); a block is an outlier block when its reference scale exceeds `outlier` (strictly), and
 * without ref its own scale is the reference.
 *   hist[j]   += number of blocks whose amax exceeds (strictly) exactly j of the nedges edges
 *   counts[0] += regular blocks, counts[1] += outlier blocks,
 *   counts[2] += regular blocks with amax > ref, counts[3] += outlier blocks with amax > ref
 *   sums[0]   += sqerr over regular blocks, sums[1] += over outlier blocks (sqerr may be NULL),
 *   sums[2]   += amax over regular blocks,  sums[3] += over outlier blocks            (fp64) */
int oracle_block_stats_summary(const float *amax, const float *sqerr, const float *ref, int64_t n, float outlier,
                               const float *edges, int nedges, uint64_t *hist, uint64_t *counts, double *sums) {
    if (!amax || nedges < 0 || (nedges > 0 && !edges)) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        float r = ref ? ref[i] : amax[i];
        int outl = r > outlier;
        if (counts) {
            counts[outl] += 1;
            if (ref && amax[i] > r) counts[2 + outl] += 1;
        }
        if (sums) {
            if (sqerr) sums[outl] += (double)sqerr[i];
            sums[2 + outl] += (double)amax[i];
        }
        if (hist) {
            int bin = 0;
            for (int e = 0; e < nedges; ++e)
                if (amax[i] > edges[e]) bin += 1;
            hist[bin] += 1;
        }
    }
    return ORACLE_OK;
}

/* deq[r][k] = value(code) * 2^(scale - 127), fp64 (exact). */
int oracle_mxfp4_dequantize(const uint8_t *codes, const uint8_t *scales, int64_t M, int64_t K,
                            double *out) {
    if (!codes || !scales || !out || K % 32) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = codes[r * (K / 2) + k / 2];
            int code = (k & 1) ? (byte >> 4) : (byte & 0xF);
            out[r * K + k] = oracle_e2m1_value(code) * oracle_e8m0_value(scales[r * (K / 32) + k / 32]);
        }
    return ORACLE_OK;
}

/* W4A4 product on the dequantized operands, fp64 accumulation, plain triple loop:
 *   y[i][n] = sum_k deqA[rows[i]][k] * deqW[n][k]          (i < nrows, n < N)
 *   bound[i][n] = sum_k |deqA| * |deqW|                    (for the forward-error test)
 * rows == NULL means rows[i] = i.  Either output may be NULL. */
int oracle_mxfp4_gemm(const uint8_t *aq, const uint8_t *as, const uint8_t *wq, const uint8_t *ws,
                      int64_t M, int64_t N, int64_t K, const int64_t *rows, int64_t nrows,
                      double *y, double *bound) {
    if (!aq || !as || !wq || !ws || K % 32) return ORACLE_ERR_ARG;
    if (!rows) nrows = M;
    double *wd = (double *)malloc((size_t)N * (size_t)K * sizeof(double));
    if (!wd) return ORACLE_ERR_ARG;
    oracle_mxfp4_dequantize(wq, ws, N, K, wd);
    int rc = ORACLE_OK;
#pragma omp parallel
    {
        double *ad = (double *)malloc((size_t)K * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < nrows; ++i) {
            int64_t m = rows ? rows[i] : i;
            if (!ad || m < 0 || m >= M) { rc = ORACLE_ERR_ARG; continue; }
            oracle_mxfp4_dequantize(aq + m * (K / 2), as + m * (K / 32), 1, K, ad);
            for (int64_t n = 0; n < N; ++n) {
                double acc = 0.0, bnd = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double p = ad[k] * wd[n * K + k];
                    acc += p;
                    bnd += fabs(p);
                }
                if (y) y[i * N + n] = acc;
                if (bound) bound[i * N + n] = bnd;
            }
        }
        free(ad);
    }
    free(wd);
    return rc;
}

/* Same product on unquantized fp64 operands (used for the invariance pin). */
int oracle_matmul_nt_f64(const double *a, const double *w, int64_t M, int64_t N, int64_t K, double *y) {
    if (!a || !w || !y) return ORACLE_ERR_ARG;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += a[m * K + k] * w[n * K + k];
            y[m * N + n] = acc;
        }
    return ORACLE_OK;
}
