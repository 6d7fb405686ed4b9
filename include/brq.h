/*
 * brq.h -- C ABI of the block-rotation MXFP4 hot path for MI355X (gfx950).
 *
 * The library implements the online part of "Block Rotation is All You Need for MXFP4
 * Quantization": a block-diagonal Hadamard rotation of activations along the reduction
 * axis K (Sec. 4.3, Eq. 1), MXFP4 quantization (Sec. 4.1: E2M1 elements, one power-of-two
 * E8M0 scale per 32 consecutive K elements) and the W4A4 product
 * Y = Q(X R) Q(W R)^T that the rotation leaves invariant (Sec. 2, equivalent
 * transformations).  Weights go through the same calls offline (rows of W are rows of
 * "X" with M := N).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers (HBM of the current HIP device).  The caller
 *     owns every buffer; the library allocates nothing.  The only state it keeps is a per-device
 *     set-up record (number of compute units; the declaration of the kernels that use more than
 *     64 KB of LDS), made under a lock by brq_init() or by the first call on that device.  A caller
 *     that captures calls into a HIP graph, or times the first call, calls brq_init() first.
 *   - Matrices are row-major with K contiguous.  X is [M][ldx] (ldx >= K, in elements),
 *     Y is [M][ldy].  Quantized operands come in one of two layouts (brq_layout):
 *       BRQ_LAYOUT_ROWMAJOR  codes [M][K/2] bytes, scales [M][K/32] bytes.
 *       BRQ_LAYOUT_TILED     what the product kernels stream fastest: rows in slabs of 64, K in
 *                            stages of 128 elements (64 code bytes) and superstages of 512
 *                            elements (16 scale bytes), every (slab, stage) block of codes
 *                            (4096 bytes) and every (slab, superstage) block of scales (1024
 *                            bytes) contiguous.  With Kp = K rounded up to a multiple of 512:
 *                              code byte j of row m   at ((m/64)*(Kp/128) + j/64)*4096 + (m%64)*64 + j%64
 *                              scale of group g, row m at ((m/64)*(Kp/512) + g/16)*1024 + (m%64)*16 + g%16
 *                            Buffer sizes (brq_operand_bytes): ceil64(M)*Kp/2 and ceil64(M)*Kp/32
 *                            bytes.  The quantizers write the K padding (elements K..Kp-1 of every
 *                            row) as zeros: code 0, scale byte 0; the product relies on that.
 *                            Padding rows are never read into a result and never written.
 *                            brq_to_rowmajor converts back.
 *   - codes: two E2M1 codes per byte, element 2j in the low nibble of byte j, element
 *     2j+1 in the high nibble.  A code is s<<3 | e<<1 | m (magnitudes 0, .5, 1, 1.5, 2,
 *     3, 4, 6).  A zero magnitude is always stored as code 0 (no negative zero).
 *   - scales: E8M0, byte b means 2^(b-127).  For a group with maximum magnitude amax the
 *     byte is max(exponent_field(amax) - 2, 0), i.e. floor(log2 amax) - 2 clamped.
 *     0xFF is never produced.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work is
 *     enqueued and the call returns; nothing synchronises with the host.
 *   - Argument errors are found on the host before anything is launched: the call
 *     returns the error code and touches no buffer.  BRQ_ERR_LAUNCH reports a failed
 *     kernel launch.  Asynchronous device faults surface at the caller's next sync.
 *   - Inputs must be finite and, for rotations, small enough that sums of B of them stay
 *     finite in fp32.  fp32 subnormals are honoured, not flushed.
 *   - M == 0 (or N == 0 for the product) is valid and does nothing; the data pointers of an
 *     empty matrix may be NULL.
 *   - Pointers must be 16-byte aligned and the row pitches of X and of the rotated output
 *     multiples of 16 bytes.  The product's output pitch ldy is free (>= N).
 */
#ifndef BRQ_H
#define BRQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BRQ_OK = 0,
    BRQ_ERR_NULL = 1,        /* a required pointer is NULL */
    BRQ_ERR_SHAPE = 2,       /* negative size, K % 32 != 0, ld < K, size beyond 2^31 work items */
    BRQ_ERR_BLOCK = 3,       /* B not a power of two, B < 8, B > 16384 or B does not divide K */
    BRQ_ERR_ALIGN = 4,       /* pointer or pitch not 16-byte aligned */
    BRQ_ERR_DTYPE = 5,       /* dtype is not one of brq_dtype */
    BRQ_ERR_LAUNCH = 6,      /* hipLaunchKernel failed (hipGetLastError) */
    BRQ_ERR_LAYOUT = 7,      /* layout is not one of brq_layout */
    BRQ_ERR_DEVICE = 8,      /* no current HIP device, or its one-time set-up failed */
    BRQ_STATUS_INT_RANGE_ = 0x7fffffff   /* (gives the type the range of int: see below) */
} brq_status;

/*
 * Callers reach these enums through foreign-function interfaces that pass plain ints, and the calls answer
 * an unknown value with BRQ_ERR_DTYPE / BRQ_ERR_LAYOUT.  The last enumerator of each type widens its value
 * range to that of int, so that reading such a value is defined behaviour on the library's side.
 */
typedef enum { BRQ_F32 = 0, BRQ_BF16 = 1, BRQ_DTYPE_INT_RANGE_ = 0x7fffffff } brq_dtype;

typedef enum { BRQ_LAYOUT_ROWMAJOR = 0, BRQ_LAYOUT_TILED = 1, BRQ_LAYOUT_INT_RANGE_ = 0x7fffffff } brq_layout;

/*
 * One-time set-up for the CURRENT HIP device (see the conventions above): idempotent, thread-safe,
 * launches nothing.  Optional: every call does the same on first use.
 */
brq_status brq_init(void);

/*
 * Sizes in bytes of the codes and scales buffers of a quantized [rows][K] operand in `layout`
 * (the "GEMM-consumable layout" of the quantizer's output; the definition is above).  Host
 * arithmetic only.  Either output pointer may be NULL.
 */
brq_status brq_operand_bytes(int64_t rows, int64_t K, brq_layout layout, int64_t* codes_bytes,
                             int64_t* scales_bytes);

/*
 * y = x * diag(s) * diag(H_B, ..., H_B) / sqrt(B)   (Sec. 4.3, Eq. 1 with R_i = Sylvester
 * Hadamard of order B, normalised so that R_i^T R_i = I; B = K is the global rotation
 * the paper compares with; B = 8 ... 128 is the rotation-dimension sweep of Sec. 5.2).
 * signs: NULL, or K sign bytes s_k (device memory, 16-byte aligned): element k of every row is
 * negated before the butterfly where signs[k] < 0 -- the random sign diagonal of the
 * "randomized Hadamard" rotations of Sec. 5.1; diag(s) H_B / sqrt(B) is still orthogonal, and
 * weights and activations must use the same signs.
 * Arithmetic: inputs widened exactly to fp32; stages h = 1, 2, ..., B/2 in ascending
 * order, pair (i, i+h) -> (a+b, a-b), each one IEEE fp32 operation; one fp32 multiply by
 * fl(1/sqrt(B)).  ydt = BRQ_F32 stores that value, BRQ_BF16 its round-to-nearest-even.
 * Every nonzero result has exactly these bits; a result that is an exact zero (operands that
 * cancel) may come out as +0 or -0 (the quantizers store either as code 0).
 * x [M][ldx] of xdt, y [M][ldy] of ydt; x and y must not overlap.
 * B: power of two, 8 <= B <= 16384, B divides K.
 */
brq_status brq_block_rotate(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                            int64_t B, const int8_t* signs, void* y, brq_dtype ydt, int64_t ldy,
                            void* stream);

/*
 * MXFP4 quantization of x along K (Sec. 4.1): per row and per group of 32 consecutive
 * elements one E8M0 scale from the group's maximum magnitude, elements rounded to the
 * nearest E2M1 value of x / 2^e (ties to the even code, saturation at +-6).
 * x [M][ldx] of xdt -> codes, scales in `layout`.  K % 32 == 0.
 */
brq_status brq_mxfp4_quantize(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                              uint8_t* codes, uint8_t* scales, brq_layout layout, void* stream);

/*
 * The online step of the method (Sec. 4.3, the rotation applied before a quantized
 * linear layer): brq_mxfp4_quantize(brq_block_rotate(x, B, signs) kept in fp32), in one pass
 * over x, bit-identical to that composition.  The quantization group stays 32 whatever
 * B is.  Same argument rules as the two calls above.
 */
brq_status brq_rotate_quantize_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K,
                                     int64_t ldx, int64_t B, const int8_t* signs, uint8_t* codes,
                                     uint8_t* scales, brq_layout layout, void* stream);

/*
 * The gated activation that feeds the rotated layer (Sec. 4.3: the online rotation R_4 sits before
 * down_proj; in the LLaMA models the paper evaluates, down_proj reads h = silu(gate) * up):
 *     h[m][k] = silu(gate[m][k]) * up[m][k],   silu(g) = g / (1 + exp(-g)),
 * stored as fp32 or as its bf16 rounding (nearest even).  Arithmetic: fp32 on the hardware's
 * exponential and reciprocal; the result h' satisfies
 *     |h' - h| <= (8 + 2 |g|) * 2^-24 * |h| + 2^-119 * |u|
 * (the absolute term covers gates below -87, where the result may be flushed to zero).  The last
 * bits are those of this kernel, not of a reference sequence.  The call exists as the unfused first
 * half that the fused call below is measured and checked against.
 * gate [M][ldg], up [M][ldu], both of xdt (they may be two halves of one buffer); h [M][ldh] of hdt
 * may overlap neither input.
 */
brq_status brq_swiglu(const void* gate, const void* up, brq_dtype xdt, int64_t M, int64_t K,
                      int64_t ldg, int64_t ldu, void* h, brq_dtype hdt, int64_t ldh, void* stream);

/*
 * The online step with its producer in front:
 *     brq_rotate_quantize_fused(h, B, signs)   with h = brq_swiglu(gate, up) of type hdt,
 * in one pass over gate and up; h never visits memory.  Bit-identical to that two-call sequence
 * of THIS library (hdt = BRQ_BF16 rounds h to bf16 before the rotation, as a separate activation
 * kernel storing bf16 would; BRQ_F32 keeps the fp32 value).  Against the exact activation the codes
 * and scales are those of a value within the bound stated for brq_swiglu: equal to the codes of the
 * exact h except where h (or its bf16 rounding, or the group maximum) lies within that bound of a
 * rounding boundary.
 * B as in brq_rotate_quantize_fused, or 1 for no rotation (quantization alone; signs must then be
 * NULL).
 */
brq_status brq_swiglu_rotate_quantize_fused(const void* gate, const void* up, brq_dtype xdt,
                                            int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                            brq_dtype hdt, int64_t B, const int8_t* signs,
                                            uint8_t* codes, uint8_t* scales, brq_layout layout,
                                            void* stream);

/*
 * Block rotation with caller-supplied blocks (Sec. 4.3, Eq. 1 as written: R_block =
 * diag(R_1, ..., R_n) with every R_i an orthogonal 32 x 32 matrix; the Hadamard block of
 * brq_block_rotate is one choice, learned blocks are what the conclusion proposes for the
 * online step):      y[m][32 b + j] = sum_i x[m][32 b + i] * R[b][i][j].
 * R: device pointer, [nR][32][32] fp32, nR = K/32 (one matrix per block) or 1 (shared).
 * Orthogonality is the caller's business; any matrix is multiplied as given.
 * Arithmetic: on the matrix cores, with R (and fp32 x) split into three bf16 parts and the
 * partial products accumulated in fp32: |y - exact| <= 2^-20 * sum_i |x_i| |R_ij|.  The order of
 * the additions is the hardware's, so unlike brq_block_rotate the last bits are not defined
 * here; ydt = BRQ_BF16 stores the round-to-nearest-even of the fp32 result.
 * K % 128 == 0.  x [M][ldx] of xdt, y [M][ldy] of ydt, no overlap.
 */
brq_status brq_matrix_rotate(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                             const float* R, int64_t nR, void* y, brq_dtype ydt, int64_t ldy,
                             void* stream);

/*
 * The online step with such blocks: brq_mxfp4_quantize(brq_matrix_rotate(x, R) kept in fp32) in
 * one pass over x.  Codes and scales are those of a rotated value within the error bound above:
 * they equal the codes of the exact rotation except where that value lies within the bound of a
 * rounding boundary of the encoder (or the group maximum within it of a power of two).
 */
brq_status brq_matrix_rotate_quantize_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K,
                                            int64_t ldx, const float* R, int64_t nR,
                                            uint8_t* codes, uint8_t* scales, brq_layout layout,
                                            void* stream);

/*
 * Block statistics of the paper's analysis (Sec. 4.1, 4.2, Appendix "Rotation Comparison") of
 * y = x after a transformation: B = 1 none, else the block rotation of brq_block_rotate (B = K:
 * the global rotation).  Per row and per block of 32 consecutive elements:
 *     amax[m][g]  = max_j |y[m][32 g + j]|               (the "block-wise scale")
 *     sqerr[m][g] = sum_j (y_j - deq(q(y))_j)^2          (the block's MXFP4 quantization loss)
 * and over the whole matrix, for each of nt <= 8 thresholds,
 *     count_gt[t] += #{ (m, k) : |y[m][k]| > thresholds[t] }   (strictly greater; ADDED to the
 *                                                             counter, which the caller zeroes)
 * amax and the comparisons are exact (fp32 values of the canonical rotation); sqerr is summed in
 * fp32 (within 4e-6 relative of the exact sum).  Which blocks count as "outlier blocks" is the
 * caller's threshold on amax.
 *     sqerr_bfp4[m][g] = the same loss under the FP16-scale counterpart that Sec. 3 (findings D, E)
 *         and Sec. 4.1 compare MXFP4 with (E2M1 elements, one half-precision scale per block of 32;
 *         the paper does not spell the format out, taken here): s = half(fl32(amax / 6)) rounded to
 *         nearest even and saturating at 65504, code_j = E2M1 rounding (ties to the even code,
 *         saturating) of fl32(y_j / s), dequantized value = val(code_j) * s; s = 0 encodes zeros.
 * thresholds is a HOST pointer read during the call; amax, sqerr, sqerr_bfp4 (device, [M][K/32]
 * fp32) and count_gt (device, [nt] uint64) may each be NULL.
 */
brq_status brq_block_stats(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                           int64_t B, const int8_t* signs, const float* thresholds, int64_t nt,
                           float* amax, uint64_t* count_gt, float* sqerr, float* sqerr_bfp4,
                           void* stream);

/*
 * What the paper's analysis reports from those per-block arrays (Sec. 4.1: loss of regular against
 * outlier blocks; Sec. 4.2 and the Appendix "Rotation Comparison": the distribution of the block-wise
 * scales before and after a rotation, and how many regular blocks' scales a rotation inflates).  Over
 * nblocks blocks, with amax / sqerr the outputs of brq_block_stats for the transformation under study and
 * amax_ref (optional) the block-wise scales of the reference, normally the untransformed activations
 * (B = 1); where amax_ref is NULL the block's own scale stands in for it:
 *     class(i)   = outlier if ref[i] > outlier_threshold, else regular        (strictly greater)
 *     hist[j]   += #{ i : amax[i] exceeds exactly j of the nedges <= 32 edges }  (strictly; nedges + 1 bins;
 *                  the edges must ascend: edges[0] <= edges[1] <= ..., else BRQ_ERR_SHAPE)
 *     counts[0] += #regular, counts[1] += #outlier,
 *     counts[2] += #{ regular i : amax[i] > ref[i] }, counts[3] += the same over outlier blocks
 *     sums[0]   += sum of sqerr over regular blocks, sums[1] += over outlier blocks   (0 where sqerr is NULL)
 *     sums[2]   += sum of amax over regular blocks,  sums[3] += over outlier blocks
 * Every output is ADDED to (the caller zeroes it) and may be NULL.  Counts are exact; the fp64 sums are
 * accumulated in an order the schedule decides and agree with a sequential fp64 sum to 1e-12 relative.
 * edges is a HOST pointer read during the call; everything else is device memory: amax, sqerr, amax_ref
 * [nblocks] fp32; hist [nedges + 1] and counts [4] uint64; sums [4] double.
 */
brq_status brq_block_stats_summary(const float* amax, const float* sqerr, const float* amax_ref,
                                   int64_t nblocks, float outlier_threshold, const float* edges,
                                   int64_t nedges, uint64_t* hist, uint64_t* counts, double* sums,
                                   void* stream);

/*
 * W4A4 product on MXFP4 operands (Sec. 2; Sec. 4.1 "scaling factor integrated into
 * hardware"):   y[m][n] = sum_g 2^(as[m][g]-127 + ws[n][g]-127) *
 *                          sum_{j<32} val(aq[m][32g+j]) * val(wq[n][32g+j]),  fp32 accumulate.
 * (aq, as) the quantized [M][K] operand in a_layout, (wq, ws) the quantized [N][K] operand in
 * w_layout -> y [M][ldy] of ydt (fp32, or bf16 = round-to-nearest-even of the fp32 sum).
 * K % 32 == 0, ldy >= N.  The layouts do not change what is summed, only (through the choice
 * of kernel) the order of the fp32 additions.
 */
brq_status brq_mxfp4_gemm(const uint8_t* aq, const uint8_t* as, brq_layout a_layout,
                          const uint8_t* wq, const uint8_t* ws, brq_layout w_layout, int64_t M,
                          int64_t N, int64_t K, void* y, brq_dtype ydt, int64_t ldy, void* stream);

/*
 * The whole online path of a decode step in one launch (Sec. 4.3: the online rotation and the quantizer in
 * front of the quantized layer, folded into the product):
 *     y = brq_mxfp4_gemm(brq_rotate_quantize_fused(x, B, signs), (wq, ws)),
 * bit for bit that two-call sequence, for M <= 16 rows of activations.  Every workgroup quantizes all of x
 * into LDS before it streams its weight rows, so the call pays for itself only where that prologue is
 * shorter than a kernel launch (a few rows); the two-call sequence remains the general path.
 * x [M][ldx] of xdt, M <= 16; K % 512 == 0, K <= 16384; B = 32 (anything else: BRQ_ERR_BLOCK); (wq, ws) the
 * quantized [N][K] weights in w_layout; y [M][ldy] of ydt.
 */
brq_status brq_rotate_quantize_gemm_fused(const void* x, brq_dtype xdt, int64_t M, int64_t K, int64_t ldx,
                                          int64_t B, const int8_t* signs, const uint8_t* wq,
                                          const uint8_t* ws, brq_layout w_layout, int64_t N, void* y,
                                          brq_dtype ydt, int64_t ldy, void* stream);

/*
 * Tiled -> row-major copy of a quantized [rows][K] operand (for inspection and parity checks;
 * nothing on the product path needs it): codes_out [rows][K/2], scales_out [rows][K/32].
 */
brq_status brq_to_rowmajor(const uint8_t* codes_tiled, const uint8_t* scales_tiled, int64_t rows,
                           int64_t K, uint8_t* codes_out, uint8_t* scales_out, void* stream);

/* Static, human-readable text for a status code. */
const char* brq_strerror(brq_status s);

/* Library version, major*10000 + minor*100 + patch. */
int brq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BRQ_H */
