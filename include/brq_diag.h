/*
 * brq_diag.h -- measurement aids of the block-rotation MXFP4 library.  Not part of the method and not
 * on the product path: bench.py uses them to read the ceiling of the block-scaled MFMA and the clock
 * the chip holds, next to the product kernel's own time.  Same conventions as brq.h.
 */
#ifndef BRQ_DIAG_H
#define BRQ_DIAG_H

#include "brq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * `workgroups` workgroups of 4 wavefronts each issue
 * iters x 16 block-scaled fp4 MFMAs (v_mfma_scale_f32_32x32x64, the instruction of the product
 * kernels) back to back from registers, 2 * 32*32*64 flops apiece, i.e. a launch does
 * workgroups * 4 * iters * 16 * 131072 flops.  The 16 MFMAs of an iteration are the register tile of
 * the large-shape product: 4 row-operand fragments x 4 column-operand fragments, read once from
 * `operands` (8192 bytes: 16 bytes per lane and fragment, the four fragments of one operand first,
 * e.g. the first bytes of a quantized matrix, so that the arithmetic sees realistic bit patterns
 * and consecutive instructions see different ones); `sink` receives
 * workgroups * 256 floats, of which sink[0] is the number of shader-clock cycles and sink[1] the
 * number of 100 MHz reference-clock ticks that workgroup 0's first wavefront spent in the loop
 * (100 * sink[0] / sink[1] = the clock in MHz that the chip held), the rest without meaning.
 * Timing a launch gives the rate the chip sustains on this
 * instruction alone, the ceiling against which a product kernel's own losses can be read.
 */
brq_status brq_diag_mfma_ceiling(const uint8_t* operands, int64_t iters, int64_t workgroups,
                                 float* sink, void* stream);

/*
 * brq_mxfp4_gemm on a shape that the persistent large-shape kernel takes (M > 128; N a multiple of 8 for
 * bf16 and of 4 for fp32 output; K % 512 == 0 or both operands tiled; the output pitch a multiple of 16
 * bytes; anything else: BRQ_ERR_SHAPE), which in addition writes to
 * `clock` (device, 6 x uint64) what the first wavefront of the kernel's first workgroup measured:
 *   [0] shader-clock cycles and [1] 100 MHz reference-clock ticks from start to end
 *       (100 * [0] / [1] is the clock in MHz that the chip held during the product),
 *   [2] cycles inside the K loops of its output tiles, [3] cycles inside their epilogues,
 *   [4] the number of output tiles that workgroup processed, [5] cycles of the prologue.
 * y receives the product as usual.
 */
brq_status brq_diag_mxfp4_gemm_clock(const uint8_t* aq, const uint8_t* as, brq_layout a_layout,
                                     const uint8_t* wq, const uint8_t* ws, brq_layout w_layout,
                                     int64_t M, int64_t N, int64_t K, void* y, brq_dtype ydt,
                                     int64_t ldy, uint64_t* clock, void* stream);

/*
 * The large-shape product kernel WITHOUT the loads that refill its operand ring: after the first 512
 * elements of K the kernel keeps multiplying what it already holds in LDS, with every MFMA, LDS read,
 * barrier and output store of the product.  y does NOT receive the product (it is written, with values
 * without meaning).  What the launch takes is what the product would take if its operands cost nothing to
 * move from the L2 into LDS; read next to brq_mxfp4_gemm's time and the MFMA-only loop's it prices that
 * movement on a chip whose clock follows its power.  Same arguments and `clock` read-out as
 * brq_diag_mxfp4_gemm_clock; bf16 output and at least 1024 output tiles of 256 x 256 only (anything
 * else: BRQ_ERR_SHAPE).
 */
brq_status brq_diag_mxfp4_gemm_no_loads(const uint8_t* aq, const uint8_t* as, brq_layout a_layout,
                                        const uint8_t* wq, const uint8_t* ws, brq_layout w_layout,
                                        int64_t M, int64_t N, int64_t K, void* y, brq_dtype ydt,
                                        int64_t ldy, uint64_t* clock, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BRQ_DIAG_H */
