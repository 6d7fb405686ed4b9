/* Calls every entry point of libbrq with arguments that its host-side validation must refuse, so that no
 * kernel is ever launched and no GPU is needed.  Linked against a build of the library whose HOST code is
 * compiled under -fsanitize=address,undefined (tests/test_sanitizers.py): a stray read in the validation code
 * (of a pointer it must not dereference, past a table, ...) ends the run with a non-zero status. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "brq.h"
#include "brq_diag.h"

#define EXPECT(call, want) do { int got_ = (int)(call); if (got_ != (int)(want)) { fprintf(stderr, "%s -> %d, expected %d\n", #call, got_, (int)(want)); return 1; } } while (0)

int main(void) {
    void *p = (void *)(uintptr_t)0x1000, *q = (void *)(uintptr_t)0x1004;      /* never dereferenced */
    int64_t cb = 0, sb = 0;
    EXPECT(brq_operand_bytes(65, 544, BRQ_LAYOUT_TILED, &cb, &sb), BRQ_OK);
    if (cb != 128 * 512 || sb != 128 * 32) return 1;
    EXPECT(brq_operand_bytes(4, 48, BRQ_LAYOUT_ROWMAJOR, &cb, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_block_rotate(NULL, BRQ_BF16, 4, 64, 64, 32, NULL, p, BRQ_F32, 64, NULL), BRQ_ERR_NULL);
    EXPECT(brq_block_rotate(p, BRQ_BF16, 4, 64, 64, 24, NULL, p, BRQ_F32, 64, NULL), BRQ_ERR_BLOCK);
    EXPECT(brq_block_rotate(q, BRQ_BF16, 4, 64, 64, 32, NULL, p, BRQ_F32, 64, NULL), BRQ_ERR_ALIGN);
    EXPECT(brq_mxfp4_quantize(p, (brq_dtype)9, 4, 64, 64, p, p, BRQ_LAYOUT_ROWMAJOR, NULL), BRQ_ERR_DTYPE);
    EXPECT(brq_mxfp4_quantize(p, BRQ_F32, 4, 48, 48, p, p, BRQ_LAYOUT_ROWMAJOR, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_mxfp4_quantize(p, BRQ_F32, 4, 64, 64, p, p, (brq_layout)5, NULL), BRQ_ERR_LAYOUT);
    EXPECT(brq_rotate_quantize_fused(p, BRQ_BF16, 4, 64, 32, 32, NULL, p, p, BRQ_LAYOUT_TILED, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_swiglu(p, NULL, BRQ_BF16, 4, 64, 64, 64, p, BRQ_F32, 64, NULL), BRQ_ERR_NULL);
    EXPECT(brq_swiglu_rotate_quantize_fused(p, p, BRQ_BF16, 4, 64, 64, 64, BRQ_BF16, 1, p, p, p, BRQ_LAYOUT_ROWMAJOR, NULL), BRQ_ERR_BLOCK);
    EXPECT(brq_matrix_rotate(p, BRQ_BF16, 4, 128, 128, p, 3, p, BRQ_F32, 128, NULL), BRQ_ERR_BLOCK);
    EXPECT(brq_matrix_rotate_quantize_fused(p, BRQ_BF16, 4, 96, 96, p, 3, p, p, BRQ_LAYOUT_ROWMAJOR, NULL), BRQ_ERR_SHAPE);
    {
        float th[8] = {0};
        EXPECT(brq_block_stats(p, BRQ_BF16, 4, 64, 64, 32, NULL, th, 9, p, p, p, NULL, NULL), BRQ_ERR_SHAPE);
        EXPECT(brq_block_stats(p, BRQ_BF16, 4, 64, 64, 32, NULL, NULL, 2, p, p, p, NULL, NULL), BRQ_ERR_NULL);
        EXPECT(brq_block_stats_summary(p, NULL, NULL, 5, 1.0f, NULL, 3, p, p, p, NULL), BRQ_ERR_NULL);
        EXPECT(brq_block_stats_summary(p, NULL, NULL, 5, 1.0f, th, 33, p, p, p, NULL), BRQ_ERR_SHAPE);
    }
    EXPECT(brq_mxfp4_gemm(p, p, BRQ_LAYOUT_ROWMAJOR, p, NULL, BRQ_LAYOUT_ROWMAJOR, 4, 4, 64, p, BRQ_F32, 4, NULL), BRQ_ERR_NULL);
    EXPECT(brq_mxfp4_gemm(p, p, BRQ_LAYOUT_ROWMAJOR, p, p, BRQ_LAYOUT_ROWMAJOR, 4, 8, 64, p, BRQ_F32, 4, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_mxfp4_gemm(p, p, BRQ_LAYOUT_ROWMAJOR, p, p, BRQ_LAYOUT_ROWMAJOR, 0, 8, 64, p, BRQ_F32, 8, NULL), BRQ_OK);
    EXPECT(brq_rotate_quantize_gemm_fused(p, BRQ_BF16, 17, 512, 512, 32, NULL, p, p, BRQ_LAYOUT_ROWMAJOR, 64, p, BRQ_F32, 64, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_rotate_quantize_gemm_fused(p, BRQ_BF16, 4, 512, 512, 64, NULL, p, p, BRQ_LAYOUT_ROWMAJOR, 64, p, BRQ_F32, 64, NULL), BRQ_ERR_BLOCK);
    EXPECT(brq_to_rowmajor(p, p, 4, 48, p, p, NULL), BRQ_ERR_SHAPE);
    EXPECT(brq_diag_mfma_ceiling(NULL, 10, 4, p, NULL), BRQ_ERR_NULL);
    EXPECT(brq_diag_mxfp4_gemm_clock(p, p, BRQ_LAYOUT_ROWMAJOR, p, p, BRQ_LAYOUT_ROWMAJOR, 128, 256, 512, p, BRQ_F32, 256, p, NULL), BRQ_ERR_SHAPE);
    for (int s = 0; s < 12; ++s)
        if (strlen(brq_strerror((brq_status)s)) == 0) return 1;
    if (brq_version() < 100) return 1;
    printf("host api sanitizer driver ok\n");
    return 0;
}
