"""CPU-only checks of the C-ABI library: it loads, exports what include/*.h declare, and
its host-side argument validation returns error codes without launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", f) for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h")]


@pytest.fixture(scope="module")
def L():
    import paper_2511_04214_amd as brq
    return brq.lib()


def declared_symbols():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(brq_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    syms = declared_symbols()
    assert {"brq_block_rotate", "brq_operand_bytes", "brq_mxfp4_quantize", "brq_rotate_quantize_fused",
            "brq_mxfp4_gemm", "brq_to_rowmajor", "brq_strerror", "brq_version"} <= set(syms)
    for s in syms:
        assert hasattr(L, s), "%s declared in include/ but not exported" % s


def test_binding_names_match_header():
    import paper_2511_04214_amd as brq
    for s in declared_symbols():
        if s in ("brq_strerror", "brq_version", "brq_init"):
            continue
        assert hasattr(brq, s[len("brq_"):]), s
    assert set(brq.EXPORTS) == set(declared_symbols())


def test_version_and_strerror(L):
    assert L.brq_version() >= 100
    texts = [L.brq_strerror(i).decode() for i in range(9)]
    assert texts[0] == "ok" and len(set(texts)) == 9
    assert "unknown" in L.brq_strerror(99).decode()


def test_argument_errors_before_any_launch(L):
    OK, NULL, SHAPE, BLOCK, ALIGN, DTYPE, LAYOUT = 0, 1, 2, 3, 4, 5, 7
    p = 0x1000  # never dereferenced: every call below fails validation on the host
    q = ctypes.c_void_p
    # null pointers
    assert L.brq_mxfp4_quantize(None, 1, 4, 64, 64, q(p), q(p), 0, None) == NULL
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 64, 64, None, q(p), 0, None) == NULL
    assert L.brq_rotate_quantize_fused(q(p), 1, 4, 64, 64, 32, None, q(p), None, 0, None) == NULL
    assert L.brq_block_rotate(q(p), 1, 4, 64, 64, 32, None, None, 0, 64, None) == NULL
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), None, 0, 4, 4, 64, q(p), 0, 4, None) == NULL
    # block statistics: (x, xdt, M, K, ldx, B, signs, thresholds, nt, amax, count_gt, sqerr, stream)
    th = (ctypes.c_float * 8)()
    assert L.brq_block_stats(None, 1, 4, 64, 64, 32, None, th, 2, q(p), q(p), q(p), q(p), None) == NULL
    assert L.brq_block_stats(q(p), 1, 4, 64, 64, 32, None, None, 2, q(p), q(p), q(p), q(p), None) == NULL   # thresholds
    assert L.brq_block_stats(q(p), 1, 4, 64, 64, 32, None, th, 9, q(p), q(p), q(p), q(p), None) == SHAPE    # nt > 8
    assert L.brq_block_stats(q(p), 1, 4, 64, 64, 24, None, th, 2, q(p), q(p), q(p), q(p), None) == BLOCK
    assert L.brq_block_stats(q(p), 1, 4, 64, 64, 32, None, th, 2, q(p), q(p + 4), q(p), q(p), None) == ALIGN
    assert L.brq_block_stats(q(p), 1, 4, 64, 64, 32, None, th, 2, q(p), q(p), q(p), q(p + 4), None) == ALIGN
    assert L.brq_block_stats(None, 1, 0, 64, 64, 32, None, th, 2, None, None, None, None, None) == OK
    # caller-supplied blocks: (x, xdt, M, K, ldx, R, nR, ...)
    assert L.brq_matrix_rotate(q(p), 1, 4, 128, 128, None, 4, q(p), 0, 128, None) == NULL
    assert L.brq_matrix_rotate(q(p), 1, 4, 128, 128, q(p), 3, q(p), 0, 128, None) == BLOCK          # 1 or K/32 blocks
    assert L.brq_matrix_rotate(q(p), 1, 4, 96, 96, q(p), 3, q(p), 0, 96, None) == SHAPE             # K % 128
    assert L.brq_matrix_rotate_quantize_fused(q(p), 1, 4, 128, 128, q(p + 4), 1, q(p), q(p), 0, None) == ALIGN
    assert L.brq_matrix_rotate_quantize_fused(q(p), 1, 4, 128, 128, q(p), 1, q(p), q(p), 9, None) == LAYOUT
    assert L.brq_matrix_rotate_quantize_fused(q(p), 1, 4, 128, 128, q(p), 1, None, q(p), 0, None) == NULL
    assert L.brq_matrix_rotate_quantize_fused(None, 1, 0, 128, 128, q(p), 1, None, None, 0, None) == OK
    # the producer calls: (gate, up, xdt, M, K, ldg, ldu, ...)
    assert L.brq_swiglu(q(p), None, 1, 4, 64, 64, 64, q(p), 0, 64, None) == NULL
    assert L.brq_swiglu(q(p), q(p), 1, 4, 64, 64, 32, q(p), 0, 64, None) == SHAPE            # ldu < K
    assert L.brq_swiglu(q(p), q(p), 1, 4, 64, 64, 64, q(p), 9, 64, None) == DTYPE
    assert L.brq_swiglu_rotate_quantize_fused(q(p), None, 1, 4, 64, 64, 64, 1, 32, None, q(p), q(p), 0, None) == NULL
    assert L.brq_swiglu_rotate_quantize_fused(q(p), q(p + 2), 1, 4, 64, 64, 64, 1, 32, None, q(p), q(p), 0, None) == ALIGN
    assert L.brq_swiglu_rotate_quantize_fused(q(p), q(p), 1, 4, 64, 64, 64, 7, 32, None, q(p), q(p), 0, None) == DTYPE
    assert L.brq_swiglu_rotate_quantize_fused(q(p), q(p), 1, 4, 64, 64, 64, 1, 24, None, q(p), q(p), 0, None) == BLOCK
    assert L.brq_swiglu_rotate_quantize_fused(q(p), q(p), 1, 4, 64, 64, 64, 1, 1, q(p), q(p), q(p), 0, None) == BLOCK   # signs, no rotation
    assert L.brq_swiglu_rotate_quantize_fused(q(p), q(p), 1, 4, 64, 64, 64, 1, 32, None, q(p), q(p), 5, None) == LAYOUT
    assert L.brq_swiglu_rotate_quantize_fused(None, None, 1, 0, 64, 64, 64, 1, 32, None, None, None, 0, None) == OK     # empty
    # shapes
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 48, 48, q(p), q(p), 0, None) == SHAPE      # K % 32
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 64, 32, q(p), q(p), 0, None) == SHAPE      # ldx < K
    assert L.brq_mxfp4_quantize(q(p), 1, -1, 64, 64, q(p), q(p), 0, None) == SHAPE
    assert L.brq_mxfp4_quantize(q(p), 1, 1 << 40, 64, 64, q(p), q(p), 0, None) == SHAPE
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 0, 4, 8, 64, q(p), 0, 4, None) == SHAPE   # ldy < N
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 0, 4, 8, 40, q(p), 0, 8, None) == SHAPE
    # dtype
    assert L.brq_mxfp4_quantize(q(p), 7, 4, 64, 64, q(p), q(p), 0, None) == DTYPE
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 0, 4, 8, 64, q(p), 3, 8, None) == DTYPE
    # layout
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 64, 64, q(p), q(p), 2, None) == LAYOUT
    assert L.brq_rotate_quantize_fused(q(p), 1, 4, 64, 64, 32, None, q(p), q(p), -1, None) == LAYOUT
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 5, 4, 8, 64, q(p), 0, 8, None) == LAYOUT
    assert L.brq_to_rowmajor(q(p), q(p), 4, 48, q(p), q(p), None) == SHAPE
    assert L.brq_to_rowmajor(q(p), None, 4, 64, q(p), q(p), None) == NULL
    assert L.brq_to_rowmajor(q(p), q(p), 0, 64, q(p), q(p), None) == OK
    # sign vector alignment
    assert L.brq_rotate_quantize_fused(q(p), 1, 4, 64, 64, 32, q(p + 8), q(p), q(p), 0, None) == ALIGN
    assert L.brq_block_rotate(q(p), 1, 4, 64, 64, 32, q(p + 1), q(p), 0, 64, None) == ALIGN
    # rotation block
    for B in (0, 4, 48, 128, 32768):
        assert L.brq_rotate_quantize_fused(q(p), 1, 4, 64, 64, B, None, q(p), q(p), 0, None) == BLOCK, B
    assert L.brq_block_rotate(q(p), 1, 4, 96, 96, 64, None, q(p), 0, 96, None) == BLOCK   # B does not divide K
    # alignment
    assert L.brq_mxfp4_quantize(q(p + 2), 1, 4, 64, 64, q(p), q(p), 0, None) == ALIGN
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 64, 68, q(p), q(p), 0, None) == ALIGN      # pitch 136 B
    assert L.brq_mxfp4_quantize(q(p), 1, 4, 64, 64, q(p + 4), q(p), 0, None) == ALIGN
    assert L.brq_mxfp4_gemm(q(p), q(p + 8), 0, q(p), q(p), 0, 4, 6, 64, q(p), 0, 6, None) == ALIGN
    # empty problems are fine and launch nothing
    assert L.brq_mxfp4_quantize(q(p), 1, 0, 64, 64, q(p), q(p), 0, None) == OK
    assert L.brq_rotate_quantize_fused(q(p), 1, 0, 64, 64, 32, None, q(p), q(p), 0, None) == OK
    assert L.brq_block_rotate(q(p), 1, 0, 64, 64, 64, None, q(p), 0, 64, None) == OK
    # the product with the clock read-out: large shapes only, and it needs somewhere to write
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 256, 256, 512, q(p), 0, 256, None, None) == NULL
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 256, 256, 512, q(p), 0, 256, q(p + 4), None) == ALIGN
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 128, 256, 512, q(p), 0, 256, q(p), None) == SHAPE
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 256, 202, 512, q(p), 0, 208, q(p), None) == SHAPE
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 256, 256, 544, q(p), 0, 256, q(p), None) == SHAPE
    assert L.brq_diag_mxfp4_gemm_clock(q(p), q(p), 0, q(p), q(p), 0, 0, 256, 512, q(p), 0, 256, q(p), None) == SHAPE
    # the variant without refill loads: bf16 output (dtype code 1) and >= 1024 tiles of 256 x 256 only
    assert L.brq_diag_mxfp4_gemm_no_loads(q(p), q(p), 0, q(p), q(p), 0, 8192, 8192, 512, q(p), 1, 8192, None, None) == NULL
    assert L.brq_diag_mxfp4_gemm_no_loads(q(p), q(p), 0, q(p), q(p), 0, 8192, 8192, 512, q(p), 0, 8192, q(p), None) == SHAPE
    assert L.brq_diag_mxfp4_gemm_no_loads(q(p), q(p), 0, q(p), q(p), 0, 4096, 4096, 512, q(p), 1, 4096, q(p), None) == SHAPE
    # decode product with the online step inside: (x, xdt, M, K, ldx, B, signs, wq, ws, w_layout, N, y, ydt, ldy, stream)
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 17, 512, 512, 32, None, q(p), q(p), 0, 64, q(p), 0, 64, None) == SHAPE   # M > 16
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 544, 544, 32, None, q(p), q(p), 0, 64, q(p), 0, 64, None) == SHAPE    # K % 512
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 32768, 32768, 32, None, q(p), q(p), 0, 64, q(p), 0, 64, None) == SHAPE # K too large
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 512, 512, 64, None, q(p), q(p), 0, 64, q(p), 0, 64, None) == BLOCK
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 512, 512, 32, None, None, q(p), 0, 64, q(p), 0, 64, None) == NULL
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 512, 512, 32, None, q(p), q(p), 3, 64, q(p), 0, 64, None) == LAYOUT
    assert L.brq_rotate_quantize_gemm_fused(q(p), 1, 4, 512, 512, 32, None, q(p), q(p), 0, 64, q(p), 0, 32, None) == SHAPE     # ldy < N
    assert L.brq_rotate_quantize_gemm_fused(None, 1, 0, 512, 512, 32, None, None, None, 0, 64, None, 0, 64, None) == OK
    # the reductions of the block statistics
    assert L.brq_block_stats_summary(None, None, None, 5, ctypes.c_float(1.0), None, 0, q(p), q(p), q(p), None) == NULL
    assert L.brq_block_stats_summary(q(p), None, None, 5, ctypes.c_float(1.0), None, 33, q(p), q(p), q(p), None) == SHAPE
    assert L.brq_block_stats_summary(q(p), None, None, 5, ctypes.c_float(1.0), None, 3, q(p), q(p), q(p), None) == NULL       # edges
    assert L.brq_block_stats_summary(q(p), None, None, 5, ctypes.c_float(1.0), None, 0, q(p + 4), q(p), q(p), None) == ALIGN
    assert L.brq_block_stats_summary(None, None, None, 0, ctypes.c_float(1.0), None, 0, None, None, None, None) == OK
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 0, 0, 8, 64, q(p), 0, 8, None) == OK
    assert L.brq_mxfp4_gemm(q(p), q(p), 0, q(p), q(p), 0, 8, 0, 64, q(p), 0, 0, None) == OK


def test_operand_bytes(L):
    import paper_2511_04214_amd as brq
    assert brq.operand_bytes(8192, 4096, "rowmajor") == (8192 * 2048, 8192 * 128)
    assert brq.operand_bytes(8192, 4096, "tiled") == (8192 * 2048, 8192 * 128)      # already whole blocks
    assert brq.operand_bytes(16, 256, "tiled") == (64 * 256, 64 * 16)                # 64 rows x 512 elements
    assert brq.operand_bytes(65, 544, "tiled") == (128 * 512, 128 * 32)
    assert brq.operand_bytes(0, 64, "tiled") == (0, 0)
    c = ctypes.c_int64()
    assert L.brq_operand_bytes(4, 48, 0, ctypes.byref(c), None) == 2     # shape
    assert L.brq_operand_bytes(4, 64, 9, ctypes.byref(c), None) == 7     # layout
    assert L.brq_operand_bytes(4, 64, 1, None, None) == 0
    with pytest.raises(ValueError):
        brq.operand_bytes(4, 64, "columns")


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2511_04214_amd as brq
    x = torch.zeros(2, 64)
    with pytest.raises(ValueError):
        brq.mxfp4_quantize(x)
    with pytest.raises(ValueError):
        brq.rotate_quantize_fused(x, 32)


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_04214_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "brq_oracle" not in text, f
