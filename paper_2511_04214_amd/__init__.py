"""Python binding of libbrq (the gfx950 block-rotation MXFP4 library).

Argument marshalling only: every function takes torch tensors that live on the GPU,
passes their device pointers and the current HIP stream through the C ABI declared in
include/brq.h, and returns the output tensors.  No arithmetic of the method happens
here.  There is no CPU fallback: without the built library, or without a GPU tensor, the
calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbrq.so")

BRQ_F32, BRQ_BF16 = 0, 1
LAYOUTS = {"rowmajor": 0, "tiled": 1}
EXPORTS = ["brq_init", "brq_block_rotate", "brq_operand_bytes", "brq_mxfp4_quantize", "brq_rotate_quantize_fused",
           "brq_swiglu", "brq_swiglu_rotate_quantize_fused", "brq_matrix_rotate",
           "brq_matrix_rotate_quantize_fused", "brq_block_stats", "brq_block_stats_summary", "brq_mxfp4_gemm", "brq_rotate_quantize_gemm_fused", "brq_to_rowmajor", "brq_diag_mfma_ceiling", "brq_diag_mxfp4_gemm_clock", "brq_diag_mxfp4_gemm_no_loads", "brq_strerror", "brq_version"]

_lib = None


class BrqError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libbrq: %s (status %d)" % (text, status))
        self.status = status


def lib():
    """Load libbrq.so (built in-tree by `python -m paper_2511_04214_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libbrq.so is not built: run __graft_entry__.build() "
                              "(python paper_2511_04214_amd/build.py) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.brq_block_rotate.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i32, i64, vp]
        L.brq_block_rotate.restype = i32
        L.brq_operand_bytes.argtypes = [i64, i64, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.brq_operand_bytes.restype = i32
        L.brq_mxfp4_quantize.argtypes = [vp, i32, i64, i64, i64, vp, vp, i32, vp]
        L.brq_mxfp4_quantize.restype = i32
        L.brq_rotate_quantize_fused.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp, i32, vp]
        L.brq_rotate_quantize_fused.restype = i32
        L.brq_swiglu.argtypes = [vp, vp, i32, i64, i64, i64, i64, vp, i32, i64, vp]
        L.brq_swiglu.restype = i32
        L.brq_swiglu_rotate_quantize_fused.argtypes = [vp, vp, i32, i64, i64, i64, i64, i32, i64, vp, vp, vp, i32, vp]
        L.brq_swiglu_rotate_quantize_fused.restype = i32
        L.brq_matrix_rotate.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, i32, i64, vp]
        L.brq_matrix_rotate.restype = i32
        L.brq_matrix_rotate_quantize_fused.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp, i32, vp]
        L.brq_matrix_rotate_quantize_fused.restype = i32
        L.brq_block_stats.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i64, vp, vp, vp, vp, vp]
        L.brq_block_stats.restype = i32
        L.brq_block_stats_summary.argtypes = [vp, vp, vp, i64, ctypes.c_float, vp, i64, vp, vp, vp, vp]
        L.brq_block_stats_summary.restype = i32
        L.brq_mxfp4_gemm.argtypes = [vp, vp, i32, vp, vp, i32, i64, i64, i64, vp, i32, i64, vp]
        L.brq_mxfp4_gemm.restype = i32
        L.brq_rotate_quantize_gemm_fused.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp, i32, i64, vp, i32, i64, vp]
        L.brq_rotate_quantize_gemm_fused.restype = i32
        L.brq_to_rowmajor.argtypes = [vp, vp, i64, i64, vp, vp, vp]
        L.brq_to_rowmajor.restype = i32
        L.brq_diag_mxfp4_gemm_clock.argtypes = [vp, vp, i32, vp, vp, i32, i64, i64, i64, vp, i32, i64, vp, vp]
        L.brq_diag_mxfp4_gemm_clock.restype = i32
        L.brq_diag_mxfp4_gemm_no_loads.argtypes = L.brq_diag_mxfp4_gemm_clock.argtypes
        L.brq_diag_mxfp4_gemm_no_loads.restype = i32
        L.brq_diag_mfma_ceiling.argtypes = [vp, i64, i64, vp, vp]
        L.brq_diag_mfma_ceiling.restype = i32
        L.brq_init.restype = i32
        L.brq_strerror.argtypes = [i32]
        L.brq_strerror.restype = ctypes.c_char_p
        L.brq_version.restype = i32
        _lib = L
    return _lib


def init():
    """One-time set-up for the current device (brq_init); every call does the same on first use."""
    _check(lib().brq_init())


def _check(status):
    if status != 0:
        raise BrqError(status, lib().brq_strerror(status).decode())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return BRQ_F32
    if t.dtype == torch.bfloat16:
        return BRQ_BF16
    raise TypeError("libbrq takes float32 or bfloat16 tensors, got %s" % t.dtype)


def _rows(t, name):
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor (libbrq has no CPU path)" % name)
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("%s must be 2-D with contiguous rows" % name)
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else t.shape[1])


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _signs_ptr(signs, K):
    """signs: None, or an int8 GPU tensor of K sign values (negative = flip)."""
    if signs is None:
        return None
    if not (signs.is_cuda and signs.is_contiguous() and signs.dtype == torch.int8 and signs.numel() == K):
        raise ValueError("signs must be a contiguous int8 GPU tensor with K elements")
    return signs.data_ptr()


def block_rotate(x, B, out_dtype=torch.float32, out=None, stream=None, signs=None):
    """y = x * diag(signs) * diag(H_B..H_B)/sqrt(B) along the last axis (brq_block_rotate)."""
    M, K, ldx = _rows(x, "x")
    y = torch.empty((M, K), dtype=out_dtype, device=x.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    _check(lib().brq_block_rotate(x.data_ptr(), _dtype_code(x), M, K, ldx, B, _signs_ptr(signs, K), y.data_ptr(),
                                  _dtype_code(y), ldy, _stream(stream)))
    return y


def _layout_code(layout):
    if layout not in LAYOUTS:
        raise ValueError("layout must be one of %s" % sorted(LAYOUTS))
    return LAYOUTS[layout]


def operand_bytes(rows, K, layout="rowmajor"):
    """(codes_bytes, scales_bytes) of a quantized [rows][K] operand (brq_operand_bytes)."""
    c, s_ = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().brq_operand_bytes(rows, K, _layout_code(layout), ctypes.byref(c), ctypes.byref(s_)))
    return c.value, s_.value


def _alloc_q(x, M, K, codes, scales, layout):
    """Row-major operands are [M, K/2] and [M, K/32] tensors, tiled operands flat byte buffers."""
    if layout == "rowmajor":
        cshape, sshape = (M, K // 2), (M, K // 32)
    else:
        cb, sb = operand_bytes(M, K, layout)
        cshape, sshape = (cb,), (sb,)
    if codes is None:
        codes = torch.empty(cshape, dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(sshape, dtype=torch.uint8, device=x.device)
    if not (codes.is_contiguous() and scales.is_contiguous()):
        raise ValueError("codes and scales must be contiguous")
    if codes.dtype != torch.uint8 or scales.dtype != torch.uint8 or not (codes.is_cuda and scales.is_cuda):
        raise ValueError("codes and scales must be uint8 GPU tensors")
    if codes.numel() < cshape[0] * (cshape[1] if len(cshape) > 1 else 1) or \
            scales.numel() < sshape[0] * (sshape[1] if len(sshape) > 1 else 1):
        raise ValueError("codes or scales buffer too small for this operand and layout")
    return codes, scales


def mxfp4_quantize(x, codes=None, scales=None, stream=None, layout="rowmajor"):
    """x -> (codes, scales) in `layout` (brq_mxfp4_quantize)."""
    M, K, ldx = _rows(x, "x")
    lc = _layout_code(layout)
    codes, scales = _alloc_q(x, M, K, codes, scales, layout)
    _check(lib().brq_mxfp4_quantize(x.data_ptr(), _dtype_code(x), M, K, ldx, codes.data_ptr(), scales.data_ptr(),
                                    lc, _stream(stream)))
    return codes, scales


def rotate_quantize_fused(x, B, codes=None, scales=None, stream=None, layout="rowmajor", signs=None):
    """Block rotation fused with MXFP4 quantization (brq_rotate_quantize_fused)."""
    M, K, ldx = _rows(x, "x")
    lc = _layout_code(layout)
    codes, scales = _alloc_q(x, M, K, codes, scales, layout)
    _check(lib().brq_rotate_quantize_fused(x.data_ptr(), _dtype_code(x), M, K, ldx, B, _signs_ptr(signs, K),
                                           codes.data_ptr(), scales.data_ptr(), lc, _stream(stream)))
    return codes, scales


def swiglu(gate, up, out_dtype=torch.float32, out=None, stream=None):
    """h = silu(gate) * up, within the error bound stated in brq.h (brq_swiglu)."""
    M, K, ldg = _rows(gate, "gate")
    M2, K2, ldu = _rows(up, "up")
    if (M, K) != (M2, K2) or gate.dtype != up.dtype:
        raise ValueError("gate and up must agree in shape and dtype")
    h = torch.empty((M, K), dtype=out_dtype, device=gate.device) if out is None else out
    _, _, ldh = _rows(h, "out")
    _check(lib().brq_swiglu(gate.data_ptr(), up.data_ptr(), _dtype_code(gate), M, K, ldg, ldu, h.data_ptr(),
                            _dtype_code(h), ldh, _stream(stream)))
    return h


def swiglu_rotate_quantize_fused(gate, up, B, h_dtype=torch.float32, codes=None, scales=None, stream=None,
                                 layout="rowmajor", signs=None):
    """silu(gate) * up -> block rotation -> MXFP4, in one pass (brq_swiglu_rotate_quantize_fused).

    h_dtype: torch.bfloat16 rounds the activation to bf16 before the rotation, torch.float32
    keeps it.  B = 1 quantizes without rotating.
    """
    M, K, ldg = _rows(gate, "gate")
    M2, K2, ldu = _rows(up, "up")
    if (M, K) != (M2, K2) or gate.dtype != up.dtype:
        raise ValueError("gate and up must agree in shape and dtype")
    if h_dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("h_dtype must be torch.float32 or torch.bfloat16")
    lc = _layout_code(layout)
    codes, scales = _alloc_q(gate, M, K, codes, scales, layout)
    _check(lib().brq_swiglu_rotate_quantize_fused(gate.data_ptr(), up.data_ptr(), _dtype_code(gate), M, K, ldg, ldu,
                                                  BRQ_BF16 if h_dtype == torch.bfloat16 else BRQ_F32, B,
                                                  _signs_ptr(signs, K), codes.data_ptr(), scales.data_ptr(), lc,
                                                  _stream(stream)))
    return codes, scales


def _blocks(R, K):
    """R: float32 GPU tensor [32, 32] (shared) or [K/32, 32, 32] -> (tensor, nR)."""
    if not (R.is_cuda and R.is_contiguous() and R.dtype == torch.float32):
        raise ValueError("R must be a contiguous float32 GPU tensor")
    if R.dim() == 2:
        R = R.unsqueeze(0)
    if R.dim() != 3 or tuple(R.shape[1:]) != (32, 32):
        raise ValueError("R must be [32, 32] or [K/32, 32, 32]")
    return R, R.shape[0]


def matrix_rotate(x, R, out_dtype=torch.float32, out=None, stream=None):
    """y = x * diag(R_1..R_n), 32 x 32 blocks given by the caller (brq_matrix_rotate)."""
    M, K, ldx = _rows(x, "x")
    R, nR = _blocks(R, K)
    y = torch.empty((M, K), dtype=out_dtype, device=x.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    _check(lib().brq_matrix_rotate(x.data_ptr(), _dtype_code(x), M, K, ldx, R.data_ptr(), nR, y.data_ptr(),
                                   _dtype_code(y), ldy, _stream(stream)))
    return y


def matrix_rotate_quantize_fused(x, R, codes=None, scales=None, stream=None, layout="rowmajor"):
    """Rotation by caller-supplied blocks fused with MXFP4 quantization (brq_matrix_rotate_quantize_fused)."""
    M, K, ldx = _rows(x, "x")
    R, nR = _blocks(R, K)
    lc = _layout_code(layout)
    codes, scales = _alloc_q(x, M, K, codes, scales, layout)
    _check(lib().brq_matrix_rotate_quantize_fused(x.data_ptr(), _dtype_code(x), M, K, ldx, R.data_ptr(), nR,
                                                  codes.data_ptr(), scales.data_ptr(), lc, _stream(stream)))
    return codes, scales


def block_stats(x, B, thresholds=(), signs=None, counts=None, want_amax=True, want_sqerr=True, stream=None,
                amax=None, sqerr=None, sqerr_bfp4=None, want_bfp4=False):
    """(amax [M, K/32] f32 or None, counts [nt] int64 or None, sqerr [M, K/32] f32 or None) of x after the
    rotation with block B (1 = none, K = global) (brq_block_stats).  `counts` is added to when given;
    `amax` / `sqerr` / `sqerr_bfp4` may be given as output tensors.  With want_bfp4 (or sqerr_bfp4) a fourth
    element is returned: the loss under the FP16-scale counterpart of MXFP4."""
    M, K, ldx = _rows(x, "x")
    th = (ctypes.c_float * max(1, len(thresholds)))(*[float(t) for t in thresholds])
    for t, n in ((amax, "amax"), (sqerr, "sqerr"), (sqerr_bfp4, "sqerr_bfp4")):
        if t is not None and not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
                                  and tuple(t.shape) == (M, K // 32)):
            raise ValueError("%s must be a contiguous float32 GPU tensor [M, K/32]" % n)
    if amax is None and want_amax:
        amax = torch.empty((M, K // 32), dtype=torch.float32, device=x.device)
    if sqerr is None and want_sqerr:
        sqerr = torch.empty((M, K // 32), dtype=torch.float32, device=x.device)
    four = want_bfp4 or sqerr_bfp4 is not None
    if sqerr_bfp4 is None and want_bfp4:
        sqerr_bfp4 = torch.empty((M, K // 32), dtype=torch.float32, device=x.device)
    if counts is None and len(thresholds):
        counts = torch.zeros((len(thresholds),), dtype=torch.int64, device=x.device)
    if counts is not None and not (counts.is_cuda and counts.is_contiguous() and counts.dtype == torch.int64
                                   and counts.numel() == len(thresholds)):
        raise ValueError("counts must be a contiguous int64 GPU tensor with one element per threshold")
    _check(lib().brq_block_stats(x.data_ptr(), _dtype_code(x), M, K, ldx, B, _signs_ptr(signs, K), th,
                                 len(thresholds), None if amax is None else amax.data_ptr(),
                                 None if counts is None else counts.data_ptr(),
                                 None if sqerr is None else sqerr.data_ptr(),
                                 None if sqerr_bfp4 is None else sqerr_bfp4.data_ptr(), _stream(stream)))
    return (amax, counts, sqerr, sqerr_bfp4) if four else (amax, counts, sqerr)


def block_stats_summary(amax, sqerr=None, amax_ref=None, outlier_threshold=0.0, edges=(), hist=None, counts=None,
                        sums=None, stream=None):
    """(hist [len(edges) + 1] int64, counts [4] int64, sums [4] float64) over the per-block arrays of block_stats
    (brq_block_stats_summary).  Outputs given by the caller are added to."""
    n = amax.numel()
    for t, nm in ((amax, "amax"), (sqerr, "sqerr"), (amax_ref, "amax_ref")):
        if t is not None and not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and t.numel() == n):
            raise ValueError("%s must be a contiguous float32 GPU tensor with one element per block" % nm)
    ed = (ctypes.c_float * max(1, len(edges)))(*[float(e) for e in edges])
    if hist is None:
        hist = torch.zeros((len(edges) + 1,), dtype=torch.int64, device=amax.device)
    if counts is None:
        counts = torch.zeros((4,), dtype=torch.int64, device=amax.device)
    if sums is None:
        sums = torch.zeros((4,), dtype=torch.float64, device=amax.device)
    for t, nm, dt, ne in ((hist, "hist", torch.int64, len(edges) + 1), (counts, "counts", torch.int64, 4), (sums, "sums", torch.float64, 4)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() == ne):
            raise ValueError("%s must be a contiguous GPU tensor of %d elements of %s" % (nm, ne, dt))
    _check(lib().brq_block_stats_summary(amax.data_ptr(), None if sqerr is None else sqerr.data_ptr(),
                                         None if amax_ref is None else amax_ref.data_ptr(), n, float(outlier_threshold), ed,
                                         len(edges), hist.data_ptr(), counts.data_ptr(), sums.data_ptr(), _stream(stream)))
    return hist, counts, sums


def to_rowmajor(codes_tiled, scales_tiled, rows, K, stream=None):
    """Tiled operand -> (codes [rows, K/2], scales [rows, K/32]) (brq_to_rowmajor)."""
    cb, sb = operand_bytes(rows, K, "tiled")
    for t, n, need in ((codes_tiled, "codes_tiled", cb), (scales_tiled, "scales_tiled", sb)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.uint8 and t.numel() >= need):
            raise ValueError("%s must be a contiguous uint8 GPU tensor of at least %d bytes" % (n, need))
    codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=codes_tiled.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=codes_tiled.device)
    _check(lib().brq_to_rowmajor(codes_tiled.data_ptr(), scales_tiled.data_ptr(), rows, K, codes.data_ptr(),
                                 scales.data_ptr(), _stream(stream)))
    return codes, scales


def mxfp4_gemm(aq, as_, wq, ws, out_dtype=torch.float32, out=None, stream=None, a_layout="rowmajor",
               w_layout="rowmajor", M=None, N=None, K=None, clock=None, no_loads=False):
    """Y[M, N] = deq(aq, as) @ deq(wq, ws)^T on the block-scaled MFMA (brq_mxfp4_gemm).

    Row-major operands are 2-D tensors that carry their shape; a tiled operand is a flat byte
    buffer, so its rows (M or N) and K must be given.  `clock` (an int64 GPU tensor of 6 elements;
    large shapes only, brq_diag_mxfp4_gemm_clock) receives the shader-clock cycles and the 100 MHz
    ticks that the kernel's first workgroup ran for, and their split over K loops and epilogues.
    `no_loads` (with `clock`; brq_diag_mxfp4_gemm_no_loads) runs the measurement variant without refill
    loads instead: `out` is written with values without meaning.
    """
    for t, n in ((aq, "aq"), (as_, "as"), (wq, "wq"), (ws, "ws")):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.uint8):
            raise ValueError("%s must be a contiguous uint8 GPU tensor" % n)
    la, lw = _layout_code(a_layout), _layout_code(w_layout)
    if a_layout == "rowmajor":
        if aq.dim() != 2 or (M is not None and M != aq.shape[0]) or (K is not None and K != aq.shape[1] * 2):
            raise ValueError("row-major aq must be [M, K/2]")
        M, K = aq.shape[0], aq.shape[1] * 2
    if w_layout == "rowmajor":
        if wq.dim() != 2 or (N is not None and N != wq.shape[0]) or (K is not None and K != wq.shape[1] * 2):
            raise ValueError("row-major wq must be [N, K/2] with the K of the other operand")
        N, K = wq.shape[0], wq.shape[1] * 2
    if M is None or N is None or K is None:
        raise ValueError("M, N and K must be given for tiled operands")
    for (c, s_, rows, lay, n) in ((aq, as_, M, a_layout, "a"), (wq, ws, N, w_layout, "w")):
        cb, sb = operand_bytes(rows, K, lay)
        if c.numel() < cb or s_.numel() < sb or (lay == "rowmajor" and tuple(s_.shape) != (rows, K // 32)):
            raise ValueError("operand %s: buffers do not match its shape and layout" % n)
    y = torch.empty((M, N), dtype=out_dtype, device=aq.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    if y.shape[0] != M or y.shape[1] != N:
        raise ValueError("out must be [M, N]")
    if clock is not None:
        if not (clock.is_cuda and clock.is_contiguous() and clock.dtype == torch.int64 and clock.numel() == 6):
            raise ValueError("clock must be a contiguous int64 GPU tensor of 6 elements")
        fn = lib().brq_diag_mxfp4_gemm_no_loads if no_loads else lib().brq_diag_mxfp4_gemm_clock
        _check(fn(aq.data_ptr(), as_.data_ptr(), la, wq.data_ptr(), ws.data_ptr(), lw, M, N, K,
                  y.data_ptr(), _dtype_code(y), ldy, clock.data_ptr(), _stream(stream)))
        return y
    if no_loads:
        raise ValueError("no_loads is a measurement variant and needs `clock`")
    _check(lib().brq_mxfp4_gemm(aq.data_ptr(), as_.data_ptr(), la, wq.data_ptr(), ws.data_ptr(), lw, M, N, K,
                                y.data_ptr(), _dtype_code(y), ldy, _stream(stream)))
    return y


def rotate_quantize_gemm_fused(x, B, wq, ws, N, out_dtype=torch.float32, out=None, stream=None, w_layout="rowmajor",
                               signs=None):
    """Y = mxfp4_gemm(rotate_quantize_fused(x, B), (wq, ws)) in one launch, M <= 16 (brq_rotate_quantize_gemm_fused)."""
    M, K, ldx = _rows(x, "x")
    for t, n in ((wq, "wq"), (ws, "ws")):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.uint8):
            raise ValueError("%s must be a contiguous uint8 GPU tensor" % n)
    cb, sb = operand_bytes(N, K, w_layout)
    if wq.numel() < cb or ws.numel() < sb:
        raise ValueError("weight buffers do not match N, K and the layout")
    y = torch.empty((M, N), dtype=out_dtype, device=x.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    if y.shape[0] != M or y.shape[1] != N:
        raise ValueError("out must be [M, N]")
    _check(lib().brq_rotate_quantize_gemm_fused(x.data_ptr(), _dtype_code(x), M, K, ldx, B, _signs_ptr(signs, K),
                                                wq.data_ptr(), ws.data_ptr(), _layout_code(w_layout), N, y.data_ptr(),
                                                _dtype_code(y), ldy, _stream(stream)))
    return y


def diag_mxfp4_gemm_clock(aq, as_, wq, ws, clock, **kw):
    """mxfp4_gemm on a large shape with the clock read-out (brq_diag_mxfp4_gemm_clock): after the launch has
    finished, 0.1 * clock[0] / clock[1] is the shader clock in GHz that the chip held during the product."""
    return mxfp4_gemm(aq, as_, wq, ws, clock=clock, **kw)


def diag_mxfp4_gemm_no_loads(aq, as_, wq, ws, clock, **kw):
    """The large-shape product kernel without its refill loads (brq_diag_mxfp4_gemm_no_loads): a timing aid, the
    output is NOT the product."""
    return mxfp4_gemm(aq, as_, wq, ws, clock=clock, no_loads=True, **kw)


def diag_mfma_ceiling(operands, iters, workgroups, sink=None, stream=None):
    """Launch the MFMA-only measurement loop (brq_diag_mfma_ceiling); returns the flops it does.  After the
    launch has finished, 0.1 * sink[0] / sink[1] is the shader clock in GHz that the chip held in the loop."""
    if not (operands.is_cuda and operands.is_contiguous() and operands.dtype == torch.uint8 and operands.numel() >= 8192):
        raise ValueError("operands must be a contiguous uint8 GPU tensor of at least 8192 bytes")
    if sink is None:
        sink = torch.empty((workgroups * 256,), dtype=torch.float32, device=operands.device)
    if not (sink.is_cuda and sink.is_contiguous() and sink.dtype == torch.float32 and sink.numel() >= workgroups * 256):
        raise ValueError("sink must be a contiguous float32 GPU tensor of workgroups * 256 elements")
    _check(lib().brq_diag_mfma_ceiling(operands.data_ptr(), iters, workgroups, sink.data_ptr(), _stream(stream)))
    return workgroups * 4 * iters * 16 * 131072
