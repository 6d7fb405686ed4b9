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
EXPORTS = ["brq_block_rotate", "brq_mxfp4_quantize", "brq_rotate_quantize_fused", "brq_mxfp4_gemm",
           "brq_strerror", "brq_version"]

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
        L.brq_block_rotate.argtypes = [vp, i32, i64, i64, i64, i64, vp, i32, i64, vp]
        L.brq_block_rotate.restype = i32
        L.brq_mxfp4_quantize.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp]
        L.brq_mxfp4_quantize.restype = i32
        L.brq_rotate_quantize_fused.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp]
        L.brq_rotate_quantize_fused.restype = i32
        L.brq_mxfp4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i32, i64, vp]
        L.brq_mxfp4_gemm.restype = i32
        L.brq_strerror.argtypes = [i32]
        L.brq_strerror.restype = ctypes.c_char_p
        L.brq_version.restype = i32
        _lib = L
    return _lib


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


def block_rotate(x, B, out_dtype=torch.float32, out=None, stream=None):
    """y = x * diag(H_B..H_B)/sqrt(B) along the last axis (brq_block_rotate)."""
    M, K, ldx = _rows(x, "x")
    y = torch.empty((M, K), dtype=out_dtype, device=x.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    _check(lib().brq_block_rotate(x.data_ptr(), _dtype_code(x), M, K, ldx, B, y.data_ptr(), _dtype_code(y), ldy,
                                  _stream(stream)))
    return y


def _alloc_q(x, M, K, codes, scales):
    if codes is None:
        codes = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((M, K // 32), dtype=torch.uint8, device=x.device)
    if not (codes.is_contiguous() and scales.is_contiguous()):
        raise ValueError("codes and scales must be contiguous")
    return codes, scales


def mxfp4_quantize(x, codes=None, scales=None, stream=None):
    """x -> (codes [M, K/2] u8, scales [M, K/32] u8) (brq_mxfp4_quantize)."""
    M, K, ldx = _rows(x, "x")
    codes, scales = _alloc_q(x, M, K, codes, scales)
    _check(lib().brq_mxfp4_quantize(x.data_ptr(), _dtype_code(x), M, K, ldx, codes.data_ptr(), scales.data_ptr(),
                                    _stream(stream)))
    return codes, scales


def rotate_quantize_fused(x, B, codes=None, scales=None, stream=None):
    """Block rotation fused with MXFP4 quantization (brq_rotate_quantize_fused)."""
    M, K, ldx = _rows(x, "x")
    codes, scales = _alloc_q(x, M, K, codes, scales)
    _check(lib().brq_rotate_quantize_fused(x.data_ptr(), _dtype_code(x), M, K, ldx, B, codes.data_ptr(),
                                           scales.data_ptr(), _stream(stream)))
    return codes, scales


def mxfp4_gemm(aq, as_, wq, ws, out_dtype=torch.float32, out=None, stream=None):
    """Y[M, N] = deq(aq, as) @ deq(wq, ws)^T on the block-scaled MFMA (brq_mxfp4_gemm)."""
    for t, n in ((aq, "aq"), (as_, "as"), (wq, "wq"), (ws, "ws")):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.uint8 and t.dim() == 2):
            raise ValueError("%s must be a contiguous 2-D uint8 GPU tensor" % n)
    M, K = aq.shape[0], aq.shape[1] * 2
    N = wq.shape[0]
    if wq.shape[1] * 2 != K or tuple(as_.shape) != (M, K // 32) or tuple(ws.shape) != (N, K // 32):
        raise ValueError("operand shapes disagree")
    y = torch.empty((M, N), dtype=out_dtype, device=aq.device) if out is None else out
    _, _, ldy = _rows(y, "out")
    _check(lib().brq_mxfp4_gemm(aq.data_ptr(), as_.data_ptr(), wq.data_ptr(), ws.data_ptr(), M, N, K, y.data_ptr(),
                                _dtype_code(y), ldy, _stream(stream)))
    return y
