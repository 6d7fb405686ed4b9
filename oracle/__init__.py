"""ctypes front for the CPU oracle (oracle/brq_oracle.c).

TEST INFRASTRUCTURE ONLY: nothing in the product package imports this module.  Only
tests, the smoke entry and the benchmark's cpu_baseline leg use it.  It carries no
arithmetic of its own: every function marshals numpy arrays into the C routines.

bf16 tensors are numpy uint16 arrays holding the bit patterns; fp32 tensors are float32.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_brq.so")

F32, BF16 = 0, 1


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB



def _bind(path):
    L = ctypes.CDLL(path)
    i64, vp, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    L.oracle_set_threads.argtypes = [i32]
    L.oracle_get_threads.restype = i32
    L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
    L.oracle_bf16_to_f32.restype = ctypes.c_float
    L.oracle_bf16_to_f32_array.argtypes = [vp, i64, vp]
    L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
    L.oracle_f32_to_bf16.restype = ctypes.c_uint16
    L.oracle_hadamard_entry.argtypes = [i32, i32, i32]
    L.oracle_hadamard_entry.restype = i32
    L.oracle_hadamard_sylvester.argtypes = [i32, vp]
    L.oracle_rotate_dense_f64.argtypes = [vp, i64, i64, i64, vp]
    L.oracle_rotation_norm.argtypes = [i64]
    L.oracle_rotation_norm.restype = ctypes.c_float
    L.oracle_block_rotate.argtypes = [vp, i32, i64, i64, i64, i64, vp, i32, i64]
    L.oracle_block_rotate_signed.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i32, i64]
    L.oracle_e2m1_value.argtypes = [i32]
    L.oracle_e2m1_value.restype = ctypes.c_double
    L.oracle_e8m0_from_amax.argtypes = [ctypes.c_float]
    L.oracle_e8m0_from_amax.restype = ctypes.c_uint8
    L.oracle_e8m0_value.argtypes = [ctypes.c_uint8]
    L.oracle_e8m0_value.restype = ctypes.c_double
    L.oracle_e2m1_encode.argtypes = [ctypes.c_float, ctypes.c_uint8]
    L.oracle_e2m1_encode.restype = ctypes.c_uint8
    L.oracle_mxfp4_quantize.argtypes = [vp, i32, i64, i64, i64, vp, vp]
    L.oracle_rotate_quantize_fused.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp]
    L.oracle_rotate_quantize_fused_signed.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp]
    L.oracle_swiglu_elem.argtypes = [ctypes.c_float, ctypes.c_float]
    L.oracle_swiglu_elem.restype = ctypes.c_float
    L.oracle_swiglu_f64.argtypes = [ctypes.c_double, ctypes.c_double]
    L.oracle_swiglu_f64.restype = ctypes.c_double
    L.oracle_f64_to_bf16.argtypes = [ctypes.c_double]
    L.oracle_f64_to_bf16.restype = ctypes.c_uint16
    L.oracle_swiglu.argtypes = [vp, vp, i32, i64, i64, i64, i64, vp, i32, i64]
    L.oracle_swiglu_f64_array.argtypes = [vp, vp, i32, i64, i64, i64, i64, vp]
    L.oracle_swiglu_rotate_quantize_fused.argtypes = [vp, vp, i32, i64, i64, i64, i64, i32, i64, vp, vp, vp]
    L.oracle_matrix_rotate_f64.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp]
    L.oracle_matrix_rotate_quantize_fused.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp]
    L.oracle_mxfp4_encode_with_scales.argtypes = [vp, vp, i64, i64, vp]
    L.oracle_block_stats.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i32, vp, vp, vp, vp]
    L.oracle_block_stats_summary.argtypes = [vp, vp, vp, i64, ctypes.c_float, vp, i32, vp, vp, vp]
    L.oracle_round_to_f16.argtypes = [ctypes.c_float]
    L.oracle_round_to_f16.restype = ctypes.c_float
    L.oracle_mxfp4_dequantize.argtypes = [vp, vp, i64, i64, vp]
    L.oracle_mxfp4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i64, vp, vp]
    L.oracle_matmul_nt_f64.argtypes = [vp, vp, i64, i64, i64, vp]
    return L


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s: bad arguments (rc=%d)" % (what, rc))


def _dt(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32, or uint16 holding bf16 bits; got %s" % a.dtype)


def _signs(signs, K):
    sg = np.ascontiguousarray(signs, dtype=np.int8)
    if sg.shape != (K,):
        raise ValueError("signs must have K elements")
    return sg


def _rows(a):
    """2-D array with contiguous rows -> (array, M, K, row pitch in elements)."""
    if a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        raise ValueError("need a 2-D array with contiguous rows")
    ld = a.strides[0] // a.itemsize if a.shape[0] > 1 else a.shape[1]   # a single row has no pitch
    return a, a.shape[0], a.shape[1], ld


class Oracle:
    """One loaded build of the oracle library.  The default build is `oracle.default()`;
    tests that plant a mistake in a copy of the C source load that copy through this class."""

    def __init__(self, path):
        self.L = _bind(path)

    def set_threads(self, n):
        self.L.oracle_set_threads(int(n))

    def get_threads(self):
        return int(self.L.oracle_get_threads())

    def bf16_to_f32(self, bits):
        """uint16 bf16 bit patterns -> float32 (exact widening, done by the C routine)."""
        b = np.ascontiguousarray(bits, dtype=np.uint16)
        out = np.empty(b.shape, dtype=np.float32)
        self.L.oracle_bf16_to_f32_array(_p(b), b.size, _p(out))
        return out

    def f32_to_bf16(self, f):
        return int(self.L.oracle_f32_to_bf16(float(np.float32(f))))

    def hadamard_sylvester(self, B):
        out = np.zeros((B, B), dtype=np.int32)
        _check(self.L.oracle_hadamard_sylvester(B, _p(out)), "hadamard_sylvester")
        return out

    def hadamard_entry(self, B, i, j):
        return int(self.L.oracle_hadamard_entry(B, i, j))

    def rotate_dense_f64(self, x, B):
        x = np.ascontiguousarray(x, dtype=np.float64)
        y = np.empty_like(x)
        _check(self.L.oracle_rotate_dense_f64(_p(x), x.shape[0], x.shape[1], B, _p(y)), "rotate_dense_f64")
        return y

    def rotation_norm(self, B):
        return np.float32(self.L.oracle_rotation_norm(B))

    def block_rotate(self, x, B, out_bf16=False, signs=None):
        x, M, K, ldx = _rows(x)
        y = np.empty((M, K), dtype=np.uint16 if out_bf16 else np.float32)
        if signs is None:
            _check(self.L.oracle_block_rotate(_p(x), _dt(x), M, K, ldx, B, _p(y), BF16 if out_bf16 else F32, K),
                   "block_rotate")
        else:
            sg = _signs(signs, K)
            _check(self.L.oracle_block_rotate_signed(_p(x), _dt(x), M, K, ldx, B, _p(sg), _p(y),
                                                     BF16 if out_bf16 else F32, K), "block_rotate_signed")
        return y

    def e2m1_value(self, code):
        return float(self.L.oracle_e2m1_value(int(code)))

    def e8m0_from_amax(self, amax):
        return int(self.L.oracle_e8m0_from_amax(float(np.float32(amax))))

    def e8m0_value(self, byte):
        return float(self.L.oracle_e8m0_value(int(byte)))

    def e2m1_encode(self, y, scale_byte):
        return int(self.L.oracle_e2m1_encode(float(np.float32(y)), int(scale_byte)))

    def mxfp4_quantize(self, x):
        x, M, K, ldx = _rows(x)
        codes = np.empty((M, K // 2), dtype=np.uint8)
        scales = np.empty((M, K // 32), dtype=np.uint8)
        _check(self.L.oracle_mxfp4_quantize(_p(x), _dt(x), M, K, ldx, _p(codes), _p(scales)), "mxfp4_quantize")
        return codes, scales

    def rotate_quantize_fused(self, x, B, signs=None):
        x, M, K, ldx = _rows(x)
        codes = np.empty((M, K // 2), dtype=np.uint8)
        scales = np.empty((M, K // 32), dtype=np.uint8)
        if signs is None:
            _check(self.L.oracle_rotate_quantize_fused(_p(x), _dt(x), M, K, ldx, B, _p(codes), _p(scales)),
                   "rotate_quantize_fused")
        else:
            sg = _signs(signs, K)
            _check(self.L.oracle_rotate_quantize_fused_signed(_p(x), _dt(x), M, K, ldx, B, _p(sg), _p(codes),
                                                              _p(scales)), "rotate_quantize_fused_signed")
        return codes, scales

    def swiglu_elem(self, g, u):
        return np.float32(self.L.oracle_swiglu_elem(float(np.float32(g)), float(np.float32(u))))

    def swiglu_f64(self, g, u):
        return float(self.L.oracle_swiglu_f64(float(g), float(u)))

    def f64_to_bf16(self, x):
        return int(self.L.oracle_f64_to_bf16(float(x)))

    def swiglu_exact(self, gate, up):
        """h = silu(gate) * up in fp64, unrounded."""
        gate, M, K, ldg = _rows(gate)
        up, M2, K2, ldu = _rows(up)
        if (M, K) != (M2, K2) or gate.dtype != up.dtype:
            raise ValueError("gate and up must agree in shape and type")
        h = np.empty((M, K), dtype=np.float64)
        _check(self.L.oracle_swiglu_f64_array(_p(gate), _p(up), _dt(gate), M, K, ldg, ldu, _p(h)), "swiglu_f64_array")
        return h

    def swiglu(self, gate, up, out_bf16=False):
        """h = silu(gate) * up: the fp64 definition rounded once to fp32, or once to bf16 (bits)."""
        gate, M, K, ldg = _rows(gate)
        up, M2, K2, ldu = _rows(up)
        if (M, K) != (M2, K2) or gate.dtype != up.dtype:
            raise ValueError("gate and up must agree in shape and type")
        h = np.empty((M, K), dtype=np.uint16 if out_bf16 else np.float32)
        _check(self.L.oracle_swiglu(_p(gate), _p(up), _dt(gate), M, K, ldg, ldu, _p(h), BF16 if out_bf16 else F32, K),
               "swiglu")
        return h

    def swiglu_rotate_quantize_fused(self, gate, up, B, h_bf16=False, signs=None):
        gate, M, K, ldg = _rows(gate)
        up, M2, K2, ldu = _rows(up)
        if (M, K) != (M2, K2) or gate.dtype != up.dtype:
            raise ValueError("gate and up must agree in shape and type")
        codes = np.empty((M, K // 2), dtype=np.uint8)
        scales = np.empty((M, K // 32), dtype=np.uint8)
        sg = None if signs is None else _signs(signs, K)
        _check(self.L.oracle_swiglu_rotate_quantize_fused(_p(gate), _p(up), _dt(gate), M, K, ldg, ldu,
                                                          BF16 if h_bf16 else F32, B,
                                                          None if sg is None else _p(sg), _p(codes), _p(scales)),
               "swiglu_rotate_quantize_fused")
        return codes, scales

    @staticmethod
    def _blocks(R, K):
        R = np.ascontiguousarray(R, dtype=np.float32)
        if R.ndim == 2:
            R = R[None]
        if R.shape[1:] != (32, 32) or R.shape[0] not in (1, K // 32):
            raise ValueError("R must be [32, 32] or [K/32, 32, 32]")
        return R

    def matrix_rotate_f64(self, x, R, want_bound=False):
        """y = x diag(R_1..R_n) in fp64 (R[b][i][j]: input i -> output j); optionally sum |x||R|."""
        x, M, K, ldx = _rows(x)
        R = self._blocks(R, K)
        y = np.empty((M, K), dtype=np.float64)
        bound = np.empty((M, K), dtype=np.float64) if want_bound else None
        _check(self.L.oracle_matrix_rotate_f64(_p(x), _dt(x), M, K, ldx, _p(R), R.shape[0], _p(y),
                                               _p(bound) if want_bound else None), "matrix_rotate_f64")
        return (y, bound) if want_bound else y

    def matrix_rotate_quantize_fused(self, x, R):
        x, M, K, ldx = _rows(x)
        R = self._blocks(R, K)
        codes = np.empty((M, K // 2), dtype=np.uint8)
        scales = np.empty((M, K // 32), dtype=np.uint8)
        _check(self.L.oracle_matrix_rotate_quantize_fused(_p(x), _dt(x), M, K, ldx, _p(R), R.shape[0], _p(codes),
                                                          _p(scales)), "matrix_rotate_quantize_fused")
        return codes, scales

    def mxfp4_encode_with_scales(self, y, scales):
        y = np.ascontiguousarray(y, dtype=np.float32)
        scales = np.ascontiguousarray(scales, dtype=np.uint8)
        M, K = y.shape
        codes = np.empty((M, K // 2), dtype=np.uint8)
        _check(self.L.oracle_mxfp4_encode_with_scales(_p(y), _p(scales), M, K, _p(codes)), "mxfp4_encode_with_scales")
        return codes

    def round_to_f16(self, f):
        return np.float32(self.L.oracle_round_to_f16(float(np.float32(f))))

    def block_stats(self, x, B, thresholds=(), signs=None, want_bfp4=False):
        """(amax [M, K/32] f32, counts [nt] u64, sqerr [M, K/32] f64[, sqerr_bfp4 [M, K/32] f64]) of x after the
        rotation with block B (B = 1: no rotation)."""
        x, M, K, ldx = _rows(x)
        th = np.ascontiguousarray(thresholds, dtype=np.float32)
        amax = np.empty((M, K // 32), dtype=np.float32)
        sqerr = np.empty((M, K // 32), dtype=np.float64)
        bfp4 = np.empty((M, K // 32), dtype=np.float64) if want_bfp4 else None
        count = np.zeros(th.size, dtype=np.uint64)
        sg = None if signs is None else _signs(signs, K)
        _check(self.L.oracle_block_stats(_p(x), _dt(x), M, K, ldx, B, None if sg is None else _p(sg),
                                         _p(th) if th.size else None, th.size, _p(amax), _p(count), _p(sqerr),
                                         None if bfp4 is None else _p(bfp4)), "block_stats")
        return (amax, count, sqerr, bfp4) if want_bfp4 else (amax, count, sqerr)

    def block_stats_summary(self, amax, sqerr=None, ref=None, outlier=0.0, edges=()):
        """(hist [len(edges) + 1] u64, counts [4] u64, sums [4] f64) over per-block statistics."""
        amax = np.ascontiguousarray(amax, dtype=np.float32).ravel()
        sq = None if sqerr is None else np.ascontiguousarray(sqerr, dtype=np.float32).ravel()
        rf = None if ref is None else np.ascontiguousarray(ref, dtype=np.float32).ravel()
        ed = np.ascontiguousarray(edges, dtype=np.float32)
        hist = np.zeros(ed.size + 1, dtype=np.uint64)
        counts = np.zeros(4, dtype=np.uint64)
        sums = np.zeros(4, dtype=np.float64)
        _check(self.L.oracle_block_stats_summary(_p(amax), None if sq is None else _p(sq), None if rf is None else _p(rf),
                                                 amax.size, float(outlier), _p(ed) if ed.size else None, ed.size,
                                                 _p(hist), _p(counts), _p(sums)), "block_stats_summary")
        return hist, counts, sums

    def mxfp4_dequantize(self, codes, scales):
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        scales = np.ascontiguousarray(scales, dtype=np.uint8)
        M, K = codes.shape[0], codes.shape[1] * 2
        out = np.empty((M, K), dtype=np.float64)
        _check(self.L.oracle_mxfp4_dequantize(_p(codes), _p(scales), M, K, _p(out)), "mxfp4_dequantize")
        return out

    def mxfp4_gemm(self, aq, as_, wq, ws, rows=None, want_bound=True):
        """fp64 product of the dequantized operands; returns (y, bound) for the chosen rows."""
        aq = np.ascontiguousarray(aq, dtype=np.uint8)
        as_ = np.ascontiguousarray(as_, dtype=np.uint8)
        wq = np.ascontiguousarray(wq, dtype=np.uint8)
        ws = np.ascontiguousarray(ws, dtype=np.uint8)
        M, K = aq.shape[0], aq.shape[1] * 2
        N = wq.shape[0]
        if wq.shape[1] * 2 != K or as_.shape != (M, K // 32) or ws.shape != (N, K // 32):
            raise ValueError("operand shapes disagree")
        if rows is None:
            rp, nrows = None, M
        else:
            rows = np.ascontiguousarray(rows, dtype=np.int64)
            rp, nrows = _p(rows), rows.size
        y = np.empty((nrows, N), dtype=np.float64)
        bound = np.empty((nrows, N), dtype=np.float64) if want_bound else None
        _check(self.L.oracle_mxfp4_gemm(_p(aq), _p(as_), _p(wq), _p(ws), M, N, K, rp, nrows, _p(y),
                                        _p(bound) if want_bound else None), "mxfp4_gemm")
        return y, bound

    def matmul_nt_f64(self, a, w):
        a = np.ascontiguousarray(a, dtype=np.float64)
        w = np.ascontiguousarray(w, dtype=np.float64)
        y = np.empty((a.shape[0], w.shape[0]), dtype=np.float64)
        _check(self.L.oracle_matmul_nt_f64(_p(a), _p(w), a.shape[0], w.shape[0], a.shape[1], _p(y)), "matmul_nt")
        return y


_default = None


def default():
    """The oracle built from oracle/brq_oracle.c as committed."""
    global _default
    if _default is None:
        _default = Oracle(build())
    return _default


def __getattr__(name):
    # module-level shorthand: oracle.mxfp4_quantize(x) == oracle.default().mxfp4_quantize(x)
    if name.startswith("_"):
        raise AttributeError(name)
    return getattr(default(), name)
