"""GPU parity of the decode-size product that carries the online step in its own prologue (Sec. 4.3: the
online rotation and the quantizer in front of the quantized layer), through the C ABI: against the oracle
(its rotation + quantization of the activations, then its fp64 product: the 1e-5 forward-error rule) and,
bit for bit, against the library's own two-call sequence that it promises to reproduce."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host
from paper_2511_04214_amd.inputs import f32_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def brq():
    import paper_2511_04214_amd as b
    b.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return b


def make(M, N, K, seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(4, size=(M, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    return (f32_to_bf16_bits(x) if dtype == "bf16" else x), f32_to_bf16_bits(w)


def check(brq, orc, x, w, layout, signs=None, xd=None):
    M, K = x.shape
    N = w.shape[0]
    sg = None if signs is None else torch.from_numpy(signs).cuda()
    xd = to_dev(x) if xd is None else xd
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32, layout=layout, signs=sg)
    y32 = brq.rotate_quantize_gemm_fused(xd, 32, wq, ws, N, w_layout=layout, signs=sg)
    y16 = brq.rotate_quantize_gemm_fused(xd, 32, wq, ws, N, w_layout=layout, signs=sg, out_dtype=torch.bfloat16)
    # the two-call sequence of the library
    aq, as_ = brq.rotate_quantize_fused(xd, 32, signs=sg)
    z32 = brq.mxfp4_gemm(aq, as_, wq, ws, w_layout=layout, N=N, K=K)
    z16 = brq.mxfp4_gemm(aq, as_, wq, ws, w_layout=layout, N=N, K=K, out_dtype=torch.bfloat16)
    assert torch.equal(y32, z32) and torch.equal(y16, z16), "differs from the two-call sequence"
    # the oracle
    oa, oas = orc.rotate_quantize_fused(x, 32, signs=signs)
    ow, ows = orc.rotate_quantize_fused(w, 32, signs=signs)
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
    err = np.abs(to_host(y32).astype(np.float64) - ref)
    assert (err <= 1e-5 * bound + 2.0 ** -126).all(), "max err/bound = %g" % float((err / (bound + 2.0 ** -126)).max())


@pytest.mark.parametrize("layout", ["rowmajor", "tiled"])
@pytest.mark.parametrize("M,N,K,dtype", [(1, 256, 512, "bf16"), (2, 1000, 1536, "bf16"), (4, 384, 2048, "f32"),
                                         (7, 130, 1024, "bf16"), (16, 640, 2560, "bf16"), (16, 128, 16384, "bf16"),
                                         (3, 77, 3584, "f32")])
def test_matches_oracle_and_two_call_sequence(brq, orc, M, N, K, dtype, layout):
    x, w = make(M, N, K, 800 + M + N + K, dtype)
    check(brq, orc, x, w, layout)


def test_signs_and_strided_activations(brq, orc):
    M, N, K = 5, 300, 1024
    x, w = make(M, N, K + 64, 810)
    signs = np.random.default_rng(811).choice([-1, 1], size=K).astype(np.int8)
    xd = to_dev(x)[:, 32:32 + K]                          # pitch K + 64, offset start
    check(brq, orc, np.ascontiguousarray(x[:, 32:32 + K]), np.ascontiguousarray(w[:, :K]), "tiled", signs=signs, xd=xd)


@pytest.mark.parametrize("M", [1, 16])
def test_decode_full_size(brq, orc, M):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["decode"]
    x = inputs.make_x(cfg, M=16)[:M]
    w = inputs.make_w(cfg)
    check(brq, orc, x, w, "tiled")


def test_output_pitch_and_argument_errors(brq):
    x, w = make(4, 256, 512, 820)
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32)
    buf = torch.full((4, 256 + 24), -7.0, dtype=torch.float32, device="cuda")
    brq.rotate_quantize_gemm_fused(to_dev(x), 32, wq, ws, 256, out=buf[:, :256])
    assert (buf[:, 256:] == -7.0).all()
    assert torch.equal(buf[:, :256], brq.rotate_quantize_gemm_fused(to_dev(x), 32, wq, ws, 256))
    x17 = torch.zeros((17, 512), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(brq.BrqError) as e:
        brq.rotate_quantize_gemm_fused(x17, 32, wq, ws, 256)
    assert e.value.status == 2
    with pytest.raises(brq.BrqError) as e:
        brq.rotate_quantize_gemm_fused(to_dev(x), 64, wq, ws, 256)
    assert e.value.status == 3
    y = brq.rotate_quantize_gemm_fused(to_dev(x)[:0], 32, wq, ws, 256)       # no rows: nothing launched
    assert y.shape == (0, 256)
