"""Seeded sweeps over shapes, layouts, types and pitches: the product's dispatcher picks one of five
kernels from M, N, K and the operand layouts, the row-wise entry points one of four from B, K and the
pitches; the hand-picked shapes of the other test files sit on the known boundaries, these draw the
rest of the space.  Same bars as there: codes and scales bit for bit, the product within
1e-5 * sum |a w| per element."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host
from test_gpu_layout import to_tiled

pytestmark = pytest.mark.gpu

RTOL = 1e-5
FLOOR = 2.0 ** -126


@pytest.fixture(scope="module")
def brq():
    import paper_2511_04214_amd as b
    b.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return b


def gemm_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.choice([rng.integers(1, 17), rng.integers(17, 129), rng.integers(129, 400)]))
        N = int(rng.choice([rng.integers(1, 700), 256 * rng.integers(1, 4)]))
        K = int(rng.choice([32 * rng.integers(1, 73), 512 * rng.integers(1, 6)]))
        out.append((M, N, K, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2)), 8 * int(rng.integers(0, 3))))
    return out


@pytest.mark.parametrize("M,N,K,a_tiled,w_tiled,bf16,pad", gemm_cases(40, 9001))
def test_product_sweep(brq, orc, M, N, K, a_tiled, w_tiled, bf16, pad):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(M, K, seed=M * 31 + K)
    wq, ws = inputs.random_mxfp4(N, K, seed=N * 17 + K + 1)
    a = [to_dev(t) for t in (to_tiled(aq, as_) if a_tiled else (aq, as_))]
    w = [to_dev(t) for t in (to_tiled(wq, ws) if w_tiled else (wq, ws))]
    dt = torch.bfloat16 if bf16 else torch.float32
    buf = torch.full((M, N + pad), -7.0, dtype=dt, device="cuda")
    brq.mxfp4_gemm(a[0], a[1], w[0], w[1], out=buf[:, :N], a_layout="tiled" if a_tiled else "rowmajor",
                   w_layout="tiled" if w_tiled else "rowmajor", M=M, N=N, K=K)
    assert (buf[:, N:] == -7.0).all(), "wrote outside the N columns"
    ref, bound = orc.mxfp4_gemm(aq, as_, wq, ws)
    got = buf[:, :N].float().cpu().numpy().astype(np.float64)
    tol = RTOL * bound + FLOOR + (np.abs(ref) * 2.0 ** -8 if bf16 else 0.0)      # bf16: half an ulp of the output
    err = np.abs(got - ref)
    assert (err <= tol).all(), "max err/tol = %g" % float((err / tol).max())


def rowwise_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.integers(1, 260))
        K = int(rng.choice([32 * rng.integers(1, 81), 2 ** rng.integers(5, 13)]))
        pows = [b for b in (8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096) if K % b == 0]
        B = int(rng.choice(pows + [1]))
        out.append((M, K, B, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2)), 8 * int(rng.integers(0, 3))))
    return out


@pytest.mark.parametrize("M,K,B,bf16,tiled,signed,pad", rowwise_cases(40, 9002))
def test_rotate_quantize_sweep(brq, orc, M, K, B, bf16, tiled, signed, pad):
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(M * 7 + K + B)
    x = rng.standard_t(4, size=(M, K + pad)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    xh = f32_to_bf16_bits(x) if bf16 else x
    signs = rng.choice([-1, 1], size=K).astype(np.int8) if (signed and B > 1) else None
    xd = to_dev(xh)[:, :K]                                             # pitch K + pad
    xv = np.ascontiguousarray(xh[:, :K])
    sg = None if signs is None else torch.from_numpy(signs).cuda()
    lay = "tiled" if tiled else "rowmajor"
    if B == 1:
        c, s = brq.mxfp4_quantize(xd, layout=lay)
        rc, rs = orc.mxfp4_quantize(xv)
    else:
        c, s = brq.rotate_quantize_fused(xd, B, layout=lay, signs=sg)
        rc, rs = orc.rotate_quantize_fused(xv, B, signs=signs)
    if tiled:
        c, s = brq.to_rowmajor(c, s, M, K)
    assert np.array_equal(to_host(s), rs), "scales differ"
    assert np.array_equal(to_host(c), rc), "codes differ"
    if B > 1:
        y = to_host(brq.block_rotate(xd, B, signs=sg))
        ry = orc.block_rotate(xv, B, signs=signs)
        ua, ub = y.view(np.uint32), ry.view(np.uint32)      # the sign of an exact zero is not defined
        assert ((ua == ub) | (((ua | ub) & np.uint32(0x7FFFFFFF)) == 0)).all(), "rotated values differ"
