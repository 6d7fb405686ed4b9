"""Seeded sweeps over shapes, layouts, types and pitches: the product's dispatcher picks one of five
kernels from M, N, K and the operand layouts, the row-wise entry points one of four from B, K and the
pitches; the hand-picked shapes of the other test files sit on the known boundaries, these draw the
rest of the space.  Same bars as there: codes and scales bit for bit (by the interval rule where the
interface states an error bound instead of an operation sequence), the product within
1e-5 * sum |a w| per element."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host
from test_gpu_layout import to_tiled

import os

pytestmark = pytest.mark.gpu

# BRQ_SWEEP_SCALE=k draws k times as many cases from other seeds (a longer run by hand; default 1)
SCALE = max(1, int(os.environ.get("BRQ_SWEEP_SCALE", "1")))
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


@pytest.mark.parametrize("M,N,K,a_tiled,w_tiled,bf16,pad", gemm_cases(40 * SCALE, 9001 + SCALE - 1))
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


@pytest.mark.parametrize("M,K,B,bf16,tiled,signed,pad", rowwise_cases(40 * SCALE, 9002 + SCALE - 1))
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


def producer_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.integers(1, 200))
        K = int(rng.choice([32 * rng.integers(1, 65), 2 ** rng.integers(5, 12)]))
        pows = [b for b in (8, 16, 32, 64, 128, 256, 512, 1024) if K % b == 0]
        out.append((M, K, int(rng.choice(pows + [1])), bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2)),
                    bool(rng.integers(2))))
    return out


@pytest.mark.parametrize("M,K,B,bf16,h_bf16,tiled,shared", producer_cases(20 * SCALE, 9003 + SCALE - 1))
def test_swiglu_fused_sweep(brq, orc, M, K, B, bf16, h_bf16, tiled, shared):
    # gate and up as two matrices or as the halves of one [M, 2K] buffer
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(M * 5 + K + B)
    gu = (rng.standard_t(4, size=(M, 2 * K)) * 1.5).astype(np.float32)
    gu[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 8.0
    gh = f32_to_bf16_bits(gu) if bf16 else gu
    g, u = np.ascontiguousarray(gh[:, :K]), np.ascontiguousarray(gh[:, K:])
    if shared:
        buf = to_dev(gh)
        gd, ud = buf[:, :K], buf[:, K:]
    else:
        gd, ud = to_dev(g), to_dev(u)
    lay = "tiled" if tiled else "rowmajor"
    c, s = brq.swiglu_rotate_quantize_fused(gd, ud, B, h_dtype=torch.bfloat16 if h_bf16 else torch.float32, layout=lay)
    if tiled:
        c, s = brq.to_rowmajor(c, s, M, K)
    # the activation is judged by its stated error bound, the codes and scales behind it by the interval
    # that bound leaves open (the oracle is the fp64 definition, not an fp32 operation sequence)
    from interval_check import check_swiglu_fused, swiglu_bound
    same_c, same_s = check_swiglu_fused(orc, g, u, B, h_bf16, None, to_host(c), to_host(s))
    assert same_c > 0.99 and same_s > 0.99, (same_c, same_s)
    h = to_host(brq.swiglu(gd, ud)).astype(np.float64)
    exact = orc.swiglu_exact(g, u)
    g64 = (orc.bf16_to_f32(g) if bf16 else g).astype(np.float64)
    u64 = (orc.bf16_to_f32(u) if bf16 else u).astype(np.float64)
    assert (np.abs(h - exact) <= swiglu_bound(g64, u64, exact)).all(), "activation outside its bound"


def stats_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.integers(1, 200))
        K = int(rng.choice([32 * rng.integers(1, 65), 2 ** rng.integers(5, 12)]))
        pows = [b for b in (8, 16, 32, 64, 128, 256, 512, 1024, 2048) if K % b == 0]
        out.append((M, K, int(rng.choice(pows + [1])), bool(rng.integers(2)), int(rng.integers(0, 9)), bool(rng.integers(2))))
    return out


@pytest.mark.parametrize("M,K,B,bf16,nt,signed", stats_cases(16 * SCALE, 9004 + SCALE - 1))
def test_block_stats_sweep(brq, orc, M, K, B, bf16, nt, signed):
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(M * 3 + K + B + nt)
    x = rng.standard_t(4, size=(M, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    xh = f32_to_bf16_bits(x) if bf16 else x
    th = tuple(float(t) for t in np.sort(rng.uniform(0.1, 8.0, size=nt)).astype(np.float32))
    signs = rng.choice([-1, 1], size=K).astype(np.int8) if (signed and B > 1) else None
    sg = None if signs is None else torch.from_numpy(signs).cuda()
    amax, counts, sq, sqb = brq.block_stats(to_dev(xh), B, th, signs=sg, want_bfp4=True)
    ra, rc, rs, rb = orc.block_stats(xh, B, th, signs=signs, want_bfp4=True)
    assert np.array_equal(to_host(amax).view(np.uint32), ra.view(np.uint32)), "block scales differ"
    if nt:
        assert np.array_equal(to_host(counts).astype(np.uint64), rc)
    for got, want in ((sq, rs), (sqb, rb)):
        g = to_host(got).astype(np.float64)
        assert (np.abs(g - want) <= 4e-6 * want + 1e-44).all()


@pytest.mark.parametrize("M,K,bf16,shared,tiled", [(37, 128, True, False, False), (150, 896, True, True, True),
                                                   (64, 2048, False, False, True), (9, 384, False, True, False),
                                                   (200, 1152, True, False, True), (1, 256, True, True, False)])
def test_matrix_blocks_sweep(brq, orc, M, K, bf16, shared, tiled):
    from test_gpu_matrix_rotate import check_fused_within_bound, orthogonal_blocks
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(M + K)
    x = rng.standard_t(4, size=(M, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    xh = f32_to_bf16_bits(x) if bf16 else x
    R = orthogonal_blocks(1 if shared else K // 32, seed=M * 11 + K)
    c, s = brq.matrix_rotate_quantize_fused(to_dev(xh), torch.from_numpy(R).cuda(), layout="tiled" if tiled else "rowmajor")
    if tiled:
        c, s = brq.to_rowmajor(c, s, M, K)
    same_c, same_s = check_fused_within_bound(orc, xh, R, to_host(c), to_host(s))
    assert same_c > 0.995 and same_s > 0.995
