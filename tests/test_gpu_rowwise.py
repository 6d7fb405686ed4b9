"""GPU parity: rotation, MXFP4 quantization and their fusion, through the C ABI, against the
CPU oracle on the same seeded inputs.  Codes and scales are compared bit for bit; rotated
fp32 values for exact equality (the sign of an exact zero is the one thing left open)."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def brq():
    import paper_2511_04214_amd as b
    b.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return b


def finite_bf16(bits):
    bits = bits.copy()
    bits[(bits & 0x7F80) == 0x7F80] ^= 0x4000      # Inf/NaN -> some finite value
    return bits


def windowed_bf16(rng, M, K, lo=1, hi=250, width=8):
    """Random bf16 bits whose exponent fields lie within `width` binades below a per-group top
    exponent: every group exercises all codes, rounding boundaries and saturation."""
    top = rng.integers(lo + width, hi, size=(M, K // 32, 1))
    e = np.clip(top - rng.integers(0, width, size=(M, K // 32, 32)), 0, 254)
    e[:, :, 0] = np.clip(top[:, :, 0], 0, 254)
    mant = rng.integers(0, 128, size=(M, K // 32, 32))
    sign = rng.integers(0, 2, size=(M, K // 32, 32))
    return ((sign << 15) | (e << 7) | mant).astype(np.uint16).reshape(M, K)


def check_q(brq, orc, x_np, B=None):
    x = to_dev(x_np)
    if B is None:
        c, s = brq.mxfp4_quantize(x)
        rc, rs = orc.mxfp4_quantize(x_np)
    else:
        c, s = brq.rotate_quantize_fused(x, B)
        rc, rs = orc.rotate_quantize_fused(x_np, B)
    c, s = to_host(c), to_host(s)
    assert np.array_equal(s, rs), "scales differ in %d places" % int((s != rs).sum())
    assert np.array_equal(c, rc), "codes differ in %d bytes" % int((c != rc).sum())


# ------------------------------------------------------------------ quantize alone

def test_quantize_every_bf16_pattern(brq, orc):
    # all 65 536 bf16 bit patterns (non-finite ones remapped), shuffled into groups, so that
    # zeros, subnormals, both signs and every exponent meet the scale rule and the encoder
    rng = np.random.default_rng(100)
    bits = finite_bf16(np.arange(1 << 16, dtype=np.uint16))
    for trial in range(3):
        x = rng.permutation(bits).reshape(64, 1024)
        check_q(brq, orc, x)
    # sorted: neighbours share a binade, so groups are full of near-maximum values
    check_q(brq, orc, np.sort(bits.view(np.int16)).view(np.uint16).reshape(64, 1024))


def test_quantize_windowed_groups_bf16(brq, orc):
    rng = np.random.default_rng(101)
    check_q(brq, orc, windowed_bf16(rng, 257, 2080))                 # ragged: 257 rows, K = 65 groups
    check_q(brq, orc, windowed_bf16(rng, 64, 512, lo=-3, hi=12, width=4))   # bottom of the exponent range
    check_q(brq, orc, windowed_bf16(rng, 64, 512, lo=240, hi=255, width=6))  # top of the range


def test_quantize_fp32_boundaries(brq, orc):
    # fp32 inputs sitting on, and one ulp either side of, every rounding midpoint, under many scales
    rng = np.random.default_rng(102)
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 4.0, 7.0, 0.5, 3.0], dtype=np.float32)
    rows = []
    for sb in list(range(0, 6)) + list(range(100, 160, 7)) + [250, 251, 252]:
        scale = np.float32(2.0) ** np.float32(sb - 127) if sb > 0 else np.float32(2.0 ** -126) / 2
        g = np.zeros(32, dtype=np.float32)
        pts = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(9))])
        pts = (pts * scale).astype(np.float32)
        for k in range(0, len(pts), 30):
            g = np.zeros(32, dtype=np.float32)
            chunk = pts[k:k + 30]
            g[1:1 + len(chunk)] = chunk * rng.choice([-1, 1], size=len(chunk)).astype(np.float32)
            g[0] = np.float32(6.0) * scale           # pins the group's exponent
            rows.append(g)
    x = np.stack(rows)
    check_q(brq, orc, x)
    # random fp32 bit patterns in exponent windows, including subnormals
    top = rng.integers(0, 254, size=(300, 4, 1))
    e = np.clip(top - rng.integers(0, 10, size=(300, 4, 32)), 0, 254)
    bits = (rng.integers(0, 2, size=e.shape) << 31) | (e << 23) | rng.integers(0, 1 << 23, size=e.shape)
    check_q(brq, orc, bits.astype(np.uint32).view(np.float32).reshape(300, 128))


def test_quantize_zero_and_negative_zero(brq, orc):
    x = np.zeros((5, 64), dtype=np.float32)
    x[1, :] = -0.0
    x[2, 3] = 1.0
    x[2, 4] = -1e-6          # underflows to magnitude 0: nibble must be 0, not 8
    x[3, 40] = -2.0 ** -140
    check_q(brq, orc, x)
    c, s = brq.mxfp4_quantize(to_dev(x))
    assert not to_host(c)[0].any() and not to_host(c)[1].any() and not to_host(s)[:2].any()


def test_quantize_strided_rows(brq, orc):
    rng = np.random.default_rng(103)
    full = windowed_bf16(rng, 37, 512)
    xd = to_dev(full)[:, 64:64 + 352]            # K = 352 = 11 groups, pitch 512
    c, s = brq.mxfp4_quantize(xd)
    rc, rs = orc.mxfp4_quantize(full[:, 64:64 + 352])
    assert np.array_equal(to_host(c), rc) and np.array_equal(to_host(s), rs)
    c2, s2 = brq.rotate_quantize_fused(xd, 32)
    rc2, rs2 = orc.rotate_quantize_fused(full[:, 64:64 + 352], 32)
    assert np.array_equal(to_host(c2), rc2) and np.array_equal(to_host(s2), rs2)


# ------------------------------------------------------------------ rotation

@pytest.mark.parametrize("B", [8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_block_rotate_matches_oracle(brq, orc, B, dt):
    rng = np.random.default_rng(200 + B)
    K = max(2 * B, 256) if B < 8192 else B
    M = 19 if B < 4096 else 5
    if dt == "bf16":
        x = windowed_bf16(rng, M, K, lo=90, hi=140, width=12)
    else:
        x = (rng.standard_t(4, size=(M, K)) * 3).astype(np.float32)
        x[:, 7] *= 50
    y = to_host(brq.block_rotate(to_dev(x), B))
    ref = orc.block_rotate(x, B)
    assert y.dtype == np.float32 and np.array_equal(y, ref)
    yb = to_host(brq.block_rotate(to_dev(x), B, out_dtype=torch.bfloat16))
    refb = orc.block_rotate(x, B, out_bf16=True)
    same = (yb == refb) | (((yb | refb) & 0x7FFF) == 0)      # +0 / -0 both accepted
    assert same.all()


def test_block_rotate_integers_exact(brq, orc):
    # small integers: fp32 is exact, so any stage order gives the same bits -- and those
    # must equal the oracle's, which its own pins tie to the integer matrix product
    rng = np.random.default_rng(201)
    x = rng.integers(-64, 65, size=(8, 1024)).astype(np.float32)
    for B in (32, 128, 1024):
        assert np.array_equal(to_host(brq.block_rotate(to_dev(x), B)), orc.block_rotate(x, B))


# ------------------------------------------------------------------ randomized (signed) rotation

def same_up_to_zero_sign_f32(a, b):
    ua, ub = a.view(np.uint32), b.view(np.uint32)
    return ((ua == ub) | (((ua | ub) & np.uint32(0x7FFFFFFF)) == 0)).all()


@pytest.mark.parametrize("B", [8, 16, 32, 128, 512, 1024, 4096])
@pytest.mark.parametrize("K,M", [(4096, 37), (4096 + 8 * 32, 21)])      # chunks per row: multiple of 64, and not
def test_signed_rotation_matches_oracle(brq, orc, B, K, M):
    if K % B:
        pytest.skip("B does not divide this K")
    rng = np.random.default_rng(300 + B)
    x = windowed_bf16(rng, M, K, lo=100, hi=135, width=10)
    s = rng.choice([-1, 1], size=K).astype(np.int8)
    sd = torch.from_numpy(s).cuda()
    y = to_host(brq.block_rotate(to_dev(x), B, signs=sd))
    assert same_up_to_zero_sign_f32(y, orc.block_rotate(x, B, signs=s))
    oc, os_ = orc.rotate_quantize_fused(x, B, signs=s)
    for layout in ("rowmajor", "tiled"):
        c, sc = brq.rotate_quantize_fused(to_dev(x), B, signs=sd, layout=layout)
        if layout == "tiled":
            c, sc = brq.to_rowmajor(c, sc, M, K)
        assert np.array_equal(to_host(c), oc) and np.array_equal(to_host(sc), os_), layout
    # the signs matter, and all-plus signs are the plain rotation
    c0, s0 = brq.rotate_quantize_fused(to_dev(x), B)
    assert not np.array_equal(to_host(c0), oc)
    c1, s1 = brq.rotate_quantize_fused(to_dev(x), B, signs=torch.ones(K, dtype=torch.int8, device="cuda"))
    assert torch.equal(c0, c1) and torch.equal(s0, s1)


def test_signed_rotation_fp32_input_and_strided_rows(brq, orc):
    rng = np.random.default_rng(311)
    M, K, ld = 13, 1024, 1024 + 64
    buf = (rng.standard_t(4, size=(M, ld)) * 2).astype(np.float32)
    s = rng.choice([-1, 1], size=K).astype(np.int8)
    xd = to_dev(buf)[:, :K]
    c, sc = brq.rotate_quantize_fused(xd, 32, signs=torch.from_numpy(s).cuda())
    oc, os_ = orc.rotate_quantize_fused(np.ascontiguousarray(buf[:, :K]), 32, signs=s)
    assert np.array_equal(to_host(c), oc) and np.array_equal(to_host(sc), os_)


def test_signed_product_is_invariant(brq, orc):
    """Same signs on activations and weights: the quantized product still approximates X W^T
    (Sec. 2: R = diag(s) H / sqrt(B) is orthogonal), and matches the oracle's."""
    rng = np.random.default_rng(312)
    M, N, K = 64, 256, 512
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32
    x = f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    w = f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
    s = rng.choice([-1, 1], size=K).astype(np.int8)
    sd = torch.from_numpy(s).cuda()
    aq, as_ = brq.rotate_quantize_fused(to_dev(x), 32, signs=sd)
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32, signs=sd)
    y = to_host(brq.mxfp4_gemm(aq, as_, wq, ws)).astype(np.float64)
    oa, oas = orc.rotate_quantize_fused(x, 32, signs=s)
    ow, ows = orc.rotate_quantize_fused(w, 32, signs=s)
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
    assert (np.abs(y - ref) <= 1e-5 * bound + 2.0 ** -126).all()
    exact = bf16_bits_to_f32(x).astype(np.float64) @ bf16_bits_to_f32(w).astype(np.float64).T
    assert np.linalg.norm(y - exact) / np.linalg.norm(exact) < 0.25


# ------------------------------------------------------------------ fused

@pytest.mark.parametrize("B", [8, 16, 32, 64, 128, 256, 512, 1024, 2048, 8192])
def test_fused_matches_oracle_and_composition(brq, orc, B):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["down_sweep"]
    K = 8192 if B >= 1024 else 2048 + 512          # 2560: not a power of two
    M = 67
    x = inputs.make_x(cfg, M=M, K=K)
    check_q(brq, orc, x, B)
    xd = to_dev(x)
    c1, s1 = brq.rotate_quantize_fused(xd, B)
    c2, s2 = brq.mxfp4_quantize(brq.block_rotate(xd, B))       # fp32 intermediate
    assert torch.equal(c1, c2) and torch.equal(s1, s2)


def test_fused_wide_dynamic_range(brq, orc):
    # groups spanning > 11 binades: the order of the fp32 additions decides codes
    rng = np.random.default_rng(300)
    x = windowed_bf16(rng, 129, 1024, lo=60, hi=200, width=24)
    for B in (32, 64, 1024):
        check_q(brq, orc, x, B)
    xf = (rng.standard_normal((33, 256)) * 10.0 ** rng.integers(-6, 6, size=(33, 256))).astype(np.float32)
    for B in (32, 256):
        check_q(brq, orc, xf, B)


def test_fused_tiny_config(brq, orc):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["tiny"]
    check_q(brq, orc, inputs.make_x(cfg), 32)
    check_q(brq, orc, inputs.make_w(cfg), 32)


def test_fused_single_group_and_single_row(brq, orc):
    rng = np.random.default_rng(301)
    check_q(brq, orc, windowed_bf16(rng, 1, 32), 32)
    check_q(brq, orc, windowed_bf16(rng, 1, 8192), 32)
    check_q(brq, orc, windowed_bf16(rng, 3, 96), 32)
    check_q(brq, orc, windowed_bf16(rng, 1, 32))


def test_empty_input(brq):
    x = torch.empty((0, 256), dtype=torch.bfloat16, device="cuda")
    c, s = brq.rotate_quantize_fused(x, 32)
    assert tuple(c.shape) == (0, 128) and tuple(s.shape) == (0, 8)
    assert tuple(brq.block_rotate(x, 64).shape) == (0, 256)


def test_errors_reach_python(brq):
    x = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(brq.BrqError):
        brq.rotate_quantize_fused(x, 64)          # 64 does not divide 96
    with pytest.raises(brq.BrqError):
        brq.mxfp4_quantize(torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda"))


# ------------------------------------------------------------------ full-size workloads

@pytest.mark.parametrize("name", ["llama1b_up", "mlp8b", "decode"])
def test_fused_full_size(brq, orc, name):
    """The benchmark's launch configuration at the benchmark's sizes, every output compared."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS[name]
    x = inputs.make_x(cfg)
    check_q(brq, orc, x, 32)


def test_fused_down_sweep_full_size(brq, orc):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["down_sweep"]
    x = inputs.make_x(cfg)
    for B in cfg["B"]:
        check_q(brq, orc, x, B)


def test_many_rows_sampled(brq, orc):
    # 4 194 309 rows x 128: row and chunk indices far beyond 2^21 (and a ragged last group of 4 rows),
    # row-major and tiled; the oracle checks the first, the last and a sample of rows
    M, K = (1 << 22) + 5, 128
    gen = torch.Generator(device="cuda").manual_seed(900)
    x = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    rng = np.random.default_rng(901)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, M - 6, M - 5, M - 4, M - 1], rng.integers(0, M, 50)]))
    idx = torch.from_numpy(rows).cuda()
    rc, rs = orc.rotate_quantize_fused(to_host(x[idx].contiguous()), 32)
    c, s = brq.rotate_quantize_fused(x, 32)
    assert np.array_equal(to_host(c[idx]), rc) and np.array_equal(to_host(s[idx]), rs)
    ct, st_ = brq.rotate_quantize_fused(x, 32, layout="tiled")
    c2, s2 = brq.to_rowmajor(ct, st_, M, K)
    assert torch.equal(c2, c) and torch.equal(s2, s)
