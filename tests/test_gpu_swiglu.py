"""GPU parity of the gated-activation producer (silu(gate) * up in front of the online
rotation, Sec. 4.3) through the C ABI against the CPU oracle: the activation itself bit for
bit in fp32 and bf16, and the fused producer + rotation + MXFP4 call bit for bit in codes and
scales, in both operand layouts, with gate and up as separate matrices or as two halves of one
buffer."""
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


def finite_bf16(bits):
    bits = bits.copy()
    bits[(bits & 0x7F80) == 0x7F80] ^= 0x4000      # Inf/NaN -> some finite value
    return bits


def make_gu(M, K, seed, dtype):
    """gate ~ heavy-tailed around 0 with a few outlier channels (what gate_proj emits), up ~ N(0, 1.5)."""
    rng = np.random.default_rng(seed)
    g = (rng.standard_t(4, size=(M, K)) * 1.5).astype(np.float32)
    g[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 8.0
    u = (rng.standard_normal((M, K)) * 1.5).astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(g), f32_to_bf16_bits(u)
    return g, u


def same_bits(a, b):
    return np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a, b.view(np.uint32) if b.dtype == np.float32 else b)


# ------------------------------------------------------------------ the activation alone

def test_swiglu_every_bf16_gate(brq, orc):
    # every finite bf16 pattern as gate (zeros, subnormals, both signs, the clamps at +-86, the
    # largest values), against a handful of up values: fp32 results must agree in every bit
    bits = finite_bf16(np.arange(1 << 16, dtype=np.uint16)).reshape(64, 1024)
    for uv in (1.0, -0.5, 3.140625, 1.0e-3, 0.0):
        up = np.full(bits.shape, f32_to_bf16_bits(np.float32([uv]))[0], dtype=np.uint16)
        if uv == 3.140625:   # keep the product finite for the largest gates
            up[(bits & 0x7F80) > 0x7E00] = 0x3F80
        want = orc.swiglu(bits, up)
        got = to_host(brq.swiglu(to_dev(bits), to_dev(up)))
        bad = want.view(np.uint32) != got.view(np.uint32)
        assert not bad.any(), "u=%g: %d of %d differ, first at gate bits %#x" % (
            uv, int(bad.sum()), bad.size, int(bits[bad][0]))
        want_b = orc.swiglu(bits, up, out_bf16=True)
        got_b = to_host(brq.swiglu(to_dev(bits), to_dev(up), out_dtype=torch.bfloat16))
        assert np.array_equal(want_b, got_b)


def test_swiglu_fp32_inputs_dense_sweep(brq, orc):
    # fp32 gates: a dense sweep of the interesting range plus values whose z = g log2(e) lands on
    # or next to a half integer (the tie rule of n), and random up
    rng = np.random.default_rng(201)
    g = np.concatenate([np.linspace(-90, 90, 1 << 20), rng.standard_normal(1 << 20) * 3]).astype(np.float32)
    half = (np.arange(-60, 60, dtype=np.float64) + 0.5) / -1.4426950216293335
    for d in (-2, -1, 0, 1, 2):
        h32 = half.astype(np.float32)
        for _ in range(abs(d)):
            h32 = np.nextafter(h32, np.float32(np.sign(d) * 1e9))
        g[rng.choice(g.size, size=h32.size, replace=False)] = h32
    g = g.reshape(2048, 1024)
    u = (rng.standard_normal(g.shape) * 2).astype(np.float32)
    want = orc.swiglu(g, u)
    got = to_host(brq.swiglu(to_dev(g), to_dev(u)))
    bad = want.view(np.uint32) != got.view(np.uint32)
    assert not bad.any(), "%d differ; first g=%r u=%r want=%r got=%r" % (
        int(bad.sum()), g[bad][0], u[bad][0], want[bad][0], got[bad][0])


def test_swiglu_strided_and_ragged(brq, orc):
    # gate and up as the halves of one [M, 2K] buffer, output into a wider buffer; M and K ragged
    M, K = 37, 416
    g, u = make_gu(M, 2 * K, 202, "bf16")
    buf = to_dev(g)                                  # [M, 2K]
    gate, up = buf[:, :K], buf[:, K:]
    out = torch.zeros((M, K + 64), dtype=torch.float32, device="cuda")
    brq.swiglu(gate, up, out=out[:, :K])
    want = orc.swiglu(g[:, :K], g[:, K:])
    got = to_host(out)
    assert same_bits(np.ascontiguousarray(got[:, :K]), want)
    assert not got[:, K:].any()                      # nothing written past the row


# ------------------------------------------------------------------ fused with rotation + quantizer

def run_fused(brq, orc, g, u, B, h_bf16, layout, signs=None, views=None):
    M, K = g.shape
    gd, ud = (to_dev(g), to_dev(u)) if views is None else views
    sg = None if signs is None else torch.from_numpy(signs).cuda()
    c, s = brq.swiglu_rotate_quantize_fused(gd, ud, B, h_dtype=torch.bfloat16 if h_bf16 else torch.float32,
                                            layout=layout, signs=sg)
    if layout == "tiled":
        c, s = brq.to_rowmajor(c, s, M, K)
    rc, rs = orc.swiglu_rotate_quantize_fused(g, u, B, h_bf16=h_bf16, signs=signs)
    c, s = to_host(c), to_host(s)
    assert np.array_equal(s, rs), "scales differ in %d places" % int((s != rs).sum())
    assert np.array_equal(c, rc), "codes differ in %d bytes" % int((c != rc).sum())


@pytest.mark.parametrize("layout", ["rowmajor", "tiled"])
@pytest.mark.parametrize("M,K,B,dtype,h_bf16", [
    (64, 512, 32, "bf16", True), (64, 512, 32, "bf16", False), (301, 1024, 32, "bf16", True),
    (130, 544, 32, "bf16", True),      # K not a multiple of 128: the general row-wise kernel
    (67, 256, 1, "bf16", True),        # no rotation: quantizer alone
    (40, 384, 8, "bf16", False), (40, 384, 16, "f32", True), (96, 1024, 64, "bf16", True),
    (33, 1024, 128, "f32", False), (50, 1024, 256, "bf16", True), (20, 1024, 512, "bf16", False),
    (9, 2048, 1024, "bf16", True),     # rotation through LDS
    (5, 8192, 8192, "bf16", False),    # full-row rotation
])
def test_fused_matches_oracle(brq, orc, M, K, B, dtype, h_bf16, layout):
    g, u = make_gu(M, K, 300 + M + K + B, dtype)
    run_fused(brq, orc, g, u, B, h_bf16, layout)


@pytest.mark.parametrize("layout", ["rowmajor", "tiled"])
def test_fused_with_signs_and_shared_buffer(brq, orc, layout):
    # randomized rotation; gate and up are the two halves of one gate_up buffer (pitch 2K)
    M, K = 150, 1024
    g, _ = make_gu(M, 2 * K, 310, "bf16")
    rng = np.random.default_rng(311)
    signs = rng.choice([-1, 1], size=K).astype(np.int8)
    buf = to_dev(g)
    for B in (32, 128, 512):
        run_fused(brq, orc, np.ascontiguousarray(g[:, :K]), np.ascontiguousarray(g[:, K:]), B, True, layout,
                  signs=signs, views=(buf[:, :K], buf[:, K:]))


def test_fused_equals_unfused_two_kernel_path(brq):
    # the fused call against the library's own two-step path (activation stored as bf16, then the
    # online step reads it): identical codes and scales, which is what hdt = bf16 promises
    M, K = 512, 2048
    g, u = make_gu(M, K, 320, "bf16")
    gd, ud = to_dev(g), to_dev(u)
    h = brq.swiglu(gd, ud, out_dtype=torch.bfloat16)
    for layout in ("rowmajor", "tiled"):
        c0, s0 = brq.rotate_quantize_fused(h, 32, layout=layout)
        c1, s1 = brq.swiglu_rotate_quantize_fused(gd, ud, 32, h_dtype=torch.bfloat16, layout=layout)
        if layout == "tiled":     # compare the defined bytes only
            c0, s0 = brq.to_rowmajor(c0, s0, M, K)
            c1, s1 = brq.to_rowmajor(c1, s1, M, K)
        assert torch.equal(c0, c1) and torch.equal(s0, s1)


def test_fused_full_size_sampled_rows(brq, orc):
    # the down_proj input of the 8B MLP (intermediate size 14336) at 8192 tokens, in the launch
    # configuration the benchmark times; the oracle checks a sample of rows, the rest through the
    # unfused path's bit identity
    M, K = 8192, 14336
    rng = np.random.default_rng(330)
    gd = (torch.randn((M, 2 * K), device="cuda", generator=torch.Generator(device="cuda").manual_seed(330)) * 1.5
          ).to(torch.bfloat16)
    gate, up = gd[:, :K], gd[:, K:]
    c, s = brq.swiglu_rotate_quantize_fused(gate, up, 32, h_dtype=torch.bfloat16, layout="tiled")
    c, s = brq.to_rowmajor(c, s, M, K)
    rows = np.sort(rng.choice(M, size=24, replace=False))
    rows[0], rows[-1] = 0, M - 1
    idx = torch.from_numpy(rows).cuda()
    gs, us = to_host(gate[idx].contiguous()), to_host(up[idx].contiguous())
    rc, rs = orc.swiglu_rotate_quantize_fused(gs, us, 32, h_bf16=True)
    assert np.array_equal(to_host(s[idx]), rs) and np.array_equal(to_host(c[idx]), rc)
    h = brq.swiglu(gate, up, out_dtype=torch.bfloat16)
    c0, s0 = brq.rotate_quantize_fused(h, 32, layout="tiled")
    c0, s0 = brq.to_rowmajor(c0, s0, M, K)
    assert torch.equal(c0, c) and torch.equal(s0, s)


def test_argument_errors(brq):
    g = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(brq.BrqError) as e:
        brq.swiglu_rotate_quantize_fused(g, g, 24)                   # not a power of two
    assert e.value.status == 3
    sg = torch.ones(64, dtype=torch.int8, device="cuda")
    with pytest.raises(brq.BrqError) as e:
        brq.swiglu_rotate_quantize_fused(g, g, 1, signs=sg)          # signs without a rotation
    assert e.value.status == 3
    with pytest.raises(ValueError):
        brq.swiglu_rotate_quantize_fused(g, g[:, :32], 32)
    c, s = brq.swiglu_rotate_quantize_fused(g[:0], g[:0], 32)        # empty input: nothing launched
    assert c.numel() == 0 and s.numel() == 0
