"""GPU tests of the tiled operand layout.

The layout is bookkeeping, not arithmetic: a tiled output must hold exactly the bytes of the
row-major output (which the other GPU tests compare with the oracle) at the addresses that
include/brq.h states, and the product must not depend on the layout of its operands.  The
address formulas are written out here in numpy, independently of the kernels.
"""
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


def tiled_indices(rows, K, Kcover=None):
    """Byte index in the tiled buffers of every (row, code byte) and (row, group) of the first
    Kcover (default K) elements of a row."""
    Kp = (K + 511) // 512 * 512
    Kcover = K if Kcover is None else Kcover
    m = np.arange(rows, dtype=np.int64)[:, None]
    j = np.arange(Kcover // 2, dtype=np.int64)[None, :]
    g = np.arange(Kcover // 32, dtype=np.int64)[None, :]
    ci = ((m // 64) * (Kp // 128) + j // 64) * 4096 + (m % 64) * 64 + j % 64
    si = ((m // 64) * (Kp // 512) + g // 16) * 1024 + (m % 64) * 16 + g % 16
    return ci, si


def to_tiled(codes, scales, fill=0xEE):
    rows, K = codes.shape[0], codes.shape[1] * 2
    Kp = (K + 511) // 512 * 512
    R = (rows + 63) // 64 * 64
    ci, si = tiled_indices(rows, K)
    ct = np.full(R * Kp // 2, fill, dtype=np.uint8)
    st = np.full(R * Kp // 32, fill, dtype=np.uint8)
    cp, sp = tiled_indices(rows, K, Kcover=Kp)        # K padding of the real rows: zeros
    ct[cp] = 0
    st[sp] = 0
    ct[ci] = codes
    st[si] = scales
    return ct, st


def make_x(M, K, seed, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(4, size=(M, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    if dtype == "bf16":
        from paper_2511_04214_amd.inputs import f32_to_bf16_bits
        return f32_to_bf16_bits(x)
    return x


@pytest.mark.parametrize("M,K,B,dtype", [(16, 256, 32, "f32"), (100, 544, 32, "bf16"), (300, 1024, 64, "bf16"),
                                         (65, 96, 32, "f32"), (2048, 2048, 32, "bf16"), (130, 2048, 1024, "bf16"),
                                         (64, 512, 512, "bf16"), (1, 32, 32, "f32"), (66, 384, 128, "bf16"),
                                         (7, 128, 32, "f32"), (1027, 4096, 32, "bf16")])
def test_fused_tiled_holds_the_rowmajor_bytes(brq, M, K, B, dtype):
    x = to_dev(make_x(M, K, 11, dtype))
    c0, s0 = brq.rotate_quantize_fused(x, B)
    cb, sb = brq.operand_bytes(M, K, "tiled")
    ct = torch.full((cb,), 0xEE, dtype=torch.uint8, device="cuda")
    st = torch.full((sb,), 0xEE, dtype=torch.uint8, device="cuda")
    brq.rotate_quantize_fused(x, B, codes=ct, scales=st, layout="tiled")
    want_c, want_s = to_tiled(to_host(c0), to_host(s0))
    assert np.array_equal(to_host(ct), want_c), "codes: wrong bytes, K padding not zero or row padding touched"
    assert np.array_equal(to_host(st), want_s), "scales: wrong bytes, K padding not zero or row padding touched"
    c1, s1 = brq.to_rowmajor(ct, st, M, K)
    assert torch.equal(c1, c0) and torch.equal(s1, s0)


@pytest.mark.parametrize("M,K", [(48, 128), (257, 1536)])
def test_quantize_tiled(brq, M, K):
    x = to_dev(make_x(M, K, 12, "bf16"))
    c0, s0 = brq.mxfp4_quantize(x)
    ct, st = brq.mxfp4_quantize(x, layout="tiled")
    c1, s1 = brq.to_rowmajor(ct, st, M, K)
    assert torch.equal(c1, c0) and torch.equal(s1, s0)


def test_fused_tiled_against_the_oracle(brq, orc):
    M, K = 70, 1024
    xh = make_x(M, K, 13, "bf16")
    ct, st = brq.rotate_quantize_fused(to_dev(xh), 32, layout="tiled")
    oc, os_ = orc.rotate_quantize_fused(xh, 32)
    ci, si = tiled_indices(M, K)
    assert np.array_equal(to_host(ct)[ci], oc)
    assert np.array_equal(to_host(st)[si], os_)


# tiled persistent kernel, general 32x32-tile kernel, M <= 128 and M <= 16 kernels
@pytest.mark.parametrize("M,N,K", [(512, 768, 2048), (256, 256, 512), (100, 200, 544), (300, 64, 1024),
                                   (8, 300, 1024), (16, 48, 96), (300, 256, 1024), (65, 512, 512), (700, 256, 512),
                                   (300, 256, 544), (512, 512, 1152), (64, 256, 96)])
def test_product_does_not_depend_on_the_layout(brq, M, N, K):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(M, K, seed=21)
    wq, ws = inputs.random_mxfp4(N, K, seed=22)
    at = [to_dev(t) for t in to_tiled(aq, as_)]
    wt = [to_dev(t) for t in to_tiled(wq, ws)]
    ar = [to_dev(aq), to_dev(as_)]
    wr = [to_dev(wq), to_dev(ws)]
    for dt in (torch.float32, torch.bfloat16):
        y0 = brq.mxfp4_gemm(ar[0], ar[1], wr[0], wr[1], out_dtype=dt)
        y1 = brq.mxfp4_gemm(at[0], at[1], wt[0], wt[1], out_dtype=dt, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)
        y2 = brq.mxfp4_gemm(at[0], at[1], wr[0], wr[1], out_dtype=dt, a_layout="tiled", M=M, K=K)
        y3 = brq.mxfp4_gemm(ar[0], ar[1], wt[0], wt[1], out_dtype=dt, w_layout="tiled", N=N, K=K)
        assert torch.equal(y0, y2) and torch.equal(y0, y3)
        if K % 512 == 0 or (M > 128 and N % 256 != 0):
            assert torch.equal(y0, y1)
        elif dt == torch.float32:
            # two tiled operands with K % 512 != 0 run on the persistent or the small-batch kernel
            # (over the zero K padding), the mixed cases on the general one: same sum, another order
            d = (y1.double() - y0.double()).norm() / y0.double().norm()
            assert d < 1e-5, float(d)


def test_end_to_end_tiled_against_the_oracle(brq, orc):
    """Fused rotate+quantize of X and W straight into the tiled layout, then the product."""
    M, N, K = 256, 512, 1024
    xh, wh = make_x(M, K, 31, "bf16"), make_x(N, K, 32, "bf16")
    act, ast = brq.rotate_quantize_fused(to_dev(xh), 32, layout="tiled")
    wct, wst = brq.rotate_quantize_fused(to_dev(wh), 32, layout="tiled")
    y = to_host(brq.mxfp4_gemm(act, ast, wct, wst, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)).astype(np.float64)
    oa, oas = orc.rotate_quantize_fused(xh, 32)
    ow, ows = orc.rotate_quantize_fused(wh, 32)
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
    assert (np.abs(y - ref) <= 1e-5 * bound + 2.0 ** -126).all()


def test_tiled_product_with_k_not_a_multiple_of_512(brq, orc):
    """K = 1408 (11 stages of 128, e.g. the shape class of an 11008-wide down projection): tiled
    operands are zero-padded to 1536 by the quantizer and the persistent kernel runs over the
    padding; against the oracle on the oracle's own quantization."""
    M, N, K = 300, 512, 1408
    xh, wh = make_x(M, K, 51, "bf16"), make_x(N, K, 52, "bf16")
    act, ast = brq.rotate_quantize_fused(to_dev(xh), 32, layout="tiled")
    wct, wst = brq.rotate_quantize_fused(to_dev(wh), 32, layout="tiled")
    y = to_host(brq.mxfp4_gemm(act, ast, wct, wst, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)).astype(np.float64)
    oa, oas = orc.rotate_quantize_fused(xh, 32)
    ow, ows = orc.rotate_quantize_fused(wh, 32)
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
    assert (np.abs(y - ref) <= 1e-5 * bound + 2.0 ** -126).all()
    # the same buffers through the general kernel (row-major A forces it) agree to the tolerance
    ar, asr = brq.to_rowmajor(act, ast, M, K)
    y2 = to_host(brq.mxfp4_gemm(ar, asr, wct, wst, w_layout="tiled", N=N, K=K)).astype(np.float64)
    assert (np.abs(y2 - ref) <= 1e-5 * bound + 2.0 ** -126).all()


def test_binding_checks_tiled_buffers(brq):
    x = torch.zeros((64, 512), dtype=torch.bfloat16, device="cuda")
    small = torch.empty((100,), dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        brq.rotate_quantize_fused(x, 32, codes=small, layout="tiled")
    ct, st = brq.rotate_quantize_fused(x, 32, layout="tiled")
    with pytest.raises(ValueError):
        brq.mxfp4_gemm(ct, st, ct, st, a_layout="tiled", w_layout="tiled")      # no shape given
    with pytest.raises(ValueError):
        brq.mxfp4_gemm(ct, st, ct, st, a_layout="tiled", w_layout="tiled", M=128, N=64, K=512)   # too small


# ------------------------------------------------------------------ full-size workloads, as bench.py runs them

@pytest.mark.parametrize("name", ["mlp8b", "decode"])
def test_fused_tiled_full_size_against_the_oracle(brq, orc, name):
    """The benchmark's launch (tiled output) at the benchmark's sizes: every code and every scale
    byte against the oracle, through the address formulas above."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS[name]
    x = inputs.make_x(cfg)
    M, K = x.shape
    ct, st = brq.rotate_quantize_fused(to_dev(x), 32, layout="tiled")
    oc, os_ = orc.rotate_quantize_fused(x, 32)
    ci, si = tiled_indices(M, K)
    assert np.array_equal(to_host(ct)[ci], oc)
    assert np.array_equal(to_host(st)[si], os_)


@pytest.mark.parametrize("name,B", [("mlp8b", 32), ("down_sweep", 32), ("down_sweep", 64), ("down_sweep", 128),
                                    ("down_sweep", 8192), ("llama1b_up", 32)])
def test_product_tiled_full_size_sampled_rows(brq, orc, name, B):
    """bench.py's step on its own inputs (tiled operands, bf16 and fp32 out), for the down-projection shape
    at every rotation block of its sweep (Sec. 5.2; B = K is the global rotation); the oracle computes a
    sample of full output rows from its own rotation and quantization of the same inputs: the first and
    last row of every 128-row band (every row of output tiles), and random ones."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS[name]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    x, w = inputs.make_x(cfg), inputs.make_w(cfg)
    act, ast = brq.rotate_quantize_fused(to_dev(x), B, layout="tiled")
    wct, wst = brq.rotate_quantize_fused(to_dev(w), B, layout="tiled")
    y32 = brq.mxfp4_gemm(act, ast, wct, wst, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)
    y16 = brq.mxfp4_gemm(act, ast, wct, wst, out_dtype=torch.bfloat16, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)
    rng = np.random.default_rng(78)
    rows = sorted(set([r for t in range(0, M, 128) for r in (t, t + 127)] + [63, 64] + rng.integers(0, M, 6).tolist()))
    oa, oas = orc.rotate_quantize_fused(x[rows], B)
    ow, ows = orc.rotate_quantize_fused(w, B)
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
    got = to_host(y32).astype(np.float64)[rows]
    assert (np.abs(got - ref) <= 1e-5 * bound + 2.0 ** -126).all()
    assert np.linalg.norm(got - ref) <= 1e-5 * np.linalg.norm(ref)
    # bf16 output = round-to-nearest-even of the fp32 output, everywhere
    u = to_host(y32).view(np.uint32)
    rne = ((u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)).astype(np.uint16)
    assert np.array_equal(to_host(y16), rne)
    # the rotation leaves the product invariant before quantization (Sec. 2), so the quantized product stays
    # near X W^T whatever B is (loose sanity bound on the sampled rows)
    exact = orc.bf16_to_f32(x[rows]).astype(np.float64) @ orc.bf16_to_f32(w).astype(np.float64).T
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.35


@pytest.mark.parametrize("M", [1, 16, 24, 64, 128])
def test_product_decode_tiled_full_size(brq, orc, M):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["decode"]
    N, K = cfg["N"], cfg["K"]
    x = inputs.make_x(cfg, M=max(16, M))[:M]
    w = inputs.make_w(cfg)
    act, ast = brq.rotate_quantize_fused(to_dev(x), 32, layout="tiled")
    wct, wst = brq.rotate_quantize_fused(to_dev(w), 32, layout="tiled")
    y = to_host(brq.mxfp4_gemm(act, ast, wct, wst, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)).astype(np.float64)
    oa, oas = orc.rotate_quantize_fused(x, 32)
    ow, ows = orc.rotate_quantize_fused(w, 32)
    rows = None if M <= 16 else sorted({0, 15, 16, M - 1, M // 2, M // 3})    # the oracle takes seconds per row
    ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows, rows=rows)
    got = y if rows is None else y[rows]
    assert (np.abs(got - ref) <= 1e-5 * bound + 2.0 ** -126).all()


def test_calls_run_on_the_given_stream(brq, orc):
    """Work goes to the caller's stream: results are complete after synchronising that stream
    alone, and two streams can run the path side by side on their own buffers."""
    rng = np.random.default_rng(61)
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    M, N, K = 256, 512, 1024
    xs = [f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)) for _ in range(2)]
    w = f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
    wct, wst = brq.rotate_quantize_fused(to_dev(w), 32, layout="tiled")
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    xd = [to_dev(x) for x in xs]
    torch.cuda.synchronize()
    outs = []
    for x, st in zip(xd, streams):
        c, s_ = brq.rotate_quantize_fused(x, 32, layout="tiled", stream=st)
        outs.append(brq.mxfp4_gemm(c, s_, wct, wst, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K, stream=st))
    ow, ows = orc.rotate_quantize_fused(w, 32)
    for x, st, y in zip(xs, streams, outs):
        st.synchronize()
        oa, oas = orc.rotate_quantize_fused(x, 32)
        ref, bound = orc.mxfp4_gemm(oa, oas, ow, ows)
        assert (np.abs(to_host(y).astype(np.float64) - ref) <= 1e-5 * bound + 2.0 ** -126).all()


def test_empty_operands_in_the_tiled_layout(brq):
    x = torch.zeros((0, 512), dtype=torch.bfloat16, device="cuda")
    c, s_ = brq.rotate_quantize_fused(x, 32, layout="tiled")
    assert c.numel() == 0 and s_.numel() == 0
    w = torch.zeros((256, 512), dtype=torch.bfloat16, device="cuda")
    wc, ws = brq.rotate_quantize_fused(w, 32, layout="tiled")
    y = brq.mxfp4_gemm(c, s_, wc, ws, a_layout="tiled", w_layout="tiled", M=0, N=256, K=512)
    assert tuple(y.shape) == (0, 256)


def test_step_in_a_hip_graph(brq):
    """The two-kernel step (fused rotate+quantize, product) captured in a HIP graph: every replay
    gives the eager result, with eager launches and synchronisations between the replays."""
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(71)
    for M, N, K in ((16, 1024, 2048), (300, 512, 1024)):
        w = to_dev(f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.05).astype(np.float32)))
        wct, wst = brq.rotate_quantize_fused(w, 32, layout="tiled")
        xs = [to_dev(f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))) for _ in range(3)]
        x = xs[0].clone()
        cb, sb = brq.operand_bytes(M, K, "tiled")
        c = torch.empty((cb,), dtype=torch.uint8, device="cuda")
        s_ = torch.empty((sb,), dtype=torch.uint8, device="cuda")
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        st = torch.cuda.Stream()

        def step():
            brq.rotate_quantize_fused(x, 32, codes=c, scales=s_, layout="tiled", stream=st)
            brq.mxfp4_gemm(c, s_, wct, wst, out=y, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K, stream=st)

        eager = []
        for xi in xs:                      # eager results for three different inputs (also warms the library up)
            x.copy_(xi)
            torch.cuda.synchronize()
            step()
            st.synchronize()
            eager.append(y.clone())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            step()
        for rep in range(2):
            for xi, want in zip(xs, eager):
                x.copy_(xi)
                y.zero_()
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                assert torch.equal(y, want), (M, rep)
                step()                     # eager work between the replays
                st.synchronize()
                assert torch.equal(y, want)


def test_other_entry_points_in_a_hip_graph(brq):
    """The producer-fused step, the rotation by caller-supplied blocks (LDS-DMA loads, LDS-staged
    stores), the small-batch product and the block statistics (atomics on caller-zeroed counters)
    captured together in one HIP graph: every replay gives the eager result."""
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits
    rng = np.random.default_rng(72)
    M, N, K = 40, 640, 1024
    w = to_dev(f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.05).astype(np.float32)))
    wct, wst = brq.rotate_quantize_fused(w, 32, layout="tiled")
    R = to_dev(np.stack([np.linalg.qr(rng.standard_normal((32, 32)))[0] for _ in range(K // 32)]).astype(np.float32))
    gus = [to_dev(f32_to_bf16_bits(rng.standard_normal((M, 2 * K)).astype(np.float32))) for _ in range(3)]
    gu = gus[0].clone()
    cb, sb = brq.operand_bytes(M, K, "tiled")
    c1, c2 = (torch.empty((cb,), dtype=torch.uint8, device="cuda") for _ in range(2))
    s1, s2 = (torch.empty((sb,), dtype=torch.uint8, device="cuda") for _ in range(2))
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    amax = torch.empty((M, K // 32), dtype=torch.float32, device="cuda")
    sqerr = torch.empty((M, K // 32), dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()

    def step():
        brq.swiglu_rotate_quantize_fused(gu[:, :K], gu[:, K:], 32, h_dtype=torch.bfloat16, codes=c1, scales=s1,
                                         layout="tiled", stream=st)
        brq.mxfp4_gemm(c1, s1, wct, wst, out=y, a_layout="tiled", w_layout="tiled", M=M, N=N, K=K, stream=st)
        brq.matrix_rotate_quantize_fused(gu[:, :K], R, codes=c2, scales=s2, layout="tiled", stream=st)
        with torch.cuda.stream(st):
            counts.zero_()                 # a fill kernel, not a memset node
        brq.block_stats(gu[:, K:], 32, (0.5, 2.0), counts=counts, amax=amax, sqerr=sqerr, stream=st)

    def snapshot():
        return [t.clone() for t in (y, c2, s2, counts, amax, sqerr)]

    eager = []
    for g_ in gus:
        gu.copy_(g_)
        torch.cuda.synchronize()
        step()
        st.synchronize()
        eager.append(snapshot())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        step()
    for rep in range(2):
        for g_, want in zip(gus, eager):
            gu.copy_(g_)
            y.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, w_ in zip(snapshot(), want):
                assert torch.equal(got, w_), rep
            step()                         # eager work between the replays
            st.synchronize()
