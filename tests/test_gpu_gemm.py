"""GPU parity of the MXFP4 product against the oracle's fp64 product of the dequantized
operands.

Tolerance (fp32 accumulation, stated bar 1e-5): for every output
    |y_gpu - y_ref| <= 1e-5 * sum_k |a_k w_k|  +  2^-126
and   ||y_gpu - y_ref||_F <= 1e-5 * ||y_ref||_F.
The first is the forward-error form of an fp32-accumulated dot product (relative to the
magnitude that was summed, so that cancellation does not make the test meaningless); the
2^-126 floor is the smallest normal fp32, below which an fp32 result cannot carry relative
accuracy.  bf16 output must equal the round-to-nearest-even of the fp32 output exactly.
"""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu

RTOL = 1e-5
FLOOR = 2.0 ** -126


@pytest.fixture(scope="module")
def brq():
    import paper_2511_04214_amd as b
    b.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return b


def bf16_rne(a):
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)).astype(np.uint16)


def check_gemm(brq, orc, aq, as_, wq, ws, rows=None, ldy=None):
    daq, das, dwq, dws = to_dev(aq), to_dev(as_), to_dev(wq), to_dev(ws)
    M, N = aq.shape[0], wq.shape[0]
    if ldy is None:
        y = brq.mxfp4_gemm(daq, das, dwq, dws)
    else:
        buf = torch.full((M, ldy), -7.0, dtype=torch.float32, device="cuda")
        y = brq.mxfp4_gemm(daq, das, dwq, dws, out=buf[:, :N])
        assert (buf[:, N:] == -7.0).all(), "wrote outside the N columns"
    y = to_host(y).astype(np.float64)
    ref, bound = orc.mxfp4_gemm(aq, as_, wq, ws, rows=rows)
    got = y if rows is None else y[np.asarray(rows)]
    err = np.abs(got - ref)
    assert (err <= RTOL * bound + FLOOR).all(), "max err/bound = %g" % float((err / (bound + FLOOR)).max())
    assert np.linalg.norm(got - ref) <= RTOL * np.linalg.norm(ref) + FLOOR
    yb = to_host(brq.mxfp4_gemm(daq, das, dwq, dws, out_dtype=torch.bfloat16))
    y32 = to_host(brq.mxfp4_gemm(daq, das, dwq, dws))
    assert np.array_equal(yb, bf16_rne(y32)), "bf16 output is not RNE of the fp32 output"
    return y32


@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (33, 70, 96), (128, 256, 512), (1, 16, 32), (100, 36, 2080),
                                   (256, 256, 1024), (300, 520, 768), (17, 1000, 256),
                                   (256, 256, 512), (512, 768, 2048), (768, 256, 1536), (2304, 512, 512),
                                   # ragged M in the persistent tiled kernel (N % 256 == 0, K % 512 == 0)
                                   (300, 256, 512), (257, 512, 1024), (17, 256, 512), (1000, 768, 2048),
                                   (255, 256, 512), (64, 256, 512), (513, 256, 512)])
def test_gemm_random_codes(brq, orc, M, N, K):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(M, K, seed=M * 7 + K)
    wq, ws = inputs.random_mxfp4(N, K, seed=N * 13 + K)
    check_gemm(brq, orc, aq, as_, wq, ws)


@pytest.mark.parametrize("M", [1, 2, 4, 7, 16])
@pytest.mark.parametrize("N,K", [(64, 128), (100, 1056), (2048, 8192)])
def test_gemm_skinny(brq, orc, M, N, K):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(M, K, seed=1000 + M)
    wq, ws = inputs.random_mxfp4(N, K, seed=2000 + N)
    check_gemm(brq, orc, aq, as_, wq, ws)


def test_gemm_padded_output_pitch(brq, orc):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(40, 256, seed=5)
    wq, ws = inputs.random_mxfp4(70, 256, seed=6)
    check_gemm(brq, orc, aq, as_, wq, ws, ldy=77)
    aq, as_ = inputs.random_mxfp4(4, 256, seed=7)
    check_gemm(brq, orc, aq, as_, wq, ws, ldy=96)


def test_gemm_exact_cases(brq):
    # all ones (code 2, byte 127): Y = K exactly; one scale byte +1 adds exactly 32
    for M, N, K in ((48, 80, 4096), (4, 32, 4096), (256, 256, 512)):
        q = lambda r: torch.full((r, K // 2), 0x22, dtype=torch.uint8, device="cuda")
        s = lambda r: torch.full((r, K // 32), 127, dtype=torch.uint8, device="cuda")
        y = brq.mxfp4_gemm(q(M), s(M), q(N), s(N))
        assert (y == K).all()
        sa = s(M)
        sa[M - 1, 5] = 128
        y = brq.mxfp4_gemm(q(M), sa, q(N), s(N))
        assert (y[:M - 1] == K).all() and (y[M - 1] == K + 32).all()
        # every code against itself: sum over a group of v*v
        codes = torch.arange(16, dtype=torch.uint8, device="cuda")
        row = (codes | (codes << 4)).repeat(K // 32)[: K // 2].contiguous()
        a = row.repeat(M, 1).contiguous()
        w = row.repeat(N, 1).contiguous()
        vals = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6], dtype=torch.float64)
        want = float((vals * vals).sum() * 4) * (K // 32)
        assert (brq.mxfp4_gemm(a, s(M), w, s(N)) == want).all()


def test_gemm_extreme_scales(brq, orc):
    # products that overflow the small end of fp32 must come out as (near) zero, large ones exact
    from paper_2511_04214_amd import inputs
    aq, _ = inputs.random_mxfp4(32, 128, seed=9)
    wq, _ = inputs.random_mxfp4(32, 128, seed=10)
    for sa, sw in ((0, 0), (0, 127), (127, 240), (150, 180), (60, 70)):
        as_ = np.full((32, 4), sa, dtype=np.uint8)
        ws = np.full((32, 4), sw, dtype=np.uint8)
        check_gemm(brq, orc, aq, as_, wq, ws)


def test_tiny_config_end_to_end(brq, orc):
    """Config 'tiny': rotate + quantize X and W on the GPU, multiply, compare with the oracle's
    product of the oracle's own quantization (codes are bit-identical, so operands agree)."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["tiny"]
    x, w = inputs.make_x(cfg), inputs.make_w(cfg)
    aq, as_ = brq.rotate_quantize_fused(to_dev(x), 32)
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32)
    raq, ras = orc.rotate_quantize_fused(x, 32)
    rwq, rws = orc.rotate_quantize_fused(w, 32)
    assert np.array_equal(to_host(aq), raq) and np.array_equal(to_host(wq), rwq)
    assert np.array_equal(to_host(as_), ras) and np.array_equal(to_host(ws), rws)
    y = check_gemm(brq, orc, raq, ras, rwq, rws)
    # and the quantized product approximates the unquantized one (sanity, loose)
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.linalg.norm(y - exact) / np.linalg.norm(exact) < 0.25


@pytest.mark.parametrize("name", ["llama1b_up", "down_sweep", "mlp8b"])
def test_gemm_full_size_sampled_rows(brq, orc, name):
    """Benchmark shapes in the benchmark's launch configuration; the oracle computes a sample of full
    output rows: the first and last row of every 128-row band (so of every row of output tiles, 256 or
    128 rows high, wherever the tile walk puts it), rows next to the 32-row MFMA tile edges, and random ones."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS[name]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    x, w = inputs.make_x(cfg), inputs.make_w(cfg)
    aq, as_ = brq.rotate_quantize_fused(to_dev(x), 32)
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32)
    rng = np.random.default_rng(77)
    rows = sorted(set([r for t in range(0, M, 128) for r in (t, t + 127)] + [1, 31, 32, M - 257] + rng.integers(0, M, 8).tolist()))
    check_gemm(brq, orc, to_host(aq), to_host(as_), to_host(wq), to_host(ws), rows=rows)


def test_gemm_half_tiles_several_per_workgroup(brq, orc):
    """4096 x 2560: 160 tiles of 256 x 256 would leave CUs idle, so the kernel runs 320 tiles of
    128 x 256 and some workgroups take two of them (ring running across a tile boundary); ragged
    variant: M = 4000."""
    from paper_2511_04214_amd import inputs
    for M in (4096, 4000):
        N, K = 2560, 1024
        aq, as_ = inputs.random_mxfp4(M, K, seed=41)
        wq, ws = inputs.random_mxfp4(N, K, seed=42)
        rng = np.random.default_rng(43)
        rows = sorted(set([0, 63, 64, 127, 128, 255, 256, M - 129, M - 128, M - 1] + rng.integers(0, M, 12).tolist()))
        check_gemm(brq, orc, aq, as_, wq, ws, rows=rows)


@pytest.mark.parametrize("K", [512, 1024, 1536])
def test_gemm_full_tiles_ragged_last_row(brq, orc, K):
    """4100 x 4096: 17 x 16 = 272 tiles of 256 x 256, enough for the full-height tile kernel, whose last
    tile row has 4 live rows: clamped A loads (row-major and tiled operands take different paths there)
    and masked stores.  Rows next to the ragged edge, of every tile row, and random ones.  Sixteen workgroups
    take two tiles: with K of one, two and three superstages the second tile's first stage (which carries
    the first tile's output) is also, precedes, or is two before the workgroup's last superstage."""
    from paper_2511_04214_amd import inputs
    from test_gpu_layout import to_tiled
    M, N = 4100, 4096
    aq, as_ = inputs.random_mxfp4(M, K, seed=45)
    wq, ws = inputs.random_mxfp4(N, K, seed=46)
    rng = np.random.default_rng(47)
    rows = sorted(set([r for t in range(0, 4096, 256) for r in (t, t + 255)] + [4096, 4097, 4098, 4099, 3840, 4095]
                      + rng.integers(0, M, 8).tolist()))
    y32 = check_gemm(brq, orc, aq, as_, wq, ws, rows=rows)
    # the same product on tiled operands (slab-clamped A loads): same kernel, same summation order
    at, wt = [to_dev(t) for t in to_tiled(aq, as_)], [to_dev(t) for t in to_tiled(wq, ws)]
    buf = torch.full((M + 3, N), -7.0, dtype=torch.float32, device="cuda")
    brq.mxfp4_gemm(at[0], at[1], wt[0], wt[1], out=buf[:M], a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)
    assert np.array_equal(to_host(buf[:M]), y32)
    assert (buf[M:] == -7.0).all(), "wrote below the last row"


# N not a multiple of 256 in the persistent tiled kernel: the last tile column clamps its W loads into the
# operand (row-major: per-lane rows; tiled: the slab index) and masks its stores by 16-byte chunk.  bf16
# output needs N % 8 == 0 and fp32 N % 4 == 0 (else the general kernel takes the call: N = 130 below).
@pytest.mark.parametrize("M,N,K", [(300, 264, 512), (257, 8, 1024), (200, 64, 512), (1000, 1160, 1024), (513, 520, 1536),
                                   (300, 260, 512), (129, 130, 512), (384, 248, 2048)])
def test_gemm_ragged_last_tile_column(brq, orc, M, N, K):
    from paper_2511_04214_amd import inputs
    from test_gpu_layout import to_tiled
    aq, as_ = inputs.random_mxfp4(M, K, seed=M * 5 + N)
    wq, ws = inputs.random_mxfp4(N, K, seed=N * 11 + K)
    y32 = check_gemm(brq, orc, aq, as_, wq, ws, ldy=N + 24)         # also: nothing written right of column N - 1
    at, wt = [to_dev(t) for t in to_tiled(aq, as_)], [to_dev(t) for t in to_tiled(wq, ws)]
    for dt in (torch.float32, torch.bfloat16):
        buf = torch.full((M + 2, N + 16), -7.0, dtype=dt, device="cuda")
        brq.mxfp4_gemm(at[0], at[1], wt[0], wt[1], out=buf[:M, :N], a_layout="tiled", w_layout="tiled", M=M, N=N, K=K)
        got = to_host(buf[:M, :N])
        assert np.array_equal(got, y32 if dt == torch.float32 else bf16_rne(y32))
        assert (buf[M:] == -7.0).all() and (buf[:, N:] == -7.0).all(), "wrote outside the M x N block"


def test_gemm_full_tiles_ragged_row_and_column(brq, orc):
    """4100 x 4104: 17 x 17 = 289 tiles of 256 x 256 (the full-height kernel), 4 live rows in the last tile row
    and 8 live columns in the last tile column; rows of every tile row, all columns."""
    from paper_2511_04214_amd import inputs
    M, N, K = 4100, 4104, 512
    aq, as_ = inputs.random_mxfp4(M, K, seed=48)
    wq, ws = inputs.random_mxfp4(N, K, seed=49)
    rng = np.random.default_rng(50)
    rows = sorted(set([r for t in range(0, 4096, 256) for r in (t, t + 255)] + [4096, 4099] + rng.integers(0, M, 6).tolist()))
    check_gemm(brq, orc, aq, as_, wq, ws, rows=rows, ldy=N + 8)


# 16 < M <= 128: the weight-streaming kernel that shares the activations through LDS (1 to 4 tiles of 32
# rows, ragged M inside the last tile, ragged N inside the last workgroup and wavefront; K of 1 to 7
# superstages, so that the main loop runs 0, 1 and 2 times with 0, 1 and 2 superstages left over);
# 129 rows take the neighbouring code path
@pytest.mark.parametrize("M,N,K", [(17, 1000, 512), (32, 256, 1024), (33, 320, 1536), (64, 4096, 2048), (50, 130, 512),
                                   (48, 64, 512), (20, 16, 3584), (63, 75, 1024), (65, 1000, 512), (128, 384, 2048),
                                   (100, 130, 1536), (96, 40, 1024), (17, 200, 1536), (33, 128, 2560), (97, 256, 3072),
                                   (128, 129, 512), (127, 128, 3584), (80, 257, 2560), (129, 256, 1024)])
def test_gemm_small_batches(brq, orc, M, N, K):
    from paper_2511_04214_amd import inputs
    aq, as_ = inputs.random_mxfp4(M, K, seed=51)
    wq, ws = inputs.random_mxfp4(N, K, seed=52)
    check_gemm(brq, orc, aq, as_, wq, ws)
    check_gemm(brq, orc, aq, as_, wq, ws, ldy=N + 12)


@pytest.mark.parametrize("M", [1, 4, 16])
def test_gemm_decode_full_size(brq, orc, M):
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["decode"]
    N, K = cfg["N"], cfg["K"]
    x = inputs.make_x(cfg, M=16)[:M]
    w = inputs.make_w(cfg)
    aq, as_ = brq.rotate_quantize_fused(to_dev(x), 32)
    wq, ws = brq.rotate_quantize_fused(to_dev(w), 32)
    check_gemm(brq, orc, to_host(aq), to_host(as_), to_host(wq), to_host(ws))


def test_measurement_loop_reports_its_clock(brq):
    # the MFMA-only loop: sink[0] shader-clock cycles, sink[1] 100 MHz ticks of workgroup 0's loop
    ops = torch.randint(0, 256, (8192,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros((8 * 256,), dtype=torch.float32, device="cuda")
    flops = brq.diag_mfma_ceiling(ops, 400, 8, sink=sink)
    torch.cuda.synchronize()
    cycles, ticks = sink[:2].tolist()
    assert flops == 8 * 4 * 400 * 16 * 131072
    assert cycles >= 400 * 16 * 32 and ticks > 0          # at least the MFMAs' own 32 cycles apiece
    assert 0.2 < 0.1 * cycles / ticks < 3.0               # GHz


def test_product_reports_its_clock(brq):
    # the large-shape kernel with the clock read-out: same product, plausible clock
    from paper_2511_04214_amd import inputs
    M, N, K = 512, 512, 2048
    aq, as_ = inputs.random_mxfp4(M, K, seed=71)
    wq, ws = inputs.random_mxfp4(N, K, seed=72)
    ops = [to_dev(t) for t in (aq, as_, wq, ws)]
    clk = torch.zeros(6, dtype=torch.int64, device="cuda")
    y0 = brq.mxfp4_gemm(*ops, out_dtype=torch.bfloat16)
    y1 = brq.mxfp4_gemm(*ops, out_dtype=torch.bfloat16, clock=clk)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    cycles, ticks, loop, epi, tiles, pro = clk.tolist()
    assert cycles >= 16 * 32 * 32 and ticks > 0           # at least the MFMAs of one tile's K loop
    assert 0.2 < 0.1 * cycles / ticks < 3.0               # GHz
    assert tiles >= 1 and loop >= tiles * 16 * 16 * 32 and epi > 0 and pro > 0 and loop + epi + pro <= cycles
    with pytest.raises(brq.BrqError) as e:                # a shape that another kernel takes
        brq.mxfp4_gemm(ops[0][:64], ops[1][:64], ops[2], ops[3], clock=clk)
    assert e.value.status == 2


def test_no_loads_variant_runs_and_leaves_the_product_alone(brq):
    """The measurement instantiation without refill loads: accepted only for bf16 output and >= 1024 tiles of
    256 x 256, reports a clock, runs in fewer cycles than the product, and a product launch after it is unchanged."""
    from paper_2511_04214_amd import inputs
    M, N, K = 8192, 8192, 1024
    aq, as_ = [to_dev(t) for t in inputs.random_mxfp4(M, K, seed=91)]
    wq, ws = [to_dev(t) for t in inputs.random_mxfp4(N, K, seed=92)]
    y0 = brq.mxfp4_gemm(aq, as_, wq, ws, out_dtype=torch.bfloat16)
    clk = torch.zeros(6, dtype=torch.int64, device="cuda")
    brq.diag_mxfp4_gemm_clock(aq, as_, wq, ws, clk, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    full = clk.tolist()
    scratch = torch.empty_like(y0)
    brq.diag_mxfp4_gemm_no_loads(aq, as_, wq, ws, clk, out=scratch)
    torch.cuda.synchronize()
    nl = clk.tolist()
    assert nl[4] == full[4] == 4 and 0 < nl[0] and 500 < 100.0 * nl[0] / nl[1] < 3000      # 4 tiles each; a plausible clock in MHz
    assert nl[2] < full[2] * 1.05, (nl, full)
    y1 = brq.mxfp4_gemm(aq, as_, wq, ws, out_dtype=torch.bfloat16)
    assert torch.equal(y0, y1)
    with pytest.raises(brq.BrqError) as err:
        brq.diag_mxfp4_gemm_no_loads(aq, as_, wq, ws, clk, out_dtype=torch.float32)         # fp32 output
    assert err.value.status == 2
    with pytest.raises(brq.BrqError) as err:
        brq.diag_mxfp4_gemm_no_loads(aq[:4096], as_[:4096], wq[:4096], ws[:4096], clk, out_dtype=torch.bfloat16)   # 256 tiles
    assert err.value.status == 2
