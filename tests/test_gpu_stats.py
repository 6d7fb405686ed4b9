"""GPU parity of the block statistics (block-wise scale, share of data above a threshold,
per-block MXFP4 loss; Sec. 4.1, 4.2, Appendix "Rotation Comparison") through the C ABI against the
CPU oracle: scales and counts bit for bit, the loss (an fp32 sum of 32 squares against the oracle's
fp64 sum) within 4e-6 relative."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host
from paper_2511_04214_amd.inputs import f32_to_bf16_bits

pytestmark = pytest.mark.gpu

TH = [0.25, 1.5, 3.0, 20.0, 1.0e30]


@pytest.fixture(scope="module")
def brq():
    import paper_2511_04214_amd as b
    b.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return b


def make_x(M, K, seed, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(4, size=(M, K)).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    x[rng.integers(0, M), :32] = 0.0                      # an all-zero block
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def check(brq, orc, x, B, signs=None, xd=None):
    xd = to_dev(x) if xd is None else xd
    sg = None if signs is None else torch.from_numpy(signs).cuda()
    amax, counts, sqerr, bfp4 = brq.block_stats(xd, B, TH, signs=sg, want_bfp4=True)
    ra, rc, rs, rb = orc.block_stats(x, B, TH, signs=signs, want_bfp4=True)
    assert np.array_equal(to_host(amax).view(np.uint32), ra.view(np.uint32)), "block scales differ"
    assert np.array_equal(to_host(counts).astype(np.uint64), rc), (to_host(counts), rc)
    got = to_host(sqerr).astype(np.float64)
    assert (np.abs(got - rs) <= 4e-6 * rs + 1e-44).all(), "loss off by up to %.3g relative" % float(
        (np.abs(got - rs) / (rs + 1e-300)).max())
    got = to_host(bfp4).astype(np.float64)     # FP16-scale counterpart: same codes (fp32 decisions), fp32 sum
    assert (np.abs(got - rb) <= 4e-6 * rb + 1e-44).all(), "FP16-scale loss off by up to %.3g relative" % float(
        (np.abs(got - rb) / (rb + 1e-300)).max())


@pytest.mark.parametrize("M,K,B,dtype", [(64, 512, 1, "bf16"), (64, 512, 32, "bf16"), (257, 544, 32, "bf16"),
                                         (33, 256, 8, "f32"), (100, 1024, 128, "bf16"), (40, 1024, 512, "f32"),
                                         (19, 2048, 1024, "bf16"), (7, 8192, 8192, "bf16"), (301, 96, 1, "f32")])
def test_stats_match_oracle(brq, orc, M, K, B, dtype):
    check(brq, orc, make_x(M, K, 600 + M + K + B, dtype), B)


def test_fp16_scale_loss_at_the_ends_of_half_precision(brq, orc):
    # blocks whose FP16 scale is a subnormal half, rounds to zero, or saturates at 65504, next to
    # ordinary ones; and quotients on the encoder's rounding boundaries (scale exactly 1, 0.5, 1.25)
    rng = np.random.default_rng(640)
    M, K = 48, 256
    x = rng.standard_normal((M, K)).astype(np.float32)
    mags = [1.0e-4, 3.0e-6, 2.0e-7, 1.0e-7, 1.0e-9, 3.9e5, 4.0e5, 1.0e7, 1.0e12]   # fp32 squares stay finite
    for i, m in enumerate(mags):
        x[i] *= np.float32(m) / 3
    grid = np.array([0.0, 0.25, 0.5, 0.75, 1.0, 1.25, 1.5, 1.75, 2.0, 2.5, 3.0, 3.5, 4.0, 5.0, 6.0], dtype=np.float32)
    for i, smax in enumerate((6.0, 3.0, 7.5)):
        row = rng.choice(grid, size=K) * np.float32(smax / 6.0) * rng.choice([-1, 1], size=K)
        row[::32] = smax                                   # every block's maximum
        x[len(mags) + i] = row.astype(np.float32)
    check(brq, orc, x, 1)
    _, _, sq, sqb = brq.block_stats(to_dev(x), 1, (), want_bfp4=True)
    assert torch.isfinite(sqb).all() and torch.isfinite(sq).all()


def test_fp16_scale_loss_optional_and_given_output(brq, orc):
    x = make_x(40, 512, 641, "bf16")
    xd = to_dev(x)
    out = torch.full((40, 16), -1.0, dtype=torch.float32, device="cuda")
    r = brq.block_stats(xd, 32, (), sqerr_bfp4=out, want_amax=False, want_sqerr=False)
    assert len(r) == 4 and r[0] is None and r[2] is None and r[3] is out
    rb = orc.block_stats(x, 32, (), want_bfp4=True)[3]
    assert (np.abs(to_host(out).astype(np.float64) - rb) <= 4e-6 * rb + 1e-44).all()
    assert len(brq.block_stats(xd, 32, ())) == 3


def test_stats_signed_and_strided(brq, orc):
    M, K = 90, 1024
    wide = make_x(M, K + 256, 610, "bf16")
    rng = np.random.default_rng(611)
    signs = rng.choice([-1, 1], size=K).astype(np.int8)
    xd = to_dev(wide)[:, 128:128 + K]
    x = np.ascontiguousarray(wide[:, 128:128 + K])
    for B in (32, 1024):
        check(brq, orc, x, B, signs=signs, xd=xd)


def test_counts_accumulate_and_optional_outputs(brq, orc):
    x1, x2 = make_x(50, 512, 620, "bf16"), make_x(70, 512, 621, "bf16")
    counts = torch.zeros(len(TH), dtype=torch.int64, device="cuda")
    a, c, s = brq.block_stats(to_dev(x1), 32, TH, counts=counts, want_amax=False, want_sqerr=False)
    assert a is None and s is None
    brq.block_stats(to_dev(x2), 32, TH, counts=counts, want_amax=False)
    want = orc.block_stats(x1, 32, TH)[1] + orc.block_stats(x2, 32, TH)[1]
    assert np.array_equal(to_host(counts).astype(np.uint64), want)
    # no thresholds: no counter is touched
    a, c, s = brq.block_stats(to_dev(x1), 32, ())
    assert c is None and np.array_equal(to_host(a), orc.block_stats(x1, 32, ())[0])


def test_full_size_sampled_rows(brq, orc):
    # X 16384 x 8192 after the block rotation and after the global one; counts against the GPU's own
    # rotation output (exact integers), scales and loss on sampled rows against the oracle
    M, K = 16384, 8192
    gen = torch.Generator(device="cuda").manual_seed(630)
    xd = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    xd[:, ::97] *= 20
    rng = np.random.default_rng(631)
    rows = np.sort(rng.choice(M, size=6, replace=False))
    idx = torch.from_numpy(rows).cuda()
    xs = to_host(xd[idx].contiguous())
    for B in (32, 8192):
        amax, counts, sqerr = brq.block_stats(xd, B, TH)
        ra, _, rs = orc.block_stats(xs, B, TH)
        assert np.array_equal(to_host(amax[idx]), ra)
        got = to_host(sqerr[idx]).astype(np.float64)
        assert (np.abs(got - rs) <= 4e-6 * rs + 1e-44).all()
        y = brq.block_rotate(xd, B)                       # bit-identical to the oracle's rotation (its own tests)
        want = [int((y.abs() > t).sum().item()) for t in TH]
        assert to_host(counts).tolist() == want


def test_argument_errors(brq):
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(brq.BrqError) as e:
        brq.block_stats(x, 24, TH)
    assert e.value.status == 3
    with pytest.raises(brq.BrqError) as e:
        brq.block_stats(x, 32, list(range(9)))            # more than 8 thresholds
    assert e.value.status == 2
    a, c, s = brq.block_stats(x[:0], 32, TH)
    assert a.numel() == 0 and int(c.sum().item()) == 0
