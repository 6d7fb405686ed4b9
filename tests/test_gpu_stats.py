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


# ------------------------------------------------------------------ the reductions of the paper's analysis

EDGES = [0.5, 1.0, 2.0, 4.0, 8.0, 16.0, 64.0]


def check_summary(brq, orc, amax, sqerr, ref, outlier, edges):
    d = lambda t: None if t is None else to_dev(t)
    hist, counts, sums = brq.block_stats_summary(d(amax), d(sqerr), d(ref), outlier_threshold=outlier, edges=edges)
    rh, rc, rs = orc.block_stats_summary(amax, sqerr, ref, outlier=outlier, edges=edges)
    assert np.array_equal(to_host(hist).astype(np.uint64), rh), (to_host(hist), rh)
    assert np.array_equal(to_host(counts).astype(np.uint64), rc), (to_host(counts), rc)
    assert np.allclose(to_host(sums), rs, rtol=1e-12, atol=0), (to_host(sums), rs)
    return rh, rc, rs


@pytest.mark.parametrize("n", [1, 255, 256, 4097, 300000])
def test_summary_matches_oracle(brq, orc, n):
    rng = np.random.default_rng(700 + n)
    amax = (np.abs(rng.standard_t(3, size=n)) * 2).astype(np.float32)
    ref = (np.abs(rng.standard_t(3, size=n)) * 2).astype(np.float32)
    sq = rng.random(n).astype(np.float32)
    k = min(n, len(EDGES))
    amax[:k] = EDGES[:k]                                   # values on the edges and on the threshold
    ref[:k] = amax[:k]
    check_summary(brq, orc, amax, sq, ref, 4.0, EDGES)
    check_summary(brq, orc, amax, None, None, 4.0, EDGES[:3])
    check_summary(brq, orc, amax, sq, ref, 0.0, [])         # no edges: one bin
    check_summary(brq, orc, amax, sq, ref, 1.0e30, [float(i) for i in range(32)])   # the most edges


def test_summary_adds_to_its_outputs_and_takes_nothing(brq):
    amax = torch.full((1000,), 3.0, dtype=torch.float32, device="cuda")
    hist = torch.tensor([5, 0, 0], dtype=torch.int64, device="cuda")
    counts = torch.tensor([1, 2, 3, 4], dtype=torch.int64, device="cuda")
    sums = torch.tensor([1.0, 2.0, 3.0, 4.0], dtype=torch.float64, device="cuda")
    for _ in range(2):
        brq.block_stats_summary(amax, outlier_threshold=2.0, edges=[1.0, 3.0], hist=hist, counts=counts, sums=sums)
    assert hist.tolist() == [5, 2000, 0]                    # 3.0 exceeds the edge 1.0 only
    assert counts.tolist() == [1, 2002, 3, 4] and sums.tolist() == [1.0, 2.0, 3.0, 4.0 + 6000.0]
    e = torch.empty((0,), dtype=torch.float32, device="cuda")
    h, c, s_ = brq.block_stats_summary(e)                   # no blocks: nothing launched
    assert h.tolist() == [0] and c.tolist() == [0, 0, 0, 0]
    with pytest.raises(brq.BrqError) as err:
        brq.block_stats_summary(amax, edges=[float(i) for i in range(33)])
    assert err.value.status == 2
    with pytest.raises(brq.BrqError) as err:
        brq.block_stats_summary(amax, edges=[1.0, 3.0, 2.0])       # edges must ascend
    assert err.value.status == 2


def test_rotation_comparison_full_size(brq, orc):
    """The paper's comparison (Sec. 4.2, Appendix "Rotation Comparison") on the benchmark's activations
    X 16384 x 8192: block-wise scales and losses after no, block and global rotation, classified into
    regular and outlier blocks by the untransformed scale.  The GPU's per-block arrays and their reductions
    against the oracle on a sample of rows (arrays bit for bit / 4e-6, reductions exact / 1e-12), and the
    paper's observations on the whole matrix: a global rotation inflates the scale of most regular blocks, a
    block rotation of few."""
    from paper_2511_04214_amd import inputs
    cfg = inputs.CONFIGS["decode"]
    x = inputs.make_x(cfg)
    M, K = x.shape
    xd = to_dev(x)
    thr = 60.0                                              # above the bulk, below the x20 outlier channels' tails
    per = {}
    for B in (1, 32, K):
        amax, _, sqerr = brq.block_stats(xd, B)
        per[B] = (amax, sqerr)
    rows = np.sort(np.random.default_rng(710).choice(M, size=8, replace=False))
    idx = torch.from_numpy(rows).cuda()
    ref_rows = None
    for B in (1, 32, K):
        ra, _, rs = orc.block_stats(x[rows], B)
        ga, gs = to_host(per[B][0][idx]), to_host(per[B][1][idx]).astype(np.float64)
        assert np.array_equal(ga.view(np.uint32), ra.view(np.uint32))
        assert (np.abs(gs - rs) <= 4e-6 * rs + 1e-44).all()
        if B == 1:
            ref_rows = ra
        check_summary(brq, orc, ga, to_host(per[B][1][idx]), ref_rows, thr, EDGES)
    res = {B: brq.block_stats_summary(per[B][0].view(-1), per[B][1].view(-1), per[1][0].view(-1), outlier_threshold=thr, edges=EDGES)
           for B in (1, 32, K)}
    c1, cb, cg = (to_host(res[B][1]) for B in (1, 32, K))
    s1, sb_, sg = (to_host(res[B][2]) for B in (1, 32, K))
    assert c1[0] + c1[1] == M * K // 32 and c1[2] == 0 and c1[3] == 0 and 0 < c1[1] < 0.1 * c1[0]
    assert cg[2] > 0.6 * cg[0] and cb[2] < 0.5 * cg[2]
    # (these activations have an outlier channel in about a quarter of their blocks, most of them below the
    # threshold: the MEAN regular-block scale need not grow under the global rotation, and is not asserted)
    assert sb_[2] < s1[2] and sb_[2] < sg[2]               # the block rotation gives the smallest regular-block scales
    for B in (1, 32, K):
        assert int(to_host(res[B][0]).sum()) == M * K // 32
