"""The interval rule itself (tests/interval_check.py), on the CPU: the oracle's own nominal result
must pass it, a planted wrong code or scale must not, and the bound must be tight enough to reject a
value one E2M1 step away."""
import numpy as np
import pytest

from interval_check import check_codes_within, check_swiglu_fused, unpack


def _gu(M, K, seed):
    rng = np.random.default_rng(seed)
    g = (rng.standard_t(4, size=(M, K)) * 1.5).astype(np.float32)
    u = (rng.standard_normal((M, K)) * 1.5).astype(np.float32)
    return g, u


@pytest.mark.parametrize("B,h_bf16", [(1, False), (1, True), (8, True), (32, False), (32, True), (128, True)])
def test_nominal_result_is_inside(orc, B, h_bf16):
    g, u = _gu(6, 256, 70 + B)
    signs = None if B == 1 else np.random.default_rng(71).choice([-1, 1], size=256).astype(np.int8)
    c, s = orc.swiglu_rotate_quantize_fused(g, u, B, h_bf16=h_bf16, signs=signs)
    same_c, same_s = check_swiglu_fused(orc, g, u, B, h_bf16, signs, c, s)
    assert same_c == 1.0 and same_s == 1.0


def test_planted_mistakes_are_outside(orc):
    g, u = _gu(4, 128, 80)
    c, s = orc.swiglu_rotate_quantize_fused(g, u, 32, h_bf16=True)
    # one code moved by one step of the E2M1 grid, somewhere away from a rounding boundary
    moved = 0
    for j in range(c.shape[1]):
        bad = c.copy()
        lo = bad[0, j] & 0x7
        bad[0, j] = (bad[0, j] & 0xF8) | ((lo + 1) if lo < 7 else (lo - 1))
        try:
            check_swiglu_fused(orc, g, u, 32, True, None, bad, s)
        except AssertionError:
            moved += 1
    assert moved >= c.shape[1] - 2          # (a value that sits on a boundary may legitimately take either code)
    bad_s = s.copy()
    bad_s[1, 2] += 1
    with pytest.raises(AssertionError):
        check_swiglu_fused(orc, g, u, 32, True, None, c, bad_s)
    # a result computed WITHOUT the rotation is rejected
    c1, s1 = orc.swiglu_rotate_quantize_fused(g, u, 1, h_bf16=True)
    with pytest.raises(AssertionError):
        check_swiglu_fused(orc, g, u, 32, True, None, c1, s1)
    # ... and so are the wrong signs
    sg = np.ones(128, np.int8)
    sg[5] = -1
    with pytest.raises(AssertionError):
        check_swiglu_fused(orc, g, u, 32, True, sg, c, s)


def test_plain_interval(orc):
    # a point interval reproduces the quantizer exactly; negative zero codes are refused
    rng = np.random.default_rng(90)
    y = rng.standard_normal((3, 64)).astype(np.float32)
    c, s = orc.mxfp4_quantize(y)
    check_codes_within(orc, y.astype(np.float64), np.zeros(y.shape), c, s)
    z = np.zeros((1, 32), dtype=np.float32)
    z[0, 0] = 1.0
    c, s = orc.mxfp4_quantize(z)
    assert (unpack(c)[0, 1:] == 0).all()
    c[0, 1] = 0x08                                  # element 2 as "negative zero"
    with pytest.raises(AssertionError):
        check_codes_within(orc, z.astype(np.float64), np.zeros(z.shape), c, s)
