"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Each pin is a plain function taking an `oracle.Oracle` build, so that the same pins run
against the committed oracle (test_oracle_pins.py) and against copies of its source with
a mistake planted in them (test_oracle_mutants.py, where at least one pin must fail).

Nothing here re-types the oracle's own formulas: expected values are hand-worked text
fixtures (tests/golden/), library routines the oracle does not call (scipy's Hadamard,
numpy matmul, Python's float.hex / math.frexp on literals), closed forms and invariants.
"""
import math
import os

import numpy as np
import scipy.linalg

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
E2M1_MAGS = None  # filled from the golden file


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def golden_e2m1():
    return {int(r[0]): float(r[1]) for r in _golden_rows("e2m1_values.txt")}


def _f32bits(x):
    return int(np.float32(x).view(np.uint32))


def _group(x0, n=32):
    g = np.zeros((1, n), dtype=np.float32)
    g[0, 0] = x0
    return g


def _unpack(codes):
    """[M, K/2] packed bytes -> [M, K] 4-bit codes, even element in the low nibble."""
    out = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = codes & 0xF
    out[:, 1::2] = codes >> 4
    return out


# --------------------------------------------------------------------------- Hadamard

def pin_hadamard_matches_scipy_and_is_orthogonal(o):
    for B in (1, 2, 4, 8, 32, 64, 128):
        H = o.hadamard_sylvester(B).astype(np.int64)
        assert np.array_equal(H, scipy.linalg.hadamard(B).astype(np.int64))  # Sylvester construction
        assert np.array_equal(H @ H.T, B * np.eye(B, dtype=np.int64))        # R^T R = I after 1/sqrt(B)
        assert np.array_equal(H, H.T)
        for i in range(0, B, max(1, B // 8)):
            for j in range(B):
                assert o.hadamard_entry(B, i, j) == H[i, j]


def pin_norm_constant_bits(o):
    # 1/sqrt(B) rounded to fp32: sqrt(2)/2 = 0x3F3504F3, scaled by exact powers of two.
    want = {2: 0x3F3504F3, 4: 0x3F000000, 8: 0x3EB504F3, 16: 0x3E800000, 32: 0x3E3504F3,
            64: 0x3E000000, 128: 0x3DB504F3, 8192: 0x3C3504F3}
    for B, bits in want.items():
        assert _f32bits(o.rotation_norm(B)) == bits, B


def pin_butterfly_exact_on_small_integers(o):
    # small integers: every partial sum fits 24 bits, so fp32 is exact and the result
    # must equal the integer matrix product (scipy's H) times fl32(1/sqrt(B)).
    rng = np.random.default_rng(5)
    for B in (32, 64, 128, 1024):
        x = rng.integers(-64, 65, size=(3, 2 * B)).astype(np.float32)
        y = o.block_rotate(x, B)
        H = scipy.linalg.hadamard(B).astype(np.int64)
        want = np.concatenate([x[:, :B].astype(np.int64) @ H, x[:, B:].astype(np.int64) @ H], axis=1)
        c = np.float32(1.0 / math.sqrt(B))
        assert np.array_equal(y, want.astype(np.float32) * c), B


def pin_butterfly_stage_order(o):
    # Hand-worked, B = 4 (norm 0.5, exact).  x = [2^24, 1, 1, 1].
    # ascending stages: h=1 -> [2^24 (tie of 2^24+1 to even), 2^24-1, 2, 0]
    #                   h=2 -> [2^24+2, 2^24-1, 2^24-2, 2^24-1]
    # (a descending order would swap the values in positions 1 and 2).
    x = np.array([[16777216.0, 1.0, 1.0, 1.0]], dtype=np.float32)
    y = o.block_rotate(x, 4)
    assert y.tolist() == [[8388609.0, 8388607.5, 8388607.0, 8388607.5]]
    # B = 2: [a, b] -> [(a+b), (a-b)] / sqrt(2); sign convention of the second output.
    y2 = o.block_rotate(np.array([[3.0, 1.0]], dtype=np.float32), 2)
    c = np.float32(1.0 / math.sqrt(2))
    assert y2.tolist() == [[float(np.float32(4.0) * c), float(np.float32(2.0) * c)]]


def pin_one_hot_spreads_over_its_block_only(o):
    # Sec. 4.3: an outlier is redistributed over its own block, nothing leaks outside.
    B, K = 32, 128
    cB = np.float32(1.0 / math.sqrt(B))
    H = scipy.linalg.hadamard(B)
    for j in (0, 1, 7, 31):
        x = np.zeros((1, K), dtype=np.float32)
        x[0, B + j] = 20.0
        y = o.block_rotate(x, B)
        assert np.array_equal(y[0, B:2 * B], (np.float32(20.0) * H[j]).astype(np.float32) * cB)
        assert not y[0, :B].any() and not y[0, 2 * B:].any()


def pin_rotation_invariants(o):
    rng = np.random.default_rng(6)
    for B in (32, 64, 256):
        x = rng.standard_normal((4, 2 * B)).astype(np.float32)
        y = o.block_rotate(x, B)
        # Sec. 4.2: rotation leaves the L2 norm unchanged (per block)
        for b in range(2):
            nx = np.linalg.norm(x[:, b * B:(b + 1) * B].astype(np.float64), axis=1)
            ny = np.linalg.norm(y[:, b * B:(b + 1) * B].astype(np.float64), axis=1)
            assert np.allclose(nx, ny, rtol=1e-6)
        # H/sqrt(B) is symmetric and orthogonal, hence an involution
        assert np.allclose(o.block_rotate(y, B), x, atol=1e-5)
        # block independence (Eq. 1): changing block 1 leaves block 0 bit-identical
        x2 = x.copy()
        x2[:, B:] += 1.0
        y2 = o.block_rotate(x2, B)
        assert np.array_equal(y2[:, :B], y[:, :B]) and not np.array_equal(y2[:, B:], y[:, B:])
        # fp32 butterfly vs the fp64 definition: (log2 B + 1) half-ulps of c*sum|x|
        yd = o.rotate_dense_f64(x.astype(np.float64), B)
        H = scipy.linalg.hadamard(B).astype(np.float64) / math.sqrt(B)
        assert np.allclose(yd[:, :B], x[:, :B].astype(np.float64) @ H, rtol=0, atol=1e-12)
        assert np.allclose(yd[:, B:], x[:, B:].astype(np.float64) @ H, rtol=0, atol=1e-12)
        for b in range(2):
            s = np.abs(x[:, b * B:(b + 1) * B]).astype(np.float64).sum(axis=1, keepdims=True)
            bound = (math.log2(B) + 1) * 2.0 ** -24 * s / math.sqrt(B) * 1.0001
            assert (np.abs(y[:, b * B:(b + 1) * B] - yd[:, b * B:(b + 1) * B]) <= bound).all()


def pin_bf16_conversions(o):
    # widening is exact; narrowing is RNE (hand-worked bit patterns)
    assert o.bf16_to_f32(np.array([0x3F80, 0xC000, 0x0001, 0x7F7F], dtype=np.uint16)).view(np.uint32).tolist() == \
        [0x3F800000, 0xC0000000, 0x00010000, 0x7F7F0000]
    assert o.f32_to_bf16(1.0) == 0x3F80
    assert o.f32_to_bf16(np.uint32(0x3F808000).view(np.float32)) == 0x3F80   # tie -> even (down)
    assert o.f32_to_bf16(np.uint32(0x3F808001).view(np.float32)) == 0x3F81   # just above the tie
    assert o.f32_to_bf16(np.uint32(0x3F818000).view(np.float32)) == 0x3F82   # tie -> even (up)
    assert o.f32_to_bf16(np.uint32(0xBF817FFF).view(np.float32)) == 0xBF81   # just below the tie
    x = np.array([[1.0, 1.0]], dtype=np.float32)
    # bf16 output of block_rotate is RNE of the fp32 value: 2/sqrt(2) = 1.41421354 -> 0x3FB5
    assert o.block_rotate(x, 2, out_bf16=True).tolist() == [[0x3FB5, 0x0000]]
    # bf16 input is widened, not reinterpreted
    xb = np.array([[0x3F80, 0x3F80]], dtype=np.uint16)
    assert np.array_equal(o.block_rotate(xb, 2), o.block_rotate(x, 2))


# --------------------------------------------------------------------------- E2M1 / E8M0

def pin_e2m1_table(o):
    g = golden_e2m1()
    assert len(g) == 16
    for code, val in g.items():
        got = o.e2m1_value(code)
        assert got == val and math.copysign(1.0, got) == math.copysign(1.0, val), code
    # encode(decode(c)) = c at scale 2^0 (code 8, "-0", is never produced: it maps to 0)
    for code, val in g.items():
        assert o.e2m1_encode(val, 127) == (0 if code == 8 else code)


def pin_thresholds_and_ties(o):
    for r, code in _golden_rows("threshold_cases.txt"):
        r, code = float(r), int(code)
        assert o.e2m1_encode(r, 127) == code, r
        assert o.e2m1_encode(-r, 127) == (code | 8 if code else 0), r
    # one fp32 step either side of each midpoint
    mids = [(0.25, 0, 1), (0.75, 1, 2), (1.25, 2, 3), (1.75, 3, 4), (2.5, 4, 5), (3.5, 5, 6), (5.0, 6, 7)]
    for m, lo, hi in mids:
        dn = np.nextafter(np.float32(m), np.float32(0))
        up = np.nextafter(np.float32(m), np.float32(10))
        assert o.e2m1_encode(dn, 127) == lo and o.e2m1_encode(up, 127) == hi, m
    # the same decisions under another scale: r = y / 2^e
    for sb in (100, 120, 130, 200):
        s = 2.0 ** (sb - 127)
        for r, code in _golden_rows("threshold_cases.txt"):
            assert o.e2m1_encode(float(r) * s, sb) == int(code), (r, sb)


def pin_scale_rule(o):
    g = golden_e2m1()
    for x, sb, code, deq in _golden_rows("rne_cases.txt"):
        x, sb, code, deq = float(x), int(sb), int(code), float(deq)
        codes, scales = o.mxfp4_quantize(_group(x))
        assert scales.shape == (1, 1) and codes.shape == (1, 16)
        assert int(scales[0, 0]) == sb, x
        assert int(codes[0, 0]) == code, x          # element 0 in the LOW nibble, element 1 = 0
        assert not codes[0, 1:].any()
        assert g[code] * 2.0 ** (sb - 127) == deq
        assert o.e8m0_from_amax(abs(x)) == sb
    # the maximum is taken over all 32 positions of the group, and over magnitudes
    for pos in (0, 1, 15, 16, 30, 31):
        for val in (7.0, -7.0):
            gq = np.full((1, 32), 0.3, dtype=np.float32)
            gq[0, pos] = val
            cq, sq = o.mxfp4_quantize(gq)
            assert int(sq[0, 0]) == 127
            u = _unpack(cq)[0]
            assert int(u[pos]) == (7 if val > 0 else 15) and (np.delete(u, pos) == 1).all()
    # E8M0 byte b means 2^(b-127)
    assert o.e8m0_value(127) == 1.0 and o.e8m0_value(0) == 2.0 ** -127 and o.e8m0_value(254) == 2.0 ** 127
    # closed form on the fp32 exponent field: byte = max(field - 2, 0); never 0xFF
    for bits in (0x00000000, 0x00000001, 0x007FFFFF, 0x00800000, 0x01000000, 0x01800000, 0x3F800000,
                 0x3FFFFFFF, 0x40000000, 0x7F7FFFFF):
        a = np.uint32(bits).view(np.float32)
        assert o.e8m0_from_amax(a) == max((bits >> 23) - 2, 0), hex(bits)
    # amax / 2^e lies in [4, 8) whenever the byte is not clamped; scale monotone in amax
    rng = np.random.default_rng(7)
    a = np.sort(np.abs(rng.standard_normal(200)).astype(np.float32) * np.float32(1e3) + np.float32(1e-3))
    b = [o.e8m0_from_amax(v) for v in a]
    assert all(b[i] <= b[i + 1] for i in range(len(b) - 1))
    for v, sb in zip(a, b):
        r = math.ldexp(float(v), 127 - sb)
        assert 4.0 <= r < 8.0


def pin_group_structure(o):
    # groups are 32 consecutive elements of a row; nibble order; row-major scales
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 96)).astype(np.float32)
    codes, scales = o.mxfp4_quantize(x)
    assert codes.shape == (3, 48) and scales.shape == (3, 3) and codes.dtype == np.uint8
    x2 = x.copy()
    x2[1, 40] = 1000.0   # group 1 of row 1 only
    c2, s2 = o.mxfp4_quantize(x2)
    diff_s = np.argwhere(s2 != scales)
    assert diff_s.tolist() == [[1, 1]]
    assert np.array_equal(np.unique(np.argwhere(c2 != codes)[:, 0]), [1])
    assert set(np.argwhere(c2 != codes)[:, 1] // 16) == {1}
    assert (c2[1, 20] & 0xF) == 6 or (c2[1, 20] & 0xF) == 7      # element 40 -> byte 20, low nibble
    # scaling a whole group by 2^k shifts the byte by k and leaves the codes unchanged
    c3, s3 = o.mxfp4_quantize(x * np.float32(2.0 ** 7))
    assert np.array_equal(c3, codes) and np.array_equal(s3.astype(int), scales.astype(int) + 7)
    # an all-zero group, and negative values too small to survive, give code 0 (no "-0")
    z = np.zeros((1, 32), dtype=np.float32)
    z[0, 5] = -0.0
    cz, sz = o.mxfp4_quantize(z)
    assert not cz.any() and int(sz[0, 0]) == 0
    t = _group(4.0)
    t[0, 1] = -0.2   # r = -0.2 -> magnitude code 0 -> nibble 0, not 8
    ct, _ = o.mxfp4_quantize(t)
    assert int(ct[0, 0]) == 0x06


def pin_round_trip_of_representable_blocks(o):
    g = golden_e2m1()
    rng = np.random.default_rng(9)
    for sb in (3, 100, 127, 140, 250):
        code = rng.integers(0, 16, size=(8, 64)).astype(np.uint8)
        code[code == 8] = 0
        code[:, 0] = 7          # a 6 in group 0, a 4 in group 1: pins the shared exponent
        code[:, 32] = 14
        vals = np.vectorize(g.get)(code) * 2.0 ** (sb - 127)
        x = vals.astype(np.float32)
        assert np.array_equal(x.astype(np.float64), vals)
        codes, scales = o.mxfp4_quantize(x)
        assert (scales == sb).all()
        assert np.array_equal(_unpack(codes), code)
        assert np.array_equal(o.mxfp4_dequantize(codes, scales), vals)


def pin_bf16_and_f32_inputs_agree(o):
    rng = np.random.default_rng(10)
    bits = rng.integers(0, 1 << 16, size=(4, 64)).astype(np.uint16)
    bits[(bits & 0x7F80) == 0x7F80] = 0x3F80      # no Inf/NaN
    wide = (bits.astype(np.uint32) << 16).view(np.float32)
    cb, sb = o.mxfp4_quantize(bits)
    cf, sf = o.mxfp4_quantize(wide)
    assert np.array_equal(cb, cf) and np.array_equal(sb, sf)
    assert np.array_equal(o.block_rotate(bits, 32), o.block_rotate(wide, 32))


def pin_fused_is_the_composition(o):
    rng = np.random.default_rng(11)
    x = (rng.standard_t(4, size=(5, 256)) * 3).astype(np.float32)
    for B in (32, 64, 256):
        c1, s1 = o.rotate_quantize_fused(x, B)
        c2, s2 = o.mxfp4_quantize(o.block_rotate(x, B))
        assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    # and it is NOT the quantizer alone: the rotation must have happened
    c0, _ = o.mxfp4_quantize(x)
    assert not np.array_equal(c0, o.rotate_quantize_fused(x, 32)[0])


def pin_signed_rotation(o):
    # Randomized Hadamard (Sec. 5.1): R = diag(s) H_B / sqrt(B).  Closed form of its entries from
    # the one-hot rows; orthogonality; and the sign acts on the INPUT side, element by element:
    # rotating x with signs equals rotating the pre-flipped x (flips are exact), which is not the
    # same as flipping the output.
    rng = np.random.default_rng(21)
    for B in (8, 16, 32, 64):
        K = 2 * B
        s = rng.choice([-1, 1], size=K).astype(np.int8)
        s[1] = -1
        s[B] = -1
        s[0] = 1
        R = o.block_rotate(np.eye(K, dtype=np.float32), B, signs=s).astype(np.float64)
        H = scipy.linalg.hadamard(B).astype(np.float64)
        want = np.zeros((K, K))
        for b in range(2):
            want[b * B:(b + 1) * B, b * B:(b + 1) * B] = (s[b * B:(b + 1) * B, None] * H) / np.sqrt(B)
        assert np.allclose(R, want, rtol=0, atol=1e-7), B
        assert np.allclose(R @ R.T, np.eye(K), rtol=0, atol=1e-6)
        x = (rng.standard_t(4, size=(4, K)) * 3).astype(np.float32)
        a = o.block_rotate(x, B, signs=s)
        assert np.array_equal(a.view(np.uint32), o.block_rotate(x * s.astype(np.float32), B).view(np.uint32))
        assert not np.array_equal(a, o.block_rotate(x, B) * s.astype(np.float32))
        # all-plus signs change nothing
        assert np.array_equal(o.block_rotate(x, B, signs=np.ones(K, np.int8)), o.block_rotate(x, B))
    # the product is still invariant when both operands use the same signs (fp64 route through the
    # fp32 rotation: tolerance of fp32 rounding)
    X = rng.standard_normal((5, 64)).astype(np.float32)
    W = rng.standard_normal((4, 64)).astype(np.float32)
    s = rng.choice([-1, 1], size=64).astype(np.int8)
    got = o.block_rotate(X, 32, signs=s).astype(np.float64) @ o.block_rotate(W, 32, signs=s).astype(np.float64).T
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.allclose(got, ref, rtol=0, atol=1e-5 * np.abs(ref).max())
    # ... and broken when they do not
    bad = o.block_rotate(X, 32, signs=s).astype(np.float64) @ o.block_rotate(W, 32).astype(np.float64).T
    assert not np.allclose(bad, ref, rtol=0, atol=1e-3 * np.abs(ref).max())


def pin_fused_small_blocks_and_signs(o):
    # Rotation blocks smaller than the 32-element quantization group (Sec. 5.2 sweeps the
    # rotation dimension) and signed rotations: still the composition, group stays 32.
    rng = np.random.default_rng(22)
    x = (rng.standard_t(4, size=(5, 128)) * 3).astype(np.float32)
    s = rng.choice([-1, 1], size=128).astype(np.int8)
    for B in (8, 16, 32, 128):
        for sg in (None, s):
            c1, s1 = o.rotate_quantize_fused(x, B, signs=sg)
            c2, s2 = o.mxfp4_quantize(o.block_rotate(x, B, signs=sg))
            assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
            assert s1.shape == (5, 4)
    # B = 16 (norm 1/4, exact): a one-hot of 32 spreads as +-8 over its 16-block only; the
    # group's scale comes from amax 8 = 1.0 * 2^3 (exponent 3 - 2 = 1, byte 128) and the 16 other
    # codes of the group are 0
    x1 = np.zeros((1, 32), dtype=np.float32)
    x1[0, 20] = 32.0
    c, sc = o.rotate_quantize_fused(x1, 16)
    vals = o.mxfp4_dequantize(c, sc)[0]
    assert sc[0, 0] == 128
    assert np.count_nonzero(vals) == 16 and np.all(vals[:16] == 0)
    assert np.array_equal(np.abs(vals[16:]), np.full(16, 8.0))
    # the same with a flipped sign on the hot element: every output changes sign, magnitudes stay
    sg = np.ones(32, np.int8)
    sg[20] = -1
    c2, sc2 = o.rotate_quantize_fused(x1, 16, signs=sg)
    assert np.array_equal(o.mxfp4_dequantize(c2, sc2)[0], -vals) and sc2[0, 0] == 128


# --------------------------------------------------------------------------- producer (SwiGLU)

def _bf16_bits_torch(x32):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def pin_swiglu_is_the_definition(o):
    # h = silu(g) * u with silu(g) = g * sigmoid(g) (the gated activation in front of down_proj,
    # Sec. 4.3).  Against torch's float64 silu (a library routine the oracle does not call), against
    # values and identities that the mathematics fixes, and the roundings against numpy's / torch's.
    import torch
    rng = np.random.default_rng(31)
    g = np.concatenate([np.linspace(-100, 100, 200001), rng.standard_normal(100000) * 4,
                        [0.0, -0.0, 1e-30, -1e-30, 700.0, -700.0, 3.0e38, -3.0e38]]).astype(np.float32)
    u = (rng.standard_normal(g.size) * 2).astype(np.float32)
    u[-2:] = 0.5                                           # keeps the product of the largest gates finite in fp32
    exact = o.swiglu_exact(g[None, :], u[None, :])[0]
    want = (torch.nn.functional.silu(torch.from_numpy(g.astype(np.float64))) * torch.from_numpy(u.astype(np.float64))).numpy()
    assert np.all(np.abs(exact - want) <= 1e-15 * np.abs(want))        # a few fp64 ulp between two evaluations
    # rounded once to fp32: numpy's conversion of the fp64 value; torch's own value rounds to the same
    # fp32 except where the two fp64 evaluations straddle a rounding boundary
    h32 = o.swiglu(g[None, :], u[None, :])[0]
    assert np.array_equal(h32.view(np.uint32), exact.astype(np.float32).view(np.uint32))
    assert (h32.view(np.uint32) == want.astype(np.float32).view(np.uint32)).mean() > 0.99999
    # not symmetric in its arguments: silu acts on the first one
    assert abs(o.swiglu_f64(1.0, 3.0) - 3.0 * 0.7310585786300049) < 1e-15         # sigmoid(1) = 0.73105857863...
    assert abs(o.swiglu_f64(3.0, 1.0) - 3.0 * 0.9525741268224334) < 1e-15         # sigmoid(3) = 0.95257412682...
    assert abs(o.swiglu_f64(-1.0, 1.0) + 0.2689414213699951) < 1e-16              # -sigmoid(-1)
    # silu(g) - silu(-g) = g sigmoid(g) + g (1 - sigmoid(g)) = g
    for gv in (0.1, 0.5, 1.0, 2.5, 7.0, 20.0, 50.0):
        assert abs((o.swiglu_f64(gv, 1.0) - o.swiglu_f64(-gv, 1.0)) - gv) <= 2e-16 * gv
    # the minimum of silu: value -0.27846454276107..., where g = -1.27846454276107... (silu'(g) = 0 there
    # means silu(g) = g + 1 ... i.e. the minimum value is g_min + 1)
    gmin = -1.2784645427610738
    assert abs(o.swiglu_f64(gmin, 1.0) - (gmin + 1.0)) < 1e-15
    assert o.swiglu_f64(gmin - 1e-3, 1.0) > o.swiglu_f64(gmin, 1.0) < o.swiglu_f64(gmin + 1e-3, 1.0)
    # limits: silu(0) = 0; silu(g) -> g for large g (exp(-g) below half an ulp of 1); silu(g) -> -0 far below
    assert o.swiglu_f64(0.0, 7.0) == 0.0
    for gv in (40.0, 86.0, 100.0, float(np.float32(3.0e38))):
        assert o.swiglu_f64(gv, 1.0) == gv and float(o.swiglu_elem(gv, -0.5)) == -0.5 * gv
    assert abs(o.swiglu_f64(-40.0, 1.0) + 40.0 * math.exp(-40.0)) < 1e-30
    assert o.swiglu_f64(-800.0, 1.0) == 0.0 and float(o.swiglu_elem(-3.0e38, 2.0)) == 0.0
    # u is a plain factor
    for gv in (-3.0, 0.7, 5.0):
        assert o.swiglu_f64(gv, 4.0) == 4.0 * o.swiglu_f64(gv, 1.0)
        assert o.swiglu_f64(gv, -1.0) == -o.swiglu_f64(gv, 1.0)
    # bf16 inputs are widened exactly: the same values given as bf16 bits or as fp32 agree
    gb, ub = _bf16_bits_torch(g[:4096]), _bf16_bits_torch(u[:4096])
    gw, uw = o.bf16_to_f32(gb), o.bf16_to_f32(ub)
    assert np.array_equal(o.swiglu(gb[None, :], ub[None, :]), o.swiglu(gw[None, :], uw[None, :]))
    # bf16 output: ONE rounding of the fp64 value to nearest even.  Hand-worked double-rounding trap:
    # 1 + 2^-8 + 2^-30 lies above the midpoint of 1 and 1 + 2^-7, so it rounds up (0x3F81); through fp32
    # it would first become the midpoint itself and then tie down to 1 (0x3F80)
    assert o.f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81
    assert o.f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80 and o.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82      # ties to even
    assert o.f64_to_bf16(-2.5) == 0xC020 and o.f64_to_bf16(0.0) == 0 and o.f64_to_bf16(-0.0) == 0x8000
    assert o.f64_to_bf16(2.0 ** -133) == 1 and o.f64_to_bf16(2.0 ** -134) == 0 and o.f64_to_bf16(1.5 * 2.0 ** -133) == 2
    # ... and it equals torch's conversion (which goes through fp32) wherever the fp32 value is not itself
    # a bf16 midpoint, i.e. wherever rounding twice cannot differ from rounding once
    x64 = rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000)
    got = np.array([o.f64_to_bf16(v) for v in x64], dtype=np.uint16)
    t = torch.from_numpy(x64).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    safe = (x64.astype(np.float32).view(np.uint32) & np.uint32(0xFFFF)) != 0x8000
    assert safe.mean() > 0.999 and np.array_equal(got[safe], t[safe])
    hb = o.swiglu(gw[None, :], uw[None, :], out_bf16=True)[0]
    ex = o.swiglu_exact(gw[None, :], uw[None, :])[0]
    assert np.array_equal(hb, np.array([o.f64_to_bf16(v) for v in ex], dtype=np.uint16))


def pin_swiglu_fused_is_the_composition(o):
    rng = np.random.default_rng(32)
    M, K = 5, 256
    # gate and up as the two halves of one [M, 2K + 8] buffer: different pitches from K, and the
    # up half starts elsewhere than the gate half
    buf = (rng.standard_normal((M, 2 * K + 8)) * 3).astype(np.float32)
    gate, up = buf[:, :K], buf[:, K + 8:]
    wide = (rng.standard_normal((M, K + 32)) * 3).astype(np.float32)
    up2 = wide[:, :K]                      # a third pitch
    s = rng.choice([-1, 1], size=K).astype(np.int8)
    for g_, u_ in ((gate, up), (gate, up2)):
        h32 = o.swiglu(np.ascontiguousarray(g_), np.ascontiguousarray(u_))
        hb = o.swiglu(np.ascontiguousarray(g_), np.ascontiguousarray(u_), out_bf16=True)
        for B in (8, 32, 128):
            for sg in (None, s):
                c1, s1 = o.swiglu_rotate_quantize_fused(g_, u_, B, h_bf16=False, signs=sg)
                c2, s2 = o.rotate_quantize_fused(h32, B, signs=sg)
                assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
                c3, s3 = o.swiglu_rotate_quantize_fused(g_, u_, B, h_bf16=True, signs=sg)
                c4, s4 = o.rotate_quantize_fused(hb, B, signs=sg)       # hb: bf16 bits, widened exactly
                assert np.array_equal(c3, c4) and np.array_equal(s3, s4)
        # B = 1: no rotation, the quantizer alone
        c5, s5 = o.swiglu_rotate_quantize_fused(g_, u_, 1)
        c6, s6 = o.mxfp4_quantize(h32)
        assert np.array_equal(c5, c6) and np.array_equal(s5, s6)
        assert not np.array_equal(c5, o.swiglu_rotate_quantize_fused(g_, u_, 32)[0])
    # passing through bf16 is visible in the codes of a long enough row (a value near a rounding
    # boundary of the encoder moves across it)
    big_g = (rng.standard_normal((8, 4096)) * 3).astype(np.float32)
    big_u = (rng.standard_normal((8, 4096)) * 3).astype(np.float32)
    assert not np.array_equal(o.swiglu_rotate_quantize_fused(big_g, big_u, 32, h_bf16=False)[0],
                              o.swiglu_rotate_quantize_fused(big_g, big_u, 32, h_bf16=True)[0])


# --------------------------------------------------------------------------- arbitrary orthogonal blocks

def _random_orthogonal_blocks(rng, n):
    q = np.stack([np.linalg.qr(rng.standard_normal((32, 32)))[0] for _ in range(n)])
    return q.astype(np.float32)


def pin_matrix_rotation_is_the_per_block_product(o):
    # Eq. (1) with arbitrary blocks: y_b = x_b R_b.  numpy's matmul per block (a library routine
    # the oracle does not call) on non-symmetric, per-block different matrices: a transposed R, a
    # wrong block or a wrong pitch all show.
    rng = np.random.default_rng(41)
    M, K = 7, 128
    wide = (rng.standard_t(4, size=(M, K + 32)) * 2).astype(np.float32)
    x = wide[:, :K]                                   # pitch K + 32
    R = rng.standard_normal((K // 32, 32, 32)).astype(np.float32)
    y, bound = o.matrix_rotate_f64(x, R, want_bound=True)
    want = np.concatenate([np.float64(x[:, 32 * b:32 * b + 32]) @ np.float64(R[b]) for b in range(K // 32)], axis=1)
    mag = np.concatenate([np.abs(np.float64(x[:, 32 * b:32 * b + 32])) @ np.abs(np.float64(R[b])) for b in range(K // 32)], axis=1)
    assert np.allclose(y, want, rtol=0, atol=1e-13 * mag.max())
    assert np.allclose(bound, mag, rtol=1e-14)
    # one shared matrix = that matrix repeated
    y1 = o.matrix_rotate_f64(x, R[2])
    assert np.array_equal(y1, o.matrix_rotate_f64(x, np.repeat(R[2:3], K // 32, axis=0)))
    assert not np.array_equal(y1, y)
    # identity and a signed permutation are exact
    assert np.array_equal(o.matrix_rotate_f64(x, np.eye(32, dtype=np.float32)), np.float64(x))
    perm = rng.permutation(32)
    sgn = rng.choice([-1.0, 1.0], size=32)
    P = np.zeros((32, 32), dtype=np.float32)
    P[perm, np.arange(32)] = sgn                      # output j takes input perm[j], times sgn[j]
    yp = o.matrix_rotate_f64(x, P)
    for b in range(K // 32):
        assert np.array_equal(yp[:, 32 * b:32 * b + 32], np.float64(x[:, 32 * b:32 * b + 32])[:, perm] * sgn)
    # the Hadamard block is one such R: same result as the dense Hadamard rotation (R holds the
    # fp32 rounding of 1/sqrt(32), hence the 1e-7)
    H = (scipy.linalg.hadamard(32) / math.sqrt(32)).astype(np.float32)
    assert np.allclose(o.matrix_rotate_f64(x, H), o.rotate_dense_f64(np.float64(x), 32), rtol=0, atol=1e-6)
    # orthogonal blocks preserve the norm of every block, and the product X W^T (Sec. 2)
    Q = _random_orthogonal_blocks(rng, K // 32)
    yq = o.matrix_rotate_f64(x, Q)
    for b in range(K // 32):
        assert np.allclose(np.linalg.norm(yq[:, 32 * b:32 * b + 32], axis=1),
                           np.linalg.norm(np.float64(x[:, 32 * b:32 * b + 32]), axis=1), rtol=1e-5)
    w = (rng.standard_normal((5, K)) * 0.02).astype(np.float32)
    assert np.allclose(yq @ o.matrix_rotate_f64(w, Q).T, np.float64(x) @ np.float64(w).T, rtol=0, atol=1e-5)


def pin_matrix_rotation_fused_and_encode_with_scales(o):
    rng = np.random.default_rng(42)
    M, K = 6, 96
    x = (rng.standard_t(4, size=(M, K)) * 3).astype(np.float32)
    Q = _random_orthogonal_blocks(rng, K // 32)
    c, s = o.matrix_rotate_quantize_fused(x, Q)
    c2, s2 = o.mxfp4_quantize(np.float32(o.matrix_rotate_f64(x, Q)))
    assert np.array_equal(c, c2) and np.array_equal(s, s2)
    assert not np.array_equal(c, o.mxfp4_quantize(x)[0])
    # a signed permutation only moves and flips the codes of the plain quantizer inside each group
    perm = rng.permutation(32)
    sgn = rng.choice([-1.0, 1.0], size=32)
    P = np.zeros((32, 32), dtype=np.float32)
    P[perm, np.arange(32)] = sgn
    cp, sp = o.matrix_rotate_quantize_fused(x, P)
    xp = np.concatenate([x[:, 32 * b:32 * b + 32][:, perm] * np.float32(sgn) for b in range(K // 32)], axis=1)
    cq, sq = o.mxfp4_quantize(np.ascontiguousarray(xp, dtype=np.float32))
    assert np.array_equal(cp, cq) and np.array_equal(sp, sq) and np.array_equal(sp, o.mxfp4_quantize(x)[1])
    # encode under given scales: the quantizer's own scales give its codes back; every
    # representable value under any scale returns its own code (table from the golden file)
    assert np.array_equal(o.mxfp4_encode_with_scales(xp, sq), cq)
    g = golden_e2m1()
    for sb in (100, 127, 140):
        vals = np.array([[g[cde] * 2.0 ** (sb - 127) for cde in range(16)] * 2], dtype=np.float32)
        got = _unpack(o.mxfp4_encode_with_scales(vals, np.array([[sb]], dtype=np.uint8)))[0]
        want = np.array(list(range(16)) * 2)
        want[want == 8] = 0                           # a zero magnitude is code 0 whatever the sign
        assert np.array_equal(got, want)
    # the scale byte is looked up per group of 32, not per row
    two = np.concatenate([np.full((1, 32), 1.0, np.float32), np.full((1, 32), 4.0, np.float32)], axis=1)
    got = _unpack(o.mxfp4_encode_with_scales(two, np.array([[127, 129]], dtype=np.uint8)))[0]
    assert (got == 2).all()


# --------------------------------------------------------------------------- block statistics

def pin_block_stats(o):
    # The three statistics against numpy reductions over the oracle's separately pinned rotation,
    # quantizer and dequantizer, and against hand-worked blocks.
    rng = np.random.default_rng(51)
    M, K = 9, 256
    x = (rng.standard_t(4, size=(M, K)) * 1.2).astype(np.float32)
    x[:, [7, 130]] *= 25.0                                       # two outlier channels
    th = np.array([0.5, 1.5, 3.0, 1.0e9], dtype=np.float32)
    for B in (1, 32, 256):
        y = x if B == 1 else o.block_rotate(x, B)
        amax, count, sqerr = o.block_stats(x, B, th)
        assert np.array_equal(amax, np.abs(y).reshape(M, K // 32, 32).max(axis=2))
        assert np.array_equal(count, [(np.abs(y) > t).sum() for t in th])
        c, s = o.mxfp4_quantize(y)
        d = np.float64(y) - o.mxfp4_dequantize(c, s)
        assert np.allclose(sqerr, (d * d).reshape(M, K // 32, 32).sum(axis=2), rtol=1e-13, atol=0)
    # signs pass through to the rotation
    sg = rng.choice([-1, 1], size=K).astype(np.int8)
    a1, _, _ = o.block_stats(x, 32, (), signs=sg)
    assert np.array_equal(a1, np.abs(o.block_rotate(x, 32, signs=sg)).reshape(M, K // 32, 32).max(axis=2))
    # hand-worked block: values 1 (x29), 5, -7.5, 0.2 -> amax 7.5 = 1.875 * 2^2, scale 2^0;
    # 5 ties to 4 (loss 1), -7.5 saturates to -6 (loss 2.25), 0.2 rounds to 0 (loss 0.04), ones are exact
    blk = np.ones((1, 32), dtype=np.float32)
    blk[0, 3], blk[0, 17], blk[0, 30] = 5.0, -7.5, 0.2
    amax, count, sqerr = o.block_stats(blk, 1, [1.0, 0.2, 7.5, 7.4])
    assert amax[0, 0] == 7.5
    assert list(count) == [2, 31, 0, 1]                          # strictly greater: 1.0, 0.2 and 7.5 themselves do not count
    assert abs(sqerr[0, 0] - (1.0 + 2.25 + np.float64(np.float32(0.2)) ** 2)) < 1e-15
    # the paper's observations on activations with outlier channels (Sec. 4.2, Appendix): a global
    # rotation removes the largest values but raises the share of mid-size ones and the scale of most
    # regular blocks; a block rotation leaves the blocks without an outlier channel as they were in scale
    X = (rng.standard_t(4, size=(64, 1024))).astype(np.float32)
    X[:, [5, 700]] *= 40.0
    a_none, c_none, _ = o.block_stats(X, 1, [1.5, 20.0])
    a_glob, c_glob, _ = o.block_stats(X, 1024, [1.5, 20.0])
    a_blk, c_blk, _ = o.block_stats(X, 32, [1.5, 20.0])
    assert c_glob[1] < c_none[1] and c_glob[0] > 1.5 * c_none[0]
    regular = np.ones(1024 // 32, dtype=bool)
    regular[[5 // 32, 700 // 32]] = False
    assert (a_glob[:, regular] > a_none[:, regular]).mean() > 0.7
    assert np.median(a_blk[:, regular] / a_none[:, regular]) < 1.2 < np.median(a_glob[:, regular] / a_none[:, regular])


def pin_block_stats_summary(o):
    # The reductions of the paper's analysis over per-block statistics, against numpy (searchsorted and masked
    # sums, which the oracle does not call) and a hand-worked case.
    rng = np.random.default_rng(55)
    n = 5000
    amax = np.abs(rng.standard_t(3, size=n)).astype(np.float32) * 2
    ref = np.abs(rng.standard_t(3, size=n)).astype(np.float32) * 2
    sq = rng.random(n).astype(np.float32)
    edges = np.array([0.5, 1.0, 2.0, 4.0, 8.0], dtype=np.float32)
    amax[:6] = [0.5, 1.0, 2.0, 4.0, 8.0, 8.5]                 # values on the edges: strictly greater decides
    ref[:6] = [3.0, 1.0, 2.0, 5.0, 8.0, 9.0]                  # ... and on the outlier threshold / equal to amax
    hist, counts, sums = o.block_stats_summary(amax, sq, ref, outlier=3.0, edges=edges)
    want_hist = np.bincount(np.searchsorted(edges, amax, side="left"), minlength=6)       # number of edges < amax
    assert np.array_equal(hist, want_hist) and hist.sum() == n
    outl = ref > np.float32(3.0)
    grew = amax > ref
    assert list(counts) == [int((~outl).sum()), int(outl.sum()), int((grew & ~outl).sum()), int((grew & outl).sum())]
    want = [np.float64(sq)[~outl].sum(), np.float64(sq)[outl].sum(), np.float64(amax)[~outl].sum(), np.float64(amax)[outl].sum()]
    assert np.allclose(sums, want, rtol=1e-12, atol=0)
    # the first six by hand: amax on an edge falls into the bin below it; ref = 3.0 is regular (not > 3); equal scales did not grow
    h6, c6, s6 = o.block_stats_summary(amax[:6], sq[:6], ref[:6], outlier=3.0, edges=edges)
    assert list(h6) == [1, 1, 1, 1, 1, 1]
    assert list(c6) == [3, 3, 0, 0]
    # without a reference the block's own scale classifies it and nothing "grew"; without sqerr no loss sums
    h0, c0, s0 = o.block_stats_summary(amax, None, None, outlier=3.0, edges=edges)
    own = amax > np.float32(3.0)
    assert list(c0) == [int((~own).sum()), int(own.sum()), 0, 0] and s0[0] == 0.0 and s0[1] == 0.0
    assert np.array_equal(h0, want_hist)
    # no edges: one bin with everything
    h1, _, _ = o.block_stats_summary(amax, sq, ref, outlier=3.0)
    assert list(h1) == [n]
    # the paper's comparison on activations with outlier channels (Appendix): classify blocks by the
    # untransformed scale; a global rotation inflates the scale of most regular blocks, a block rotation of
    # few, and removes the bulk of that inflation in the mean regular-block scale
    X = (rng.standard_t(4, size=(64, 1024))).astype(np.float32)
    X[:, [5, 700]] *= 40.0
    a_none, _, q_none = o.block_stats(X, 1)
    thr = float(np.quantile(np.abs(X), 0.999))                # top 0.1 % of magnitudes (Sec. 4.1)
    res = {}
    for B in (32, 1024):
        a, _, q = o.block_stats(X, B)
        _, c, s_ = o.block_stats_summary(a, q.astype(np.float32), a_none, outlier=thr)
        res[B] = (c, s_)
    _, c_n, s_n = o.block_stats_summary(a_none, q_none.astype(np.float32), a_none, outlier=thr)
    assert c_n[1] > 0 and c_n[0] > 10 * c_n[1] and c_n[2] == 0 and c_n[3] == 0
    assert res[1024][0][2] > 0.6 * res[1024][0][0]            # most regular blocks' scales grow under the global rotation (the paper: > 70 %)
    assert res[32][0][2] < 0.5 * res[1024][0][2]              # ... far fewer under the block rotation
    infl_glob = res[1024][1][2] - s_n[2]
    infl_blk = res[32][1][2] - s_n[2]
    assert infl_glob > 0 and infl_blk < 0.2 * infl_glob        # block rotation removes > 80 % of that inflation


def pin_bfp4_loss(o):
    # The FP16-scale counterpart (Sec. 3, 4.1): half-precision rounding against numpy's float16 (a
    # conversion the oracle does not call), the loss against a composition of separately pinned
    # parts, hand-worked blocks, and the paper's observation that the power-of-two scale loses more.
    rng = np.random.default_rng(61)
    f = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 6, 20000),
                        [0.0, 65504.0, 65519.9, 65520.0, 1.0e9, 6.1e-5, 5.96e-8, 2.9e-8, 3.0e-8, -1.0009765625]]).astype(np.float32)
    want = np.clip(f.astype(np.float64), -65519.99, 65519.99).astype(np.float16).astype(np.float32)
    want = np.where(np.abs(f) >= 65520.0, np.sign(f) * np.float32(65504.0), want)
    got = np.array([o.round_to_f16(v) for v in f], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    M, K = 7, 128
    x = (rng.standard_t(4, size=(M, K)) * 1.3).astype(np.float32)
    x[:, 9] *= 30.0
    for B in (1, 32):
        y = x if B == 1 else o.block_rotate(x, B)
        amax, _, sq, sqb = o.block_stats(x, B, (), want_bfp4=True)
        s = np.array([[o.round_to_f16(np.float32(a) / np.float32(6.0)) for a in row] for row in amax], dtype=np.float32)
        r = (y.reshape(M, K // 32, 32) / s[:, :, None]).astype(np.float32).reshape(M, K)     # IEEE fp32 division
        codes = o.mxfp4_encode_with_scales(r, np.full((M, K // 32), 127, dtype=np.uint8))
        deq = o.mxfp4_dequantize(codes, np.full((M, K // 32), 127, dtype=np.uint8)) * np.repeat(np.float64(s), 32, axis=1)
        d = np.float64(y) - deq
        assert np.allclose(sqb, (d * d).reshape(M, K // 32, 32).sum(axis=2), rtol=1e-13, atol=0)
    # Sec. 3, finding E: over many blocks the power-of-two scale loses more than the FP16 scale, with
    # and without rotation
    big = rng.standard_t(3, size=(256, 1024)).astype(np.float32)
    for B in (1, 32):
        _, _, sq, sqb = o.block_stats(big, B, (), want_bfp4=True)
        assert sqb.mean() < 0.9 * sq.mean()
    # hand-worked: maximum 7.5 -> s = 1.25: 7.5 is exactly 6 s (no saturation loss, where MXFP4 loses
    # 2.25); the ones become 0.8 -> code 1.0 -> 1.25, each 0.0625 off in square
    blk = np.ones((1, 32), dtype=np.float32)
    blk[0, 17] = -7.5
    _, _, sq, sqb = o.block_stats(blk, 1, (), want_bfp4=True)
    assert abs(sq[0, 0] - 2.25) < 1e-15 and abs(sqb[0, 0] - 31 * 0.0625) < 1e-12
    # an all-zero block, and one whose scale vanishes in half precision: nothing is representable
    z = np.zeros((1, 64), dtype=np.float32)
    z[0, 32:] = 1.0e-9
    _, _, _, sqb = o.block_stats(z, 1, (), want_bfp4=True)
    assert sqb[0, 0] == 0.0 and abs(sqb[0, 1] - 32 * np.float64(np.float32(1.0e-9)) ** 2) < 1e-30


# --------------------------------------------------------------------------- product

def pin_equivalent_transformation(o):
    # Sec. 2 / Eq. (1): (X R)(W R)^T = X W^T for orthogonal R, before quantization
    rng = np.random.default_rng(12)
    X = rng.standard_normal((6, 128))
    W = rng.standard_normal((5, 128))
    ref = X @ W.T
    for B in (32, 64, 128):
        got = o.matmul_nt_f64(o.rotate_dense_f64(X, B), o.rotate_dense_f64(W, B))
        assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    assert np.allclose(o.matmul_nt_f64(X, W), ref, rtol=0, atol=1e-12)


def pin_gemm_against_brute_force(o):
    g = golden_e2m1()
    rng = np.random.default_rng(13)
    M, N, K = 5, 7, 96
    aq = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    wq = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    as_ = rng.integers(120, 135, size=(M, K // 32), dtype=np.uint8)
    ws = rng.integers(120, 135, size=(N, K // 32), dtype=np.uint8)
    lut = np.array([g[c] for c in range(16)])

    def deq(q, s):
        return lut[_unpack(q)] * np.repeat(2.0 ** (s.astype(np.float64) - 127), 32, axis=1)

    A, W = deq(aq, as_), deq(wq, ws)
    assert np.array_equal(o.mxfp4_dequantize(aq, as_), A)
    y, bound = o.mxfp4_gemm(aq, as_, wq, ws)
    want = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            for k in range(K):
                want[m, n] += A[m, k] * W[n, k]
    assert np.allclose(y, want, rtol=1e-14, atol=0)
    assert np.allclose(bound, np.abs(A) @ np.abs(W).T, rtol=1e-14)
    # a row subset returns exactly those rows
    ys, _ = o.mxfp4_gemm(aq, as_, wq, ws, rows=[3, 0])
    assert np.array_equal(ys, y[[3, 0]])
    # all ones (code 2, byte 127) -> Y = K exactly
    ones_q = np.full((2, K // 2), 0x22, dtype=np.uint8)
    ones_s = np.full((2, K // 32), 127, dtype=np.uint8)
    y1, _ = o.mxfp4_gemm(ones_q, ones_s, ones_q, ones_s)
    assert (y1 == K).all()
    # bumping one scale byte doubles exactly that group's contribution
    s2 = ones_s.copy()
    s2[1, 2] += 1
    y2, _ = o.mxfp4_gemm(ones_q, s2, ones_q, ones_s)
    assert (y2[0] == K).all() and (y2[1] == K + 32).all()
    # one-hot A (element 33 = 6, high nibble of byte 16) picks a single product
    oh = np.zeros((1, K // 2), dtype=np.uint8)
    oh[0, 16] = 0x70
    yo, _ = o.mxfp4_gemm(oh, ones_s[:1], wq, ws)
    assert np.array_equal(yo[0], 6.0 * W[:, 33])


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
