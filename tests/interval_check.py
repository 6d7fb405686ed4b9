"""Interval parity for paths whose last bits are not defined by an operation sequence (the rotation
by caller-supplied blocks on the matrix cores, the gated activation on the hardware's exponential):
the interface states an error bound on the value that reaches the quantizer, and codes and scales
must be ones that SOME value within that bound produces under the oracle's scale rule and element
encoder.  Everything here runs on the CPU and calls only the oracle."""
import numpy as np


def outward32(lo, hi):
    """float64 interval -> float32 interval that contains it."""
    l32, h32 = lo.astype(np.float32), hi.astype(np.float32)
    l32 = np.where(l32.astype(np.float64) > lo, np.nextafter(l32, np.float32(-np.inf)), l32)
    h32 = np.where(h32.astype(np.float64) < hi, np.nextafter(h32, np.float32(np.inf)), h32)
    return l32, h32


def unpack(codes):
    out = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = codes & 0xF
    out[:, 1::2] = codes >> 4
    return out


def check_codes_within(orc, y, d, codes, scales):
    """y [M, K] fp64: centre of the value that reaches the quantizer, d >= 0 its half width.  codes /
    scales (row-major, from the GPU) must be reachable from a value in [y - d, y + d]."""
    M, K = y.shape
    lo32, hi32 = outward32(y - d, y + d)
    # scale bytes: the group maximum lies between max(|y| - d) and max(|y| + d)
    a_lo = np.maximum(np.abs(y) - d, 0).reshape(M, K // 32, 32).max(axis=2)
    a_hi = (np.abs(y) + d).reshape(M, K // 32, 32).max(axis=2)
    a_lo32, a_hi32 = outward32(a_lo, a_hi)
    a_lo32 = np.maximum(a_lo32, 0)
    s_lo = orc.mxfp4_quantize(np.ascontiguousarray(np.repeat(a_lo32, 32, axis=1)))[1]
    s_hi = orc.mxfp4_quantize(np.ascontiguousarray(np.repeat(a_hi32, 32, axis=1)))[1]
    assert ((s_lo <= scales) & (scales <= s_hi)).all(), "scale bytes outside the interval in %d groups" % int(
        ((scales < s_lo) | (scales > s_hi)).sum())
    # codes under the GPU's own scale bytes: between the codes of the interval's ends (the encoder is monotone)
    val = np.array([orc.e2m1_value(c) for c in range(16)])
    v_lo = val[unpack(orc.mxfp4_encode_with_scales(lo32, scales))]
    v_hi = val[unpack(orc.mxfp4_encode_with_scales(hi32, scales))]
    v = val[unpack(codes)]
    bad = (v < v_lo) | (v > v_hi)
    assert not bad.any(), "%d codes outside their interval, first at %s" % (int(bad.sum()), np.argwhere(bad)[0])
    assert not (unpack(codes) == 8).any()        # a zero magnitude is code 0


# ---- the gated activation h = silu(g) * u and what follows it

def swiglu_bound(g64, u64, exact):
    """The bound brq.h states for brq_swiglu: (8 + 2 |g|) 2^-24 |h| + 2^-119 |u|."""
    return (8.0 + 2.0 * np.abs(g64)) * 2.0 ** -24 * np.abs(exact) + 2.0 ** -119 * np.abs(u64)


def swiglu_h_interval(orc, g, u, h_bf16):
    """(lo, hi) fp64 arrays: every value the library's activation may hand to the rotation, for gate g and
    up u (float32, or uint16 bf16 bits): the exact value +- the stated bound, moved outward to fp32 and,
    for h_bf16, rounded to bf16 (rounding is monotone, so the ends bracket the result)."""
    from paper_2511_04214_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32
    exact = orc.swiglu_exact(g, u)
    g64 = (orc.bf16_to_f32(g) if g.dtype == np.uint16 else g).astype(np.float64)
    u64 = (orc.bf16_to_f32(u) if u.dtype == np.uint16 else u).astype(np.float64)
    d = swiglu_bound(g64, u64, exact)
    lo32, hi32 = outward32(exact - d, exact + d)
    if h_bf16:
        lo32, hi32 = bf16_bits_to_f32(f32_to_bf16_bits(lo32)), bf16_bits_to_f32(f32_to_bf16_bits(hi32))
    return lo32.astype(np.float64), hi32.astype(np.float64)


def check_swiglu_fused(orc, g, u, B, h_bf16, signs, codes, scales):
    """Codes and scales of brq_swiglu_rotate_quantize_fused against the fp64 definition: the activation
    lies in swiglu_h_interval; the rotation (exact in fp64 here) maps the box of a rotation block to
    centre +- sum of the half widths / sqrt(B), to which the fp32 butterfly adds at most
    (log2 B + 1) 2^-24 / sqrt(B) * sum |h| (each of its log2 B add stages and the final multiply rounds
    once, on partial sums bounded by sum |h|).  Returns the fractions of code bytes and of scale bytes
    that equal the oracle's nominal result (the definition rounded once, then rotated and quantized)."""
    M, K = g.shape
    lo, hi = swiglu_h_interval(orc, g, u, h_bf16)
    c, w = 0.5 * (lo + hi), 0.5 * (hi - lo)
    if B == 1:
        y, d = c, w
    else:
        if signs is not None:
            c = c * np.where(np.asarray(signs) < 0, -1.0, 1.0)[None, :]
        y = orc.rotate_dense_f64(c, B)
        wsum = w.reshape(M, K // B, B).sum(axis=2) / np.sqrt(B)
        asum = (np.abs(c) + w).reshape(M, K // B, B).sum(axis=2) / np.sqrt(B)
        d = np.repeat(wsum + (np.log2(B) + 1) * 2.0 ** -24 * asum, B, axis=1)
    check_codes_within(orc, y, d + 2.0 ** -140, codes, scales)
    rc, rs = orc.swiglu_rotate_quantize_fused(g, u, B, h_bf16=h_bf16, signs=signs)
    return float((rc == codes).mean()), float((rs == scales).mean())
