"""The seeded synthetic inputs are reproducible bit for bit (tests/golden/input_sha256.txt), have
the structure their recipe states (outlier channels, heavy tails, weight scale), and the bf16
helpers of the input module agree with the oracle's conversions."""
import hashlib
import os
import sys

import numpy as np

from paper_2511_04214_amd import inputs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "input_sha256.txt")


def digests(name):
    cfg = inputs.CONFIGS[name]
    return {"x": hashlib.sha256(np.ascontiguousarray(inputs.make_x(cfg)).tobytes()).hexdigest(),
            "w": hashlib.sha256(np.ascontiguousarray(inputs.make_w(cfg)).tobytes()).hexdigest()}


def test_inputs_are_reproducible():
    want = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            cfg, buf, h = line.split()
            want.setdefault(cfg, {})[buf] = h
    assert set(want) == {"tiny", "llama1b_up"}
    for cfg in want:
        assert digests(cfg) == want[cfg], cfg


def test_inputs_have_the_stated_structure(orc):
    cfg = inputs.CONFIGS["llama1b_up"]
    x = orc.bf16_to_f32(inputs.make_x(cfg))
    w = orc.bf16_to_f32(inputs.make_w(cfg))
    ch = inputs.outlier_channels(cfg)
    assert len(ch) == round(0.01 * cfg["K"]) or len(ch) >= 1
    rms = np.sqrt((x.astype(np.float64) ** 2).mean(axis=0))
    others = np.delete(rms, ch)
    assert rms[ch].min() > 8 * np.median(others)                 # whole columns scaled up
    assert abs(w.std() - 0.02) < 0.002 and abs(w.mean()) < 1e-3
    kurt = ((x[:, np.delete(np.arange(cfg["K"]), ch)].astype(np.float64)) ** 4).mean() / others.mean() ** 4
    assert kurt > 4                                              # heavier tails than a normal (3)
    # the module's bf16 helpers are the oracle's conversions
    f = (np.random.default_rng(5).standard_normal(4096) * 3).astype(np.float32)
    bits = inputs.f32_to_bf16_bits(f)
    assert all(int(b) == orc.f32_to_bf16(v) for b, v in zip(bits[:512], f[:512]))
    assert np.array_equal(inputs.bf16_bits_to_f32(bits), orc.bf16_to_f32(bits))


if __name__ == "__main__" and "--write" in sys.argv:
    for name in ("tiny", "llama1b_up"):
        for buf, h in digests(name).items():
            print(name, buf, h)
