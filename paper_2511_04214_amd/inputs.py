"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on LLaMA / Mistral / Qwen activations and weights (Sec. 3, Sec. 5).
None of those is available here; these generators stand in for them.  They reproduce the
structure the paper describes for LLM activations (Sec. 4.1-4.2): heavy tails, a few
outlier channels that carry most of the energy, most 32-groups "regular".

This module holds data generation only -- none of the method's arithmetic (no rotation,
no scale rule, no E2M1 encoding).  Both the HIP path and the CPU oracle are fed from
here.  numpy only; no torch import.

bf16 tensors are returned as uint16 arrays of bit patterns.
"""
import numpy as np

# name -> workload.  B lists the rotation block sizes exercised; "K" means full-K.
CONFIGS = {
    "tiny": dict(M=16, K=256, N=256, dtype="f32", dist="normal", outlier_channels=[3, 77],
                 outlier_scale=20.0, B=[32], seed=0),
    "llama1b_up": dict(M=2048, K=2048, N=8192, dtype="bf16", dist="student_t4", outlier_frac=0.01,
                       outlier_scale=20.0, B=[32], seed=1),
    "down_sweep": dict(M=4096, K=8192, N=2048, dtype="bf16", dist="student_t4", outlier_frac=0.01,
                       outlier_scale=20.0, B=[32, 64, 128, 8192], seed=2),
    "mlp8b": dict(M=8192, K=4096, N=14336, dtype="bf16", dist="student_t4", outlier_frac=0.005,
                  outlier_scale=50.0, B=[32], seed=3),
    "decode": dict(M=16384, K=8192, N=28672, dtype="bf16", dist="student_t4", outlier_frac=0.01,
                   outlier_scale=20.0, B=[32], seed=4, gemm_M=[1, 4, 16]),
}
CONFIG_ORDER = ["tiny", "llama1b_up", "down_sweep", "mlp8b", "decode"]

W_STD = 0.02  # weights ~ N(0, std = 0.02)


def f32_to_bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even (finite values)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _streams(seed):
    sx, sw = np.random.SeedSequence(seed).spawn(2)
    return np.random.default_rng(sx), np.random.default_rng(sw)


def outlier_channels(cfg, K=None):
    """Indices of the activation channels that are scaled up (whole columns)."""
    K = cfg["K"] if K is None else K
    if "outlier_channels" in cfg:
        return np.array([c for c in cfg["outlier_channels"] if c < K], dtype=np.int64)
    rng = np.random.default_rng(np.random.SeedSequence([cfg["seed"], 7]))
    n = int(round(cfg["outlier_frac"] * K))
    return np.sort(rng.choice(K, size=n, replace=False))


def make_x(cfg, M=None, K=None, chunk_rows=1024):
    """Activations [M, K]: float32 for 'f32' configs, uint16 bf16 bits otherwise.

    M / K override the config's shape (used for reduced and ragged parity cases; the
    distribution and the outlier-channel fraction stay those of the config).
    """
    M = cfg["M"] if M is None else M
    K = cfg["K"] if K is None else K
    rng, _ = _streams(cfg["seed"])
    cols = outlier_channels(cfg, K)
    out = np.empty((M, K), dtype=np.float32)
    for r0 in range(0, M, chunk_rows):
        r1 = min(M, r0 + chunk_rows)
        if cfg["dist"] == "normal":
            blk = rng.standard_normal((r1 - r0, K))
        else:
            blk = rng.standard_t(4, size=(r1 - r0, K))
        blk[:, cols] *= cfg["outlier_scale"]
        out[r0:r1] = blk.astype(np.float32)
    return out if cfg["dtype"] == "f32" else f32_to_bf16_bits(out)


def make_w(cfg, N=None, K=None, chunk_rows=2048):
    """Weights [N, K] ~ N(0, 0.02), same dtype convention as make_x."""
    N = cfg["N"] if N is None else N
    K = cfg["K"] if K is None else K
    _, rng = _streams(cfg["seed"])
    out = np.empty((N, K), dtype=np.float32)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        out[r0:r1] = rng.standard_normal((r1 - r0, K), dtype=np.float32) * np.float32(W_STD)
    return out if cfg["dtype"] == "f32" else f32_to_bf16_bits(out)


def random_mxfp4(rows, K, seed, scale_lo=110, scale_hi=135):
    """Uniformly random packed E2M1 codes [rows, K/2] and E8M0 bytes [rows, K/32].

    For GEMM parity cases that should not depend on the quantizer: every code value and
    a band of scale bytes around 2^0 appear.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 11]))
    codes = rng.integers(0, 256, size=(rows, K // 2), dtype=np.uint8)
    scales = rng.integers(scale_lo, scale_hi + 1, size=(rows, K // 32), dtype=np.uint8)
    return codes, scales
