"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random numbers and rounds them once to the 16-bit storage
format; it contains none of the arithmetic of the method under test.  Both the CPU
oracle and the HIP path consume the *same* uint16 bit patterns produced here, so the
input quantisation is common to both sides and never shows up as a difference.

Formats: "f16" is IEEE binary16, "bf16" is the upper half of IEEE binary32; both
are produced with round-to-nearest-even.
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f16", "bf16")


def round_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32/fp64 array to `dtype` (RNE) and return the uint16 bit patterns."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        b = x32.view(np.uint32)
        lsb = (b >> np.uint32(16)) & np.uint32(1)
        r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
        return r.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def uniform_bits(shape, dtype: str, seed: int) -> np.ndarray:
    """i.i.d. uniform[-1, 1) entries, rounded once to `dtype`."""
    rng = np.random.default_rng(seed)
    x = rng.random(size=shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    return round_to_bits(x, dtype)


def normal_bits(shape, dtype: str, seed: int, scale: float) -> np.ndarray:
    """i.i.d. N(0, 1) * scale entries, rounded once to `dtype`."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(scale)
    return round_to_bits(x, dtype)


def small_int_bits(shape, dtype: str, seed: int, lo: int = -3, hi: int = 4) -> np.ndarray:
    """Small integers in [lo, hi): exactly representable, so products and sums are exact."""
    rng = np.random.default_rng(seed)
    x = rng.integers(lo, hi, size=shape).astype(np.float32)
    return round_to_bits(x, dtype)


def gemm_inputs(M: int, N: int, K: int, dtype: str, seed: int, dist: str, batch: int | None = None):
    """A[M,K] and B[K,N] (or [batch,M,K], [batch,K,N]) as uint16 bit patterns.

    dist = "uniform"  -> U[-1,1)            (the 256^3 and ragged bf16 workloads)
    dist = "normal"   -> N(0,1)/sqrt(K)     (the 4096^3, 8192^3 and batched workloads)
    """
    sa = (M, K) if batch is None else (batch, M, K)
    sb = (K, N) if batch is None else (batch, K, N)
    if dist == "uniform":
        return uniform_bits(sa, dtype, seed), uniform_bits(sb, dtype, seed + 1)
    if dist == "normal":
        s = 1.0 / np.sqrt(K)
        return normal_bits(sa, dtype, seed, s), normal_bits(sb, dtype, seed + 1, s)
    if dist == "int":
        return small_int_bits(sa, dtype, seed), small_int_bits(sb, dtype, seed + 1)
    raise ValueError(dist)


def conv_inputs(N: int, C: int, H: int, W: int, K: int, R: int, S: int, dtype: str, seed: int,
                dist: str = "normal"):
    """NCHW input and KCRS filter, N(0,1)/sqrt(C*R*S), as uint16 bit patterns."""
    if dist == "int":
        return (small_int_bits((N, C, H, W), dtype, seed), small_int_bits((K, C, R, S), dtype, seed + 1))
    s = 1.0 / np.sqrt(C * R * S)
    return (normal_bits((N, C, H, W), dtype, seed, s), normal_bits((K, C, R, S), dtype, seed + 1, s))


# The benchmark / parity configurations (shapes, distributions and seeds of the workloads).
CONFIGS = {
    "c1_f16_256": dict(kind="gemm", M=256, N=256, K=256, dtype="f16", out="f16", dist="uniform", seed=0,
                       tile=(64, 64, 32)),
    "c2_f16_4096": dict(kind="gemm", M=4096, N=4096, K=4096, dtype="f16", out="f16", dist="normal", seed=0),
    "c3_bf16_ragged": dict(kind="gemm", M=3001, N=5003, K=1999, dtype="bf16", out="f32", dist="uniform", seed=0),
    "c4_f16_bmm": dict(kind="bmm", batch=32, M=2048, N=2048, K=512, dtype="f16", out="f16", dist="normal", seed=0),
    "p_f16_8192": dict(kind="gemm", M=8192, N=8192, K=8192, dtype="f16", out="f16", dist="normal", seed=0),
    "f1_f16_addmm": dict(kind="addmm", M=4096, N=4096, K=4096, dtype="f16", out="f16", dist="normal", seed=0, alpha=1.0, beta=1.0),
    "f1_f16_bias_gelu": dict(kind="addmm", M=4096, N=4096, K=4096, dtype="f16", out="f16", dist="normal", seed=0, alpha=1.0, beta=1.0,
                             bias="row", act="gelu_tanh"),
    "f3_f16_add": dict(kind="add", n=16777216, dtype="f16", out="f16", seed=0),
    "f3_f16_silu": dict(kind="silu", n=16777216, dtype="f16", out="f16", seed=0),
    "f3_f16_softmax": dict(kind="softmax", rows=4096, cols=4096, dtype="f16", out="f16", seed=0),
    "f3_f16_rms_norm": dict(kind="rms_norm", rows=4096, cols=4096, dtype="f16", out="f16", seed=0, eps=1e-6),
    "f4_f16_sdpa": dict(kind="sdpa", B=4, H=48, S=1024, D=64, dtype="f16", out="f16", seed=0),
    "f4_bf16_sdpa": dict(kind="sdpa", B=4, H=48, S=1024, D=64, dtype="bf16", out="bf16", seed=0),
    "f4_f16_sdpa_4k": dict(kind="sdpa", B=1, H=48, S=4096, D=64, dtype="f16", out="f16", seed=0),
    "c5_f16_conv": dict(kind="conv", N=32, C=256, H=56, W=56, K=256, R=3, S=3, stride=1, pad=1,
                        dtype="f16", out="f16", seed=0),
    # the same convolution with its filter stored channels-last, (f, r, s, c): the order in which the kernel for 256 filters walks
    # the reduction, so that it reads the filter as it is instead of copying it first
    "c5_f16_conv_krsc": dict(kind="conv", filter="krsc", N=32, C=256, H=56, W=56, K=256, R=3, S=3, stride=1, pad=1,
                             dtype="f16", out="f16", seed=0),
    # the same convolution written by the caller as an arrangement (Section 4.3) and run through the view interface
    "f2_f16_conv_views": dict(kind="conv", via="views", N=32, C=256, H=56, W=56, K=256, R=3, S=3, stride=1, pad=1,
                              dtype="f16", out="f16", seed=0),
    # the conv2d task of the paper's kernel list (Section 5.1): few output tiles, a long reduction
    "c6_f16_conv_paper": dict(kind="conv", N=4, C=512, H=14, W=14, K=512, R=3, S=3, stride=1, pad=0,
                              dtype="f16", out="f16", seed=0),
}
