"""fp64 oracle of the memory-bound kernels (test infrastructure only).

The paper lists `add`, `silu`, `softmax` and `rms_norm` among its kernels (Section 5.1) and
prints the arrangement of the first (Section 4.1: every vector tiled into blocks of
BLOCK_SIZE, application `output = input + other`).  Each function below is the plain
definition of the operation, evaluated in fp64 on the exactly decoded 16-bit inputs:

  add       out[i] = x[i] + y[i]
  silu      out[i] = x[i] / (1 + exp(-x[i]))
  softmax   out[r, c] = exp(x[r, c] - max_c x[r, :]) / sum_c exp(x[r, c] - max_c x[r, :])
  rms_norm  out[r, c] = x[r, c] / sqrt(mean_c x[r, :]^2 + eps)            (no weight)

`encode` rounds an fp64 array once (nearest even) to a 16-bit format; it exists so that tests
can state what a correctly rounded result is, independently of the input generators.
"""
from __future__ import annotations

import numpy as np

from . import numeric as _num


def decode(bits, dtype: str) -> np.ndarray:
    return _num.decode(bits, dtype)


def encode(x, dtype: str) -> np.ndarray:
    """fp64 -> 16-bit patterns, one round-to-nearest-even step, computed on the integers."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)            # numpy rounds binary64 -> binary16 directly
    if dtype == "bf16":
        b = x.view(np.uint64)
        sign = (b >> np.uint64(63)).astype(np.uint16) << np.uint16(15)
        mag = np.abs(x)
        out = np.zeros(x.shape, dtype=np.uint16)
        nz = mag > 0
        # bf16 = 8 exponent bits (bias 127), 7 fraction bits; spacing of normal numbers in [2^e, 2^(e+1)) is 2^(e-7)
        _, ex = np.frexp(mag)                                   # mag = m * 2^ex, m in [0.5, 1): binade exponent ex - 1
        e = np.clip(ex.astype(np.int64) - 1, -126, 127)         # subnormals share the spacing of the smallest normal binade
        q = np.ldexp(mag, (7 - e).astype(np.int64))             # in units of the spacing: [128, 256) for normals
        r = np.rint(q)                                          # rint rounds half to even
        val = r.astype(np.int64)
        # value = val * 2^(e-7); encode: normals val in [128,256] (256 -> next binade), subnormals val < 128 at e = -126
        exp_field = np.where(val >= 128, e + 127, 0)
        bump = val == 256
        exp_field = np.where(bump, exp_field + 1, exp_field)
        frac = np.where(bump, 0, np.where(val >= 128, val - 128, val))
        code = (exp_field << 7) | frac
        code = np.where(exp_field >= 255, 0x7F80, code)         # overflow -> infinity
        out[nz] = code[nz].astype(np.uint16)
        out = out | sign
        out = np.where(np.isnan(x), np.uint16(0x7FC0), out)
        out = np.where(np.isinf(x), sign | np.uint16(0x7F80), out)
        return out.astype(np.uint16)
    raise ValueError(dtype)


def add(x_bits, y_bits, dtype: str) -> np.ndarray:
    """Section 4.1: output = input + other, element by element (exact in fp64 for 16-bit inputs)."""
    return decode(x_bits, dtype) + decode(y_bits, dtype)


def silu(x_bits, dtype: str) -> np.ndarray:
    x = decode(x_bits, dtype)
    return x / (1.0 + np.exp(-x))


def softmax(x_bits, dtype: str) -> np.ndarray:
    """Along the last axis."""
    x = decode(x_bits, dtype)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def rms_norm(x_bits, dtype: str, eps: float) -> np.ndarray:
    """Along the last axis, without a weight."""
    x = decode(x_bits, dtype)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
