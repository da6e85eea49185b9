"""fp64 oracle of scaled dot-product attention (test infrastructure only).

The paper lists `scaled_dot_product_attention` among its kernels and states that both of its
implementations follow the FlashAttention-2 algorithm (Section 5.1); that algorithm reaches,
up to rounding, the plain definition below, so the definition is the oracle:

    O[b, h, i, :] = sum_j softmax_j( scale * <Q[b, h, i, :], K[b, h, j, :]> ) * V[b, h, j, :]

No mask, no dropout (the task passes three tensors only).  Inputs are the 16-bit patterns the GPU
receives, decoded exactly; everything is evaluated in fp64 with numpy.
"""
from __future__ import annotations

import numpy as np

from . import numeric as _num


def sdpa(q_bits, k_bits, v_bits, dtype: str, scale: float | None = None) -> np.ndarray:
    """q [..., Sq, D], k [..., Sk, D], v [..., Sk, Dv] -> [..., Sq, Dv] in fp64."""
    q, k, v = (_num.decode(np.ascontiguousarray(x), dtype) for x in (q_bits, k_bits, v_bits))
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[-1])
    s = np.matmul(q, np.swapaxes(k, -1, -2)) * scale
    p = np.exp(s - s.max(axis=-1, keepdims=True))
    p /= p.sum(axis=-1, keepdims=True)
    return np.matmul(p, v)
