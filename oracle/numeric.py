"""fp64 numerical oracle (test infrastructure only): ctypes front end of nt_oracle.c.

Every function takes the 16-bit input patterns the GPU receives (numpy uint16 arrays,
possibly strided views) plus the format name, and returns fp64 results computed by the
plain definitions in nt_oracle.c:
  gemm / bmm        -- Section 4.2: C = sum_k A[:,k] B[k,:]
  conv2d            -- Section 4.3: direct cross-correlation the implicit GEMM must equal
  addmm             -- Section 5.1 task list: beta * input + alpha * (A . B)
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_DT = {"f16": 0, "bf16": 1}
_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        i64, p = C.c_int64, C.c_void_p
        L.nto_decode.argtypes = [p, i64, C.c_int, p]
        L.nto_decode.restype = None
        L.nto_gemm.argtypes = [p, i64, i64, p, i64, i64, p, i64, i64, i64, C.c_int, C.c_int]
        L.nto_gemm.restype = C.c_int
        L.nto_gemm_samples.argtypes = [p, i64, i64, p, i64, i64, i64, C.c_int, p, p, i64, p]
        L.nto_gemm_samples.restype = None
        L.nto_conv2d.argtypes = [p, p, p] + [i64] * 13 + [C.c_int, C.c_int]
        L.nto_conv2d.restype = None
        L.nto_conv2d_samples.argtypes = [p, p] + [i64] * 9 + [C.c_int, p, i64, p]
        L.nto_conv2d_samples.restype = None
        _lib = L
    return _lib


def _u16(a):
    a = np.asarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _strides_elems(a):
    return [s // a.itemsize for s in a.strides]


def decode(bits, dtype: str) -> np.ndarray:
    bits = np.ascontiguousarray(_u16(bits))
    out = np.empty(bits.shape, dtype=np.float64)
    lib().nto_decode(bits.ctypes.data, bits.size, _DT[dtype], out.ctypes.data)
    return out


def gemm(A, B, dtype: str, nthreads: int = 1) -> np.ndarray:
    """C[M,N] in fp64; A [M,K] and B [K,N] may be arbitrary strided uint16 views."""
    A, B = _u16(A), _u16(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.float64)
    sa, sb = _strides_elems(A), _strides_elems(B)
    rc = lib().nto_gemm(A.ctypes.data, sa[0], sa[1], B.ctypes.data, sb[0], sb[1],
                        out.ctypes.data, M, N, K, _DT[dtype], nthreads)
    if rc != 0:
        raise MemoryError("oracle gemm")
    return out


def bmm(A, B, dtype: str, nthreads: int = 1) -> np.ndarray:
    """Batched product: the same definition applied per batch index."""
    A, B = _u16(A), _u16(B)
    return np.stack([gemm(A[b], B[b], dtype, nthreads) for b in range(A.shape[0])])


def gemm_samples(A, B, dtype: str, ms, ns) -> np.ndarray:
    A, B = _u16(A), _u16(B)
    K = A.shape[1]
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    out = np.empty(ms.size, dtype=np.float64)
    sa, sb = _strides_elems(A), _strides_elems(B)
    lib().nto_gemm_samples(A.ctypes.data, sa[0], sa[1], B.ctypes.data, sb[0], sb[1], K, _DT[dtype],
                           ms.ctypes.data, ns.ctypes.data, ms.size, out.ctypes.data)
    return out


def addmm(inp, A, B, dtype: str, alpha: float = 1.0, beta: float = 1.0, inp_dtype: str | None = None,
          nthreads: int = 1) -> np.ndarray:
    """beta * input + alpha * (A . B) in fp64 (the addmm task of Section 5.1; the definition is the
    one the paper's PyTorch baseline evaluates).  `inp` broadcasts against [M, N]; it is either an
    fp64 / fp32 array of exact values or 16-bit patterns in format `inp_dtype`.  beta = 0 drops
    the input altogether (its values, NaN included, do not reach the result)."""
    prod = gemm(A, B, dtype, nthreads)
    if beta == 0:
        return float(alpha) * prod
    inp = np.asarray(inp)
    vals = decode(inp, inp_dtype) if inp.dtype == np.uint16 else inp.astype(np.float64)
    return float(beta) * np.broadcast_to(vals, prod.shape) + float(alpha) * prod


def activation(x, act) -> np.ndarray:
    """The activations an epilogue may fuse, by their textbook definitions, in fp64:
    relu max(x, 0); silu x / (1 + exp(-x)); gelu_tanh 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    x = np.asarray(x, dtype=np.float64)
    if act in (None, "none"):
        return x
    if act == "relu":
        return np.maximum(x, 0.0)
    if act == "silu":
        return x / (1.0 + np.exp(-x))
    if act == "gelu_tanh":
        return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))
    raise ValueError(act)


def addmm_act(inp, A, B, dtype: str, act, alpha: float = 1.0, beta: float = 1.0, inp_dtype: str | None = None,
              nthreads: int = 1) -> np.ndarray:
    """act(beta * input + alpha * (A . B)): addmm followed by an element-wise activation."""
    return activation(addmm(inp, A, B, dtype, alpha, beta, inp_dtype, nthreads), act)


def conv_out_size(H: int, R: int, stride: int, pad: int) -> int:
    """P = floor((H + 2*pad - R) / stride) + 1: number of filter positions that fit."""
    return (H + 2 * pad - R) // stride + 1


def conv2d(X, Wt, dtype: str, stride=(1, 1), pad=(0, 0), nthreads: int = 1) -> np.ndarray:
    X = np.ascontiguousarray(_u16(X))
    Wt = np.ascontiguousarray(_u16(Wt))
    N, Cc, H, W = X.shape
    F, C2, R, S = Wt.shape
    assert Cc == C2
    P = conv_out_size(H, R, stride[0], pad[0])
    Q = conv_out_size(W, S, stride[1], pad[1])
    Y = np.empty((N, F, P, Q), dtype=np.float64)
    lib().nto_conv2d(X.ctypes.data, Wt.ctypes.data, Y.ctypes.data, N, Cc, H, W, F, R, S, P, Q,
                     stride[0], stride[1], pad[0], pad[1], _DT[dtype], nthreads)
    return Y


def conv2d_samples(X, Wt, dtype: str, idx, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    X = np.ascontiguousarray(_u16(X))
    Wt = np.ascontiguousarray(_u16(Wt))
    _, Cc, H, W = X.shape
    _, _, R, S = Wt.shape
    idx = np.ascontiguousarray(idx, dtype=np.int64).reshape(-1, 4)
    out = np.empty(idx.shape[0], dtype=np.float64)
    lib().nto_conv2d_samples(X.ctypes.data, Wt.ctypes.data, Cc, H, W, R, S,
                             stride[0], stride[1], pad[0], pad[1], _DT[dtype],
                             idx.ctypes.data, idx.shape[0], out.ctypes.data)
    return out
