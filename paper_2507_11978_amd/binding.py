"""ctypes binding of include/nt.h -- argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnt.so")
MAX_DIMS, MAX_LEVELS = 8, 8

OP_TILE, OP_EXPAND, OP_SQUEEZE, OP_PERMUTE, OP_FLATTEN, OP_RAVEL, OP_DESCEND, OP_ASCEND = range(8)
_DTYPES = {"f16": 0, "bf16": 1, "f32": 2}
_STATUS = {1: "NT_ERR_INVALID_ARG", 2: "NT_ERR_SHAPE_MISMATCH", 3: "NT_ERR_UNSUPPORTED",
           4: "NT_ERR_BUFFER_TOO_SMALL", 5: "NT_ERR_DEVICE"}


class NtError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status
        self.name = _STATUS.get(status, str(status))


class TensorDesc(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("size", C.c_int64 * MAX_DIMS), ("stride", C.c_int64 * MAX_DIMS)]


class MetaOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n", C.c_int32), ("a", C.c_int64 * MAX_DIMS), ("b", C.c_int64 * MAX_DIMS),
                ("c", C.c_int64 * MAX_DIMS), ("d", C.c_int64 * MAX_DIMS), ("e", C.c_int64 * MAX_DIMS)]


class TileCfg(C.Structure):
    _fields_ = [("bm", C.c_int32), ("bn", C.c_int32), ("bk", C.c_int32)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


class _Recorder:
    """Stands in for the library while prepare() runs a binding function: notes the one C call it makes."""

    def __init__(self, lib):
        self._lib, self.call = lib, None

    def __getattr__(self, name):
        fn = getattr(self._lib, name)

        def note(*args):
            self.call = (fn, args)
            return 0
        return note


_recorder = None


def prepare(op, *args, **kwargs):
    """The C call that `op(*args, **kwargs)` (any launching function of this module) would make, marshalled once:
    returns a function of no arguments that makes it.  For loops that repeat one call on the same tensors (the tensors
    must stay alive and in place, the stream is the one current now): it skips the per-call marshalling, nothing else."""
    global _recorder
    lib = load()
    _recorder = _Recorder(lib)
    try:
        op(*args, **kwargs)
        fn, cargs = _recorder.call
    finally:
        _recorder = None
    keep = (args, kwargs)                                   # the tensors: their memory must outlive the prepared call

    def call():
        _check(fn(*cargs))
    call.keep = keep
    return call


def load():
    """Load libnt.so (built beforehand by paper_2507_11978_amd/build.py); never falls back."""
    global _lib
    if _recorder is not None:
        return _recorder
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_2507_11978_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    P, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    D, O = C.POINTER(TensorDesc), C.POINTER(MetaOp)
    L.nt_arrange_levels.argtypes = [D, O, i32, P, P, P]
    L.nt_arrange_tile.argtypes = [D, O, i32, i64, P, i32, P, P, C.c_size_t, P, P, P, P]
    arr_tail = [TileCfg, P, P, i32, i64, i64, P, P, C.c_size_t, P]
    L.nt_arrange_gemm.argtypes = [D, D, D] + arr_tail
    L.nt_arrange_bmm.argtypes = [D, D, D] + arr_tail
    L.nt_arrange_conv2d.argtypes = [D, D, D, i32, i32, i32, i32] + arr_tail
    L.nt_program_order.argtypes = [i64, i64, i64, P]
    L.nt_tile_supported.argtypes = [TileCfg]
    L.nt_tile_supported.restype = i32
    L.nt_gemm.argtypes = [P, D, P, D, P, D, i32, i32, TileCfg, P]
    L.nt_gemm_noalloc.argtypes = [P, D, P, D, P, D, i32, i32, TileCfg, P]
    L.nt_bmm.argtypes = [P, D, P, D, P, D, i32, i32, TileCfg, P]
    L.nt_addmm.argtypes = [P, D, P, D, P, D, P, D, C.c_float, C.c_float, i32, i32, TileCfg, P]
    L.nt_addmm_act.argtypes = [P, D, P, D, P, D, P, D, C.c_float, C.c_float, i32, i32, i32, TileCfg, P]
    L.nt_conv2d_implicit.argtypes = [P, D, P, D, P, D, i32, i32, i32, i32, i32, i32, TileCfg, P]
    L.nt_matmul_views.argtypes = [P, D, O, i32, P, D, O, i32, P, D, O, i32, i32, i32, TileCfg, P]
    L.nt_sdpa.argtypes = [P, D, P, D, P, D, P, D, C.c_float, i32, P]
    L.nt_add.argtypes = [P, D, P, D, P, D, i32, i64, P]
    L.nt_silu.argtypes = [P, D, P, D, i32, i64, P]
    L.nt_softmax.argtypes = [P, D, P, D, i32, P]
    L.nt_rms_norm.argtypes = [P, D, P, D, C.c_float, i32, P]
    L.nt_mfma_probe.argtypes = [P, i64, i32, i32, i32, P, P]
    L.nt_trace_tile.argtypes = [i32, D, D, D, i32, i32, i32, i32, TileCfg, i32, i64, i64, P, P, C.c_size_t, P]
    L.nt_trace_loader_slice.argtypes = [i32, P, D, P, D, D, i32, i32, i32, i32, i32, i32, TileCfg, i32, i64, i64, P, C.c_size_t, P]
    for name in ("nt_arrange_levels", "nt_arrange_tile", "nt_arrange_gemm", "nt_arrange_bmm", "nt_arrange_conv2d",
                 "nt_program_order", "nt_gemm", "nt_gemm_noalloc", "nt_addmm", "nt_addmm_act", "nt_bmm", "nt_conv2d_implicit", "nt_trace_tile", "nt_trace_loader_slice",
                 "nt_add", "nt_silu", "nt_softmax", "nt_rms_norm", "nt_matmul_views", "nt_sdpa", "nt_mfma_probe"):
        getattr(L, name).restype = i32
    L.nt_last_kernel_path.restype = i32
    L.nt_last_k_split.restype = i32
    L.nt_last_error.restype = C.c_char_p
    L.nt_version.restype = C.c_char_p
    _lib = L
    return L


def _check(st: int):
    if st != 0:
        raise NtError(st, load().nt_last_error().decode())


def version() -> str:
    return load().nt_version().decode()


# ------------------------------------------------------------------ marshalling helpers
def make_desc(shape: Sequence[int], strides: Sequence[int] | None = None) -> TensorDesc:
    shape = [int(s) for s in shape]
    if strides is None:
        strides, acc = [], 1
        for s in reversed(shape):
            strides.append(acc)
            acc *= max(s, 1)
        strides.reverse()
    d = TensorDesc()
    d.ndim = len(shape)
    for i, (s, t) in enumerate(zip(shape, strides)):
        d.size[i], d.stride[i] = int(s), int(t)
    return d


_desc_cache: dict = {}


def _desc_of(t) -> TensorDesc:
    """Descriptor of a torch tensor (sizes and element strides) or a (shape, strides) pair.  Descriptors of tensors
    are read-only inputs of the library and are kept by (shape, strides): a call on a layout seen before builds none."""
    if isinstance(t, TensorDesc):
        return t
    if hasattr(t, "data_ptr"):
        key = (tuple(t.shape), tuple(t.stride()))
        d = _desc_cache.get(key)
        if d is None:
            if len(_desc_cache) > 4096:
                _desc_cache.clear()
            d = _desc_cache[key] = make_desc(*key)
        return d
    return make_desc(*t)


def make_ops(ops) -> tuple:
    """ops: tuples ("tile", shape[, strides[, pad[, dilation]]]), ("expand", shape), ("squeeze", dim),
    ("permute", order), ("flatten", start, end), ("ravel",), ("descend",), ("ascend",);
    pad is a sequence of (low, high) pairs."""
    arr = (MetaOp * max(len(ops), 1))()
    for o, op in zip(arr, ops):
        kind = op[0]
        vals = {"a": [], "b": [], "c": [], "d": [], "e": []}
        if kind == "tile":
            o.kind, vals["a"] = OP_TILE, list(op[1])
            if len(op) > 2 and op[2] is not None:
                vals["b"] = list(op[2])
            if len(op) > 3 and op[3] is not None:
                vals["c"], vals["d"] = [p[0] for p in op[3]], [p[1] for p in op[3]]
            if len(op) > 4 and op[4] is not None:
                vals["e"] = list(op[4])
        elif kind == "expand":
            o.kind, vals["a"] = OP_EXPAND, list(op[1])
        elif kind == "squeeze":
            o.kind, vals["a"] = OP_SQUEEZE, [op[1]]
        elif kind == "permute":
            o.kind, vals["a"] = OP_PERMUTE, list(op[1])
        elif kind == "flatten":
            o.kind, vals["a"] = OP_FLATTEN, [op[1], op[2]]
        elif kind == "ravel":
            o.kind = OP_RAVEL
        elif kind == "descend":
            o.kind = OP_DESCEND
        elif kind == "ascend":
            o.kind = OP_ASCEND
        else:
            raise ValueError(kind)
        o.n = len(vals["a"])
        for f, v in vals.items():
            for i, x in enumerate(v):
                getattr(o, f)[i] = int(x)
    return arr, len(ops)


def _cfg(tile) -> TileCfg:
    if tile is None:
        return TileCfg(0, 0, 0)
    if isinstance(tile, TileCfg):
        return tile
    return TileCfg(*[int(x) for x in tile])


# ------------------------------------------------------------------------ arrangement
def arrange_levels(shape, strides, ops):
    d = make_desc(shape, strides)
    arr, n = make_ops(ops)
    nl = C.c_int32()
    nd = (C.c_int32 * MAX_LEVELS)()
    sh = (C.c_int64 * (MAX_LEVELS * MAX_DIMS))()
    _check(load().nt_arrange_levels(C.byref(d), arr, n, C.byref(nl), nd, sh))
    return [tuple(sh[l * MAX_DIMS + i] for i in range(nd[l])) for l in range(nl.value)]


def arrange_tile(shape, strides, ops, program_id, mid=(), capacity=None):
    """Returns (offsets int64[], mask uint8[], tile_shape, grid_shape)."""
    d = make_desc(shape, strides)
    arr, n = make_ops(ops)
    tshape, gshape = (C.c_int64 * MAX_DIMS)(), (C.c_int64 * MAX_DIMS)()
    tnd, gnd = C.c_int32(), C.c_int32()
    midv = (C.c_int64 * max(len(mid), 1))(*[int(m) for m in mid])
    L = load()
    _check(L.nt_arrange_tile(C.byref(d), arr, n, int(program_id), midv, len(mid), None, None, 0,
                             tshape, C.byref(tnd), gshape, C.byref(gnd)))
    ts = tuple(tshape[i] for i in range(tnd.value))
    gs = tuple(gshape[i] for i in range(gnd.value))
    count = int(np.prod(ts)) if ts else 1
    cap = count if capacity is None else capacity
    off = np.empty(max(cap, 1), dtype=np.int64)
    mask = np.empty(max(cap, 1), dtype=np.uint8)
    _check(L.nt_arrange_tile(C.byref(d), arr, n, int(program_id), midv, len(mid), off.ctypes.data, mask.ctypes.data,
                             cap, tshape, C.byref(tnd), gshape, C.byref(gnd)))
    return off[:count], mask[:count], ts, gs


def _arrange_problem(fn, descs, extra, tile, operand, program_id, k):
    grid = (C.c_int64 * 3)()
    kt = C.c_int64()
    tshape = (C.c_int64 * 2)()
    cfg = _cfg(tile)
    ds = [C.byref(_desc_of(d)) for d in descs]
    if operand is None:
        _check(fn(*ds, *extra, cfg, grid, C.byref(kt), 0, 0, 0, None, None, 0, None))
        return tuple(grid), kt.value
    _check(fn(*ds, *extra, cfg, grid, C.byref(kt), int(operand), int(program_id), int(k), None, None, 0, tshape))
    count = tshape[0] * tshape[1]
    off = np.empty(max(count, 1), dtype=np.int64)
    mask = np.empty(max(count, 1), dtype=np.uint8)
    _check(fn(*ds, *extra, cfg, grid, C.byref(kt), int(operand), int(program_id), int(k),
              off.ctypes.data, mask.ctypes.data, count, tshape))
    return off[:count], mask[:count], (tshape[0], tshape[1]), tuple(grid), kt.value


def arrange_gemm(dA, dB, dC, tile=None, operand=None, program_id=0, k=0):
    return _arrange_problem(load().nt_arrange_gemm, (dA, dB, dC), (), tile, operand, program_id, k)


def arrange_bmm(dA, dB, dC, tile=None, operand=None, program_id=0, k=0):
    return _arrange_problem(load().nt_arrange_bmm, (dA, dB, dC), (), tile, operand, program_id, k)


def arrange_conv2d(dx, dw, dy, stride=(1, 1), pad=(0, 0), tile=None, operand=None, program_id=0, k=0):
    extra = (int(stride[0]), int(stride[1]), int(pad[0]), int(pad[1]))
    return _arrange_problem(load().nt_arrange_conv2d, (dx, dw, dy), extra, tile, operand, program_id, k)


def program_order(batch: int, mt: int, nt: int) -> np.ndarray:
    out = np.empty(max(batch * mt * nt, 1), dtype=np.int64)
    _check(load().nt_program_order(batch, mt, nt, out.ctypes.data))
    return out[:batch * mt * nt]


def tile_supported(tile) -> bool:
    return bool(load().nt_tile_supported(_cfg(tile)))


# ---------------------------------------------------------------------------- kernels
_dtype_names: dict = {}


def _torch_dtype_name(t) -> str:
    if not _dtype_names:
        import torch
        _dtype_names.update({torch.float16: "f16", torch.bfloat16: "bf16", torch.float32: "f32"})
    return _dtype_names[t.dtype]


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _require_cuda(*ts):
    for t in ts:
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU (no CPU path exists)")


def gemm(A, B, Cout, tile=None, stream=None):
    """Cout[M,N] = A[M,K] @ B[K,N] on the GPU; tensors may be any strided views."""
    _require_cuda(A, B, Cout)
    _check(load().nt_gemm(A.data_ptr(), C.byref(_desc_of(A)), B.data_ptr(), C.byref(_desc_of(B)),
                          Cout.data_ptr(), C.byref(_desc_of(Cout)), _DTYPES[_torch_dtype_name(A)],
                          _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
    return Cout


def gemm_noalloc(A, B, Cout, tile=None, stream=None):
    """gemm() through the entry point that allocates no device memory (a k split uses the library's fixed scratch array)."""
    _require_cuda(A, B, Cout)
    _check(load().nt_gemm_noalloc(A.data_ptr(), C.byref(_desc_of(A)), B.data_ptr(), C.byref(_desc_of(B)),
                                  Cout.data_ptr(), C.byref(_desc_of(Cout)), _DTYPES[_torch_dtype_name(A)],
                                  _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
    return Cout


def mfma_probe(data, out, iters=2000, blocks=1024, stream=None):
    """Matrix-instruction-only loop on the 16-bit elements of `data` (see nt_mfma_probe); returns the flop count of the call."""
    _require_cuda(data, out)
    if out.numel() < blocks * 256:
        raise ValueError("out must hold blocks * 256 floats")
    _check(load().nt_mfma_probe(data.data_ptr(), data.numel(), _DTYPES[_torch_dtype_name(data)], int(iters), int(blocks), out.data_ptr(), _stream_ptr(stream)))
    return 2.0 * 16 * 16 * 32 * 64 * iters * 4 * blocks


PATH_GENERIC, PATH_STAGED, PATH_DIRECT, PATH_CONV, PATH_CONV_DIRECT, PATH_CONV_UNFOLD, PATH_CONV_TAP = 0, 1, 2, 3, 4, 5, 6


def last_kernel_path() -> int:
    """Kernel launched by this thread's last gemm / addmm / bmm / conv2d_implicit call (-1: none)."""
    return int(load().nt_last_kernel_path())


def last_k_split() -> int:
    """Into how many parts the reduction of this thread's last product / convolution call was split (1: not split)."""
    return int(load().nt_last_k_split())


ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "silu": 2, "gelu_tanh": 3}


def addmm(inp, A, B, Cout, alpha=1.0, beta=1.0, tile=None, stream=None, act=None):
    """Cout[M,N] = act(beta * inp + alpha * (A[M,K] @ B[K,N])); inp has Cout's dtype and is handed over as
    an [M, N] view (stride 0 along broadcast axes).  act: None, "relu", "silu" or "gelu_tanh" (fused into the
    epilogue); inp may be None when beta is 0."""
    if act is not None or inp is None:
        if act not in ACTIVATIONS:
            raise ValueError(f"unknown activation {act!r}")
        _require_cuda(A, B, Cout)
        view = None
        if inp is not None:
            _require_cuda(inp)
            if inp.dtype != Cout.dtype:
                raise ValueError("input must have the output's dtype")
            try:
                view = inp.expand(Cout.shape)
            except RuntimeError:
                view = inp
        _check(load().nt_addmm_act(view.data_ptr() if view is not None else None, C.byref(_desc_of(view)) if view is not None else None,
                                   A.data_ptr(), C.byref(_desc_of(A)), B.data_ptr(), C.byref(_desc_of(B)),
                                   Cout.data_ptr(), C.byref(_desc_of(Cout)), float(alpha), float(beta), ACTIVATIONS[act],
                                   _DTYPES[_torch_dtype_name(A)], _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
        return Cout
    _require_cuda(inp, A, B, Cout)
    if inp.dtype != Cout.dtype:
        raise ValueError("input must have the output's dtype")
    try:
        view = inp.expand(Cout.shape)
    except RuntimeError:
        view = inp                                    # not broadcastable: the library reports the mismatch
    _check(load().nt_addmm(view.data_ptr(), C.byref(_desc_of(view)), A.data_ptr(), C.byref(_desc_of(A)),
                           B.data_ptr(), C.byref(_desc_of(B)), Cout.data_ptr(), C.byref(_desc_of(Cout)),
                           float(alpha), float(beta), _DTYPES[_torch_dtype_name(A)],
                           _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
    return Cout


def add(x, y, out, block_size=0, stream=None):
    """out = x + y over 1-D tensors (16-bit floating point, any stride)."""
    _require_cuda(x, y, out)
    _check(load().nt_add(x.data_ptr(), C.byref(_desc_of(x)), y.data_ptr(), C.byref(_desc_of(y)), out.data_ptr(),
                         C.byref(_desc_of(out)), _DTYPES[_torch_dtype_name(x)], int(block_size), _stream_ptr(stream)))
    return out


def silu(x, out, block_size=0, stream=None):
    _require_cuda(x, out)
    _check(load().nt_silu(x.data_ptr(), C.byref(_desc_of(x)), out.data_ptr(), C.byref(_desc_of(out)),
                          _DTYPES[_torch_dtype_name(x)], int(block_size), _stream_ptr(stream)))
    return out


def softmax(x, out, stream=None):
    """Row-wise softmax of a 2-D tensor."""
    _require_cuda(x, out)
    _check(load().nt_softmax(x.data_ptr(), C.byref(_desc_of(x)), out.data_ptr(), C.byref(_desc_of(out)),
                             _DTYPES[_torch_dtype_name(x)], _stream_ptr(stream)))
    return out


def rms_norm(x, out, eps=1e-6, stream=None):
    """Row-wise x / sqrt(mean(x^2) + eps) of a 2-D tensor (no weight)."""
    _require_cuda(x, out)
    _check(load().nt_rms_norm(x.data_ptr(), C.byref(_desc_of(x)), out.data_ptr(), C.byref(_desc_of(out)),
                              float(eps), _DTYPES[_torch_dtype_name(x)], _stream_ptr(stream)))
    return out


def matmul_views(A, ops_a, B, ops_b, Cout, ops_c, tile=None, stream=None):
    """Cview = Aview @ Bview, each view being the tensor run through a meta-operation program
    (see make_ops) that ends in one level of rank 2 or 3."""
    _require_cuda(A, B, Cout)
    oa, na = make_ops(ops_a)
    ob, nb = make_ops(ops_b)
    oc, nc = make_ops(ops_c)
    _check(load().nt_matmul_views(A.data_ptr(), C.byref(_desc_of(A)), oa, na, B.data_ptr(), C.byref(_desc_of(B)), ob, nb,
                                  Cout.data_ptr(), C.byref(_desc_of(Cout)), oc, nc, _DTYPES[_torch_dtype_name(A)],
                                  _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
    return Cout


def sdpa(q, k, v, out, scale=0.0, stream=None):
    """out = softmax(scale * q @ k^T) @ v per (batch, head); tensors [batch, heads, seq, 64]; scale 0 = 1/sqrt(64)."""
    _require_cuda(q, k, v, out)
    _check(load().nt_sdpa(q.data_ptr(), C.byref(_desc_of(q)), k.data_ptr(), C.byref(_desc_of(k)), v.data_ptr(), C.byref(_desc_of(v)),
                          out.data_ptr(), C.byref(_desc_of(out)), float(scale), _DTYPES[_torch_dtype_name(q)], _stream_ptr(stream)))
    return out


def bmm(A, B, Cout, tile=None, stream=None):
    _require_cuda(A, B, Cout)
    _check(load().nt_bmm(A.data_ptr(), C.byref(_desc_of(A)), B.data_ptr(), C.byref(_desc_of(B)),
                         Cout.data_ptr(), C.byref(_desc_of(Cout)), _DTYPES[_torch_dtype_name(A)],
                         _DTYPES[_torch_dtype_name(Cout)], _cfg(tile), _stream_ptr(stream)))
    return Cout


def conv2d_implicit(x, w, y, stride=(1, 1), pad=(0, 0), tile=None, stream=None):
    _require_cuda(x, w, y)
    _check(load().nt_conv2d_implicit(x.data_ptr(), C.byref(_desc_of(x)), w.data_ptr(), C.byref(_desc_of(w)),
                                     y.data_ptr(), C.byref(_desc_of(y)), int(stride[0]), int(stride[1]),
                                     int(pad[0]), int(pad[1]), _DTYPES[_torch_dtype_name(x)],
                                     _DTYPES[_torch_dtype_name(y)], _cfg(tile), _stream_ptr(stream)))
    return y


def trace_loader_slice(kind, a, b, c, operand, program_id, slice_index, tile=None, stride=(1, 1), pad=(0, 0), stream=None):
    """What the matrix-instruction kernel's own loader leaves in LDS for one operand (0 = A, 1 = B) of program `program_id` and
    32-k slice `slice_index`: a numpy uint16 array [256, 32] of 16-bit patterns, row r = row of the operand's tile, 0xFFFF in
    the rows past the tile's.  a, b: device tensors (read); c: a tensor of the output's shape and dtype (not written)."""
    import numpy as np
    import torch
    kinds = {"gemm": 0, "bmm": 1, "conv2d": 2}
    _require_cuda(a, b, c)
    out = torch.full((256 * 32,), -1, dtype=torch.int16, device="cuda")
    _check(load().nt_trace_loader_slice(kinds[kind], a.data_ptr(), C.byref(_desc_of(a)), b.data_ptr(), C.byref(_desc_of(b)),
                                        C.byref(_desc_of(c)), int(stride[0]), int(stride[1]), int(pad[0]), int(pad[1]),
                                        _DTYPES[_torch_dtype_name(a)], _DTYPES[_torch_dtype_name(c)], _cfg(tile), int(operand),
                                        int(program_id), int(slice_index), out.data_ptr(), out.numel(), _stream_ptr(stream)))
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16).reshape(256, 32)


def trace_tile(kind, d0, d1, d2, tile, operand, program_id, k, stride=(1, 1), pad=(0, 0), stream=None):
    """Device twin of arrange_*: returns (offsets, mask) numpy arrays computed on the GPU."""
    import torch
    kinds = {"gemm": 0, "bmm": 1, "conv2d": 2}
    cfg = _cfg(tile)
    if cfg.bm == 0:
        raise ValueError("trace_tile needs an explicit tile")
    cap = max(cfg.bm * cfg.bk, cfg.bk * cfg.bn, cfg.bm * cfg.bn)
    off = torch.full((cap,), -7, dtype=torch.int64, device="cuda")
    mask = torch.full((cap,), 9, dtype=torch.uint8, device="cuda")
    _check(load().nt_trace_tile(kinds[kind], C.byref(_desc_of(d0)), C.byref(_desc_of(d1)), C.byref(_desc_of(d2)),
                                int(stride[0]), int(stride[1]), int(pad[0]), int(pad[1]), cfg, int(operand),
                                int(program_id), int(k), off.data_ptr(), mask.data_ptr(), cap, _stream_ptr(stream)))
    torch.cuda.synchronize()
    n = [cfg.bm * cfg.bk, cfg.bk * cfg.bn, cfg.bm * cfg.bn][operand]
    return off[:n].cpu().numpy(), mask[:n].cpu().numpy()
