"""Arrangement enumerator of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

A hierarchical tensor (Section 3.1.2) is kept as a list of *levels*, outermost first,
each level being a shape tuple, together with an index function that takes one index
per dimension of every level and returns the coordinates in the source tensor plus a
validity flag.  Every meta-operation of Table 1 returns a new hierarchical tensor whose
index function is the old one composed with a local rule; nothing is simplified or
fused, so each rule can be read against the paper on its own:

  tile      Algorithm 1 for the shapes (outer = ceil(size / tile), inner = tile); the
            `strides` argument is the interval between tiles (Section 3.1.3), default
            = tile shape, -1 = default.  Element t of tile o sits at o*stride + t of the
            tiled dimension and is valid only inside it: this is where masks come from.
  expand    a singleton dimension is repeated; its index is ignored.
  squeeze   a singleton dimension is removed.
  permute   dimensions are reordered.
  flatten   dimensions [start_dim, end_dim) of one level are merged, first one slowest.
  ravel     all levels are concatenated into one level (Section 3.1.3, the (N,P,Q) +
            (C,R,S) -> (N,P,Q,C,R,S) example).
  .dtype    the next-inner level (Section 3.1.2); an operation called on it acts there.

Tile-to-program mapping (Section 3.2.1): the outermost level's shape is the grid, one
program per outermost index, and all arranged parameters must agree on that shape.
Source-to-target mapping (Section 3.2.2): for a program and an index into the levels
between outermost and innermost, the innermost level's elements are enumerated in
row-major order as (element offset, mask).

Readings adopted where the paper is silent (conventions of this repository):
  * program id -> outermost index is row-major (last dimension fastest);
  * a strided tile over size S with tile T, stride st has ceil((S - T) / st) + 1 outer
    positions -- this equals Algorithm 1 for st == T and H - R + 1 for st == 1;
  * flatten's end_dim is exclusive (the printed conv shapes require it);
  * a tile shape of -1 means the whole dimension;
  * masked elements report offset -1 and read as zero;
  * optional low/high padding of a tile (needed for padded convolution) shifts the
    tile origin by -pad_lo and extends the tiled extent to S + pad_lo + pad_hi.
"""
from __future__ import annotations

import numpy as np


class ShapeMismatch(ValueError):
    """An arrangement that is not proper (Section 3.2.1) or an illegal meta-operation."""


def _ceil_div(a: int, b: int) -> int:
    return -((-a) // b)


class Arranged:
    """A hierarchical view of one source tensor.  `cursor` is the level that
    meta-operations act on; `.dtype` returns the same tensor with cursor + 1."""

    def __init__(self, src_shape, src_strides, levels, fn, cursor=0):
        self.src_shape = tuple(int(s) for s in src_shape)
        self.src_strides = tuple(int(s) for s in src_strides)
        self.levels = [tuple(int(x) for x in lv) for lv in levels]
        self.fn = fn
        self.cursor = cursor

    # ------------------------------------------------------------------ basics
    @property
    def shape(self):
        return self.levels[self.cursor]

    @property
    def ndim(self):
        return len(self.shape)

    def _with(self, levels, fn):
        return Arranged(self.src_shape, self.src_strides, levels, fn, self.cursor)

    @property
    def dtype(self):
        if self.cursor + 1 >= len(self.levels):
            raise ShapeMismatch("no inner level to descend into")
        return Arranged(self.src_shape, self.src_strides, self.levels, self.fn, self.cursor + 1)

    @dtype.setter
    def dtype(self, inner):
        if inner.cursor != self.cursor + 1:
            raise ShapeMismatch("dtype must be assigned a tensor one level further in")
        self.levels, self.fn = inner.levels, inner.fn

    # ---------------------------------------------------------- meta-operations
    def tile(self, tile_shape, strides=None, pad=None, dilation=None):
        """Element j of tile o along a dimension is source coordinate o * stride + j * dilation - pad_low (the paper's tile
        has dilation 1 and no padding; both are extensions, with the usual meaning for convolutions).  A tile then
        spans (t - 1) * dilation + 1 source coordinates, and as many tiles exist as start inside the padded extent
        with their whole span (the last one may overhang: ceiling)."""
        L, S = self.cursor, self.shape
        if len(tile_shape) != len(S):
            raise ShapeMismatch("tile_shape rank differs from the level's rank")
        T, st, lo, dil, outer = [], [], [], [], []
        for i, size in enumerate(S):
            t = size if tile_shape[i] == -1 else int(tile_shape[i])
            s = t if strides is None or strides[i] == -1 else int(strides[i])
            d = 1 if dilation is None or dilation[i] in (-1, 0) else int(dilation[i])
            p_lo, p_hi = (0, 0) if pad is None else (int(pad[i][0]), int(pad[i][1]))
            if t <= 0 and not (t == 0 and size == 0):
                raise ShapeMismatch("tile sizes must be positive")
            if d < 1:
                raise ShapeMismatch("dilation must be positive")
            if s <= 0:
                s = 1
            span = (t - 1) * d + 1 if t > 0 else 0
            if size + p_lo + p_hi > 0:
                o = max(_ceil_div(size + p_lo + p_hi - span, s) + 1, 0)
            else:                       # empty dimension: "-1" still yields its one (empty) tile
                o = 1 if tile_shape[i] == -1 else 0
            T.append(t), st.append(s), lo.append(p_lo), dil.append(d), outer.append(o)
        old_fn = self.fn

        def fn(idx, L=L, S=S, st=tuple(st), lo=tuple(lo), dil=tuple(dil)):
            parent, ok = [], True
            for i in range(len(S)):
                x = idx[L][i] * st[i] + idx[L + 1][i] * dil[i] - lo[i]
                ok = ok & (x >= 0) & (x < S[i])
                parent.append(x)
            coords, valid = old_fn(idx[:L] + [parent] + idx[L + 2:])
            return coords, valid & ok

        return self._with(self.levels[:L] + [tuple(outer), tuple(T)] + self.levels[L + 1:], fn)

    def expand(self, shape):
        L, S = self.cursor, self.shape
        if len(shape) != len(S):
            raise ShapeMismatch("expand rank differs from the level's rank")
        new, bcast = [], []
        for i, size in enumerate(S):
            if shape[i] == -1 or shape[i] == size:
                new.append(size), bcast.append(False)
            elif size == 1:
                new.append(int(shape[i])), bcast.append(True)
            else:
                raise ShapeMismatch("expand of a non-singleton dimension")
        old_fn = self.fn

        def fn(idx, L=L, bcast=tuple(bcast)):
            here = [x * 0 if b else x for x, b in zip(idx[L], bcast)]
            return old_fn(idx[:L] + [here] + idx[L + 1:])

        return self._with(self.levels[:L] + [tuple(new)] + self.levels[L + 1:], fn)

    def squeeze(self, dim):
        L, S = self.cursor, self.shape
        if not 0 <= dim < len(S) or S[dim] != 1:
            raise ShapeMismatch("squeeze of a non-singleton dimension")
        old_fn = self.fn

        def fn(idx, L=L, dim=dim):
            here = list(idx[L])
            here.insert(dim, np.int64(0))
            return old_fn(idx[:L] + [here] + idx[L + 1:])

        return self._with(self.levels[:L] + [S[:dim] + S[dim + 1:]] + self.levels[L + 1:], fn)

    def permute(self, order):
        L, S = self.cursor, self.shape
        if sorted(order) != list(range(len(S))):
            raise ShapeMismatch("permute needs a permutation of the level's dimensions")
        old_fn = self.fn

        def fn(idx, L=L, order=tuple(order)):
            here = [None] * len(order)
            for new_pos, old_pos in enumerate(order):
                here[old_pos] = idx[L][new_pos]
            return old_fn(idx[:L] + [here] + idx[L + 1:])

        return self._with(self.levels[:L] + [tuple(S[o] for o in order)] + self.levels[L + 1:], fn)

    def flatten(self, start_dim=0, end_dim=None):
        L, S = self.cursor, self.shape
        end_dim = len(S) if end_dim is None else end_dim
        if not 0 <= start_dim <= end_dim <= len(S):
            raise ShapeMismatch("flatten range outside the level")
        merged = S[start_dim:end_dim]
        total = 1
        for m in merged:
            total *= m
        old_fn = self.fn

        def fn(idx, L=L, a=start_dim, merged=merged):
            here = list(idx[L])
            rem = here[a]
            parts = []
            for m in reversed(merged):          # last merged dimension is the fastest
                parts.append(rem % m if m else rem * 0)
                rem = rem // m if m else rem * 0
            parts.reverse()
            return old_fn(idx[:L] + [here[:a] + parts + here[a + 1:]] + idx[L + 1:])

        return self._with(self.levels[:L] + [S[:start_dim] + (total,) + S[end_dim:]] + self.levels[L + 1:], fn)

    def ravel(self):
        L = self.cursor
        lens = [len(lv) for lv in self.levels[L:]]
        flat = tuple(x for lv in self.levels[L:] for x in lv)
        old_fn = self.fn

        def fn(idx, L=L, lens=tuple(lens)):
            here, split, pos = list(idx[L]), [], 0
            for n in lens:
                split.append(here[pos:pos + n])
                pos += n
            return old_fn(idx[:L] + split)

        return self._with(self.levels[:L] + [flat], fn)


def Tensor(shape, strides=None) -> Arranged:
    """A source tensor with concrete sizes; strides (in elements) default to row-major."""
    shape = tuple(int(s) for s in shape)
    if strides is None:
        strides, acc = [], 1
        for s in reversed(shape):
            strides.append(acc)
            acc *= max(s, 1)
        strides = tuple(reversed(strides))

    def fn(idx, shape=shape):
        coords, valid = list(idx[0]), True
        for x, s in zip(coords, shape):
            valid = valid & (x >= 0) & (x < s)
        return coords, valid

    return Arranged(shape, strides, [shape], fn)


# ----------------------------------------------------------------- arrangement programs
def run_program(t: Arranged, ops) -> Arranged:
    """Apply a list of meta-operations given as tuples:
    ("tile", tile_shape[, strides[, pad[, dilation]]]), ("expand", shape), ("squeeze", dim),
    ("permute", order), ("flatten", start, end), ("ravel",), ("descend",), ("ascend",).
    descend / ascend stand for taking `.dtype` and assigning the result back."""
    stack = []
    for op in ops:
        kind = op[0]
        if kind == "descend":
            stack.append(t)
            t = t.dtype
        elif kind == "ascend":
            outer = stack.pop()
            outer.dtype = t
            t = outer
        elif kind == "tile":
            t = t.tile(*op[1:])
        elif kind == "expand":
            t = t.expand(op[1])
        elif kind == "squeeze":
            t = t.squeeze(op[1])
        elif kind == "permute":
            t = t.permute(op[1])
        elif kind == "flatten":
            t = t.flatten(op[1], op[2])
        elif kind == "ravel":
            t = t.ravel()
        else:
            raise ValueError(kind)
    while stack:
        outer = stack.pop()
        outer.dtype = t
        t = outer
    return t


def mm_programs(Mt_Nt, BM, BN, BK):
    """Meta-operation programs of the matrix-multiplication arrangement (Section 4.2):
    C is tiled (BM, BN); A is tiled (BM, BK), its grid of blocks re-tiled into row sets
    (1, -1), the row sets repeated across the Nt block columns of C, and the singleton
    left in the middle level dropped; B mirrors this with column sets."""
    Mt, Nt = Mt_Nt
    a = [("tile", (BM, BK)), ("tile", (1, -1)), ("expand", (-1, Nt)), ("descend",), ("squeeze", 0), ("ascend",)]
    b = [("tile", (BK, BN)), ("tile", (-1, 1)), ("expand", (Mt, -1)), ("descend",), ("squeeze", 1), ("ascend",)]
    c = [("tile", (BM, BN))]
    return a, b, c


def mm_arrangement(A: Arranged, B: Arranged, Cm: Arranged, BM, BN, BK):
    """Arrange A [M,K], B [K,N], C [M,N] (2-D levels, possibly themselves arranged)."""
    c_arr = Cm.tile((BM, BN))
    pa, pb, _ = mm_programs(c_arr.shape, BM, BN, BK)
    return run_program(A, pa), run_program(B, pb), c_arr


def bmm_arrangement(A: Arranged, B: Arranged, Cm: Arranged, BM, BN, BK):
    """Batched matmul: the paper lists the kernel without printing its arrangement; the
    reading taken is the matmul arrangement with a leading batch dimension tiled by 1,
    giving grid (batch, Mt, Nt), middle level (Kt,), inner blocks 2-D."""
    c_arr = run_program(Cm, [("tile", (1, BM, BN)), ("descend",), ("squeeze", 0), ("ascend",)])
    _, Mt, Nt = c_arr.shape
    pa = [("tile", (1, BM, BK)), ("tile", (1, 1, -1)), ("expand", (-1, -1, Nt)),
          ("descend",), ("squeeze", 0), ("squeeze", 0), ("descend",), ("squeeze", 0), ("ascend",), ("ascend",)]
    pb = [("tile", (1, BK, BN)), ("tile", (1, -1, 1)), ("expand", (-1, Mt, -1)),
          ("descend",), ("squeeze", 0), ("squeeze", 1), ("descend",), ("squeeze", 0), ("ascend",), ("ascend",)]
    return run_program(A, pa), run_program(B, pb), c_arr


def conv2d_operand_programs(R, S, C, stride=(1, 1), pad=(0, 0), P=None, Q=None, H=None, W=None, dilation=(1, 1)):
    """Programs turning input (N,C,H,W), filter (K,C,R,S), output (N,K,P,Q) into the
    implicit-GEMM matrices (N*P*Q, C*R*S), (C*R*S, K), (N*P*Q, K) (Section 4.3).
    The paper's listing has stride 1 and no padding; stride and padding are carried by
    the tile's strides and pad arguments.  pad_hi is chosen so that exactly P (Q) filter
    positions exist, P being the usual floor formula."""
    pads = None
    if pad != (0, 0) or stride != (1, 1) or dilation != (1, 1):
        hi_h = (P - 1) * stride[0] + (R - 1) * dilation[0] + 1 - H - pad[0]
        hi_w = (Q - 1) * stride[1] + (S - 1) * dilation[1] + 1 - W - pad[1]
        pads = ((0, 0), (0, 0), (pad[0], hi_h), (pad[1], hi_w))
    tile = ("tile", (1, C, R, S), (-1, -1, stride[0], stride[1])) + ((pads,) if pads else ())
    if dilation != (1, 1):
        tile = tile + ((-1, -1, dilation[0], dilation[1]),)
    x = [tile, ("squeeze", 1), ("descend",), ("squeeze", 0), ("ascend",), ("ravel",),
         ("flatten", 0, 3), ("flatten", 1, 4)]
    w = [("flatten", 1, 4), ("permute", (1, 0))]
    y = [("permute", (0, 2, 3, 1)), ("flatten", 0, 3)]
    return x, w, y


def grouped_conv2d_view_programs(G, Cg, Kg, R, S, stride=(1, 1), pad=(0, 0), P=None, Q=None, H=None, W=None, dilation=(1, 1)):
    """A grouped convolution (input (N, G*Cg, H, W), filter (G*Kg, Cg, R, S), output (N, G*Kg, P, Q); group g's filters see
    only group g's channels) written as ONE batched matrix product over the groups, with the meta-operations of Table 1
    only: programs that turn the three tensors into the single-level views (G, N*P*Q, Cg*R*S), (G, Cg*R*S, Kg) and
    (G, N*P*Q, Kg).  The input is tiled as in Section 4.3, the channel axis in tiles of Cg, so that the outer level gains
    the group index; G = 1 gives the implicit-GEMM views of Section 4.3 with a leading batch axis of one.  Depthwise:
    Cg = Kg = 1."""
    hi_h = (P - 1) * stride[0] + (R - 1) * dilation[0] + 1 - H - pad[0]
    hi_w = (Q - 1) * stride[1] + (S - 1) * dilation[1] + 1 - W - pad[1]
    pads = ((0, 0), (0, 0), (pad[0], hi_h), (pad[1], hi_w))
    x = [("tile", (1, Cg, R, S), (-1, -1, stride[0], stride[1]), pads, (-1, -1, dilation[0], dilation[1])),   # (N, G, P, Q) of (1, Cg, R, S)
         ("permute", (1, 0, 2, 3)), ("descend",), ("squeeze", 0), ("ascend",), ("ravel",),                    # (G, N, P, Q, Cg, R, S)
         ("flatten", 1, 4), ("flatten", 2, 5)]
    w = [("flatten", 1, 4), ("tile", (Kg, -1)), ("ravel",), ("squeeze", 1), ("permute", (0, 2, 1))]           # (G, Cg R S, Kg)
    y = [("tile", (-1, Kg, -1, -1)), ("ravel",), ("squeeze", 0), ("squeeze", 1), ("squeeze", 1),              # (G, N, Kg, P, Q)
         ("permute", (0, 1, 3, 4, 2)), ("flatten", 1, 4)]
    return x, w, y


def conv2d_arrangement(X: Arranged, Wt: Arranged, Y: Arranged, BM, BN, BK, stride=(1, 1), pad=(0, 0), dilation=(1, 1)):
    _, C, H, W = X.shape
    _, _, R, S = Wt.shape
    _, _, P, Q = Y.shape
    px, pw, py = conv2d_operand_programs(R, S, C, stride, pad, P, Q, H, W, dilation)
    return mm_arrangement(run_program(X, px), run_program(Wt, pw), run_program(Y, py), BM, BN, BK)


# ------------------------------------------------------------ the two mappings
def grid_shape(arranged) -> tuple:
    """Tile-to-program mapping: the common outermost shape, or ShapeMismatch."""
    arranged = list(arranged)
    g = arranged[0].levels[0]
    for a in arranged[1:]:
        if a.levels[0] != g:
            raise ShapeMismatch(f"outermost shapes differ: {g} vs {a.levels[0]}")
    return g


def num_programs(arranged) -> int:
    n = 1
    for s in grid_shape(arranged):
        n *= s
    return n


def _unravel(flat: int, shape):
    out = []
    for s in reversed(shape):
        out.append(flat % s if s else 0)
        flat = flat // s if s else 0
    return list(reversed(out))


def tile_index_set(a: Arranged, pid: int, mid=()):
    """Source-to-target mapping for one tile: element offsets (row-major over the
    innermost level, -1 where masked), masks (uint8) and the innermost shape.
    `mid` lists the indices of all levels strictly between outermost and innermost."""
    levels = a.levels
    inner = levels[-1] if len(levels) > 1 else ()
    n_mid = sum(len(lv) for lv in levels[1:-1])
    if len(mid) != n_mid:
        raise ShapeMismatch(f"expected {n_mid} middle indices, got {len(mid)}")
    idx = [[np.int64(v) for v in _unravel(pid, levels[0])]]
    pos = 0
    for lv in levels[1:-1]:
        part = []
        for s in lv:
            if not 0 <= mid[pos] < s:
                raise IndexError("middle index out of range")
            part.append(np.int64(mid[pos]))
            pos += 1
        idx.append(part)
    if len(levels) > 1:
        grids = np.indices(inner, dtype=np.int64).reshape(len(inner), -1) if inner else np.zeros((0, 1), np.int64)
        idx.append([grids[d] for d in range(len(inner))])
    coords, valid = a.fn(idx)
    n = int(np.prod(inner)) if inner else 1
    off = np.zeros(n, dtype=np.int64)
    for x, s in zip(coords, a.src_strides):
        off = off + np.asarray(x, dtype=np.int64) * np.int64(s)
    valid = np.broadcast_to(np.asarray(valid, dtype=bool), (n,))
    off = np.where(valid, off, np.int64(-1))
    return off, valid.astype(np.uint8), inner


def view_index_set(a: Arranged):
    """A single-level arranged tensor (a view) written out: the offset of every element of the
    view (-1 where it falls outside the source) and the mask, both shaped like the view."""
    if len(a.levels) != 1:
        raise ShapeMismatch("a view has a single level")
    shape = a.levels[0]
    grids = np.indices(shape, dtype=np.int64).reshape(len(shape), -1)
    coords, valid = a.fn([[grids[d] for d in range(len(shape))]])
    n = int(np.prod(shape)) if shape else 1
    off = np.zeros(n, dtype=np.int64)
    for x, s in zip(coords, a.src_strides):
        off = off + np.asarray(x, dtype=np.int64) * np.int64(s)
    valid = np.broadcast_to(np.asarray(valid, dtype=bool), (n,))
    return np.where(valid, off, np.int64(-1)).reshape(shape), valid.reshape(shape)


def _dot_by_definition(A, B):
    """sum_k A[..., m, k] * B[..., k, n] in fp64, the terms added one k after another (no library product)."""
    out = np.zeros(A.shape[:-1] + (B.shape[-1],), dtype=np.float64)
    for k in range(A.shape[-1]):
        out += A[..., :, k, None] * B[..., k, None, :]
    return out


def matmul_views(a_view: Arranged, b_view: Arranged, c_view: Arranged, a_flat, b_flat, c_flat):
    """C_view = A_view . B_view (Sections 4.2 / 4.3: the matrix product over operands that are
    themselves arranged tensors) on flat fp64 source arrays: elements of A_view / B_view outside
    their tensor read as zero, elements of C_view outside C are dropped.  Views are [rows, cols]
    or [batch, rows, cols].  Returns the updated copy of c_flat."""
    oa, ma = view_index_set(a_view)
    ob, mb = view_index_set(b_view)
    oc, mc = view_index_set(c_view)
    A = np.where(ma, np.asarray(a_flat, dtype=np.float64)[np.where(ma, oa, 0)], 0.0)
    B = np.where(mb, np.asarray(b_flat, dtype=np.float64)[np.where(mb, ob, 0)], 0.0)
    if A.ndim != B.ndim or A.ndim != oc.ndim or A.shape[-1] != B.shape[-2] or oc.shape[-2:] != (A.shape[-2], B.shape[-1]) \
            or A.shape[:-2] != B.shape[:-2] or A.shape[:-2] != oc.shape[:-2]:
        raise ShapeMismatch("view shapes do not form a matrix product")
    prod = _dot_by_definition(A, B)
    out = np.array(c_flat, dtype=np.float64, copy=True)
    out[oc[mc]] = prod[mc]
    return out


# --------------------------------------------------- application on arranged tiles
def apply_mm(a_arr, b_arr, c_arr, a_flat, b_flat, c_flat):
    """The matrix-multiplication application (Section 4.2) executed serially, one
    program after another, on flat fp64 source arrays through the index sets above:
    a zero accumulator of the output tile's shape, one dot product per k, store."""
    n_prog = num_programs((a_arr, b_arr, c_arr))
    kt = a_arr.levels[1][0]
    if b_arr.levels[1][0] != kt:
        raise ShapeMismatch("A and B disagree on the number of k tiles")
    for pid in range(n_prog):
        c_off, c_mask, c_shape = tile_index_set(c_arr, pid)
        acc = np.zeros(c_shape, dtype=np.float64)
        for k in range(kt):
            a_off, a_mask, a_shape = tile_index_set(a_arr, pid, (k,))
            b_off, b_mask, b_shape = tile_index_set(b_arr, pid, (k,))
            a_tile = np.where(a_mask != 0, a_flat[np.maximum(a_off, 0)], 0.0).reshape(a_shape)
            b_tile = np.where(b_mask != 0, b_flat[np.maximum(b_off, 0)], 0.0).reshape(b_shape)
            acc += _dot_by_definition(a_tile, b_tile)
        keep = c_mask != 0
        c_flat[c_off[keep]] = acc.reshape(-1)[keep]
    return c_flat
