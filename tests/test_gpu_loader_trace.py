"""The source-to-target mapping (Section 3.2.2) as the matrix-instruction kernels execute it, against the oracle's enumerator.

Those kernels do not gather through the operand map: every lane derives its own addresses (swizzled LDS slots, range-checked
loads, for the convolution the unfolded input generated on the fly with its padding fix-ups).  The operand is filled with its
elements' own offsets (+1, 16 bits at a time), one workgroup of the real kernel loads one 32-k slice, and what it left in LDS
is read back element by element: the offset must be the oracle's, bit for bit, wherever the oracle's tile has an element, and
zero must have been fed wherever a masked element can reach an output that is stored."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
from oracle import arrangement as arr

pytestmark = pytest.mark.gpu

TDT = {"f16": torch.float16, "bf16": torch.bfloat16}


def coded(shape, strides, dt, part):
    """Device view (shape, strides in elements) of a buffer whose element at offset o from the view's first holds 16 bits
    (part 0: low, 1: high) of o + 1."""
    span = 1 + sum((n - 1) * s for n, s in zip(shape, strides))
    o = np.arange(span, dtype=np.int64) + 1
    bits = ((o >> (16 * part)) & 0xffff).astype(np.uint16)
    buf = torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt])
    return torch.as_strided(buf, shape, strides)


def loader_offsets(kind, shape_a, strides_a, shape_b, strides_b, shape_c, dt, operand, pid, sl, tile=None, stride=(1, 1), pad=(0, 0),
                   want_path=None):
    """[256, 32] int64: the source offset of every element of the slice as loaded (-1: a zero was fed; -2: row past the tile)."""
    c = torch.empty(shape_c, dtype=TDT[dt], device="cuda")
    parts = []
    for part in (0, 1):
        a = coded(shape_a, strides_a, dt, part if operand == 0 else 0)
        b = coded(shape_b, strides_b, dt, part if operand == 1 else 0)
        parts.append(nt.trace_loader_slice(kind, a, b, c, operand, pid, sl, tile=tile, stride=stride, pad=pad).astype(np.int64))
        if want_path is not None:
            assert nt.last_kernel_path() == want_path
    lo, hi = parts
    past = (lo == 0xffff) & (hi == 0xffff)
    return np.where(past, -2, (lo | (hi << 16)) - 1)


def contiguous(shape):
    s, acc = [], 1
    for n in reversed(shape):
        s.append(acc)
        acc *= n
    return tuple(reversed(s))


# ---------------------------------------------------------------- plain products
def check_product(M, N, K, dt, tile, ta, tb, lda_pad=0, ldb_pad=0, batch=None):
    BM, BN, BK = tile
    # A[m, k]: row-major with pitch K + pad, or (ta) stored as K rows of pitch M + pad; B likewise
    sa = (1, M + lda_pad) if ta else (K + lda_pad, 1)
    sb = (1, K + ldb_pad) if tb else (N + ldb_pad, 1)
    sha, shb, shc = (M, K), (K, N), (M, N)
    if batch:
        sa = ((M + lda_pad) * (K + lda_pad),) + sa
        sb = ((N + ldb_pad) * (K + ldb_pad),) + sb
        sha, shb, shc = (batch,) + sha, (batch,) + shb, (batch,) + shc
        a_arr, b_arr, c_arr = arr.bmm_arrangement(arr.Tensor(sha, sa), arr.Tensor(shb, sb), arr.Tensor(shc), BM, BN, BK)
        kind = "bmm"
    else:
        a_arr, b_arr, c_arr = arr.mm_arrangement(arr.Tensor(sha, sa), arr.Tensor(shb, sb), arr.Tensor(shc), BM, BN, BK)
        kind = "gemm"
    mt, ntl = -(-M // BM), -(-N // BN)
    n_prog = (batch or 1) * mt * ntl
    n_slices = -(-K // 32)
    for pid in sorted({0, n_prog - 1, n_prog // 2}):
        i, j = (pid % (mt * ntl)) // ntl, pid % ntl
        for sl in sorted({0, n_slices - 1, n_slices // 2}):
            k_tile, half = sl // 2, sl % 2
            for operand, view in ((0, a_arr), (1, b_arr)):
                got = loader_offsets(kind, sha, sa, shb, sb, shc, dt, operand, pid, sl, tile=tile, want_path=nt.PATH_DIRECT)
                o_off, o_mask, shp = arr.tile_index_set(view, pid, (k_tile,))
                o_off, o_mask = o_off.reshape(shp), o_mask.reshape(shp)
                if operand == 0:
                    rows, ref, msk = BM, o_off[:, 32 * half:32 * half + 32], o_mask[:, 32 * half:32 * half + 32]
                    inside = (i * BM + np.arange(BM)) < M
                else:
                    rows, ref, msk = BN, o_off[32 * half:32 * half + 32, :].T, o_mask[32 * half:32 * half + 32, :].T
                    inside = (j * BN + np.arange(BN)) < N
                assert (got[rows:] == -2).all()
                g = got[:rows]
                what = (M, N, K, dt, tile, ta, tb, "AB"[operand], pid, sl)
                assert np.array_equal(g[msk == 1], ref[msk == 1]), what
                # the k past K must read as zero on every row that is stored
                k_past = (32 * sl + np.arange(32)) >= K
                assert (g[np.ix_(inside, k_past)] == -1).all(), what
                # (rows past M / N: whatever was fetched only reaches outputs that are never stored)
                assert (msk[inside][:, ~k_past] == 1).all()


@pytest.mark.parametrize("tile", [(128, 128, 64), (256, 128, 64), (128, 256, 64), (256, 256, 64)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_full_tiles(tile, ta, tb):
    check_product(512, 768, 192, "f16", tile, ta, tb)


@pytest.mark.parametrize("tile", [(128, 128, 64), (256, 256, 64), (128, 256, 64)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_ragged_tiles_and_odd_pitches(tile, ta, tb):
    check_product(301, 203, 151, "bf16", tile, ta, tb)             # odd pitches, every extent ragged
    check_product(300, 200, 100, "f16", tile, ta, tb, 4, 12)       # aligned rows with gaps between them, ragged K


def test_batched():
    check_product(256, 384, 128, "f16", (128, 128, 64), False, False, batch=3)
    check_product(200, 130, 72, "bf16", (128, 128, 64), False, True, batch=2)


# ---------------------------------------------------------------- convolution
def whole_matrix(view, n_row_tiles, n_col_tiles, kt, pid_of, rows_first):
    """The arrangement's whole operand matrix (offsets, -1 where masked), put together from its tiles."""
    blocks = []
    for t in range(n_row_tiles if rows_first else n_col_tiles):
        line = []
        for k in range(kt):
            off, _, shp = arr.tile_index_set(view, pid_of(t), (k,))
            line.append(off.reshape(shp))
        blocks.append(np.concatenate(line, axis=1 if rows_first else 0))
    return np.concatenate(blocks, axis=0 if rows_first else 1)


@pytest.mark.parametrize("Nn,C,H,W,F,R,S,pad,layout", [(*c, "kcrs") if len(c) == 8 else c for c in [
    (2, 32, 16, 16, 64, 3, 3, (1, 1)),        # output rows of 16 positions; left / right / top / bottom padding
    (3, 32, 14, 14, 96, 3, 3, (1, 1)),        # rows of 14 positions: the kernel numbers them with a pitch of 16
    (2, 64, 10, 10, 256, 3, 3, (0, 0)),       # no padding, rows of 8
    (2, 32, 12, 13, 130, 3, 3, (1, 0)),       # padding above and below only, rows of 11
    (1, 32, 9, 12, 64, 3, 5, (0, 1)),         # 3 x 5 filter, one column of padding
    (2, 96, 8, 8, 64, 1, 1, (0, 0)),          # 1 x 1 filter
    (2, 64, 14, 14, 256, 3, 3, (1, 1)),       # 256 filters, channels in blocks of 32: the tap-major kernel; rows of 14, padding
    (3, 32, 16, 16, 300, 3, 3, (1, 1)),       # the same with one channel block per tap, rows of 16, a ragged last filter tile
    (1, 64, 9, 9, 192, 2, 2, (0, 1)),         # 2 x 2 filter, rows of 9 (a run that starts in the right padding)
    (2, 32, 6, 20, 256, 5, 3, (1, 1)),        # 5 x 3 filter
    (2, 64, 14, 14, 256, 3, 3, (1, 1), "krsc"),   # the filter stored channels-last, (f, r, s, c): read as it is, no copy
]])
def test_convolution(Nn, C, H, W, F, R, S, pad, layout):
    dt = "f16"
    P, Q = H + 2 * pad[0] - R + 1, W + 2 * pad[1] - S + 1
    Q8 = -(-Q // 8) * 8
    K = C * R * S
    assert K % 32 == 0
    tile = (256, 256 if F > 128 else 128, 64)
    BN = tile[1]
    BNk = 64 if F <= 64 else BN                 # few filters: the same grid is run by the kernel built for 64 per program
    shx, shw, shy = (Nn, C, H, W), (F, C, R, S), (Nn, F, P, Q)
    sx, sw = contiguous(shx), contiguous(shw)
    if layout == "krsc":
        sw = (R * S * C, 1, S * C, C)
    BMo, BKo = 64, 64
    a_arr, b_arr, _ = arr.conv2d_arrangement(arr.Tensor(shx), arr.Tensor(shw, sw), arr.Tensor(shy), BMo, BN, BKo, (1, 1), pad)
    Mo = Nn * P * Q
    mto, nto, kto = -(-Mo // BMo), -(-F // BN), -(-K // BKo)
    A_ref = whole_matrix(a_arr, mto, nto, kto, lambda t: t * nto, True)[:Mo, :K]          # [positions, C R S]
    B_ref = whole_matrix(b_arr, mto, nto, kto, lambda t: t, False)[:K, :]                 # [C R S, filters (padded to the tile)]
    Mk = Nn * P * Q8                                                                       # positions as the kernel numbers them
    n_slices = K // 32
    # positions per program: the library's choice (256, 224 or 192, the first tiles possibly 32 higher than the others, whatever
    # fills the chip's rounds best); the rows past a program's height come back unwritten.  Tile row i starts where the
    # tile rows before it end.
    heights, covered = [], 0
    while covered < Mk:
        h = int((loader_offsets("conv2d", shx, sx, shw, sw, shy, dt, 0, len(heights) * nto, 0, tile=tile, pad=pad)[:, 0] != -2).sum())
        assert h in (192, 224, 256) and (not heights or h in (heights[-1], heights[-1] - 32))
        heights.append(h)
        covered += h
    mt = len(heights)
    starts = np.concatenate([[0], np.cumsum(heights)])
    with pytest.raises(nt.NtError):                            # no program past the last tile row
        loader_offsets("conv2d", shx, sx, shw, sw, shy, dt, 0, mt * nto, 0, tile=tile, pad=pad)
    for pid in sorted({0, mt * nto - 1, (mt * nto) // 2}):
        i, j = pid // nto, pid % nto
        rows = heights[i]
        for sl in sorted({0, 1, n_slices // 2, n_slices - 1}):
            ks = slice(32 * sl, 32 * sl + 32)
            got = loader_offsets("conv2d", shx, sx, shw, sw, shy, dt, 0, pid, sl, tile=tile, pad=pad)
            path = nt.last_kernel_path()
            assert path == (nt.PATH_CONV_TAP if F > 128 and C % 32 == 0 else nt.PATH_CONV_DIRECT)
            if path == nt.PATH_CONV_TAP:        # the reduction is walked tap by tap: slice sl = 32 channels of one tap
                cb = C // 32
                ks = (32 * (sl % cb) + np.arange(32)) * (R * S) + sl // cb
            assert (got[rows:] == -2).all()
            for r in range(rows):
                m = int(starts[i]) + r
                n, p, q = m // (P * Q8), (m % (P * Q8)) // Q8, m % Q8
                if m >= Mk or q >= Q:
                    continue                                  # a row past the last position, or one of a row's surplus positions: never stored
                ref = A_ref[(n * P + p) * Q + q, ks]
                assert np.array_equal(got[r], ref), ((Nn, C, H, W, F, R, S, pad), "x", pid, sl, r, got[r], ref)
            got = loader_offsets("conv2d", shx, sx, shw, sw, shy, dt, 1, pid, sl, tile=tile, pad=pad)
            assert (got[BNk:] == -2).all()
            for r in range(BNk):
                f = j * BN + r
                if f >= F:
                    continue                                  # a filter past the last: never stored
                assert np.array_equal(got[r], B_ref[ks, f]), ((Nn, C, H, W, F, R, S, pad), "w", pid, sl, r)


def test_refusals():
    dt = "f16"
    a, b, c = (torch.zeros(s, dtype=torch.float16, device="cuda") for s in ((64, 64), (64, 64), (64, 64)))
    with pytest.raises(nt.NtError) as e:                     # a tile that the operand-map kernel runs
        nt.trace_loader_slice("gemm", a, b, c, 0, 0, 0, tile=(64, 64, 32))
    assert e.value.name == "NT_ERR_UNSUPPORTED"
    a, b, c = (torch.zeros(s, dtype=torch.float16, device="cuda") for s in ((256, 64), (64, 256), (256, 256)))
    for bad in ((0, 4, 0), (0, 0, 2), (2, 0, 0)):
        with pytest.raises(nt.NtError) as e:
            nt.trace_loader_slice("gemm", a, b, c, bad[0], bad[1], bad[2], tile=(128, 128, 64))
        assert e.value.name == "NT_ERR_INVALID_ARG"
