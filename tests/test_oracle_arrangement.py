"""Pins for the oracle's arrangement enumerator (CPU only).

Every check compares the enumerator with something fixed outside it: shapes the paper
prints, Algorithm 1's formula, hand-worked offsets, brute-force counting arguments, or
the plain triple-loop / direct-convolution results.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import arrangement as arr
from oracle import numeric as onum
import synthetic_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def _tup(s):
    return tuple(int(x) for x in s.split(",") if x.strip())


# ------------------------------------------------------------- shapes printed in the paper
def test_paper_printed_shapes():
    rows = {ln.split("|")[0].strip(): [c.strip() for c in ln.split("|")[1:3]] for ln in _golden_lines("paper_shapes.txt")}
    src, res = rows["tile_4x4_by_2x2"]
    t = arr.Tensor(_tup(src)).tile((2, 2))
    assert t.levels == [_tup(x) for x in res.split(";")]
    src, res = rows["squeeze_1x2"]
    assert arr.Tensor(_tup(src)).squeeze(0).levels == [_tup(res)]
    src, res = rows["ravel_npq_crs"]
    outer, inner = (_tup(x) for x in src.split(";"))
    # build a two-level tensor with exactly these level shapes: tile a 6-D... simpler: a 3-D
    # tensor of sizes outer*inner tiled by inner
    t = arr.Tensor(tuple(o * i for o, i in zip(outer, inner))).tile(inner)
    assert t.levels == [outer, inner]
    assert t.ravel().levels == [_tup(res)]
    src, res = rows["mm_grid_2x2"]
    a, b, c = arr.mm_arrangement(arr.Tensor((4, 6)), arr.Tensor((6, 8)), arr.Tensor((4, 8)), 2, 4, 3)
    assert a.levels[0] == b.levels[0] == c.levels[0] == _tup(src)
    assert arr.num_programs((a, b, c)) == int(res)


@pytest.mark.parametrize("size,tile", [(3001, 64), (5003, 256), (1999, 32), (7, 7), (1, 64), (64, 1), (65, 64)])
def test_algorithm1_outer_is_ceil(size, tile):
    t = arr.Tensor((size,)).tile((tile,))
    assert t.levels == [((size + tile - 1) // tile,), (tile,)]


def test_conv_shape_chain_matches_section_4_3():
    N, C, H, W, K, R, S = 2, 3, 5, 6, 4, 3, 2
    P, Q = H - R + 1, W - S + 1
    x = arr.Tensor((N, C, H, W)).tile((1, C, R, S), strides=(-1, -1, 1, 1))
    assert x.levels == [(N, 1, P, Q), (1, C, R, S)]
    x = x.squeeze(1)
    x.dtype = x.dtype.squeeze(0)
    assert x.levels == [(N, P, Q), (C, R, S)]
    x = x.ravel()
    assert x.levels == [(N, P, Q, C, R, S)]
    x = x.flatten(end_dim=3).flatten(start_dim=1)
    assert x.levels == [(N * P * Q, C * R * S)]
    w = arr.Tensor((K, C, R, S)).flatten(start_dim=1).permute((1, 0))
    assert w.levels == [(C * R * S, K)]
    y = arr.Tensor((N, K, P, Q)).permute((0, 2, 3, 1)).flatten(end_dim=3)
    assert y.levels == [(N * P * Q, K)]


def test_mm_level_structure():
    # Section 4.2: after the squeeze the k range is input.shape[0] and tiles are input[k], other[k]
    M, N, K, BM, BN, BK = 10, 9, 7, 4, 2, 3
    a, b, c = arr.mm_arrangement(arr.Tensor((M, K)), arr.Tensor((K, N)), arr.Tensor((M, N)), BM, BN, BK)
    assert a.levels == [(3, 5), (3,), (BM, BK)]
    assert b.levels == [(3, 5), (3,), (BK, BN)]
    assert c.levels == [(3, 5), (BM, BN)]


def test_mismatched_outermost_shapes_is_an_error():
    a = arr.Tensor((8, 8)).tile((4, 4))
    b = arr.Tensor((8, 8)).tile((2, 4))
    with pytest.raises(arr.ShapeMismatch):
        arr.grid_shape((a, b))
    with pytest.raises(arr.ShapeMismatch):
        arr.Tensor((2, 3)).expand((5, -1))
    with pytest.raises(arr.ShapeMismatch):
        arr.Tensor((2, 3)).squeeze(0)


def test_defaults_of_tile_strides():
    # default stride == tile shape, -1 == default (Section 3.1.3)
    a = arr.Tensor((9, 10)).tile((2, 5))
    b = arr.Tensor((9, 10)).tile((2, 5), strides=(-1, -1))
    c = arr.Tensor((9, 10)).tile((2, 5), strides=(2, 5))
    for pid in range(10):
        oa = arr.tile_index_set(a, pid)
        for other in (b, c):
            oo = arr.tile_index_set(other, pid)
            assert np.array_equal(oa[0], oo[0]) and np.array_equal(oa[1], oo[1])
    assert arr.Tensor((9, 10)).tile((-1, 5)).levels == [(1, 2), (9, 5)]


# --------------------------------------------------------------------- hand-worked offsets
def test_hand_worked_tile_offsets():
    ln = [x for x in _golden_lines("hand_worked.txt") if x.startswith("tile_4x6_by_2x4_pid3")][0]
    kv = dict(p.split("=") for p in ln.split()[1:])
    off, mask, shape = arr.tile_index_set(arr.Tensor((4, 6)).tile((2, 4)), 3)
    assert shape == (2, 4)
    assert off.tolist() == list(_tup(kv["offsets"]))
    assert mask.tolist() == list(_tup(kv["mask"]))


def test_strides_are_honoured():
    # a transposed view: element (i,j) of the logical 3x5 tensor sits at j*3 + i
    t = arr.Tensor((3, 5), strides=(1, 3)).tile((2, 2))
    off, mask, _ = arr.tile_index_set(t, 1 * 3 + 2)   # tile (1,2): rows 2..3, cols 4..5
    assert off.tolist() == [4 * 3 + 2, -1, -1, -1]
    assert mask.tolist() == [1, 0, 0, 0]


# ----------------------------------------------------------------- brute-force coverage
@pytest.mark.parametrize("M,N,K,BM,BN,BK", [(5, 7, 3, 2, 4, 2), (4, 4, 4, 2, 2, 2), (1, 9, 5, 3, 2, 4), (6, 5, 1, 4, 4, 4)])
def test_exactly_once_coverage(M, N, K, BM, BN, BK):
    a, b, c = arr.mm_arrangement(arr.Tensor((M, K)), arr.Tensor((K, N)), arr.Tensor((M, N)), BM, BN, BK)
    Mt, Nt = -(-M // BM), -(-N // BN)
    Kt = -(-K // BK)
    G = arr.num_programs((a, b, c))
    assert G == Mt * Nt and a.levels[1] == (Kt,)
    c_count = np.zeros(M * N, int)
    a_count = np.zeros(M * K, int)
    b_count = np.zeros(K * N, int)
    triples = {}
    for pid in range(G):
        co, cm, _ = arr.tile_index_set(c, pid)
        np.add.at(c_count, co[cm != 0], 1)
        for k in range(Kt):
            ao, am, _ = arr.tile_index_set(a, pid, (k,))
            bo, bm, _ = arr.tile_index_set(b, pid, (k,))
            np.add.at(a_count, ao[am != 0], 1)
            np.add.at(b_count, bo[bm != 0], 1)
            A2, B2 = ao.reshape(BM, BK), bo.reshape(BK, BN)
            C2 = co.reshape(BM, BN)
            for r, kk, n in itertools.product(range(BM), range(BK), range(BN)):
                if A2[r, kk] >= 0 and B2[kk, n] >= 0 and C2[r, n] >= 0:
                    m_, k_ = divmod(A2[r, kk], K)
                    k2_, n_ = divmod(B2[kk, n], N)
                    assert k_ == k2_ and C2[r, n] == m_ * N + n_
                    triples[(m_, k_, n_)] = triples.get((m_, k_, n_), 0) + 1
    assert (c_count == 1).all()              # every output element stored exactly once
    assert (a_count == Nt).all()             # every A element read by the Nt programs of its block row
    assert (b_count == Mt).all()
    assert len(triples) == M * K * N and set(triples.values()) == {1}


def test_edge_mask_closed_forms():
    M, N, BM, BN = 3001, 5003, 256, 256
    c = arr.Tensor((M, N)).tile((BM, BN))
    Mt, Nt = c.levels[0]
    assert (Mt, Nt) == (12, 20)
    off, mask, _ = arr.tile_index_set(c, (Mt - 1) * Nt + (Nt - 1))
    rows, cols = M - (Mt - 1) * BM, N - (Nt - 1) * BN
    assert mask.sum() == rows * cols == 185 * 139
    assert mask.reshape(BM, BN)[:rows, :cols].all()
    good = off[mask != 0]
    assert len(set(good.tolist())) == good.size and good.max() == M * N - 1
    off, mask, _ = arr.tile_index_set(c, 0)
    assert mask.all() and off[0] == 0 and off[-1] == 255 * N + 255


# ------------------------------------------------- application on index sets == definition
@pytest.mark.parametrize("M,N,K,BM,BN,BK,dt", [(5, 7, 3, 2, 4, 2, "f16"), (9, 4, 11, 4, 4, 4, "bf16"), (8, 8, 8, 4, 4, 2, "f16")])
def test_apply_mm_equals_triple_loop(M, N, K, BM, BN, BK, dt):
    A, B = si.gemm_inputs(M, N, K, dt, seed=3, dist="uniform")
    a, b, c = arr.mm_arrangement(arr.Tensor((M, K)), arr.Tensor((K, N)), arr.Tensor((M, N)), BM, BN, BK)
    out = arr.apply_mm(a, b, c, onum.decode(A, dt).ravel(), onum.decode(B, dt).ravel(), np.full(M * N, np.nan))
    ref = onum.gemm(A, B, dt)
    assert np.allclose(out.reshape(M, N), ref, rtol=0, atol=1e-12)


def test_apply_bmm_equals_triple_loop():
    Bn, M, N, K = 3, 5, 6, 7
    A, B = si.gemm_inputs(M, N, K, "f16", seed=5, dist="uniform", batch=Bn)
    a, b, c = arr.bmm_arrangement(arr.Tensor((Bn, M, K)), arr.Tensor((Bn, K, N)), arr.Tensor((Bn, M, N)), 2, 4, 3)
    assert a.levels == [(3, 3, 2), (3,), (2, 3)] and b.levels == [(3, 3, 2), (3,), (3, 4)]
    assert c.levels == [(3, 3, 2), (2, 4)]
    out = arr.apply_mm(a, b, c, onum.decode(A, "f16").ravel(), onum.decode(B, "f16").ravel(), np.full(Bn * M * N, np.nan))
    assert np.allclose(out.reshape(Bn, M, N), onum.bmm(A, B, "f16"), rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape,stride,pad", [
    ((2, 3, 5, 6, 4, 3, 2), (1, 1), (0, 0)),      # the paper's case: stride 1, no padding
    ((1, 2, 6, 5, 3, 3, 3), (1, 1), (1, 1)),      # same-size output
    ((2, 2, 7, 8, 2, 3, 2), (2, 2), (1, 0)),      # stride 2, extent not divisible
    ((1, 1, 4, 4, 1, 1, 1), (1, 1), (0, 0)),      # 1x1 filter
    ((1, 3, 5, 5, 2, 3, 3), (2, 1), (2, 1)),
])
def test_implicit_gemm_equals_direct_convolution(shape, stride, pad):
    N, C, H, W, K, R, S = shape
    X, Wt = si.conv_inputs(N, C, H, W, K, R, S, "f16", seed=11)
    ref = onum.conv2d(X, Wt, "f16", stride, pad)
    P, Q = ref.shape[2:]
    a, b, c = arr.conv2d_arrangement(arr.Tensor((N, C, H, W)), arr.Tensor((K, C, R, S)), arr.Tensor((N, K, P, Q)),
                                     4, 2, 5, stride, pad)
    assert a.levels[0] == (-(-N * P * Q // 4), -(-K // 2))
    out = arr.apply_mm(a, b, c, onum.decode(X, "f16").ravel(), onum.decode(Wt, "f16").ravel(), np.full(ref.size, np.nan))
    assert np.allclose(out.reshape(ref.shape), ref, rtol=0, atol=1e-12)


def test_conv_index_map_closed_form():
    # A[m,kk] of the implicit GEMM must address X[n, c, p+r-pad, q+s-pad] (Section 4.3 shape names)
    N, C, H, W, K, R, S, pad = 2, 3, 4, 5, 2, 3, 3, 1
    P, Q = H, W
    px, _, _ = arr.conv2d_operand_programs(R, S, C, (1, 1), (pad, pad), P, Q, H, W)
    x = arr.run_program(arr.Tensor((N, C, H, W)), px).tile((1, 1))       # one element per program
    assert x.levels[0] == (N * P * Q, C * R * S)
    for m, kk in [(0, 0), (7, 13), (N * P * Q - 1, C * R * S - 1), (5, 4), (21, 26)]:
        n, p, q = m // (P * Q), (m // Q) % P, m % Q
        c, r, s = kk // (R * S), (kk // S) % R, kk % S
        h, w = p + r - pad, q + s - pad
        off, mask, _ = arr.tile_index_set(x, m * (C * R * S) + kk)
        inside = 0 <= h < H and 0 <= w < W
        assert mask[0] == int(inside)
        assert off[0] == (((n * C + c) * H + h) * W + w if inside else -1)


def test_k_zero_leaves_zero_output():
    a, b, c = arr.mm_arrangement(arr.Tensor((3, 0)), arr.Tensor((0, 4)), arr.Tensor((3, 4)), 2, 2, 2)
    assert a.levels[1] == (0,)
    out = arr.apply_mm(a, b, c, np.zeros(0), np.zeros(0), np.full(12, np.nan))
    assert (out == 0).all()


def test_planted_mistakes_are_caught():
    """The pins above must fail for plausible slips: check a few mutated enumerators."""
    M, N, K, BM, BN, BK = 5, 7, 3, 2, 4, 2
    A, B = si.gemm_inputs(M, N, K, "f16", seed=3, dist="uniform")
    ref = onum.gemm(A, B, "f16")
    fa, fb = onum.decode(A, "f16").ravel(), onum.decode(B, "f16").ravel()

    def run(pa, pb, pc):
        a = arr.run_program(arr.Tensor((M, K)), pa)
        b = arr.run_program(arr.Tensor((K, N)), pb)
        c = arr.run_program(arr.Tensor((M, N)), pc)
        return arr.apply_mm(a, b, c, fa, fb, np.full(M * N, np.nan)).reshape(M, N)

    pa, pb, pc = arr.mm_programs((3, 2), BM, BN, BK)
    assert np.allclose(run(pa, pb, pc), ref, atol=1e-12)
    # slip 1: A's row sets and B's column sets swapped in the second tiling
    bad_a = [pa[0], ("tile", (-1, 1))] + pa[2:]
    with pytest.raises((arr.ShapeMismatch, ValueError, IndexError)):
        run(bad_a, pb, pc)
    # slip 2: wrong BK for B only -> different k tiling, result differs or shapes clash
    bad_b = [("tile", (BK + 1, BN))] + pb[1:]
    try:
        wrong = run(pa, bad_b, pc)
        assert not np.allclose(wrong, ref, atol=1e-9)
    except (arr.ShapeMismatch, ValueError):
        pass


def test_matmul_views_equals_direct_convolution_and_plain_products():
    """The product over arranged operands: with the Section 4.3 programs it must equal the direct
    convolution (7 loops, here numpy's own sliding windows), with empty programs a plain product,
    with a permute a transposed one."""
    rng = np.random.default_rng(3)
    for (N, C, H, W, K, R, S), stride, pad in [((2, 3, 7, 6, 4, 3, 2), (1, 1), (0, 0)), ((1, 2, 8, 9, 3, 3, 3), (2, 1), (1, 2))]:
        x = rng.integers(-3, 4, (N, C, H, W)).astype(np.float64)
        w = rng.integers(-3, 4, (K, C, R, S)).astype(np.float64)
        P = (H + 2 * pad[0] - R) // stride[0] + 1
        Q = (W + 2 * pad[1] - S) // stride[1] + 1
        px, pw, py = arr.conv2d_operand_programs(R, S, C, stride, pad, P, Q, H, W)
        X, Wt, Y = arr.Tensor((N, C, H, W)), arr.Tensor((K, C, R, S)), arr.Tensor((N, K, P, Q))
        got = arr.matmul_views(arr.run_program(X, px), arr.run_program(Wt, pw), arr.run_program(Y, py),
                               x.ravel(), w.ravel(), np.full(N * K * P * Q, np.nan)).reshape(N, K, P, Q)
        xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
        ref = np.zeros((N, K, P, Q))
        for p in range(P):
            for q in range(Q):
                patch = xp[:, :, p * stride[0]:p * stride[0] + R, q * stride[1]:q * stride[1] + S]
                ref[:, :, p, q] = np.einsum("ncrs,kcrs->nk", patch, w)
        assert np.array_equal(got, ref)
    a, b = rng.integers(-3, 4, (5, 4)).astype(np.float64), rng.integers(-3, 4, (4, 6)).astype(np.float64)
    A, B, Cc = arr.Tensor((5, 4)), arr.Tensor((4, 6)), arr.Tensor((5, 6))
    assert np.array_equal(arr.matmul_views(A, B, Cc, a.ravel(), b.ravel(), np.zeros(30)).reshape(5, 6), a @ b)
    # B handed over as its transpose's storage and viewed back through a permute
    Bt = arr.run_program(arr.Tensor((6, 4)), [("permute", (1, 0))])
    assert np.array_equal(arr.matmul_views(A, Bt, Cc, a.ravel(), b.T.copy().ravel(), np.zeros(30)).reshape(5, 6), a @ b)
    # every second row of A (a tile of height 1 every 2 rows, squeezed): a strided gather expressed as an arrangement
    A2 = arr.run_program(arr.Tensor((5, 4)), [("tile", (1, -1), (2, -1)), ("squeeze", 1), ("descend",), ("squeeze", 0), ("ascend",), ("ravel",)])
    C3 = arr.Tensor((3, 6))
    assert np.array_equal(arr.matmul_views(A2, B, C3, a.ravel(), b.ravel(), np.zeros(18)).reshape(3, 6), a[::2] @ b)
