"""Pins for the extensions of the tile operation that the convolution views need (dilation; a grouped convolution written
as one batched view): the oracle's arrangement machinery against the textbook definition of the convolution, written out
as loops on tiny inputs, and against closed forms of the index map."""
import itertools

import numpy as np
import pytest

from oracle import arrangement as arr


def conv_by_definition(x, w, stride, pad, dilation, groups):
    """y[n, f, p, q] = sum over c, r, s of x[n, g Cg + c, p sh + r dh - ph, q sw + s dw - pw] * w[f, c, r, s], g = f // Kg."""
    N, C, H, W = x.shape
    F, Cg, R, S = w.shape
    Kg = F // groups
    P = (H + 2 * pad[0] - (R - 1) * dilation[0] - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - (S - 1) * dilation[1] - 1) // stride[1] + 1
    y = np.zeros((N, F, P, Q))
    for n, f, p, q in itertools.product(range(N), range(F), range(P), range(Q)):
        g = f // Kg
        acc = 0.0
        for c, r, s in itertools.product(range(Cg), range(R), range(S)):
            h, ww = p * stride[0] + r * dilation[0] - pad[0], q * stride[1] + s * dilation[1] - pad[1]
            if 0 <= h < H and 0 <= ww < W:
                acc += x[n, g * Cg + c, h, ww] * w[f, c, r, s]
        y[n, f, p, q] = acc
    return y


def test_dilated_tile_closed_form():
    """Tile o, element j of a 1-D tensor of n elements with unit stride in memory: offset o * stride + j * dilation - pad,
    masked outside [0, n); as many tiles as fit with their span (t - 1) * dilation + 1, rounded up."""
    n, t, st, dil, lo, hi = 23, 4, 3, 2, 2, 1
    a = arr.Tensor((n,)).tile((t,), (st,), ((lo, hi),), (dil,))
    span = (t - 1) * dil + 1
    n_tiles = -(-(n + lo + hi - span) // st) + 1
    assert a.levels == [(n_tiles,), (t,)]
    for o in range(n_tiles):
        off, mask, shp = arr.tile_index_set(a, o)
        want = o * st + np.arange(t) * dil - lo
        ok = (want >= 0) & (want < n)
        assert shp == (t,) and np.array_equal(mask, ok.astype(np.uint8)) and np.array_equal(off, np.where(ok, want, -1))
    # dilation 1 is the tile of the paper
    b, c = arr.Tensor((n,)).tile((t,), (st,), ((lo, hi),)), arr.Tensor((n,)).tile((t,), (st,), ((lo, hi),), (1,))
    for o in range(b.levels[0][0]):
        assert all(np.array_equal(u, v) for u, v in zip(arr.tile_index_set(b, o)[:2], arr.tile_index_set(c, o)[:2]))


@pytest.mark.parametrize("stride,pad,dilation", [((1, 1), (0, 0), (2, 2)), ((1, 1), (2, 2), (2, 2)), ((2, 1), (1, 3), (1, 3)),
                                                 ((2, 2), (2, 1), (2, 1)), ((1, 1), (1, 1), (1, 1))])
def test_dilated_convolution_through_the_arrangement(stride, pad, dilation):
    rng = np.random.default_rng(5)
    N, C, H, W, F, R, S = 2, 3, 9, 8, 4, 3, 2
    x = rng.integers(-3, 4, (N, C, H, W)).astype(np.float64)
    w = rng.integers(-3, 4, (F, C, R, S)).astype(np.float64)
    want = conv_by_definition(x, w, stride, pad, dilation, 1)
    P, Q = want.shape[2:]
    a, b, c = arr.conv2d_arrangement(arr.Tensor(x.shape), arr.Tensor(w.shape), arr.Tensor(want.shape), 8, 4, 8, stride, pad, dilation)
    got = arr.apply_mm(a, b, c, x.ravel(), w.ravel(), np.full(want.size, np.nan)).reshape(want.shape)
    assert np.array_equal(got, want)
    # the same through the single-level views and the view product
    px, pw, py = arr.conv2d_operand_programs(R, S, C, stride, pad, P, Q, H, W, dilation)
    got = arr.matmul_views(arr.run_program(arr.Tensor(x.shape), px), arr.run_program(arr.Tensor(w.shape), pw),
                           arr.run_program(arr.Tensor(want.shape), py), x.ravel(), w.ravel(), np.full(want.size, np.nan))
    assert np.array_equal(got.reshape(want.shape), want)


@pytest.mark.parametrize("G,Cg,Kg", [(2, 3, 2), (4, 1, 1), (3, 2, 1), (1, 4, 3)])
@pytest.mark.parametrize("stride,pad,dilation", [((1, 1), (1, 1), (1, 1)), ((2, 1), (0, 2), (1, 2))])
def test_grouped_convolution_as_one_batched_view(G, Cg, Kg, stride, pad, dilation):
    rng = np.random.default_rng(11 * G + Cg)
    N, H, W, R, S = 2, 7, 6, 3, 3
    x = rng.integers(-3, 4, (N, G * Cg, H, W)).astype(np.float64)
    w = rng.integers(-3, 4, (G * Kg, Cg, R, S)).astype(np.float64)
    want = conv_by_definition(x, w, stride, pad, dilation, G)
    P, Q = want.shape[2:]
    px, pw, py = arr.grouped_conv2d_view_programs(G, Cg, Kg, R, S, stride, pad, P, Q, H, W, dilation)
    va, vb, vc = arr.run_program(arr.Tensor(x.shape), px), arr.run_program(arr.Tensor(w.shape), pw), arr.run_program(arr.Tensor(want.shape), py)
    assert va.levels == [(G, N * P * Q, Cg * R * S)] and vb.levels == [(G, Cg * R * S, Kg)] and vc.levels == [(G, N * P * Q, Kg)]
    got = arr.matmul_views(va, vb, vc, x.ravel(), w.ravel(), np.full(want.size, np.nan))
    assert np.array_equal(got.reshape(want.shape), want)
    # every output element is written exactly once: the output view is a permutation of the tensor
    off, mask = arr.view_index_set(vc)
    assert mask.all() and np.array_equal(np.sort(off.ravel()), np.arange(want.size))
