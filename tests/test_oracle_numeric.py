"""Pins for the oracle's fp64 numerics (CPU only): exact special cases, hand-worked
products, closed forms, algebraic identities and an independent numpy second opinion."""
import os

import numpy as np
import pytest

from oracle import numeric as onum
import synthetic_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _hand(name):
    with open(os.path.join(GOLDEN, "hand_worked.txt")) as f:
        for ln in f:
            if ln.startswith(name + " "):
                return dict(p.split("=") for p in ln.split()[1:])
    raise KeyError(name)


def _mat(s):
    return np.array([[float(x) for x in row.split(",")] for row in s.split(";")])


def _bits(x, dt):
    return si.round_to_bits(np.asarray(x, dtype=np.float32), dt)


def test_decode_known_bit_patterns():
    f16 = {0x0000: 0.0, 0x3C00: 1.0, 0xC000: -2.0, 0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24,
           0x0400: 2.0 ** -14, 0x7BFF: 65504.0, 0x3555: 0.333251953125, 0xBC01: -(1 + 2.0 ** -10)}
    got = onum.decode(np.array(list(f16), dtype=np.uint16), "f16")
    assert got.tolist() == list(f16.values())
    bf = {0x3F80: 1.0, 0x4049: 3.140625, 0xBF00: -0.5, 0x0080: 2.0 ** -126, 0x3F81: 1.0078125}
    got = onum.decode(np.array(list(bf), dtype=np.uint16), "bf16")
    assert got.tolist() == list(bf.values())
    # exhaustive agreement with numpy's binary16 (finite values)
    allbits = np.arange(65536, dtype=np.uint16)
    ref = allbits.view(np.float16).astype(np.float64)
    got = onum.decode(allbits, "f16")
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin]) and np.isnan(got[np.isnan(ref)]).all()


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_hand_worked_products(dt):
    for name in ("gemm2", "gemm3"):
        kv = _hand(name)
        A, B, C = _mat(kv["A"]), _mat(kv["B"]), _mat(kv["C"])
        assert np.array_equal(onum.gemm(_bits(A, dt), _bits(B, dt), dt), C)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_identity_and_permutation(dt):
    A, _ = si.gemm_inputs(7, 7, 5, dt, seed=1, dist="uniform")
    Ad = onum.decode(A, dt)
    eye = _bits(np.eye(5), dt)
    assert np.array_equal(onum.gemm(A, eye, dt), Ad)                 # A . I = A, exactly
    perm = np.random.default_rng(0).permutation(5)
    Pm = np.zeros((5, 5)); Pm[perm, np.arange(5)] = 1.0               # column j picks row perm[j]
    assert np.array_equal(onum.gemm(A, _bits(Pm, dt), dt), Ad[:, perm])
    Pl = np.zeros((7, 7)); Pl[np.arange(7), np.random.default_rng(1).permutation(7)] = 1.0
    rows = Pl.argmax(1)
    assert np.array_equal(onum.gemm(_bits(Pl, dt), A.reshape(7, 5), dt), Ad[rows, :])


def test_all_ones_closed_form_and_non_commutativity():
    M, N, K = 6, 9, 37
    ones_a, ones_b = _bits(np.ones((M, K)), "f16"), _bits(np.ones((K, N)), "f16")
    assert np.array_equal(onum.gemm(ones_a, ones_b, "f16"), np.full((M, N), float(K)))
    # rank-1: (u 1^T)(1 v^T) = K u v^T -- catches a transposed operand
    u = np.arange(1, M + 1, dtype=np.float32)[:, None] * np.ones((1, K), np.float32)
    v = np.ones((K, 1), np.float32) * np.arange(1, N + 1, dtype=np.float32)[None, :]
    assert np.array_equal(onum.gemm(_bits(u, "f16"), _bits(v, "f16"), "f16"), K * np.outer(np.arange(1, M + 1), np.arange(1, N + 1)))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_transpose_identity_through_strides(dt):
    A, B = si.gemm_inputs(11, 13, 17, dt, seed=4, dist="uniform")
    C = onum.gemm(A, B, dt)
    Ct = onum.gemm(B.T, A.T, dt)              # strided (non-contiguous) views
    assert np.allclose(Ct, C.T, rtol=0, atol=1e-13)
    # column-major copies of the same matrices give the same product
    Af = np.asfortranarray(A)
    assert np.array_equal(onum.gemm(Af, B, dt), C)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_numpy_second_opinion_and_samples(dt):
    A, B = si.gemm_inputs(33, 29, 41, dt, seed=9, dist="normal")
    ref = onum.decode(A, dt) @ onum.decode(B, dt)
    C = onum.gemm(A, B, dt)
    assert np.allclose(C, ref, rtol=1e-13, atol=1e-14)
    assert np.array_equal(onum.gemm(A, B, dt, nthreads=4), C)
    ms, ns = np.array([0, 5, 32, 17]), np.array([28, 0, 3, 17])
    assert np.allclose(onum.gemm_samples(A, B, dt, ms, ns), C[ms, ns], rtol=1e-13, atol=1e-15)


def test_bmm_is_per_batch_gemm():
    A, B = si.gemm_inputs(5, 6, 7, "f16", seed=2, dist="uniform", batch=3)
    C = onum.bmm(A, B, "f16")
    for b in range(3):
        assert np.allclose(C[b], onum.decode(A[b], "f16") @ onum.decode(B[b], "f16"), rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_addmm_hand_worked_and_special_cases(dt):
    for name in ("addmm2", "addmm2_bias"):
        kv = _hand(name)
        A, B, I, C = _mat(kv["A"]), _mat(kv["B"]), _mat(kv["I"]), _mat(kv["C"])
        got = onum.addmm(I, _bits(A, dt), _bits(B, dt), dt, alpha=float(kv["alpha"]), beta=float(kv["beta"]))
        assert np.array_equal(got, C)
        # the same input handed over as 16-bit patterns
        got = onum.addmm(_bits(I, dt), _bits(A, dt), _bits(B, dt), dt, alpha=float(kv["alpha"]), beta=float(kv["beta"]), inp_dtype=dt)
        assert np.array_equal(got, C)
    A, B = si.gemm_inputs(9, 11, 6, dt, seed=3, dist="int")
    I = np.random.default_rng(5).integers(-8, 8, (9, 11)).astype(np.float64)
    prod = onum.gemm(A, B, dt)
    assert np.array_equal(onum.addmm(I, A, B, dt, alpha=1, beta=0), prod)                  # reduces to the product
    assert np.array_equal(onum.addmm(I, A, np.zeros_like(B), dt, alpha=7, beta=1), I)       # A . 0 = 0
    assert np.array_equal(onum.addmm(I, A, B, dt, alpha=-2, beta=0.5), 0.5 * I - 2 * prod)  # linearity (exact: small integers)
    nan = np.full((9, 11), np.nan)
    assert np.array_equal(onum.addmm(nan, A, B, dt, alpha=1, beta=0), prod)                 # beta = 0 drops the input
    # brute force, element by element
    Ad, Bd = onum.decode(A, dt), onum.decode(B, dt)
    ref = np.array([[3 * I[m, n] + 2 * sum(Ad[m, k] * Bd[k, n] for k in range(6)) for n in range(11)] for m in range(9)])
    assert np.array_equal(onum.addmm(I, A, B, dt, alpha=2, beta=3), ref)
    # column bias broadcasts along n, row bias along m
    col = np.arange(9, dtype=np.float64).reshape(9, 1)
    assert np.array_equal(onum.addmm(col, A, B, dt), prod + col)


def test_activation_pins():
    from scipy import special
    # relu: hand-worked product (tests/golden/hand_worked.txt)
    kv = _hand("addmm2_relu")
    A, B, I, C = _mat(kv["A"]), _mat(kv["B"]), _mat(kv["I"]), _mat(kv["C"])
    got = onum.addmm_act(I, _bits(A, "f16"), _bits(B, "f16"), "f16", "relu", alpha=float(kv["alpha"]), beta=float(kv["beta"]))
    assert np.array_equal(got, C)
    assert np.array_equal(onum.addmm_act(I, _bits(A, "f16"), _bits(B, "f16"), "f16", None, alpha=-1.0, beta=1.0), [[11, -52], [-93, 10]])
    x = np.linspace(-8.0, 8.0, 3201)
    for act in ("silu", "gelu_tanh"):
        y = onum.activation(x, act)
        assert onum.activation(0.0, act) == 0.0
        assert np.allclose(y - onum.activation(-x, act), x, rtol=0, atol=1e-14)      # f(x) - f(-x) = x for x * sigmoid-like gates
        assert np.allclose(onum.activation(40.0, act), 40.0) and abs(onum.activation(-40.0, act)) < 1e-15
    # silu: closed form at ln 3 (sigmoid = 3/4) and a library second opinion (logistic function)
    assert abs(onum.activation(np.log(3.0), "silu") - 0.75 * np.log(3.0)) < 1e-15
    assert np.allclose(onum.activation(x, "silu"), x * special.expit(x), rtol=1e-14, atol=1e-15)
    # gelu, tanh form: 0.5 (1 + tanh u) is the logistic function of 2u; and it approximates the
    # erf-based definition x Phi(x) to within 5e-4 (a wrong cubic coefficient or a dropped term leaves that band)
    u = np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)
    assert np.allclose(onum.activation(x, "gelu_tanh"), x * special.expit(2.0 * u), rtol=1e-13, atol=1e-15)
    exact = 0.5 * x * (1.0 + special.erf(x / np.sqrt(2.0)))
    assert np.abs(onum.activation(x, "gelu_tanh") - exact).max() < 5e-4
    assert np.abs(0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * x)) - exact).max() > 5e-3   # the planted mistake is visible
    assert np.array_equal(onum.activation(x, "relu"), np.where(x > 0, x, 0.0))


def test_conv_hand_worked():
    kv = _hand("conv_3x3_2x2")
    X, W, Y = _mat(kv["X"]), _mat(kv["W"]), _mat(kv["Y"])
    got = onum.conv2d(_bits(X[None, None], "f16"), _bits(W[None, None], "f16"), "f16")
    assert np.array_equal(got[0, 0], Y)
    Y2 = _mat(_hand("conv_3x3_ones_pad1")["Y"])
    got = onum.conv2d(_bits(X[None, None], "f16"), _bits(np.ones((1, 1, 3, 3)), "f16"), "f16", pad=(1, 1))
    assert np.array_equal(got[0, 0], Y2)


def test_conv_1x1_is_a_gemm():
    N, C, H, W, K = 2, 5, 3, 4, 6
    X, Wt = si.conv_inputs(N, C, H, W, K, 1, 1, "f16", seed=7)
    Y = onum.conv2d(X, Wt, "f16")
    # Y[n,:,p,q] = Wt[K,C] . X[n,:,p,q]
    Xm = X.transpose(1, 0, 2, 3).reshape(C, N * H * W)
    ref = onum.gemm(Wt.reshape(K, C), Xm, "f16").reshape(K, N, H, W).transpose(1, 0, 2, 3)
    assert np.allclose(Y, ref, rtol=0, atol=1e-14)


@pytest.mark.parametrize("stride,pad", [((1, 1), (0, 0)), ((1, 1), (1, 1)), ((2, 2), (1, 0)), ((2, 1), (2, 1))])
def test_conv_numpy_second_opinion(stride, pad):
    N, C, H, W, K, R, S = 2, 3, 7, 6, 4, 3, 2
    X, Wt = si.conv_inputs(N, C, H, W, K, R, S, "bf16", seed=8)
    Y = onum.conv2d(X, Wt, "bf16", stride, pad, nthreads=2)
    Xd = np.pad(onum.decode(X, "bf16"), ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    Wd = onum.decode(Wt, "bf16")
    win = np.lib.stride_tricks.sliding_window_view(Xd, (R, S), axis=(2, 3))[:, :, ::stride[0], ::stride[1]]
    ref = np.einsum("ncpqrs,kcrs->nkpq", win, Wd)
    assert Y.shape == ref.shape
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-14)
    idx = np.array([[0, 0, 0, 0], [1, 3, Y.shape[2] - 1, Y.shape[3] - 1], [1, 2, 1, 0]])
    got = onum.conv2d_samples(X, Wt, "bf16", idx, stride, pad)
    assert np.allclose(got, Y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]], rtol=1e-13, atol=1e-15)


def test_input_rounding_is_nearest_even():
    # bf16: 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7 -> rounds to 1.0; 1 + 3*2^-8 ties up
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    assert onum.decode(si.round_to_bits(x, "bf16"), "bf16").tolist() == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]
    # f16: 2049 is a tie between 2048 and 2050 -> 2048 (even)
    assert onum.decode(si.round_to_bits(np.array([2049.0, 2051.0]), "f16"), "f16").tolist() == [2048.0, 2052.0]
