"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element
on sizes the oracle finishes in seconds, covering several tiles, ragged tails, every operand
orientation, both input formats, all output formats and the degenerate cases."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import arrangement as arr
from oracle import numeric as onum
from gpu_util import TORCH_DT, assert_gates, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def run_gemm(A, B, dt, out, tile, M, N):
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.gemm(to_gpu(A, dt), to_gpu(B, dt), C, tile=tile)
    torch.cuda.synchronize()
    return to_f64(C)


def test_c1_256_cubed_tile_64x64x32():
    cfg = si.CONFIGS["c1_f16_256"]
    A, B = si.gemm_inputs(256, 256, 256, "f16", cfg["seed"], cfg["dist"])
    ref = onum.gemm(A, B, "f16")
    got = run_gemm(A, B, "f16", "f16", (64, 64, 32), 256, 256)
    assert_gates(got, ref, "f16", "c1")
    got32 = run_gemm(A, B, "f16", "f32", (64, 64, 32), 256, 256)
    assert_gates(got32, ref, "f32", "c1 f32 out")


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [(64, 64, 32), (128, 128, 64), (256, 128, 64), (128, 256, 64), (256, 256, 64), None])
@pytest.mark.parametrize("M,N,K", [(300, 260, 200), (512, 512, 256), (257, 129, 65), (1, 1, 1), (129, 520, 72)])
def test_gemm_shapes_and_tiles(dt, tile, M, N, K):
    A, B = si.gemm_inputs(M, N, K, dt, seed=M + N + K, dist="uniform")
    ref = onum.gemm(A, B, dt)
    got = run_gemm(A, B, dt, "f32", tile, M, N)
    assert_gates(got, ref, "f32", f"{dt} {M}x{N}x{K} tile {tile}")


@pytest.mark.parametrize("out", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_output_formats_round_to_nearest_even(dt, out):
    M, N, K = 200, 264, 136
    A, B = si.gemm_inputs(M, N, K, dt, seed=5, dist="normal")
    ref = onum.gemm(A, B, dt)
    got = run_gemm(A, B, dt, out, (128, 128, 64), M, N)
    assert_gates(got, ref, out, f"{dt}->{out}")
    if out != "f32":
        # the stored value must be the fp32 accumulator rounded once: compare with the fp32 run
        acc = torch.from_numpy(run_gemm(A, B, dt, "f32", (128, 128, 64), M, N)).to(torch.float32)
        assert np.array_equal(to_f64(acc.to(TORCH_DT[out])), got)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [(64, 64, 32), (128, 128, 64), (256, 256, 64)])
def test_integer_inputs_are_exact(dt, tile):
    # small integers: every product and partial sum is exact in fp32, so the result is bit exact
    M, N, K = 260, 300, 190
    A, B = si.gemm_inputs(M, N, K, dt, seed=2, dist="int")
    ref = onum.gemm(A, B, dt)
    got = run_gemm(A, B, dt, "f32", tile, M, N)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("tc", [False, True])
@pytest.mark.parametrize("M,N,K,tile", [(384, 256, 192, (128, 128, 64)), (301, 263, 131, (128, 128, 64)),
                                        (301, 263, 131, (64, 64, 32)), (512, 512, 128, (256, 256, 64))])
def test_operand_orientations(ta, tb, tc, M, N, K, tile):
    """A, B, C given as transposed views (unit stride along the other axis)."""
    dt = "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=9, dist="uniform")
    ref = onum.gemm(A, B, dt)
    At = to_gpu(A.T.copy(), dt).t() if ta else to_gpu(A, dt)
    Bt = to_gpu(B.T.copy(), dt).t() if tb else to_gpu(B, dt)
    Cs = torch.full((N, M) if tc else (M, N), float("nan"), dtype=torch.float32, device="cuda")
    Cv = Cs.t() if tc else Cs
    assert At.shape == (M, K) and Bt.shape == (K, N) and Cv.shape == (M, N)
    nt.gemm(At, Bt, Cv, tile=tile)
    torch.cuda.synchronize()
    assert_gates(to_f64(Cv), ref, "f32", f"ta={ta} tb={tb} tc={tc}")



@pytest.mark.parametrize("tile", [(128, 128, 64), (256, 256, 64)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
@pytest.mark.parametrize("r", [1, 2, 3, 4, 5, 6, 7, 8, 9, 15])
def test_ragged_remainders_of_every_length(r, ta, tb, tile):
    """Every possible length of the partial vector at the ragged end of M, N and K, for both
    memory orientations of A and B; small integers make the comparison bit exact, and NaNs
    planted right behind the operands must never reach the result."""
    dt = "bf16"
    M, N, K = tile[0] + r, tile[1] + 16 - r, 64 + r
    A, B = si.gemm_inputs(M, N, K, dt, seed=100 + r, dist="int")
    ref = onum.gemm(A, B, dt)

    def planted(X, transposed):
        X = X.T.copy() if transposed else X
        buf = torch.full((X.size + 64,), float("nan"), dtype=TORCH_DT[dt], device="cuda")
        buf[:X.size] = to_gpu(X, dt).reshape(-1)
        v = buf[:X.size].view(X.shape)
        return v.t() if transposed else v

    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.gemm(planted(A, ta), planted(B, tb), C, tile=tile)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), ref)


@pytest.mark.parametrize("M,N,K", [(300, 7, 100), (7, 300, 100), (300, 300, 7), (300, 8, 8), (8, 8, 8), (300, 300, 9)])
def test_axes_shorter_than_one_vector(M, N, K):
    """Operands shorter than one 16-byte vector along an axis (the vector loaders' lower limit)."""
    dt = "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=M + 3 * N + 5 * K, dist="int")
    ref = onum.gemm(A, B, dt)
    for tile in [(128, 128, 64), (256, 256, 64)]:
        for ta in (False, True):
            for tb in (False, True):
                At = to_gpu(A.T.copy(), dt).t() if ta else to_gpu(A, dt)
                Bt = to_gpu(B.T.copy(), dt).t() if tb else to_gpu(B, dt)
                C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
                nt.gemm(At, Bt, C, tile=tile)
                torch.cuda.synchronize()
                assert np.array_equal(to_f64(C), ref), (tile, ta, tb)



@pytest.mark.parametrize("out", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("M,N,K,tile", [(256, 256, 128, (128, 128, 64)), (512, 512, 256, (256, 256, 64)), (300, 264, 200, (128, 128, 64)),
                                        (301, 263, 131, (256, 256, 64)), (150, 170, 90, (64, 64, 32)), (512, 768, 128, None)])
def test_addmm_full_input(M, N, K, tile, out):
    """beta * input + alpha * (A . B) on the direct, staged and operand-map kernels."""
    dt = "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=21, dist="normal")
    rng = np.random.default_rng(23)
    Ival = rng.standard_normal((M, N)).astype(np.float32)
    Iten = torch.from_numpy(Ival).to(TORCH_DT[out]).cuda()
    ref = onum.addmm(to_f64(Iten), A, B, dt, alpha=0.75, beta=-1.5)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.addmm(Iten, to_gpu(A, dt), to_gpu(B, dt), C, alpha=0.75, beta=-1.5, tile=tile)
    torch.cuda.synchronize()
    assert_gates(to_f64(C), ref, out, f"addmm {M}x{N}x{K} {tile} {out}")


@pytest.mark.parametrize("tile", [(64, 64, 32), (128, 128, 64), (256, 256, 64)])
def test_addmm_bias_broadcast_and_exact_integers(tile):
    dt, M, N, K = "bf16", 260, 300, 72
    A, B = si.gemm_inputs(M, N, K, dt, seed=31, dist="int")
    prod = onum.gemm(A, B, dt)
    rng = np.random.default_rng(32)
    row = torch.from_numpy(rng.integers(-8, 8, (N,)).astype(np.float32)).cuda()
    col = torch.from_numpy(rng.integers(-8, 8, (M, 1)).astype(np.float32)).cuda()
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    for inp, alpha, beta in [(row, 1.0, 1.0), (col, 2.0, -3.0), (row, -1.0, 0.5)]:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(inp, a, b, C, alpha=alpha, beta=beta, tile=tile)
        torch.cuda.synchronize()
        ref = onum.addmm(inp.cpu().numpy().astype(np.float64), A, B, dt, alpha=alpha, beta=beta)
        assert np.array_equal(to_f64(C), ref), (tile, alpha, beta)
    # beta = 0: the input is not read (NaNs in it must not reach C); alpha alone scales
    nan = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.addmm(nan, a, b, C, alpha=2.0, beta=0.0, tile=tile)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), 2.0 * prod)
    # in place: C doubles as the input
    C = torch.from_numpy(rng.integers(-8, 8, (M, N)).astype(np.float32)).cuda()
    ref = onum.addmm(to_f64(C), A, B, dt, alpha=1.0, beta=1.0)
    nt.addmm(C, a, b, C, tile=tile)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), ref)


def test_addmm_strided_input_transposed_output_and_k_zero():
    dt, M, N, K = "f16", 200, 136, 96
    A, B = si.gemm_inputs(M, N, K, dt, seed=41, dist="int")
    rng = np.random.default_rng(42)
    It = torch.from_numpy(rng.integers(-8, 8, (N, M)).astype(np.float32)).cuda()      # input given transposed
    ref = onum.addmm(to_f64(It.t()), A, B, dt, alpha=1.0, beta=2.0)
    for tile in [(64, 64, 32), (128, 128, 64)]:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(It.t(), to_gpu(A, dt), to_gpu(B, dt), C, alpha=1.0, beta=2.0, tile=tile)
        Ct = torch.full((N, M), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(It.t(), to_gpu(A, dt), to_gpu(B, dt), Ct.t(), alpha=1.0, beta=2.0, tile=tile)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(C), ref) and np.array_equal(to_f64(Ct.t()), ref)
    # K = 0: C = beta * input
    A0 = torch.empty((M, 0), dtype=torch.float16, device="cuda")
    B0 = torch.empty((0, N), dtype=torch.float16, device="cuda")
    for tile in [None, (128, 128, 64)]:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(It.t(), A0, B0, C, alpha=3.0, beta=-2.0, tile=tile)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(C), -2.0 * to_f64(It.t()))
    with pytest.raises(nt.NtError):
        nt.addmm(It, to_gpu(A, dt), to_gpu(B, dt), torch.empty((M, N), dtype=torch.float32, device="cuda"))   # [N, M] input


@pytest.mark.parametrize("act", ["relu", "silu", "gelu_tanh"])
@pytest.mark.parametrize("M,N,K,tile,out,path", [(512, 512, 256, (256, 256, 64), "f16", "direct"), (256, 384, 128, (128, 128, 64), "f32", "direct"),
                                                 (301, 263, 131, (256, 256, 64), "bf16", "direct"), (300, 264, 200, (128, 256, 64), "f32", "direct"),
                                                 (301, 263, 131, (256, 256, 64), "bf16", "staged"), (300, 264, 200, (128, 256, 64), "f32", "staged"),
                                                 (150, 170, 90, (64, 64, 32), "f16", "generic")])
def test_addmm_fused_activation(M, N, K, tile, out, path, act):
    """act(beta * bias + alpha * (A . B)): the activation acts on the fp32 combined value in every epilogue."""
    dt = "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=51, dist="normal")
    A = si.round_to_bits(onum.decode(A, dt).astype(np.float32) * 12.0, dt)         # spread the results over the activations' bends
    bias = torch.from_numpy(np.random.default_rng(52).standard_normal((N,)).astype(np.float32)).to(TORCH_DT[out]).cuda()
    ref = onum.addmm_act(to_f64(bias), A, B, dt, act, alpha=0.5, beta=2.0)
    # (ragged, odd-pitched problems stream directly as well; a column-major output takes the staged kernel)
    C = torch.full((N, M), float("nan"), dtype=TORCH_DT[out], device="cuda").t() if path == "staged" else \
        torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.addmm(bias, to_gpu(A, dt), to_gpu(B, dt), C, alpha=0.5, beta=2.0, tile=tile, act=act)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == {"direct": nt.PATH_DIRECT, "staged": nt.PATH_STAGED, "generic": nt.PATH_GENERIC}[path]
    if out == "f32":
        # fp32 accumulation plus the activation's fast exponential / reciprocal (a few ulp of fp32)
        assert np.abs(to_f64(C) - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max())
    else:
        assert_gates(to_f64(C), ref, out, f"addmm_act {act} {M}x{N}x{K} {tile} {out}")
    assert (to_f64(C) < 0).any() == (act != "relu")                                 # the case does reach the negative side


def test_addmm_activation_without_input_strided_output_and_errors():
    dt, M, N, K = "bf16", 136, 200, 64
    A, B = si.gemm_inputs(M, N, K, dt, seed=61, dist="int")
    prod = onum.gemm(A, B, dt)
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    for tile in [(64, 64, 32), (128, 128, 64)]:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(None, a, b, C, alpha=-1.0, beta=0.0, tile=tile, act="relu")         # exact: small integers
        Ct = torch.full((N, M), float("nan"), dtype=torch.float32, device="cuda")
        nt.addmm(None, a, b, Ct.t(), alpha=-1.0, beta=0.0, tile=tile, act="relu")    # column-major C: element-wise store routine
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(C), np.maximum(-prod, 0.0)) and np.array_equal(to_f64(Ct.t()), np.maximum(-prod, 0.0))
    # K = 0: act(beta * input)
    inp = torch.from_numpy(np.random.default_rng(62).integers(-8, 8, (M, N)).astype(np.float32)).cuda()
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.addmm(inp, torch.empty((M, 0), dtype=torch.bfloat16, device="cuda"), torch.empty((0, N), dtype=torch.bfloat16, device="cuda"), C,
             alpha=1.0, beta=-1.0, act="relu")
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), np.maximum(-to_f64(inp), 0.0))
    with pytest.raises(ValueError):
        nt.addmm(inp, a, b, C, act="tanh")
    with pytest.raises(nt.NtError):
        nt.addmm(None, a, b, C, beta=1.0, act="relu")                                # beta != 0 needs an input


def test_general_strides_and_padded_pitch():
    dt, M, N, K = "bf16", 150, 170, 90
    A, B = si.gemm_inputs(M, N, K, dt, seed=4, dist="uniform")
    ref = onum.gemm(A, B, dt)
    # A embedded with row pitch K+3 and column step 2; B with pitch N+5; C with pitch N+7
    Abuf = torch.zeros((M, 2 * K + 3), dtype=TORCH_DT[dt], device="cuda")
    Abuf[:, 0:2 * K:2] = to_gpu(A, dt)
    Bbuf = torch.zeros((K, N + 5), dtype=TORCH_DT[dt], device="cuda")
    Bbuf[:, :N] = to_gpu(B, dt)
    Cbuf = torch.full((M, N + 7), -5.0, dtype=torch.float32, device="cuda")
    for tile in [(64, 64, 32), (128, 128, 64)]:
        Cbuf.fill_(-5.0)
        nt.gemm(Abuf[:, 0:2 * K:2], Bbuf[:, :N], Cbuf[:, :N], tile=tile)
        torch.cuda.synchronize()
        assert_gates(to_f64(Cbuf[:, :N]), ref, "f32", f"strided {tile}")
        assert (Cbuf[:, N:] == -5.0).all(), "store outside the C view"


def test_unaligned_base_pointers():
    # operands that start 2 bytes off a 16-byte boundary and have odd pitches (like the ragged bf16 case)
    dt, M, N, K = "bf16", 271, 333, 199
    A, B = si.gemm_inputs(M, N, K, dt, seed=6, dist="uniform")
    ref = onum.gemm(A, B, dt)
    Ab = torch.zeros(M * K + 1, dtype=TORCH_DT[dt], device="cuda")
    Bb = torch.zeros(K * N + 3, dtype=TORCH_DT[dt], device="cuda")
    Ab[1:] = to_gpu(A, dt).reshape(-1)
    Bb[3:] = to_gpu(B, dt).reshape(-1)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.gemm(Ab[1:].view(M, K), Bb[3:].view(K, N), C, tile=(128, 128, 64))
    torch.cuda.synchronize()
    assert_gates(to_f64(C), ref, "f32", "unaligned")


@pytest.mark.parametrize("tile", [(64, 64, 32), (128, 128, 64), None])
def test_bmm_small(tile):
    dt, Bn, M, N, K = "f16", 3, 200, 136, 72
    A, B = si.gemm_inputs(M, N, K, dt, seed=8, dist="normal", batch=Bn)
    ref = onum.bmm(A, B, dt)
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.bmm(to_gpu(A, dt), to_gpu(B, dt), C, tile=tile)
    torch.cuda.synchronize()
    assert_gates(to_f64(C), ref, "f16", f"bmm {tile}")


def test_bmm_strided_batch_views():
    dt, Bn, M, N, K = "f16", 4, 128, 128, 64
    A, B = si.gemm_inputs(M, N, K, dt, seed=12, dist="normal", batch=Bn)
    ref = onum.bmm(A, B, dt)
    # batch-minor storage: [M, batch, K] viewed as [batch, M, K]
    Ag = to_gpu(A.transpose(1, 0, 2).copy(), dt).permute(1, 0, 2)
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.bmm(Ag, to_gpu(B, dt), C, tile=(128, 128, 64))
    torch.cuda.synchronize()
    assert_gates(to_f64(C), ref, "f32", "bmm strided")


@pytest.mark.parametrize("shape,stride,pad,tile", [
    ((2, 8, 12, 14, 24, 3, 3), (1, 1), (1, 1), (64, 64, 32)),
    ((3, 16, 9, 10, 70, 3, 2), (2, 2), (1, 0), (64, 64, 32)),
    ((2, 32, 16, 16, 130, 3, 3), (1, 1), (1, 1), (128, 128, 64)),
    ((1, 5, 7, 7, 3, 1, 1), (1, 1), (0, 0), None),
    ((2, 6, 10, 8, 9, 3, 3), (2, 1), (2, 1), None),
    ((4, 64, 14, 14, 64, 3, 3), (1, 1), (1, 1), None),
])
def test_conv2d_small(shape, stride, pad, tile):
    N, Cc, H, W, K, R, S = shape
    dt = "f16"
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=13)
    ref = onum.conv2d(X, Wt, dt, stride, pad)
    Y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, stride, pad, tile=tile)
    torch.cuda.synchronize()
    assert_gates(to_f64(Y), ref, "f32", f"conv {shape} {stride} {pad}")


@pytest.mark.parametrize("dt,out", [("f16", "f32"), ("bf16", "bf16"), ("f16", "f16")])
@pytest.mark.parametrize("shape,pad,tile", [
    ((2, 32, 16, 16, 130, 3, 3), (1, 1), (256, 128, 64)),     # ragged filters and k tail
    ((3, 16, 8, 24, 256, 3, 3), (1, 1), (256, 256, 64)),      # M = 576: last tile rows masked
    ((2, 8, 10, 10, 64, 3, 3), (0, 0), (256, 128, 64)),       # no padding, M < one tile
    ((1, 8, 8, 18, 128, 3, 3), (1, 0), (256, 128, 64)),       # padding along h only
    ((2, 64, 8, 8, 128, 1, 1), (0, 0), (256, 128, 64)),       # 1x1 filter
    ((2, 4, 9, 8, 256, 5, 3), (2, 1), (256, 256, 64)),        # 5x3 filter
    ((5, 64, 24, 16, 256, 3, 3), (1, 1), None),               # library default tile
])
def test_conv2d_dense_unit_stride(shape, pad, tile, dt, out):
    """Shapes the dedicated implicit-GEMM kernel takes: contiguous NCHW, stride 1 (here with Q % 8 == 0)."""
    N, Cc, H, W, K, R, S = shape
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=21)
    ref = onum.conv2d(X, Wt, dt, (1, 1), pad)
    assert ref.shape[3] % 8 == 0
    Y = torch.full(ref.shape, float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, (1, 1), pad, tile=tile)
    torch.cuda.synchronize()
    # whole 32-k slices (C * R * S a multiple of 32) stream straight into LDS, other reductions are staged through registers
    assert nt.last_kernel_path() in ((nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP) if (Cc * R * S) % 32 == 0 else (nt.PATH_CONV,))
    assert_gates(to_f64(Y), ref, out, f"conv dense {shape} {pad} {tile}")


@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32")])
@pytest.mark.parametrize("M,N,K,tile", [(500, 512, 256, None), (1000, 520, 192, (128, 128, 64)), (264, 776, 128, (256, 256, 64)),
                                        (1032, 264, 320, (128, 256, 64)), (520, 1000, 64, (256, 128, 64)), (8, 8, 64, (128, 128, 64)),
                                        # ragged K, odd pitches (rows with 2-byte alignment), odd extents (an operand's last
                                        # element shares its 4-byte word with the byte after the operand)
                                        (301, 263, 131, (256, 256, 64)), (129, 257, 1999, None), (500, 512, 200, (128, 256, 64)),
                                        (255, 513, 95, (256, 128, 64)), (77, 33, 17, (128, 128, 64)), (64, 128, 30, None),
                                        (9, 1001, 4097, None)])
def test_overhanging_tiles_on_the_direct_kernel(M, N, K, tile, dt, out):
    """M / N not multiples of the tile, K not a multiple of the slice, rows of any alignment: the direct-to-LDS kernel
    with range-checked loads, the tail of K zeroed in LDS, and masked stores, in all four operand orientations (bit
    exact: integer inputs)."""
    A, B = si.gemm_inputs(M, N, K, dt, seed=81, dist="int")
    ref = onum.gemm(A, B, dt)
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    at, bt = a.t().contiguous().t(), b.t().contiguous().t()          # column-major A, B stored [N, K]
    for aa, bb in [(a, b), (a, bt), (at, b), (at, bt)]:
        buf = torch.full((M + 2, N + 8), float("nan"), dtype=TORCH_DT[out], device="cuda")   # what lies around C must stay untouched
        C = buf[1:M + 1, :N]
        nt.gemm(aa, bb, C, tile=tile)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == nt.PATH_DIRECT
        assert np.array_equal(to_f64(C), ref)
        assert torch.isnan(buf[0]).all() and torch.isnan(buf[M + 1]).all() and torch.isnan(buf[:, N:]).all()


def test_overhanging_tiles_bmm_and_bias_on_the_direct_kernel():
    dt, Bn, M, N, K = "f16", 3, 300, 392, 128
    A, B = si.gemm_inputs(M, N, K, dt, seed=82, dist="normal", batch=Bn)
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.bmm(to_gpu(A, dt), to_gpu(B, dt), C)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_DIRECT
    assert_gates(to_f64(C), onum.bmm(A, B, dt), "f16", "bmm with overhanging tiles")
    bias = torch.from_numpy(np.random.default_rng(83).standard_normal((N,)).astype(np.float32)).half().cuda()
    C2 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.addmm(bias, to_gpu(A[0], dt), to_gpu(B[0], dt), C2, alpha=1.0, beta=1.0, act="silu")
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_DIRECT
    assert_gates(to_f64(C2), onum.addmm_act(to_f64(bias), A[0], B[0], dt, "silu"), "f16", "bias + silu with overhanging tiles")


@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32")])
@pytest.mark.parametrize("M,N,K", [(16, 1024, 4096), (100, 520, 2048), (8, 264, 3072), (200, 256, 2048)])
def test_skinny_products_split_along_k(M, N, K, dt, out):
    """Few output tiles and a long reduction: K is dealt to several programs per tile (a batched product over equal
    parts of K into fp32 slices of the library's workspace) and a second kernel adds the slices and applies the
    epilogue.  Small integers: exact whatever the order; every operand orientation; what lies around C stays untouched."""
    A, B = si.gemm_inputs(M, N, K, dt, seed=91, dist="int")
    ref = onum.gemm(A, B, dt)
    want = torch.from_numpy(ref).to(torch.float32).to(TORCH_DT[out])      # integers below 2^24, rounded once
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    at, bt = a.t().contiguous().t(), b.t().contiguous().t()
    for aa, bb in [(a, b), (a, bt), (at, b), (at, bt)]:
        buf = torch.full((M + 2, N + 8), float("nan"), dtype=TORCH_DT[out], device="cuda")
        C = buf[1:M + 1, :N]
        nt.gemm(aa, bb, C)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() in (nt.PATH_DIRECT, nt.PATH_STAGED) and nt.last_k_split() > 1
        assert torch.equal(C.cpu(), want)
        assert torch.isnan(buf[0]).all() and torch.isnan(buf[M + 1]).all() and torch.isnan(buf[:, N:]).all()


def test_k_split_is_left_alone_where_it_does_not_pay():
    for M, N, K in [(1024, 1024, 1024), (4096, 4096, 4096), (512, 2048, 1024)]:
        A, B = si.gemm_inputs(M, N, K, "f16", seed=94, dist="int")
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        nt.gemm(to_gpu(A, "f16"), to_gpu(B, "f16"), C)
        torch.cuda.synchronize()
        assert nt.last_k_split() == 1, (M, N, K)
    assert np.array_equal(to_f64(C), onum.gemm(A, B, "f16"))


def test_skinny_addmm_split_along_k_applies_the_epilogue_once():
    # bias row + activation after the sum of the parts; transposed (column-major) output; random data against the oracle
    dt, M, N, K = "f16", 48, 640, 4096
    A, B = si.gemm_inputs(M, N, K, dt, seed=92, dist="normal")
    bias = torch.from_numpy(np.random.default_rng(93).standard_normal((N,)).astype(np.float32)).half().cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda").t()
    nt.addmm(bias, to_gpu(A, dt), to_gpu(B, dt), C, alpha=0.5, beta=2.0, act="gelu_tanh")
    C2 = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda").t()
    nt.addmm(bias, to_gpu(A, dt), to_gpu(B, dt), C2, alpha=0.5, beta=2.0, act="gelu_tanh")
    torch.cuda.synchronize()
    assert nt.last_k_split() == 8                                         # 5 programs of 128 x 128, 64 k tiles
    assert torch.equal(C, C2)                                             # fixed order of the sums: the same bits
    assert_gates(to_f64(C), onum.addmm_act(to_f64(bias), A, B, dt, "gelu_tanh", alpha=0.5, beta=2.0), "f16", "skinny addmm")


def test_kernel_paths_are_the_intended_ones():
    """Operands with unit stride along an axis stream directly into LDS (aligned full tiles with plain loads, ragged or
    unaligned problems with range-checked ones), an output without unit stride along n takes the staged kernel, other
    strides and tiny tiles the operand-map kernel; strided and widely padded convolutions unfold their input into the
    workspace unless the caller names a tile."""
    def path_of(M, N, K, tile=None, view=None):
        A, B = si.gemm_inputs(M, N, K, "f16", seed=1, dist="int")
        a, b = to_gpu(A, "f16"), to_gpu(B, "f16")
        if view == "strided_a":
            buf = torch.zeros((M, 2 * K), dtype=torch.float16, device="cuda")
            buf[:, ::2] = a
            a = buf[:, ::2]
        Cc = torch.empty((N, M), dtype=torch.float16, device="cuda").t() if view == "strided_c" else torch.empty((M, N), dtype=torch.float16, device="cuda")
        nt.gemm(a, b, Cc, tile=tile)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(Cc), onum.gemm(A, B, "f16"))
        return nt.last_kernel_path()
    assert path_of(512, 512, 256) == nt.PATH_DIRECT
    assert path_of(512, 512, 256, tile=(256, 256, 64)) == nt.PATH_DIRECT
    assert path_of(500, 512, 256) == nt.PATH_DIRECT          # ragged M, whole k tiles: range-checked direct loads
    assert path_of(504, 520, 256, tile=(128, 128, 64)) == nt.PATH_DIRECT   # ragged M and N
    assert path_of(500, 512, 200) == nt.PATH_DIRECT          # ragged K: the tail of the last slice is zeroed in LDS
    assert path_of(512, 520, 264) == nt.PATH_DIRECT          # ragged N and K
    assert path_of(512, 516, 256, tile=(128, 128, 64)) == nt.PATH_DIRECT   # pitch of B not a multiple of 8: 2-byte aligned rows
    assert path_of(501, 515, 201) == nt.PATH_DIRECT          # everything odd
    assert path_of(512, 512, 256, view="strided_c") == nt.PATH_STAGED      # C without unit stride along n
    assert path_of(512, 512, 256, view="strided_a") == nt.PATH_GENERIC
    assert path_of(256, 256, 64, tile=(64, 64, 32)) == nt.PATH_GENERIC
    X, Wt = si.conv_inputs(2, 8, 16, 16, 128, 3, 3, "f16", seed=3)
    # (unit stride with two columns of padding: the convolution kernel on a zero-padded copy of the input)
    for stride, pad, want in [((1, 1), (1, 1), nt.PATH_CONV), ((2, 2), (1, 1), nt.PATH_CONV_UNFOLD), ((1, 1), (2, 2), nt.PATH_CONV)]:
        ref = onum.conv2d(X, Wt, "f16", stride, pad)
        Y = torch.empty(ref.shape, dtype=torch.float16, device="cuda")
        nt.conv2d_implicit(to_gpu(X, "f16"), to_gpu(Wt, "f16"), Y, stride, pad)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == want, (stride, pad)
        nt.conv2d_implicit(to_gpu(X, "f16"), to_gpu(Wt, "f16"), Y, stride, pad, tile=(64, 64, 32))      # a tile named by the caller: the index map
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == nt.PATH_GENERIC, (stride, pad)
        assert_gates(to_f64(Y), ref, "f16", f"conv {stride} {pad} through the index map")
        assert_gates(to_f64(Y), ref, "f16", f"conv {stride} {pad}")


@pytest.mark.parametrize("shape,pad", [
    ((4, 16, 14, 14, 128, 3, 3), (0, 0)),      # the paper's conv task in small: Q = 12
    ((4, 16, 14, 14, 128, 3, 3), (1, 1)),      # Q = 14, right padding inside the last run
    ((3, 8, 7, 7, 130, 3, 3), (1, 1)),         # W < 8: one run per row, seven positions
    ((2, 8, 9, 11, 128, 3, 3), (1, 1)),        # Q = 11
    ((2, 8, 12, 9, 128, 1, 1), (0, 0)),        # 1 x 1 filter, Q = 9: the last run holds one position
    ((1, 8, 6, 17, 128, 3, 2), (0, 1)),        # even filter width, Q = 18
    ((8, 4, 5, 5, 128, 5, 5), (2, 1)),         # Q = 3 < 8
    ((1, 24, 28, 28, 256, 3, 3), (1, 1)),      # Q = 28
    # the same with reductions that are whole 32-k slices (the kernel that streams its operands straight into LDS)
    ((4, 32, 14, 14, 128, 3, 3), (1, 1)),
    ((4, 32, 14, 14, 128, 3, 3), (0, 0)),
    ((3, 32, 7, 7, 130, 3, 3), (1, 1)),
    ((2, 64, 12, 9, 128, 1, 1), (0, 0)),
    ((1, 16, 6, 17, 128, 3, 2), (0, 1)),
    ((8, 32, 5, 5, 128, 5, 5), (2, 1)),
    ((1, 32, 28, 28, 256, 3, 3), (1, 1)),
    ((2, 32, 9, 11, 136, 3, 3), (1, 0)),
    # 64 filters or fewer: the kernel built for 64 filters per program (40: its second half-wavefront column is ragged)
    ((4, 32, 14, 14, 40, 3, 3), (1, 1)),
    ((2, 64, 9, 11, 64, 1, 1), (0, 0)),
    ((8, 32, 16, 16, 24, 3, 3), (1, 1)),
])
def test_conv2d_dense_rows_that_are_no_multiple_of_eight(shape, pad):
    """Output rows of any length: the kernel numbers positions with the row pitch rounded up to 8 and never stores the
    surplus.  Small integers: exact, so a wrong halo element, a missed padding column or a position stored in the wrong
    place changes the result; what lies around the output must stay untouched."""
    N, Cc, H, W, K, R, S = shape
    for dt, out in (("f16", "f32"), ("bf16", "bf16")):
        X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=23, dist="int")
        ref = onum.conv2d(X, Wt, dt, (1, 1), pad)
        buf = torch.full((ref.size + 64,), float("nan"), dtype=TORCH_DT[out], device="cuda")
        Y = buf[32:32 + ref.size].view(ref.shape)
        nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, (1, 1), pad)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() in ((nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP) if (Cc * R * S) % 32 == 0 else (nt.PATH_CONV,))
        # the sums are integers below 2^24: exact in fp32, then rounded once (to nearest even) to the output format
        want = torch.from_numpy(ref).to(torch.float32).to(TORCH_DT[out])
        assert torch.equal(Y.cpu(), want), f"conv {shape} {pad} {dt} {out}"
        assert torch.isnan(buf[:32]).all() and torch.isnan(buf[32 + ref.size:]).all()


@pytest.mark.parametrize("shape,pad", [
    ((4, 64, 14, 14, 128, 3, 3), (1, 1)),      # 9 k tiles: two parts (5 + 4)
    ((2, 100, 10, 10, 96, 3, 3), (1, 1)),      # K = 900: 15 k tiles in three parts, the last one ragged; 96 filters
    ((3, 256, 8, 8, 130, 3, 3), (0, 0)),       # 36 k tiles, Q = 6
    ((2, 512, 7, 7, 256, 1, 1), (0, 0)),       # 1 x 1 filter, 8 k tiles
    ((1, 128, 7, 7, 256, 3, 3), (1, 1)),       # 49 output positions: one tile of 256 rows, 18 k tiles in four parts
])
def test_conv2d_dense_split_along_k(shape, pad):
    """Few output tiles and a long reduction: the k tiles are dealt to several programs per output tile, whose fp32
    partial tiles a second kernel adds up.  Small integers: exact whatever the order of the sums, in every output format.  The output is a
    channel slice of a larger tensor (its batch stride is not its size) and what lies around it must stay untouched;
    the calls share one workspace, which grows from one shape to the next."""
    N, Cc, H, W, K, R, S = shape
    for dt, out in (("f16", "f32"), ("bf16", "bf16"), ("f16", "f16")):
        X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=29, dist="int")
        ref = onum.conv2d(X, Wt, dt, (1, 1), pad)
        big = torch.full((N, K + 3, ref.shape[2], ref.shape[3]), float("nan"), dtype=TORCH_DT[out], device="cuda")
        Y = big[:, 2:K + 2]
        nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, (1, 1), pad)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() in ((nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP) if (Cc * R * S) % 32 == 0 else (nt.PATH_CONV,))
        assert nt.last_k_split() > 1
        # the sums are integers below 2^24: exact in fp32, then rounded once (to nearest even) to the output format
        want = torch.from_numpy(ref).to(torch.float32).to(TORCH_DT[out])
        assert torch.equal(Y.cpu(), want), f"conv split {shape} {pad} {dt} {out}"
        assert torch.isnan(big[:, :2]).all() and torch.isnan(big[:, K + 2:]).all()


def test_conv2d_dense_split_along_k_is_reproducible():
    # the partial tiles are added in a fixed order: two runs give the same bits (random data, fp32 output)
    N, Cc, H, W, K, R, S = 4, 128, 14, 14, 128, 3, 3
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, "f16", seed=30)
    ref = onum.conv2d(X, Wt, "f16", (1, 1), (1, 1))
    x, w = to_gpu(X, "f16"), to_gpu(Wt, "f16")
    Y1 = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    Y2 = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    nt.conv2d_implicit(x, w, Y1, (1, 1), (1, 1))
    nt.conv2d_implicit(x, w, Y2, (1, 1), (1, 1))
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    assert_gates(to_f64(Y1), ref, "f32", "conv split, random data")


@pytest.mark.parametrize("shape,stride,pad", [
    ((4, 32, 28, 28, 64, 3, 3), (2, 2), (1, 1)),       # the strided 3 x 3 of a residual stage
    ((2, 64, 14, 14, 128, 1, 1), (2, 2), (0, 0)),      # strided 1 x 1 (downsample)
    ((2, 3, 32, 32, 64, 7, 7), (2, 2), (3, 3)),        # a stem: wide padding, few channels (C R S = 147)
    ((3, 16, 12, 12, 40, 5, 5), (1, 1), (2, 2)),       # 5 x 5, padding 2
    ((2, 32, 9, 11, 72, 7, 7), (1, 1), (3, 3)),        # 7 x 7, padding 3; C R S = 1568 (whole 32-k slices)
    ((2, 8, 6, 5, 16, 3, 3), (1, 1), (0, 2)),          # padding along w only; planes of 6 x 9 = 54 elements (groups of 8 cross planes)
    ((1, 8, 3, 3, 8, 1, 1), (1, 1), (0, 0)),           # 9 positions, nothing padded (only the channels-last view takes the copy)
    ((2, 8, 9, 7, 24, 3, 2), (2, 1), (2, 1)),          # mixed strides, 49 > P Q = 35 positions per image, ragged everything
    ((1, 8, 5, 5, 16, 3, 3), (2, 2), (1, 1)),          # 9 positions per image
])
def test_conv2d_through_the_workspace(shape, stride, pad):
    """Convolutions the implicit kernels do not take as they are.  Strided ones: the unfolded input is written once into
    the workspace and the product runs per image on the matrix kernels.  Unit-stride ones (wide padding, channels-last
    input): a dense zero-padded copy of the input is made and the implicit kernels run on it without padding.  Small
    integers: exact; NCHW and channels-last views; what lies around the output (a channel slice of a larger tensor)
    stays untouched."""
    N, Cc, H, W, K, R, S = shape
    for dt, out in (("f16", "f32"), ("bf16", "bf16")):
        X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=31, dist="int")
        ref = onum.conv2d(X, Wt, dt, stride, pad)
        want = torch.from_numpy(ref).to(torch.float32).to(TORCH_DT[out])
        for channels_last in (False, True):
            x = to_gpu(X.transpose(0, 2, 3, 1).copy(), dt).permute(0, 3, 1, 2) if channels_last else to_gpu(X, dt)
            big = torch.full((N, K + 3, ref.shape[2], ref.shape[3]), float("nan"), dtype=TORCH_DT[out], device="cuda")
            Y = big[:, 2:K + 2]
            nt.conv2d_implicit(x, to_gpu(Wt, dt), Y, stride, pad)
            torch.cuda.synchronize()
            if stride == (1, 1):
                assert nt.last_kernel_path() in ((nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP) if (Cc * R * S) % 32 == 0 else (nt.PATH_CONV,))
            else:
                assert nt.last_kernel_path() == nt.PATH_CONV_UNFOLD
            assert torch.equal(Y.cpu(), want), f"conv {shape} {stride} {pad} {dt} {out} channels_last={channels_last}"
            assert torch.isnan(big[:, :2]).all() and torch.isnan(big[:, K + 2:]).all()


def test_conv2d_dense_integer_exact_and_padding_edges():
    # small integers: exact; a wrong halo element or a missed padding row changes the result
    N, Cc, H, W, K, R, S = 2, 8, 16, 16, 128, 3, 3
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, "f16", seed=22, dist="int")
    ref = onum.conv2d(X, Wt, "f16", (1, 1), (1, 1))
    Y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    nt.conv2d_implicit(to_gpu(X, "f16"), to_gpu(Wt, "f16"), Y, (1, 1), (1, 1), tile=(256, 128, 64))
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(Y), ref)


def test_conv2d_channels_last_views():
    # NHWC storage presented as NCHW views: the index map is stride generic
    N, Cc, H, W, K, R, S = 2, 8, 9, 9, 16, 3, 3
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, "bf16", seed=14)
    ref = onum.conv2d(X, Wt, "bf16", (1, 1), (1, 1))
    Xg = to_gpu(X.transpose(0, 2, 3, 1).copy(), "bf16").permute(0, 3, 1, 2)
    Y = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda").permute(0, 3, 1, 2)
    nt.conv2d_implicit(Xg, to_gpu(Wt, "bf16"), Y, (1, 1), (1, 1))
    torch.cuda.synchronize()
    assert_gates(to_f64(Y), ref, "f32", "conv nhwc")


def test_degenerate_shapes():
    dt = "f16"
    z = torch.zeros((0,), dtype=torch.float16, device="cuda")
    # K = 0: C is zero-filled
    C = torch.full((5, 7), float("nan"), dtype=torch.float32, device="cuda")
    nt.gemm(z.view(5, 0), z.view(0, 7), C)
    torch.cuda.synchronize()
    assert (C == 0).all()
    # M = 0 / N = 0: nothing happens, no error
    nt.gemm(z.view(0, 4), torch.zeros((4, 7), dtype=torch.float16, device="cuda"), torch.zeros((0, 7), dtype=torch.float16, device="cuda"))
    nt.bmm(z.view(0, 4, 4), z.view(0, 4, 4), z.view(0, 4, 4))
    torch.cuda.synchronize()
    with pytest.raises(nt.NtError) as e:
        nt.gemm(torch.zeros((4, 5), dtype=torch.float16, device="cuda"), torch.zeros((6, 7), dtype=torch.float16, device="cuda"),
                torch.zeros((4, 7), dtype=torch.float16, device="cuda"))
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"


# ---------------------------------------------------------------- device index maps
def test_device_address_generator_matches_oracle():
    """The address generator used inside the kernels, dumped by a trace kernel, against
    the oracle's enumerator (bit exact)."""
    # matmul, ragged
    M, N, K, tile = 150, 170, 90, (64, 64, 32)
    a, b, c = arr.mm_arrangement(arr.Tensor((M, K)), arr.Tensor((K, N)), arr.Tensor((M, N)), *tile)
    d = (((M, K), None), ((K, N), None), ((M, N), None))
    for pid in [0, 2, 8]:
        for k in [0, 2]:
            for operand, t in ((0, a), (1, b)):
                off, mask = nt.trace_tile("gemm", *d, tile, operand, pid, k)
                o_off, o_mask, _ = arr.tile_index_set(t, pid, (k,))
                assert np.array_equal(off, o_off) and np.array_equal(mask, o_mask)
        off, mask = nt.trace_tile("gemm", *d, tile, 2, pid, 0)
        o_off, o_mask, _ = arr.tile_index_set(c, pid)
        assert np.array_equal(off, o_off) and np.array_equal(mask, o_mask)
    # convolution with stride and padding
    Nn, Cc, H, W, Kf, R, S, stride, pad = 2, 5, 9, 10, 70, 3, 3, (2, 1), (1, 1)
    P, Q = (H + 2 - R) // 2 + 1, (W + 2 - S) + 1
    a, b, c = arr.conv2d_arrangement(arr.Tensor((Nn, Cc, H, W)), arr.Tensor((Kf, Cc, R, S)), arr.Tensor((Nn, Kf, P, Q)),
                                     *tile, stride, pad)
    d = (((Nn, Cc, H, W), None), ((Kf, Cc, R, S), None), ((Nn, Kf, P, Q), None))
    G = a.levels[0][0] * a.levels[0][1]
    for pid in range(G):
        for k in range(a.levels[1][0]):
            for operand, t in ((0, a), (1, b)):
                off, mask = nt.trace_tile("conv2d", *d, tile, operand, pid, k, stride, pad)
                o_off, o_mask, _ = arr.tile_index_set(t, pid, (k,))
                assert np.array_equal(off, o_off) and np.array_equal(mask, o_mask)
        off, mask = nt.trace_tile("conv2d", *d, tile, 2, pid, 0, stride, pad)
        o_off, o_mask, _ = arr.tile_index_set(c, pid)
        assert np.array_equal(off, o_off) and np.array_equal(mask, o_mask)
    # batched
    Bn = 3
    a, b, c = arr.bmm_arrangement(arr.Tensor((Bn, M, K)), arr.Tensor((Bn, K, N)), arr.Tensor((Bn, M, N)), *tile)
    d = (((Bn, M, K), None), ((Bn, K, N), None), ((Bn, M, N), None))
    for pid in [0, 10, 26]:
        off, mask = nt.trace_tile("bmm", *d, tile, 0, pid, 1)
        o_off, o_mask, _ = arr.tile_index_set(a, pid, (1,))
        assert np.array_equal(off, o_off) and np.array_equal(mask, o_mask)


def test_convolution_with_a_channels_last_filter():
    """A filter stored (f, r, s, c) and described by its strides: the kernel that walks the reduction tap by tap reads it as it
    is (that is its own order); same result, bit for bit, as with the (f, c, r, s) filter."""
    dt = "f16"
    N, Cc, H, W, K, R, S, pad = 40, 64, 28, 28, 256, 3, 3, (1, 1)
    X, Wt = si.small_int_bits((N, Cc, H, W), dt, 31), si.small_int_bits((K, Cc, R, S), dt, 32)
    ref = onum.conv2d(X, Wt, dt, (1, 1), pad, nthreads=16)
    x, w = to_gpu(X, dt), to_gpu(Wt, dt)
    w_last = w.permute(0, 2, 3, 1).contiguous().permute(0, 3, 1, 2)              # same tensor, channels-last storage
    assert w_last.stride() == (R * S * Cc, 1, S * Cc, Cc) and torch.equal(w_last, w)
    for filt in (w, w_last):
        Y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
        nt.conv2d_implicit(x, filt, Y, (1, 1), pad, tile=(256, 256, 64))
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == nt.PATH_CONV_TAP
        assert np.array_equal(to_f64(Y), ref)
