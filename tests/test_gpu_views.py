"""GPU parity of nt_matmul_views (the matrix product over operands that are themselves arranged
tensors) against the oracle's view enumerator + fp64 product."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import arrangement as arr
from oracle import numeric as onum
from gpu_util import TORCH_DT, assert_gates, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def oracle_views(a_bits, pa, b_bits, pb, c_shape, pc, dt):
    A, B, Cc = arr.Tensor(a_bits.shape), arr.Tensor(b_bits.shape), arr.Tensor(c_shape)
    out = arr.matmul_views(arr.run_program(A, pa), arr.run_program(B, pb), arr.run_program(Cc, pc),
                           onum.decode(a_bits, dt).ravel(), onum.decode(b_bits, dt).ravel(), np.full(int(np.prod(c_shape)), np.nan))
    return out.reshape(c_shape)


@pytest.mark.parametrize("shape,stride,pad", [((2, 8, 12, 10, 16, 3, 3), (1, 1), (1, 1)), ((3, 5, 9, 11, 7, 3, 2), (2, 1), (1, 0)),
                                              ((1, 16, 20, 20, 130, 5, 5), (2, 2), (2, 2))])
@pytest.mark.parametrize("tile", [(64, 64, 32), None])
def test_convolution_written_as_an_arrangement_by_the_caller(shape, stride, pad, tile):
    """The Section 4.3 programs supplied through the public interface (integers: exact)."""
    dt = "f16"
    N, Cc, H, W, K, R, S = shape
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=5)
    X = si.small_int_bits(X.shape, dt, 6)
    Wt = si.small_int_bits(Wt.shape, dt, 7)
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    px, pw, py = arr.conv2d_operand_programs(R, S, Cc, stride, pad, P, Q, H, W)
    ref = oracle_views(X, px, Wt, pw, (N, K, P, Q), py, dt)
    assert np.array_equal(ref, onum.conv2d(X, Wt, dt, stride, pad))          # the oracle's two routes agree
    Y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(to_gpu(X, dt), px, to_gpu(Wt, dt), pw, Y, py, tile=tile)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(Y), ref)


@pytest.mark.parametrize("shape,stride,pad,want", [
    ((2, 32, 20, 24, 64, 3, 3), (1, 1), (1, 1), "direct"),        # dense, unit stride: the convolution kernel that streams into LDS
    ((32, 128, 20, 24, 256, 3, 3), (1, 1), (1, 1), "tap"),         # ... and the one that walks the reduction tap by tap
    ((2, 16, 21, 21, 64, 3, 3), (2, 2), (1, 1), "unfold"),        # strided: the unfolded input + the matrix kernels
    ((2, 8, 20, 20, 32, 5, 5), (1, 1), (2, 2), "padded"),         # two columns of padding: the zero-padded copy
])
def test_a_callers_convolution_views_reach_the_convolution_kernels(shape, stride, pad, want):
    """Views that address their tensors exactly like the Section 4.3 arrangement are recognised from their lowered index maps
    and run where nt_conv2d_implicit runs: same kernels, bit-identical output."""
    dt = "f16"
    N, Cc, H, W, K, R, S = shape
    X, Wt = si.small_int_bits((N, Cc, H, W), dt, 6), si.small_int_bits((K, Cc, R, S), dt, 7)
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    px, pw, py = arr.conv2d_operand_programs(R, S, Cc, stride, pad, P, Q, H, W)
    ref = onum.conv2d(X, Wt, dt, stride, pad, nthreads=16)
    x, w = to_gpu(X, dt), to_gpu(Wt, dt)
    Y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(x, px, w, pw, Y, py)
    torch.cuda.synchronize()
    path = nt.last_kernel_path()
    assert path == {"direct": nt.PATH_CONV_DIRECT, "tap": nt.PATH_CONV_TAP, "unfold": nt.PATH_CONV_UNFOLD, "padded": nt.PATH_CONV}[want]
    assert np.array_equal(to_f64(Y), ref)
    Y2 = torch.full((N, K, P, Q), float("nan"), dtype=torch.float32, device="cuda")
    nt.conv2d_implicit(x, w, Y2, stride, pad)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == path and torch.equal(Y, Y2)


@pytest.mark.parametrize("shape,stride,pad,dilation", [((2, 16, 20, 22, 64, 3, 3), (1, 1), (2, 2), (2, 2)), ((1, 8, 17, 19, 40, 3, 2), (2, 1), (1, 3), (1, 3)),
                                                       ((2, 32, 16, 16, 96, 3, 3), (1, 1), (0, 0), (3, 2))])
def test_dilated_convolution_views(shape, stride, pad, dilation):
    """The tile operation's dilation, through the public interface: against the oracle's view product and, for its element
    offsets, the oracle's enumerator (the unfolded input + the matrix kernels run it)."""
    dt = "bf16"
    N, Cc, H, W, K, R, S = shape
    X, Wt = si.small_int_bits((N, Cc, H, W), dt, 16), si.small_int_bits((K, Cc, R, S), dt, 17)
    P = (H + 2 * pad[0] - (R - 1) * dilation[0] - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - (S - 1) * dilation[1] - 1) // stride[1] + 1
    px, pw, py = arr.conv2d_operand_programs(R, S, Cc, stride, pad, P, Q, H, W, dilation)
    ref = oracle_views(X, px, Wt, pw, (N, K, P, Q), py, dt)
    for tile, want in ((None, nt.PATH_CONV_UNFOLD), ((64, 64, 32), nt.PATH_GENERIC)):
        Y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float32, device="cuda")
        nt.matmul_views(to_gpu(X, dt), px, to_gpu(Wt, dt), pw, Y, py, tile=tile)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == want
        assert np.array_equal(to_f64(Y), ref)


@pytest.mark.parametrize("G,Cg,Kg,hw,stride,pad,dilation,want", [
    (2, 32, 64, 24, (1, 1), (1, 1), (1, 1), "direct"),      # two groups, each on the convolution kernel
    (4, 8, 8, 15, (2, 2), (1, 1), (1, 1), "unfold"),        # strided groups
    (16, 1, 1, 12, (1, 1), (1, 1), (1, 1), None),            # depthwise: reduction of 9
    (3, 4, 6, 11, (1, 2), (2, 0), (2, 1), None),            # dilated groups
])
def test_grouped_convolution_as_a_batched_view(G, Cg, Kg, hw, stride, pad, dilation, want):
    dt = "f16"
    N, H, W, R, S = 2, hw, hw + 1, 3, 3
    X, Wt = si.small_int_bits((N, G * Cg, H, W), dt, 26), si.small_int_bits((G * Kg, Cg, R, S), dt, 27)
    P = (H + 2 * pad[0] - (R - 1) * dilation[0] - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - (S - 1) * dilation[1] - 1) // stride[1] + 1
    px, pw, py = arr.grouped_conv2d_view_programs(G, Cg, Kg, R, S, stride, pad, P, Q, H, W, dilation)
    ref = oracle_views(X, px, Wt, pw, (N, G * Kg, P, Q), py, dt)
    Y = torch.full((N, G * Kg, P, Q), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(to_gpu(X, dt), px, to_gpu(Wt, dt), pw, Y, py)
    torch.cuda.synchronize()
    if want:
        assert nt.last_kernel_path() == {"direct": nt.PATH_CONV_DIRECT, "unfold": nt.PATH_CONV_UNFOLD}[want]
    assert np.array_equal(to_f64(Y), ref)
    # the same views on the operand-map kernel (a tile named by the caller): one batched launch
    Y.fill_(float("nan"))
    nt.matmul_views(to_gpu(X, dt), px, to_gpu(Wt, dt), pw, Y, py, tile=(64, 64, 32))
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_GENERIC and np.array_equal(to_f64(Y), ref)


def test_plain_transposed_gathered_and_batched_views():
    dt, M, N, K = "bf16", 300, 260, 200
    A, B = si.gemm_inputs(M, N, K, dt, seed=8, dist="int")
    ref = onum.gemm(A, B, dt)
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    Cc = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(a, [], b, [], Cc, [])                                     # empty programs: the tensors themselves
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(Cc), ref) and nt.last_kernel_path() == nt.PATH_DIRECT
    bt = to_gpu(np.ascontiguousarray(B.T), dt)                                # [N, K] storage viewed as [K, N]
    Cc.fill_(float("nan"))
    nt.matmul_views(a, [], bt, [("permute", (1, 0))], Cc, [])
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(Cc), ref) and nt.last_kernel_path() == nt.PATH_DIRECT
    # every third row of A, written as an arrangement: tiles of height 1 every 3 rows, flattened back to a matrix
    gather = [("tile", (1, -1), (3, -1)), ("squeeze", 1), ("descend",), ("squeeze", 0), ("ascend",), ("ravel",)]
    # (a strided tiling has ceil((M - 1) / 3) + 1 = 101 tiles; the last starts at row 300, outside A, and reads as zeros)
    rows = -((1 - M) // 3) + 1
    C3 = torch.full((rows, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(a, gather, b, [], C3, [])
    torch.cuda.synchronize()
    want = np.vstack([onum.gemm(A[::3], B, dt), np.zeros((rows - len(range(0, M, 3)), N))])
    assert np.array_equal(to_f64(C3), want)
    assert np.array_equal(oracle_views(A, gather, B, [], (rows, N), [], dt), want)
    # batched: A stored [M, batch, K], viewed [batch, M, K]; C stored [batch, N, M], viewed [batch, M, N]
    Bn, M2, N2, K2 = 3, 70, 90, 40
    A3, B3 = si.gemm_inputs(M2, N2, K2, dt, seed=9, dist="int", batch=Bn)
    ref3 = onum.bmm(A3, B3, dt)
    a3 = to_gpu(np.ascontiguousarray(A3.transpose(1, 0, 2)), dt)
    c3 = torch.full((Bn, N2, M2), float("nan"), dtype=torch.float32, device="cuda")
    nt.matmul_views(a3, [("permute", (1, 0, 2))], to_gpu(B3, dt), [], c3, [("permute", (0, 2, 1))])
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(c3).transpose(0, 2, 1), ref3)


def test_matmul_views_errors():
    a = torch.zeros((8, 8), dtype=torch.float16, device="cuda")
    c = torch.zeros((8, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(nt.NtError):
        nt.matmul_views(a, [("tile", (4, 4))], a, [], c, [])                  # two levels left: not a view
    with pytest.raises(nt.NtError):
        nt.matmul_views(a, [("flatten", 0, 2)], a, [], c, [])                 # rank 1
    with pytest.raises(nt.NtError):
        nt.matmul_views(a, [], torch.zeros((9, 8), dtype=torch.float16, device="cuda"), [], c, [])   # inner sizes differ
