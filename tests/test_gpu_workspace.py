"""GPU parity of the calls that go through the library's workspace when they overlap on one device, and of operands
whose last element a range-checked 16-byte load cannot fetch (odd pitches and extents, an operand that ends exactly at
the end of a page)."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import numeric as onum
from gpu_util import TORCH_DT, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def test_two_streams_share_the_workspace_without_racing():
    """Two streams issue different k-split convolutions and skinny products at the same time, several rounds, no host
    synchronisation in between: each partial-tile region is handed from one call to the next through the library's
    event, so every result must be the exact integer result of its own problem."""
    dt = "f16"
    # (a) convolution, 12 programs x 72 k tiles -> split; (b) another one with other sizes; (c), (d) skinny products
    Xa, Wa = si.conv_inputs(4, 512, 14, 14, 512, 3, 3, dt, seed=41, dist="int")
    Xb, Wb = si.conv_inputs(2, 256, 10, 10, 192, 3, 3, dt, seed=42, dist="int")
    Ac, Bc = si.gemm_inputs(16, 1024, 4096, dt, seed=43, dist="int")
    Ad, Bd = si.gemm_inputs(100, 520, 2048, dt, seed=44, dist="int")
    ref_a = onum.conv2d(Xa, Wa, dt, (1, 1), (0, 0), nthreads=16)
    ref_b = onum.conv2d(Xb, Wb, dt, (1, 1), (1, 1), nthreads=16)
    ref_c, ref_d = onum.gemm(Ac, Bc, dt), onum.gemm(Ad, Bd, dt)
    xa, wa, xb, wb = to_gpu(Xa, dt), to_gpu(Wa, dt), to_gpu(Xb, dt), to_gpu(Wb, dt)
    ac, bc, ad, bd = to_gpu(Ac, dt), to_gpu(Bc, dt), to_gpu(Ad, dt), to_gpu(Bd, dt)
    rounds = 6
    ya = [torch.full(ref_a.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    yb = [torch.full(ref_b.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    yc = [torch.full(ref_c.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    yd = [torch.full(ref_d.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for r in range(rounds):
        nt.conv2d_implicit(xa, wa, ya[r], (1, 1), (0, 0), stream=s1)
        assert nt.last_k_split() > 1
        nt.gemm(ac, bc, yc[r], stream=s2)
        assert nt.last_k_split() > 1
        nt.conv2d_implicit(xb, wb, yb[r], (1, 1), (1, 1), stream=s2)
        assert nt.last_k_split() > 1
        nt.gemm(ad, bd, yd[r], stream=s1)
        assert nt.last_k_split() > 1
    torch.cuda.synchronize()
    for r in range(rounds):
        assert np.array_equal(to_f64(ya[r]), ref_a), f"round {r}: convolution on stream 1"
        assert np.array_equal(to_f64(yb[r]), ref_b), f"round {r}: convolution on stream 2"
        assert np.array_equal(to_f64(yc[r]), ref_c), f"round {r}: product on stream 2"
        assert np.array_equal(to_f64(yd[r]), ref_d), f"round {r}: product on stream 1"


def test_two_streams_padded_copy_and_unfolded_routes():
    """The same for the convolutions whose zero-padded copy or unfolded input lives in the workspace."""
    dt = "f16"
    Xa, Wa = si.conv_inputs(4, 32, 20, 20, 64, 5, 5, dt, seed=51, dist="int")       # padding 2: padded copy
    Xb, Wb = si.conv_inputs(4, 32, 21, 21, 64, 3, 3, dt, seed=52, dist="int")       # stride 2: unfolded input
    ref_a = onum.conv2d(Xa, Wa, dt, (1, 1), (2, 2), nthreads=16)
    ref_b = onum.conv2d(Xb, Wb, dt, (2, 2), (1, 1), nthreads=16)
    xa, wa, xb, wb = to_gpu(Xa, dt), to_gpu(Wa, dt), to_gpu(Xb, dt), to_gpu(Wb, dt)
    rounds = 6
    ya = [torch.full(ref_a.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    yb = [torch.full(ref_b.shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(rounds)]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for r in range(rounds):
        nt.conv2d_implicit(xa, wa, ya[r], (1, 1), (2, 2), stream=s1)
        nt.conv2d_implicit(xb, wb, yb[r], (2, 2), (1, 1), stream=s2)
        assert nt.last_kernel_path() == nt.PATH_CONV_UNFOLD
    torch.cuda.synchronize()
    for r in range(rounds):
        assert np.array_equal(to_f64(ya[r]), ref_a), f"round {r}: padded copy"
        assert np.array_equal(to_f64(yb[r]), ref_b), f"round {r}: unfolded input"


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
@pytest.mark.parametrize("M,N,K", [(257, 259, 131), (300, 129, 97), (129, 131, 33), (255, 255, 31)])
def test_operand_that_ends_at_the_end_of_a_page(M, N, K, ta, tb):
    """Odd pitches and extents: the 4-byte word that holds an operand's last element would end 2 bytes past it, so a
    range-checked load drops it and the kernel fetches that element by itself.  Each operand is placed so that it
    ends exactly where a 4 KB page ends (NaNs follow where the allocation goes on); small integers: bit exact."""
    dt = "bf16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=7 * M + K, dist="int")
    ref = onum.gemm(A, B, dt)

    def at_page_end(X, transposed):
        X = X.T.copy() if transposed else X
        buf = torch.full((X.size + 4096,), float("nan"), dtype=TORCH_DT[dt], device="cuda")
        end = (buf.data_ptr() + 2 * X.size + 4095) // 4096 * 4096            # first page end at or after the data's size
        first = (end - buf.data_ptr()) // 2 - X.size
        v = buf[first:first + X.size]
        v.copy_(to_gpu(X, dt).reshape(-1))
        assert (v.data_ptr() + 2 * X.size) % 4096 == 0
        v = v.view(X.shape)
        return v.t() if transposed else v

    for tile in [(128, 128, 64), (256, 256, 64)]:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.gemm(at_page_end(A, ta), at_page_end(B, tb), C, tile=tile)
        torch.cuda.synchronize()
        assert nt.last_kernel_path() == nt.PATH_DIRECT
        assert np.array_equal(to_f64(C), ref), (tile, ta, tb)


def test_zero_fill_of_many_batch_entries():
    """K = 0 zero-fills C; the batch may exceed what one grid dimension holds."""
    Bn, M, N = 70000, 3, 5
    A = torch.empty((Bn, M, 0), dtype=torch.float16, device="cuda")
    B = torch.empty((Bn, 0, N), dtype=torch.float16, device="cuda")
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.bmm(A, B, C)
    torch.cuda.synchronize()
    assert (C == 0).all()
