"""The entry point that allocates nothing (nt_gemm_noalloc) against nt_gemm, through the C ABI: the same kernels run, so
the outputs must agree bit for bit (and with the oracle within the benchmark's gates); two calls in a row, the second on
a smaller input, so that the shared scratch array still holds the first call's partial tiles when the second runs."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import numeric as onum
from gpu_util import TORCH_DT, assert_gates, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def test_gemm_noalloc_matches_gemm_on_two_calls_in_a_row():
    dt, out = "f16", "f16"
    cases = [(200, 640, 4096), (48, 264, 2048)]                     # skinny products: both split along K; the second is smaller
    results = []
    for M, N, K in cases:                                           # the two no-allocation calls back to back, nothing in between
        A, B = si.gemm_inputs(M, N, K, dt, seed=60 + M, dist="normal")
        a, b = to_gpu(A, dt), to_gpu(B, dt)
        C1 = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
        nt.gemm_noalloc(a, b, C1)
        assert nt.last_kernel_path() == nt.PATH_DIRECT and nt.last_k_split() > 1, (M, N, K)
        results.append((A, B, a, b, C1, nt.last_k_split()))
    torch.cuda.synchronize()
    for (M, N, K), (A, B, a, b, C1, split) in zip(cases, results):
        C0 = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
        nt.gemm(a, b, C0)
        assert nt.last_k_split() == split
        torch.cuda.synchronize()
        assert torch.equal(C0, C1), (M, N, K)
        assert_gates(to_f64(C1), onum.gemm(A, B, dt, nthreads=8), out, f"noalloc {M}x{N}x{K}")


def test_gemm_noalloc_without_a_split_and_exact_integers():
    # a product that needs no scratch memory, an overhanging one, and integer data (exact) in fp32
    for M, N, K in [(512, 512, 256), (300, 200, 100), (16, 1024, 4096)]:
        A, B = si.gemm_inputs(M, N, K, "bf16", seed=M, dist="int")
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        nt.gemm_noalloc(to_gpu(A, "bf16"), to_gpu(B, "bf16"), C)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(C), onum.gemm(A, B, "bf16")), (M, N, K)


def test_gemm_noalloc_refuses_a_split_beyond_its_scratch():
    # 64 programs of 256 x 256 and 256 k tiles: the library would deal K to 4 parts = 64 MiB of partial tiles
    M = N = 2048
    K = 16384
    a = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    b = torch.zeros((K, N), dtype=torch.float16, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.gemm(a, b, C, tile=(256, 256, 64))
    torch.cuda.synchronize()
    assert nt.last_k_split() == 4
    C.fill_(float("nan"))
    with pytest.raises(nt.NtError) as e:
        nt.gemm_noalloc(a, b, C, tile=(256, 256, 64))
    assert e.value.status == 3 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(C).all()                                     # nothing was launched
