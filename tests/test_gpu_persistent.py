"""GPU parity of products whose 256 x 256 programs outnumber the compute units: there one workgroup per unit walks
several programs, the slices of consecutive programs forming one stream through the ring.  Every element against the
fp64 oracle, for program counts that are and are not multiples of the grid, one and several passes of the ring per
program, every operand orientation and output format, the fused epilogue, and batches dealt out over the XCDs."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import numeric as onum
from gpu_util import TORCH_DT, assert_gates, to_f64, to_gpu

pytestmark = pytest.mark.gpu

THREADS = 16
TILE = (256, 256, 64)


@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32"), ("bf16", "bf16")])
@pytest.mark.parametrize("M,N,K", [(4352, 4096, 128),      # 272 programs: 16 workgroups run a second one; one pass of the ring each
                                   (4096, 4352, 256),      # two passes
                                   (5120, 5376, 384),      # 420 programs, three passes
                                   (8192, 8448, 128)])     # 1056 programs: four or five per workgroup
def test_many_programs_per_unit(M, N, K, dt, out):
    A, B = si.gemm_inputs(M, N, K, dt, seed=31, dist="normal")
    ref = onum.gemm(A, B, dt, nthreads=THREADS)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.gemm(to_gpu(A, dt), to_gpu(B, dt), C, tile=TILE)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_DIRECT
    assert_gates(to_f64(C), ref, out, f"{M}x{N}x{K} {dt}->{out}")


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_many_programs_per_unit_orientations_exact(ta, tb):
    """Small integers: every product and sum is exact, so the result equals the oracle's bit for bit."""
    M, N, K, dt = 4352, 4096, 256, "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=33, dist="int")
    ref = onum.gemm(A, B, dt, nthreads=THREADS)
    At = to_gpu(A.T.copy(), dt).t() if ta else to_gpu(A, dt)
    Bt = to_gpu(B.T.copy(), dt).t() if tb else to_gpu(B, dt)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.gemm(At, Bt, C, tile=TILE)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_DIRECT
    assert np.array_equal(to_f64(C), ref)


@pytest.mark.parametrize("out", ["f16", "f32"])
def test_many_programs_per_unit_fused_epilogue(out):
    M, N, K, dt = 4352, 4096, 128, "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=35, dist="normal")
    rng = np.random.default_rng(37)
    Iten = torch.from_numpy(rng.standard_normal((M, N)).astype(np.float32)).to(TORCH_DT[out]).cuda()
    ref = onum.addmm(to_f64(Iten), A, B, dt, alpha=0.5, beta=-1.25)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.addmm(Iten, to_gpu(A, dt), to_gpu(B, dt), C, alpha=0.5, beta=-1.25, tile=TILE)
    torch.cuda.synchronize()
    assert_gates(to_f64(C), ref, out, f"addmm {out}")


@pytest.mark.parametrize("Bn,M,N,K", [(9, 1536, 1536, 128),     # 324 programs: a group of 8 entries, one per XCD, and one left over
                                      (20, 1024, 1024, 256),    # 320 programs: two groups of 8 and four left over
                                      (5, 2048, 2048, 128)])    # 320 programs, fewer entries than XCDs
def test_many_programs_per_unit_batched(Bn, M, N, K):
    dt = "f16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=39, dist="normal", batch=Bn)
    ref = onum.bmm(A, B, dt, nthreads=THREADS)
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.bmm(to_gpu(A, dt), to_gpu(B, dt), C, tile=TILE)
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_DIRECT
    assert_gates(to_f64(C), ref, "f16", f"bmm {Bn}x{M}x{N}x{K}")


def test_repeated_launches_agree_bit_for_bit():
    """Nothing in the walk depends on timing: two launches give identical bits."""
    M, N, K, dt = 4352, 4096, 256, "bf16"
    A, B = si.gemm_inputs(M, N, K, dt, seed=41, dist="normal")
    a, b = to_gpu(A, dt), to_gpu(B, dt)
    C1 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    C2 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    nt.gemm(a, b, C1, tile=TILE)
    nt.gemm(a, b, C2, tile=TILE)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)
