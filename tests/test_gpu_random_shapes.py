"""Seeded random problem shapes against the oracle, bit for bit (small integers: every sum is exact in fp32 and is
rounded once to the output format).  The shapes are drawn so that every route of a convolution (implicit kernels, with
and without the k split; zero-padded copy; unfolded input; operand map) and of a product (plain and range-checked
direct loads, ragged K, odd pitches, k split) comes up."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import numeric as onum
from gpu_util import TORCH_DT, to_gpu

pytestmark = pytest.mark.gpu


def _conv_cases(seed, count, long_reduction):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        N = int(rng.integers(1, 5))
        C = int(rng.choice([32, 64, 96, 128, 256] if long_reduction else [3, 8, 16, 24, 32, 64]))
        H, W = (int(rng.integers(5, 15)), int(rng.integers(5, 15))) if long_reduction else (int(rng.integers(4, 20)), int(rng.integers(4, 20)))
        K = int(rng.choice([8, 24, 40, 64, 72, 128, 136]))
        R, S = int(rng.choice([1, 3, 5, 7] if long_reduction else [1, 2, 3, 5])), int(rng.choice([1, 3, 5, 7] if long_reduction else [1, 2, 3, 5]))
        sh, sw = (1, 1) if long_reduction else (int(rng.choice([1, 1, 2])), int(rng.choice([1, 1, 2])))
        ph, pw = int(rng.integers(0, 4 if long_reduction else 3)), int(rng.integers(0, 4 if long_reduction else 3))
        dt, out = str(rng.choice(["f16", "bf16"])), str(rng.choice(["f32", "f16", "bf16"]))
        nhwc = bool(rng.integers(0, 2))
        if H + 2 * ph >= R and W + 2 * pw >= S:
            cases.append((N, C, H, W, K, R, S, sh, sw, ph, pw, dt, out, nhwc))
    return cases


@pytest.mark.parametrize("case", _conv_cases(2024, 24, False) + _conv_cases(77, 24, True), ids=lambda c: "-".join(str(v) for v in c))
def test_random_convolutions(case):
    N, C, H, W, K, R, S, sh, sw, ph, pw, dt, out, nhwc = case
    X, Wt = si.conv_inputs(N, C, H, W, K, R, S, dt, seed=100 + N + C + H + W + K, dist="int")
    ref = onum.conv2d(X, Wt, dt, (sh, sw), (ph, pw))
    want = torch.from_numpy(ref).to(torch.float32).to(TORCH_DT[out])
    x = to_gpu(X.transpose(0, 2, 3, 1).copy(), dt).permute(0, 3, 1, 2) if nhwc else to_gpu(X, dt)
    Y = torch.full(ref.shape, float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.conv2d_implicit(x, to_gpu(Wt, dt), Y, (sh, sw), (ph, pw))
    torch.cuda.synchronize()
    assert torch.equal(Y.cpu(), want), f"path {nt.last_kernel_path()}, k split {nt.last_k_split()}"


def _mm_cases(seed, count, long_reduction):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        if long_reduction:
            M, N = int(rng.integers(1, 300)), int(rng.integers(1, 300))
            K = int(rng.choice([64 * rng.integers(32, 130), rng.integers(2048, 8000)]))
        else:
            M, N = int(rng.integers(1, 600)), int(rng.integers(1, 600))
            K = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000)]))
        cases.append((M, N, K, str(rng.choice(["f16", "bf16"])), str(rng.choice(["f32", "f16", "bf16"])), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", _mm_cases(2025, 24, False) + _mm_cases(78, 24, True), ids=lambda c: "-".join(str(v) for v in c))
def test_random_products(case):
    M, N, K, dt, out, ta, tb = case
    A, B = si.gemm_inputs(M, N, K, dt, seed=300 + M + N + K, dist="int")
    want = torch.from_numpy(onum.gemm(A, B, dt)).to(torch.float32).to(TORCH_DT[out])
    a = to_gpu(A.T.copy(), dt).t() if ta else to_gpu(A, dt)
    b = to_gpu(B.T.copy(), dt).t() if tb else to_gpu(B, dt)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.gemm(a, b, C)
    torch.cuda.synchronize()
    assert torch.equal(C.cpu(), want), f"path {nt.last_kernel_path()}, k split {nt.last_k_split()}"
