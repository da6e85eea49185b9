"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the WHOLE output
of every workload against the fp64 oracle, with both gates of the benchmark definition evaluated as stated
there -- the largest absolute error over every element and the relative Frobenius error over the matrix."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import numeric as onum
from gpu_util import ABS_GATE, REL_GATE, REL_GATE_F32, TORCH_DT, to_f64, to_gpu

pytestmark = pytest.mark.gpu

THREADS = 16        # host threads of the oracle's row-partitioned loops


def check_whole(got, ref, out, abs_gate=True):
    """Both gates over every element of the output (got, ref: fp64 arrays of the same shape)."""
    assert got.shape == ref.shape
    d = got - ref
    if abs_gate:
        assert np.abs(d).max() <= ABS_GATE, f"max abs err {np.abs(d).max():.3e}"
    rel = np.linalg.norm(d.ravel()) / np.linalg.norm(ref.ravel())
    assert rel <= (REL_GATE_F32 if out == "f32" else REL_GATE), f"rel err {rel:.3e}"


check_samples = check_whole


@pytest.mark.parametrize("name", ["c2_f16_4096", "c3_bf16_ragged", "p_f16_8192"])
def test_full_size_gemm(name):
    cfg = si.CONFIGS[name]
    M, N, K, dt, out = cfg["M"], cfg["N"], cfg["K"], cfg["dtype"], cfg["out"]
    A, B = si.gemm_inputs(M, N, K, dt, cfg["seed"], cfg["dist"])
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.gemm(to_gpu(A, dt), to_gpu(B, dt), C)           # library default tile, as in the benchmark
    torch.cuda.synchronize()
    assert torch.isfinite(C).all()
    ref = onum.gemm(A, B, dt, nthreads=THREADS)        # every element of the product (Section 4.2)
    check_whole(to_f64(C), ref, out)
    if name == "c3_bf16_ragged":
        # also the bf16-output variant, gated on the relative error only (|C| reaches ~70, where
        # the bf16 spacing alone exceeds the absolute gate)
        Cb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        nt.gemm(to_gpu(A, dt), to_gpu(B, dt), Cb)
        torch.cuda.synchronize()
        check_whole(to_f64(Cb), ref, "bf16", abs_gate=False)
        assert np.array_equal(to_f64(C.to(torch.bfloat16)), to_f64(Cb))


def test_full_size_bmm():
    cfg = si.CONFIGS["c4_f16_bmm"]
    Bn, M, N, K, dt = cfg["batch"], cfg["M"], cfg["N"], cfg["K"], cfg["dtype"]
    A, B = si.gemm_inputs(M, N, K, dt, cfg["seed"], cfg["dist"], batch=Bn)
    C = torch.full((Bn, M, N), float("nan"), dtype=torch.float16, device="cuda")
    nt.bmm(to_gpu(A, dt), to_gpu(B, dt), C)
    torch.cuda.synchronize()
    assert torch.isfinite(C).all()
    ref = onum.bmm(A, B, dt, nthreads=THREADS)         # all 32 entries, every element
    check_whole(to_f64(C), ref, "f16")


def unfolded_input(Xn, R, S, pad):
    """A[m, kk] = x[c, p + r - pad, q + s - pad] of one image (Section 4.3, unit conv stride), zero outside:
    m = (p, q), kk = (c, r, s), as 16-bit patterns (the pattern 0 is +0.0 in both formats)."""
    C, H, W = Xn.shape
    P, Q = H + 2 * pad - R + 1, W + 2 * pad - S + 1
    Xp = np.zeros((C, H + 2 * pad, W + 2 * pad), dtype=np.uint16)
    Xp[:, pad:pad + H, pad:pad + W] = Xn
    U = np.empty((P, Q, C, R, S), dtype=np.uint16)
    for r in range(R):
        for s in range(S):
            U[:, :, :, r, s] = Xp[:, r:r + P, s:s + Q].transpose(1, 2, 0)
    return U.reshape(P * Q, C * R * S)


def test_full_size_conv():
    """Every output of all 32 images.  The reference for the whole tensor is the oracle's product over the
    unfolded input (the equality Section 4.3 rests on); on three whole images it is first checked, bit for bit,
    against the oracle's direct convolution (the two add the same terms in the same order, apart from the
    zeros the unfolded input holds where the direct loop skips)."""
    cfg = si.CONFIGS["c5_f16_conv"]
    N, Cc, H, W, K, R, S = (cfg[k] for k in ("N", "C", "H", "W", "K", "R", "S"))
    dt = cfg["dtype"]
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, cfg["seed"])
    Y = torch.full((N, K, H, W), float("nan"), dtype=torch.float16, device="cuda")
    nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, (1, 1), (1, 1))
    torch.cuda.synchronize()
    assert torch.isfinite(Y).all()
    Wm = Wt.reshape(K, Cc * R * S).T                   # [kk, f]
    ref = np.empty((N, K, H, W), dtype=np.float64)
    for n in range(N):
        ref[n] = onum.gemm(unfolded_input(X[n], R, S, 1), Wm, dt, nthreads=THREADS).T.reshape(K, H, W)
    for n in (0, 13, N - 1):
        direct = onum.conv2d(X[n:n + 1], Wt, dt, (1, 1), (1, 1), nthreads=THREADS)[0]
        assert np.array_equal(direct, ref[n])
    check_whole(to_f64(Y), ref, "f16")


@pytest.mark.parametrize("dt,out", [("f16", "f16"), ("bf16", "f32")])
@pytest.mark.parametrize("shape,pad", [
    ((16, 32, 56, 56, 256, 3, 3), 1),      # 1568 blocks of 32 positions on 256 units: a round of 224-position tiles, then lower ones
    ((9, 32, 60, 64, 512, 3, 3), 1),       # two tiles of filters per tile of positions
    ((33, 32, 30, 40, 256, 1, 1), 0),      # 1 x 1 filter, the last tile of the second kind ragged
    ((13, 64, 47, 53, 300, 3, 3), 1),      # rows of 53 positions (pitch 56), ragged filters
])
def test_conv_grids_of_more_programs_than_units(shape, pad, dt, out):
    """Grids of more programs than compute units: the kernel for 256 filters runs tiles of two heights (the first rounds
    32 positions higher than the last).  Every output against the oracle (reference as in test_full_size_conv)."""
    N, Cc, H, W, K, R, S = shape
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=27)
    P, Q = H + 2 * pad - R + 1, W + 2 * pad - S + 1
    Y = torch.full((N, K, P, Q), float("nan"), dtype=TORCH_DT[out], device="cuda")
    # (the tile of 256 filters is named: with reductions this short the library's own choice is the 128-filter tile)
    nt.conv2d_implicit(to_gpu(X, dt), to_gpu(Wt, dt), Y, (1, 1), (pad, pad), tile=(256, 256, 64))
    torch.cuda.synchronize()
    assert nt.last_kernel_path() == nt.PATH_CONV_TAP
    Wm = Wt.reshape(K, Cc * R * S).T
    ref = np.empty((N, K, P, Q), dtype=np.float64)
    for n in range(N):
        ref[n] = onum.gemm(unfolded_input(X[n], R, S, pad), Wm, dt, nthreads=THREADS).T.reshape(K, P, Q)
    direct = onum.conv2d(X[N - 1:N], Wt, dt, (1, 1), (pad, pad), nthreads=THREADS)[0]
    assert np.array_equal(direct, ref[N - 1])
    check_whole(to_f64(Y), ref, out)


@pytest.mark.parametrize("shape,want_split", [
    ((32, 512, 14, 14, 512, 3, 3), True),      # 56 tiles of 256 x 256, 72 k tiles: the 256-filter tile with its reduction in 4 parts (one round)
    ((8, 256, 56, 56, 256, 3, 3), None),       # 98 tiles: whatever the estimate picks
    ((64, 256, 14, 14, 512, 3, 3), None),      # 112 tiles
])
def test_conv_tile_and_split_chosen_together(shape, want_split):
    """Mid-sized grids, where the library weighs the 256-filter tile against the 128-filter one together with the split of
    the reduction: every output against the oracle (reference as in test_full_size_conv), and the same bits twice."""
    N, Cc, H, W, K, R, S = shape
    dt, pad = "f16", 1
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, seed=29)
    Y = torch.full((N, K, H, W), float("nan"), dtype=torch.float16, device="cuda")
    Y2 = torch.full((N, K, H, W), float("nan"), dtype=torch.float16, device="cuda")
    x, w = to_gpu(X, dt), to_gpu(Wt, dt)
    nt.conv2d_implicit(x, w, Y, (1, 1), (pad, pad))
    nt.conv2d_implicit(x, w, Y2, (1, 1), (pad, pad))
    torch.cuda.synchronize()
    assert nt.last_kernel_path() in (nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP)
    if want_split:
        assert nt.last_kernel_path() == nt.PATH_CONV_TAP and nt.last_k_split() > 1
    assert torch.equal(Y, Y2)
    Wm = Wt.reshape(K, Cc * R * S).T
    ref = np.empty((N, K, H, W), dtype=np.float64)
    for n in range(N):
        ref[n] = onum.gemm(unfolded_input(X[n], R, S, pad), Wm, dt, nthreads=THREADS).T.reshape(K, H, W)
    direct = onum.conv2d(X[N - 1:N], Wt[:32], dt, (1, 1), (pad, pad), nthreads=THREADS)[0]
    assert np.array_equal(direct, ref[N - 1, :32])
    check_whole(to_f64(Y), ref, "f16")


def test_full_size_conv_of_the_papers_kernel_list():
    """(4, 512, 14, 14) * (512, 512, 3, 3) in the launch configuration bench.py times (k split over 18 programs per
    output tile): every output against the oracle, and a second call gives the same bits."""
    cfg = si.CONFIGS["c6_f16_conv_paper"]
    N, Cc, H, W, K, R, S = (cfg[k] for k in ("N", "C", "H", "W", "K", "R", "S"))
    dt = cfg["dtype"]
    X, Wt = si.conv_inputs(N, Cc, H, W, K, R, S, dt, cfg["seed"])
    ref = onum.conv2d(X, Wt, dt, (1, 1), (0, 0), nthreads=THREADS)
    x, w = to_gpu(X, dt), to_gpu(Wt, dt)
    Y = torch.full(ref.shape, float("nan"), dtype=torch.float16, device="cuda")
    Y2 = torch.full(ref.shape, float("nan"), dtype=torch.float16, device="cuda")
    nt.conv2d_implicit(x, w, Y, (1, 1), (0, 0))
    nt.conv2d_implicit(x, w, Y2, (1, 1), (0, 0))
    torch.cuda.synchronize()
    assert nt.last_kernel_path() in (nt.PATH_CONV_DIRECT, nt.PATH_CONV_TAP) and nt.last_k_split() == 18
    assert torch.equal(Y, Y2)
    check_samples(to_f64(Y).ravel(), ref.ravel(), "f16")


@pytest.mark.parametrize("name", ["f1_f16_addmm", "f1_f16_bias_gelu"])
def test_full_size_addmm(name):
    cfg = si.CONFIGS[name]
    M, N, K, dt, out = cfg["M"], cfg["N"], cfg["K"], cfg["dtype"], cfg["out"]
    A, B = si.gemm_inputs(M, N, K, dt, cfg["seed"], cfg["dist"])
    row = cfg.get("bias") == "row"
    Ib = si.normal_bits((N,) if row else (M, N), out, cfg["seed"] + 2, 1.0)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DT[out], device="cuda")
    nt.addmm(to_gpu(Ib, out), to_gpu(A, dt), to_gpu(B, dt), C, alpha=cfg["alpha"], beta=cfg["beta"], act=cfg.get("act"))
    torch.cuda.synchronize()
    assert torch.isfinite(C).all()
    ref = onum.addmm_act(Ib, A, B, dt, cfg.get("act"), alpha=cfg["alpha"], beta=cfg["beta"], inp_dtype=out, nthreads=THREADS)
    check_whole(to_f64(C), ref, out)


def test_full_size_attention():
    from oracle import attention as oat
    cfg = si.CONFIGS["f4_f16_sdpa"]
    Bn, H, S, D, dt = cfg["B"], cfg["H"], cfg["S"], cfg["D"], cfg["dtype"]
    q, k, v = (si.normal_bits((Bn, H, S, D), dt, cfg["seed"] + i, 1.0) for i in range(3))
    out = torch.full((Bn, H, S, D), float("nan"), dtype=TORCH_DT[dt], device="cuda")
    nt.sdpa(to_gpu(q, dt), to_gpu(k, dt), to_gpu(v, dt), out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    # every output row is a convex combination of that head's value rows
    vd = to_f64(to_gpu(v, dt))
    od = to_f64(out)
    assert (od <= vd.max(axis=2, keepdims=True) + 1e-3).all() and (od >= vd.min(axis=2, keepdims=True) - 1e-3).all()
    # whole heads against the definition: first, last, and two in between (spread over batch entries and XCDs)
    for b, h in [(0, 0), (1, 17), (2, 30), (Bn - 1, H - 1)]:
        ref = oat.sdpa(q[b, h], k[b, h], v[b, h], dt)
        check_samples(od[b, h], ref, dt)


@pytest.mark.parametrize("name", ["f3_f16_add", "f3_f16_silu", "f3_f16_softmax", "f3_f16_rms_norm"])
def test_full_size_memory_bound_kernels(name):
    """The benchmark's inputs and launch; the whole output against the oracle (add: bit for bit; the others:
    one unit in the last place of the output format)."""
    from oracle import elementwise as oe
    cfg = si.CONFIGS[name]
    dt, kind = cfg["dtype"], cfg["kind"]
    bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    if kind in ("add", "silu"):
        n = cfg["n"]
        x = si.normal_bits((n,), dt, cfg["seed"], 2.0)
        out = torch.full((n,), float("nan"), dtype=TORCH_DT[dt], device="cuda")
        if kind == "add":
            y = si.normal_bits((n,), dt, cfg["seed"] + 1, 2.0)
            nt.add(to_gpu(x, dt), to_gpu(y, dt), out)
            torch.cuda.synchronize()
            assert np.array_equal(bits(out), oe.encode(oe.add(x, y, dt), dt))
            return
        nt.silu(to_gpu(x, dt), out)
        ref = oe.silu(x, dt)
    else:
        rows, cols = cfg["rows"], cfg["cols"]
        x = si.normal_bits((rows, cols), dt, cfg["seed"], 2.0)
        out = torch.full((rows, cols), float("nan"), dtype=TORCH_DT[dt], device="cuda")
        if kind == "softmax":
            nt.softmax(to_gpu(x, dt), out)
            ref = oe.softmax(x, dt)
        else:
            nt.rms_norm(to_gpu(x, dt), out, eps=cfg["eps"])
            ref = oe.rms_norm(x, dt, cfg["eps"])
    torch.cuda.synchronize()
    got = oe.decode(bits(out), dt)
    assert np.isfinite(got).all()
    assert (np.abs(got - ref) <= 2.0 ** -10 * np.abs(ref) + 2.0 ** -24).all()
