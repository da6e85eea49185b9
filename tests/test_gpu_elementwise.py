"""GPU parity of the memory-bound kernels (add, silu, softmax, rms_norm) against the fp64 oracle.

add is exact in fp32 for 16-bit operands up to one rounding, and that rounding is innocuous
(24 >= 2 * 11 + 2 significand bits), so its result must equal the correctly rounded sum bit for bit.
The other three are gated at one unit in the last place of the output format around the exact value
(half a unit for the final conversion, the rest for fp32 evaluation), plus the subnormal spacing."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import elementwise as oe
from gpu_util import TORCH_DT, to_gpu

pytestmark = pytest.mark.gpu

ULP = {"f16": 2.0 ** -10, "bf16": 2.0 ** -7}
TINY = {"f16": 2.0 ** -24, "bf16": 2.0 ** -133}


def bits_of(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_one_ulp(got_bits, ref, dt, what=""):
    got = oe.decode(got_bits, dt)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    bound = ULP[dt] * np.abs(ref) + TINY[dt]
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), f"{what}: |err| {err.flat[worst]:.3e} > {bound.flat[worst]:.3e} at {worst} (ref {ref.flat[worst]:.6e})"


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("n", [1, 7, 8, 1000, 1024 * 37 + 5, 1 << 20])
def test_add_is_correctly_rounded(dt, n):
    x, y = si.normal_bits((n,), dt, n, 3.0), si.normal_bits((n,), dt, n + 1, 300.0)
    out = torch.full((n,), float("nan"), dtype=TORCH_DT[dt], device="cuda")
    nt.add(to_gpu(x, dt), to_gpu(y, dt), out)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out), oe.encode(oe.add(x, y, dt), dt))


def test_add_ties_overflow_strides_alignment_and_errors():
    dt = "f16"
    x = si.round_to_bits(np.array([2048, 2050, 65504, -65504, 1, 0], dtype=np.float32), dt)
    y = si.round_to_bits(np.array([1, 1, 65504, -65504, 2.0 ** -24, -0.0], dtype=np.float32), dt)
    out = torch.empty(6, dtype=torch.float16, device="cuda")
    nt.add(to_gpu(x, dt), to_gpu(y, dt), out, block_size=4)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [2048.0, 2052.0, float("inf"), float("-inf"), 1.0, 0.0]
    # strided views, a base pointer 2 bytes off a 16-byte boundary, in place
    n = 5000
    a, b = si.normal_bits((2 * n + 1,), dt, 1, 2.0), si.normal_bits((3 * n,), dt, 2, 2.0)
    ga, gb = to_gpu(a, dt), to_gpu(b, dt)
    o = torch.zeros(n + 1, dtype=torch.float16, device="cuda")
    nt.add(ga[1::2], gb[::3], o[1:])
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(o[1:]), oe.encode(oe.add(a[1::2], b[::3], dt), dt)) and o[0].item() == 0.0
    o2 = ga[1:n + 1].clone()
    nt.add(o2, gb[:n], o2)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(o2), oe.encode(oe.add(a[1:n + 1], b[:n], dt), dt))
    with pytest.raises(nt.NtError):
        nt.add(ga[:10], gb[:11], o[:10])
    with pytest.raises(nt.NtError):
        nt.add(ga[:10], gb[:10], o[:10], block_size=-1)
    nt.add(ga[:0], gb[:0], o[:0])                                  # empty: nothing happens


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("n", [5, 4096, 1024 * 129 + 3])
def test_silu(dt, n):
    x = si.normal_bits((n,), dt, n, 4.0)
    x[:4] = si.round_to_bits(np.array([0.0, -0.0, 20.0, -20.0], dtype=np.float32), dt)[: min(4, n)]
    out = torch.full((n,), float("nan"), dtype=TORCH_DT[dt], device="cuda")
    nt.silu(to_gpu(x, dt), out)
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(out), oe.silu(x, dt), dt, f"silu {dt} {n}")
    xs = to_gpu(x, dt)
    o = torch.zeros(2 * n, dtype=TORCH_DT[dt], device="cuda")
    nt.silu(xs, o[::2])                                            # strided output
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(o[::2]), oe.silu(x, dt), dt, "silu strided")
    assert not o[1::2].any()


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("rows,cols", [(5, 8), (33, 512), (7, 520), (16, 4096), (3, 8192), (4, 8200), (9, 301), (2, 20000)])
def test_softmax_and_rms_norm(dt, rows, cols):
    x = si.normal_bits((rows, cols), dt, rows * cols, 3.0)
    gx = to_gpu(x, dt)
    out = torch.full((rows, cols), float("nan"), dtype=TORCH_DT[dt], device="cuda")
    nt.softmax(gx, out)
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(out), oe.softmax(x, dt), dt, f"softmax {dt} {rows}x{cols}")
    for eps in (0.0, 1e-5):
        out.fill_(float("nan"))
        nt.rms_norm(gx, out, eps=eps)
        torch.cuda.synchronize()
        assert_one_ulp(bits_of(out), oe.rms_norm(x, dt, eps), dt, f"rms_norm {dt} {rows}x{cols} eps={eps}")


def test_row_kernels_padded_pitch_transposed_views_and_extremes():
    dt, rows, cols = "f16", 12, 1024
    x = si.normal_bits((rows, cols), dt, 9, 2.0)
    buf = torch.zeros((rows, cols + 24), dtype=torch.float16, device="cuda")
    buf[:, 8:8 + cols] = to_gpu(x, dt)
    obuf = torch.full((rows, cols + 8), -3.0, dtype=torch.float16, device="cuda")
    nt.softmax(buf[:, 8:8 + cols], obuf[:, :cols])                  # row pitch differs from the row length
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(obuf[:, :cols]), oe.softmax(x, dt), dt, "softmax padded")
    assert (obuf[:, cols:] == -3.0).all()
    xt = to_gpu(np.ascontiguousarray(x.T), dt)                     # [cols, rows] storage, viewed as [rows, cols]
    ot = torch.empty((cols, rows), dtype=torch.float16, device="cuda")
    nt.rms_norm(xt.t(), ot.t(), eps=1e-6)
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(ot.t()), oe.rms_norm(x, dt, 1e-6), dt, "rms_norm transposed")
    # large entries must not overflow the exponentials; a dominant entry takes all the mass
    big = si.round_to_bits(np.array([[60000.0, 59990.0, -60000.0, 0.0] * 2], dtype=np.float32), dt)
    o = torch.empty((1, 8), dtype=torch.float16, device="cuda")
    nt.softmax(to_gpu(big, dt), o)
    torch.cuda.synchronize()
    assert_one_ulp(bits_of(o), oe.softmax(big, dt), dt, "softmax extremes")
    z = torch.zeros((3, 64), dtype=torch.float16, device="cuda")
    o = torch.full((3, 64), float("nan"), dtype=torch.float16, device="cuda")
    nt.rms_norm(z, o, eps=1e-6)
    torch.cuda.synchronize()
    assert not o.any()
    with pytest.raises(nt.NtError):
        nt.softmax(z, torch.empty((3, 65), dtype=torch.float16, device="cuda"))
    with pytest.raises(nt.NtError):
        nt.rms_norm(z, o, eps=-1.0)


def test_prepared_call_is_the_same_call():
    """nt.prepare marshals a call once; the function it returns repeats exactly that call."""
    x = torch.randn(4099, device="cuda").half()
    y = torch.randn(4099, device="cuda").half()
    a, b = torch.empty_like(x), torch.full_like(x, float("nan"))
    nt.add(x, y, a)
    again = nt.prepare(nt.add, x, y, b)
    assert torch.isnan(b).all()                              # preparing launches nothing
    again()
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    x.mul_(2)                                                # same memory, new contents
    again()
    nt.add(x, y, a)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
