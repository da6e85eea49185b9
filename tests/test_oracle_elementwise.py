"""Pins for the oracle of the memory-bound kernels (CPU only): hand-worked values, closed
forms, identities, rounding ties, and agreement of `encode` with independent conversions."""
import numpy as np
import pytest

from oracle import elementwise as oe
import synthetic_inputs as si


def _bits(x, dt):
    return si.round_to_bits(np.asarray(x, dtype=np.float32), dt)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_encode_is_round_to_nearest_even(dt):
    # every 16-bit value survives a round trip
    allbits = np.arange(65536, dtype=np.uint16)
    vals = oe.decode(allbits, dt)
    fin = np.isfinite(vals)
    assert np.array_equal(oe.encode(vals[fin], dt), allbits[fin])
    # midpoints between neighbours go to the even one, anything off the midpoint to the nearer one
    pos = allbits[(allbits & 0x8000) == 0]
    pos = pos[np.isfinite(oe.decode(pos + 1, dt)) & np.isfinite(oe.decode(pos, dt))]
    lo, hi = oe.decode(pos, dt), oe.decode(pos + 1, dt)
    mid = (lo + hi) / 2                                          # exact in fp64
    even = np.where(pos % 2 == 0, pos, pos + 1)
    assert np.array_equal(oe.encode(mid, dt), even)
    assert np.array_equal(oe.encode(np.nextafter(mid, np.inf), dt), pos + 1)
    assert np.array_equal(oe.encode(np.nextafter(mid, -np.inf), dt), pos)
    assert np.array_equal(oe.encode(-mid, dt), even | 0x8000)
    # agreement with the input generator's conversion (which goes through fp32) on fp32 values
    x = np.random.default_rng(0).standard_normal(20000).astype(np.float32) * np.float32(37.0)
    assert np.array_equal(oe.encode(x.astype(np.float64), dt), si.round_to_bits(x, dt))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_add_hand_worked_and_ties(dt):
    x, y = _bits([1.0, -2.5, 0.0, 100.0, 0.5], dt), _bits([2.0, 2.5, -0.0, 28.0, 0.25], dt)
    assert oe.add(x, y, dt).tolist() == [3.0, 0.0, 0.0, 128.0, 0.75]
    if dt == "f16":
        # spacing is 2 above 2048: 2048 + 1 is a tie -> 2048 (even), 2050 + 1 is a tie -> 2052
        s = oe.add(_bits([2048.0, 2050.0], dt), _bits([1.0, 1.0], dt), dt)
        assert s.tolist() == [2049.0, 2051.0]
        assert oe.decode(oe.encode(s, dt), dt).tolist() == [2048.0, 2052.0]
    else:
        # spacing is 2 above 256: 256 + 1 -> 256, 258 + 1 -> 260
        s = oe.add(_bits([256.0, 258.0], dt), _bits([1.0, 1.0], dt), dt)
        assert oe.decode(oe.encode(s, dt), dt).tolist() == [256.0, 260.0]
    # commutative, and x + (-x) = 0
    a, b = si.normal_bits((1000,), dt, 1, 3.0), si.normal_bits((1000,), dt, 2, 3.0)
    assert np.array_equal(oe.add(a, b, dt), oe.add(b, a, dt))
    assert not oe.add(a, a ^ np.uint16(0x8000), dt).any()


def test_silu_values_and_identities():
    dt = "f16"
    x = _bits([0.0, 1.0, -1.0, 8.0, -8.0], dt)
    got = oe.silu(x, dt)
    assert got[0] == 0.0
    assert abs(got[1] - 0.7310585786300049) < 1e-15            # 1 / (1 + 1/e)
    assert abs(got[2] + 0.2689414213699951) < 1e-15            # -1 / (1 + e)
    assert abs(got[3] - 8.0 / (1.0 + np.exp(-8.0))) < 1e-15
    # silu(x) - silu(-x) = x, since sigmoid(x) + sigmoid(-x) = 1
    b = si.normal_bits((5000,), dt, 3, 4.0)
    xs = oe.decode(b, dt)
    assert np.allclose(oe.silu(b, dt) - oe.silu(b ^ np.uint16(0x8000), dt), xs, rtol=0, atol=1e-13)
    # minimum of x * sigmoid(x) is about -0.27846 near x = -1.2785
    grid = _bits(np.linspace(-6, 6, 4001), dt)
    assert abs(oe.silu(grid, dt).min() + 0.2784645) < 1e-5
    # for large x it approaches x, for very negative x it approaches 0 from below
    assert abs(oe.silu(_bits([30.0], dt), dt)[0] - 30.0) < 1e-11 and -1e-11 < oe.silu(_bits([-30.0], dt), dt)[0] < 0


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_softmax_closed_forms(dt):
    # two elements: a sigmoid of the difference; equal elements: uniform
    got = oe.softmax(_bits([[1.0, 3.0], [2.0, 2.0]], dt), dt)
    assert np.allclose(got[0], [1 / (1 + np.e ** 2), 1 / (1 + np.e ** -2)], rtol=1e-15)
    assert got[1].tolist() == [0.5, 0.5]
    assert np.allclose(oe.softmax(_bits(np.full((3, 7), -5.0), dt), dt), 1 / 7, rtol=1e-15)
    # hand-worked: [0, ln 2, ln 4] -> [1, 2, 4] / 7 (the logs are rounded to the format first)
    row = _bits([[0.0, np.log(2.0), np.log(4.0)]], dt)
    e = np.exp(oe.decode(row, dt))
    assert np.allclose(oe.softmax(row, dt), e / e.sum(), rtol=1e-15)
    x = si.normal_bits((17, 300), dt, 4, 3.0)
    p = oe.softmax(x, dt)
    assert np.allclose(p.sum(axis=1), 1.0, rtol=1e-13) and (p > 0).all()
    # order preserving, invariant under a shift of the row (a shift by a power of two is exact here)
    assert np.array_equal(np.argsort(p, axis=1, kind="stable"), np.argsort(oe.decode(x, dt), axis=1, kind="stable"))
    small = si.round_to_bits(np.random.default_rng(5).integers(-8, 8, (4, 50)).astype(np.float32), dt)
    shifted = si.round_to_bits(oe.decode(small, dt).astype(np.float32) + 16.0, dt)
    assert np.allclose(oe.softmax(small, dt), oe.softmax(shifted, dt), rtol=1e-14)
    # no overflow for large entries
    assert np.isfinite(oe.softmax(_bits([[60000.0, 59000.0, -60000.0]], "f16"), "f16")).all()


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_rms_norm_closed_forms(dt):
    # hand-worked: [3, 4] has mean square 12.5
    got = oe.rms_norm(_bits([[3.0, 4.0]], dt), dt, eps=0.0)
    assert np.allclose(got, [[3 / np.sqrt(12.5), 4 / np.sqrt(12.5)]], rtol=1e-15)
    # a constant row c becomes c / sqrt(c^2 + eps)
    got = oe.rms_norm(_bits(np.full((2, 9), -2.0), dt), dt, eps=0.25)
    assert np.allclose(got, -2 / np.sqrt(4.25), rtol=1e-15)
    x = si.normal_bits((11, 257), dt, 6, 2.0)
    y = oe.rms_norm(x, dt, eps=0.0)
    assert np.allclose(np.sqrt((y * y).mean(axis=1)), 1.0, rtol=1e-13)           # unit root mean square
    # scaling the input by a power of two (exact in the format) leaves the result unchanged, a sign flip flips it
    x4 = si.round_to_bits(oe.decode(x, dt).astype(np.float32) * 4.0, dt)
    assert np.allclose(oe.rms_norm(x4, dt, eps=0.0), y, rtol=1e-14)
    assert np.allclose(oe.rms_norm(x ^ np.uint16(0x8000), dt, eps=0.0), -y, rtol=1e-14)
    # eps only ever shrinks the magnitude; a zero row stays zero
    assert (np.abs(oe.rms_norm(x, dt, eps=1e-2)) <= np.abs(y)).all()
    assert not oe.rms_norm(_bits(np.zeros((1, 8)), dt), dt, eps=1e-6).any()
