"""Pins for the attention oracle (CPU only): closed forms and invariants of the definition."""
import numpy as np
import pytest

from oracle import attention as oat
from oracle import numeric as onum
import synthetic_inputs as si


def _bits(x, dt="f16"):
    return si.round_to_bits(np.asarray(x, dtype=np.float32), dt)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_closed_forms(dt):
    rng = np.random.default_rng(0)
    v = _bits(rng.integers(-4, 5, (5, 3)), dt)
    vd = onum.decode(v, dt)
    # zero queries: every key weighs the same, the output is the mean of the values
    out = oat.sdpa(_bits(np.zeros((4, 6)), dt), _bits(rng.standard_normal((5, 6)), dt), v, dt)
    assert np.allclose(out, np.broadcast_to(vd.mean(axis=0), (4, 3)), rtol=1e-14, atol=1e-14)
    # a single key: the output is its value whatever the scores
    out = oat.sdpa(_bits(rng.standard_normal((4, 6)), dt), _bits(rng.standard_normal((1, 6)), dt), v[:1], dt)
    assert np.allclose(out, np.broadcast_to(vd[:1], (4, 3)), rtol=1e-15)
    # two keys: the weights are a sigmoid of the scaled score difference (hand-worked: q = [2, 0], k0 = [1, 0], k1 = [0, 1], scale 0.5)
    out = oat.sdpa(_bits([[2.0, 0.0]], dt), _bits([[1.0, 0.0], [0.0, 1.0]], dt), _bits([[1.0], [3.0]], dt), dt, scale=0.5)
    w0 = 1.0 / (1.0 + np.exp(-1.0))                       # scores 1 and 0
    assert np.allclose(out, [[w0 * 1.0 + (1 - w0) * 3.0]], rtol=1e-15)
    # values all equal to c: the output is c (the weights sum to one)
    out = oat.sdpa(_bits(rng.standard_normal((7, 8)), dt), _bits(rng.standard_normal((9, 8)), dt), _bits(np.full((9, 2), 2.5), dt), dt)
    assert np.allclose(out, 2.5, rtol=1e-14)


def test_invariants():
    dt = "f16"
    q, k, v = (si.normal_bits(s, dt, i, 1.0) for i, s in enumerate([(2, 3, 10, 16), (2, 3, 13, 16), (2, 3, 13, 8)]))
    ref = oat.sdpa(q, k, v, dt)
    assert ref.shape == (2, 3, 10, 8)
    # the order of the keys does not matter
    perm = np.random.default_rng(1).permutation(13)
    assert np.allclose(oat.sdpa(q, k[:, :, perm], v[:, :, perm], dt), ref, rtol=1e-12, atol=1e-14)
    # every output row is a convex combination of value rows
    vd = onum.decode(v, dt)
    assert (ref <= vd.max(axis=2, keepdims=True) + 1e-12).all() and (ref >= vd.min(axis=2, keepdims=True) - 1e-12).all()
    # a dominant score picks its value row: scale up one key that is aligned with the query
    qd, kd = onum.decode(q, dt)[0, 0, 0], onum.decode(k, dt)[0, 0]
    big = oat.sdpa(q[0, 0, :1], _bits(np.vstack([qd * 40.0, kd[1:]])), v[0, 0], dt, scale=1.0)
    assert np.allclose(big[0], vd[0, 0, 0], atol=1e-6)
    # batch and head entries are independent
    assert np.array_equal(oat.sdpa(q[1, 2], k[1, 2], v[1, 2], dt), ref[1, 2])
    # explicit triple loop on one head
    s = np.array([[sum(onum.decode(q, dt)[0, 1, i, d] * onum.decode(k, dt)[0, 1, j, d] for d in range(16)) / 4.0 for j in range(13)] for i in range(10)])
    p = np.exp(s - s.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    assert np.allclose(ref[0, 1], p @ vd[0, 1], rtol=1e-13, atol=1e-15)
    # large scores do not overflow
    assert np.isfinite(oat.sdpa(_bits(np.full((1, 4), 200.0)), _bits(np.full((3, 4), 200.0)), _bits(np.ones((3, 2))), dt, scale=1.0)).all()
