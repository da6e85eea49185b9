"""GPU parity of nt_sdpa against the fp64 oracle (plain definition of attention).

Gates: the GEMM gates of this repository (max |err| <= 2e-2, relative Frobenius error <= 1e-2): the
probabilities are rounded to the 16-bit input format before they multiply V (as in the
FlashAttention-2 scheme), which bounds the relative error of an output by about one unit in the
last place of that format, and the output is rounded once more."""
import numpy as np
import pytest
import torch

import paper_2507_11978_amd as nt
import synthetic_inputs as si
from oracle import attention as oat
from oracle import numeric as onum
from gpu_util import TORCH_DT, assert_gates, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def run(q, k, v, dt, scale=0.0):
    out = torch.full(q.shape[:-1] + (v.shape[-1],), float("nan"), dtype=TORCH_DT[dt], device="cuda")
    nt.sdpa(to_gpu(q, dt), to_gpu(k, dt), to_gpu(v, dt), out, scale=scale)
    torch.cuda.synchronize()
    return to_f64(out)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,Sq,Sk", [(1, 1, 128, 64), (2, 3, 256, 192), (1, 2, 100, 77), (1, 1, 1, 1), (2, 2, 33, 300), (1, 4, 384, 1024)])
def test_sdpa_shapes(dt, B, H, Sq, Sk):
    q, k, v = (si.normal_bits(s, dt, 10 + i, 1.0) for i, s in enumerate([(B, H, Sq, 64), (B, H, Sk, 64), (B, H, Sk, 64)]))
    ref = oat.sdpa(q, k, v, dt)
    assert_gates(run(q, k, v, dt), ref, dt, f"sdpa {dt} {B}x{H}x{Sq}x{Sk}")


def test_sdpa_closed_forms_and_scale():
    dt = "f16"
    rng = np.random.default_rng(2)
    v = si.round_to_bits(rng.integers(-4, 5, (1, 1, 200, 64)).astype(np.float32), dt)
    k = si.normal_bits((1, 1, 200, 64), dt, 3, 1.0)
    # zero queries: the mean of the values (exact up to the rounding of the weights 1/200 and of the result)
    got = run(np.zeros((1, 1, 70, 64), dtype=np.uint16), k, v, dt)
    assert np.abs(got - onum.decode(v, dt).mean(axis=2, keepdims=True)).max() < 4e-3
    # a dominant key takes all the weight: its value row comes out exactly
    q = si.normal_bits((1, 1, 5, 64), dt, 4, 1.0)
    kd = onum.decode(k, dt).copy()
    kd[0, 0, 17] = onum.decode(q, dt)[0, 0, 2] * 8.0
    k2 = si.round_to_bits(kd.astype(np.float32), dt)
    got = run(q, k2, v, dt, scale=1.0)
    assert np.array_equal(got[0, 0, 2], onum.decode(v, dt)[0, 0, 17])
    # an explicit scale against the oracle; large scores must not overflow
    q, k, v = (si.normal_bits((1, 2, 130, 64), dt, 20 + i, 3.0) for i in range(3))
    assert_gates(run(q, k, v, dt, scale=0.5), oat.sdpa(q, k, v, dt, scale=0.5), dt, "sdpa scale 0.5")


def test_sdpa_strided_views_and_errors():
    dt, B, H, S = "f16", 2, 3, 150
    q, k, v = (si.normal_bits((B, H, S, 64), dt, 30 + i, 1.0) for i in range(3))
    ref = oat.sdpa(q, k, v, dt)
    # [batch, seq, heads, 64] storage viewed as [batch, heads, seq, 64]; output into a padded buffer
    qs = to_gpu(np.ascontiguousarray(q.transpose(0, 2, 1, 3)), dt).permute(0, 2, 1, 3)
    ks = to_gpu(np.ascontiguousarray(k.transpose(0, 2, 1, 3)), dt).permute(0, 2, 1, 3)
    vbuf = torch.zeros((B, H, S, 80), dtype=torch.float16, device="cuda")
    vbuf[..., :64] = to_gpu(v, dt)
    obuf = torch.full((B, H, S + 2, 64), -7.0, dtype=torch.float16, device="cuda")
    nt.sdpa(qs, ks, vbuf[..., :64], obuf[:, :, 1:S + 1])
    torch.cuda.synchronize()
    assert_gates(to_f64(obuf[:, :, 1:S + 1]), ref, dt, "sdpa strided")
    assert (obuf[:, :, 0] == -7.0).all() and (obuf[:, :, S + 1] == -7.0).all()
    z = torch.zeros((1, 1, 8, 32), dtype=torch.float16, device="cuda")
    with pytest.raises(nt.NtError):
        nt.sdpa(z, z, z, z)                                               # head size 32 is not built
    a = torch.zeros((1, 1, 8, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(nt.NtError):
        nt.sdpa(a, a[:, :, :0], a[:, :, :0], a)                           # no keys
    with pytest.raises(nt.NtError):
        nt.sdpa(a, a, a[:, :, :4], a)                                     # K and V lengths differ


def test_sdpa_negative_scale():
    dt = "f16"
    q, k, v = (si.normal_bits((1, 2, 90, 64), dt, 40 + i, 1.0) for i in range(3))
    assert_gates(run(q, k, v, dt, scale=-0.3), oat.sdpa(q, k, v, dt, scale=-0.3), dt, "sdpa negative scale")


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_sdpa_scores_rising_along_the_keys(dt):
    """Keys grow along the sequence, so a row's maximum keeps rising (or falling) from block to block: some
    blocks stay within the band the kernel tolerates between its row reference and the running maximum, others
    force the reference up."""
    rng = np.random.default_rng(70)
    S, Sk = 96, 640
    w = rng.standard_normal(64).astype(np.float32)
    w /= np.linalg.norm(w)
    for per_block in (3.0, 11.0, 40.0):                       # rise of the top score per 64 keys, in base-2 units
        q = rng.standard_normal((1, 2, S, 64)).astype(np.float32)
        proj = np.abs(q @ w).mean()
        step = per_block / 64.0 / (proj * 0.125 * 1.4427)      # so that scale * q . k_j grows by ~per_block per block
        kf = (np.arange(Sk, dtype=np.float32)[:, None] * step) * w[None, :] + 0.05 * rng.standard_normal((Sk, 64)).astype(np.float32)
        kf = np.broadcast_to(kf, (1, 2, Sk, 64))
        qb, kb = si.round_to_bits(q, dt), si.round_to_bits(np.ascontiguousarray(kf), dt)
        vb = si.normal_bits((1, 2, Sk, 64), dt, 71, 1.0)
        assert_gates(run(qb, kb, vb, dt), oat.sdpa(qb, kb, vb, dt), dt, f"sdpa rising scores {per_block} {dt}")
