"""Helpers shared by the GPU parity tests (host <-> device plumbing and the gates)."""
import numpy as np
import torch

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}

# Correctness gates of the benchmark definition: max |err| <= 2e-2 and relative Frobenius
# error <= 1e-2 against the fp64 oracle on the same 16-bit inputs.
ABS_GATE, REL_GATE = 2e-2, 1e-2
# fp32 outputs only carry fp32 accumulation error (~ sqrt(K) * 2^-24 relative): far tighter.
REL_GATE_F32 = 2e-5


def to_gpu(bits: np.ndarray, dtype: str) -> torch.Tensor:
    """uint16 bit patterns -> device tensor of the 16-bit float type (no value conversion)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.view(TORCH_DT[dtype]).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def errors(got: np.ndarray, ref: np.ndarray):
    d = got - ref
    return float(np.abs(d).max()) if d.size else 0.0, float(np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-300))


def assert_gates(got: np.ndarray, ref: np.ndarray, out_dtype: str, what: str = ""):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    mx, rel = errors(got, ref)
    assert mx <= ABS_GATE, f"{what}: max abs err {mx:.3e} > {ABS_GATE}"
    gate = REL_GATE_F32 if out_dtype == "f32" else REL_GATE
    assert rel <= gate, f"{what}: relative Frobenius err {rel:.3e} > {gate}"
    return mx, rel
