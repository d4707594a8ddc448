"""Helpers for the GPU parity tests: host<->device marshalling of bf16 bit patterns and the two
acceptance metrics.  No arithmetic of the layer lives here."""
import numpy as np
import torch

from synth import inputs as si
from synth.device import dev_bf16, host_f64  # noqa: F401  (re-exported for the tests)

REL_TOL = 2e-2      # max |gpu - ref| / max(|ref|, rms(ref)) on outputs
COS_TOL = 0.999     # cosine similarity per gradient tensor


def f64_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    return si.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def dev_from_f64(a: np.ndarray) -> torch.Tensor:
    """Round an fp64 array to bf16 (via fp32, nearest-even) and upload."""
    return dev_bf16(f64_to_bf16_bits(a))


def rounded(a: np.ndarray) -> np.ndarray:
    """The fp64 value of `a` after rounding to bf16."""
    return si.bf16_bits_to_f64(f64_to_bf16_bits(a))


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)) - element-wise relative error with the
    denominator floored at the tensor's RMS so that near-zero reference entries do not blow up."""
    got, ref = np.asarray(got, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def cosine(a: np.ndarray, b: np.ndarray) -> float:
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    na, nb = np.linalg.norm(a), np.linalg.norm(b)
    if na == 0 and nb == 0:
        return 1.0
    return float(np.dot(a, b) / (na * nb))


def assert_close(got, ref, name, rel_tol=REL_TOL, cos_tol=COS_TOL):
    got = host_f64(got) if isinstance(got, torch.Tensor) else got
    assert got.shape == tuple(ref.shape) or got.size == ref.size, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values in GPU result"
    r, c = rel_err(got, ref), cosine(got, ref)
    assert r <= rel_tol and c >= cos_tol, f"{name}: rel_err={r:.3e} (tol {rel_tol}) cos={c:.6f} (tol {cos_tol})"
    return r, c
