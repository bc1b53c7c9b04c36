"""Helpers shared by the GPU parity tests: input staging and the error metrics."""
import numpy as np
import torch

import oracle
from paper_2311_02382_amd import synth

# Tolerances: max |gpu - ref| / max |ref| per tensor (elementwise relative error is
# undefined at zeros); lse: max |gpu - ref| / max(1, |ref|).
TOL = {"bf16": dict(t=2e-2, lse=1e-3), "f32": dict(t=1e-4, lse=1e-4)}


def rel_err(got, ref, floor=1e-30):
    """max |got - ref| / max(max |ref|, floor).  `floor` is for cases whose exact result is 0
    (a single visible key has dS = 0): there the error is measured against the size of the
    terms that cancel, which the caller states."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), floor))


def fro_err(got, ref, floor=1e-30):
    """Second metric: ||got - ref||_F / max(||ref||_F, floor)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), floor))


def lse_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite lse"
    return float((np.abs(got - ref) / np.maximum(1.0, np.abs(ref))).max())


class Staged:
    """One tensor in three forms: device tensor (what the kernels read), float64 copy of
    exactly those values (what the oracle reads)."""

    def __init__(self, x_f32: np.ndarray, kind: str, device="cuda"):
        if kind == "bf16":
            bits = synth.f32_to_bf16_bits(x_f32)
            self.f64 = synth.bf16_bits_to_f64(bits).reshape(x_f32.shape)
            self.dev = torch.from_numpy(bits.view(np.int16).reshape(x_f32.shape)).to(device).view(torch.bfloat16)
        else:
            self.f64 = x_f32.astype(np.float64)
            self.dev = torch.from_numpy(np.ascontiguousarray(x_f32)).to(device)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def stage_all(B, l_x, H, d, seed, kind, std=1.0):
    q, k, v, do = synth.make_inputs(B, l_x, H, d, seed, std)
    return tuple(Staged(a, kind) for a in (q, k, v, do))
