"""Shared helpers of the GPU parity tests (comparison metric and tolerances)."""
import numpy as np
import torch

# max |err| / RMS(ref) per output tensor: the bar the hot path is held to
TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}


def relerr(got, ref):
    got = got.detach().cpu().to(torch.float64).numpy() if isinstance(got, torch.Tensor) else np.asarray(got)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    return float(np.max(np.abs(got - ref)) / (np.sqrt(np.mean(ref * ref)) + 1e-300))


def check(name, got, ref, dtype, scale=1.0):
    e = relerr(got, ref)
    tol = TOL[dtype] * scale
    print(f"    parity {name}: {e:.3e} (tol {tol:.1e})", flush=True)
    assert e <= tol, f"{name}: max|err|/RMS(ref) = {e:.3e} > {tol:.1e}"
    return e
