"""Shared helpers of the GPU parity tests (comparison metric and tolerances).

Metric: max |got - ref| / RMS(ref) per output tensor, ref = fp64 oracle.
Bar: 1e-4 for the fp32 path, 2e-2 for the bf16 path.  A bf16 tensor cannot be closer to the oracle
than the oracle's own correctly rounded image; for Gaussian-like tensors of 10^5..10^8 elements
that storage error alone is 0.8e-2 .. 1.6e-2 in this metric (entries near 4 RMS sit in a binade
whose half-ulp is 2^-8 * 4).  The 2e-2 is therefore applied to what the computation adds on top of
that floor: tol = 2e-2 + floor * storage_error(ref), where storage_error is computed exactly (round
the oracle to bf16, measure) and floor counts the bf16 tensors of that dynamic range between the
inputs and the result (1 for path outputs; attention gradients also pass through P and dS).  The
plain metric is printed for every tensor so the margin to a flat 2e-2 stays visible.
"""
import numpy as np
import torch

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}


def _np(got):
    return got.detach().cpu().to(torch.float64).numpy() if isinstance(got, torch.Tensor) else np.asarray(got)


def relerr(got, ref):
    got = _np(got)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    rms = np.sqrt(np.mean(ref * ref))
    if rms == 0.0:      # degenerate case (e.g. a one-token softmax has zero score gradient): absolute error
        rms = 1.0
    return float(np.max(np.abs(got - ref)) / rms)


def storage_error(ref, dtype):
    """max|round(ref) - ref| / RMS(ref): what storing the exact result in `dtype` costs."""
    if dtype != torch.bfloat16:
        return 0.0
    ref = np.ascontiguousarray(np.asarray(ref, dtype=np.float64))
    if ref.size == 0:
        return 0.0
    rounded = torch.from_numpy(ref).to(torch.bfloat16).to(torch.float64).numpy()
    return relerr(rounded, ref)


def check(name, got, ref, dtype, scale=1.0, floor=None):
    e = relerr(got, ref)
    if floor is None:
        floor = 1.0 if (isinstance(got, torch.Tensor) and got.dtype == torch.bfloat16) else 0.0
    fl = storage_error(ref, torch.bfloat16) * floor if floor else 0.0
    tol = TOL[dtype] * scale + fl
    print(f"    parity {name}: {e:.3e} (tol {TOL[dtype] * scale:.1e} + storage floor {fl:.2e})", flush=True)
    assert e <= tol, f"{name}: max|err|/RMS(ref) = {e:.3e} > {tol:.2e}"
    return e
