"""Shared helpers of the GPU parity tests (comparison metric and tolerances).

Metric: max |got - ref| / RMS(ref) per output tensor, ref = fp64 oracle.
Bar: 1e-4 for the fp32 path, 2e-2 for the bf16 path.  A bf16 tensor cannot be closer to the oracle
than the oracle's own correctly rounded image; for Gaussian-like tensors of 10^5..10^8 elements
that storage error alone is 0.8e-2 .. 1.6e-2 in this metric (entries near 4 RMS sit in a binade
whose half-ulp is 2^-8 * 4).  The 2e-2 is therefore applied to what the computation adds on top of
that floor: tol = 2e-2 + floor * storage_error(ref), where storage_error is computed exactly (round
the oracle to bf16, measure) and floor counts the bf16 tensors of that dynamic range between the
inputs and the result (1 for the single-stage entry points; 3 for attention gradients, which also
pass through P and dS, and for the block, whose outputs sit behind a chain of about ten rounded
tensors whose errors add in quadrature).  The plain metric is printed for every tensor so the margin
to a flat 2e-2 stays visible.

Because a max over 10^5..10^8 entries is a noisy statistic, two size-independent checks sit beside it
for every bf16 tensor: the relative L2 error must stay below 1e-2 and the least-squares slope of got
on ref within 3e-3 of 1.  A dropped or mis-scaled term of a percent or more fails these whatever
the tensor size.
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


def l2_and_slope(got, ref):
    got = _np(got).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    rr = float(np.dot(ref, ref))
    if rr == 0.0:
        return 0.0, 1.0
    return float(np.linalg.norm(got - ref) / np.sqrt(rr)), float(np.dot(got, ref) / rr)


def check(name, got, ref, dtype, scale=1.0, floor=None):
    """dtype: the path's arithmetic type (picks the bar).  floor: see the module docstring; None means
    1 for a tensor stored in bf16 and 0 otherwise."""
    e = relerr(got, ref)
    if floor is None:
        floor = 1.0 if (isinstance(got, torch.Tensor) and got.dtype == torch.bfloat16) else 0.0
    fl = storage_error(ref, torch.bfloat16) * floor if floor else 0.0
    tol = TOL[dtype] * scale + fl
    l2, slope = l2_and_slope(got, ref)
    print(f"    parity {name}: max/rms {e:.3e} (tol {TOL[dtype] * scale:.1e} + floor {fl:.2e})  l2 {l2:.2e}  "
          f"slope-1 {slope - 1:+.1e}", flush=True)
    assert e <= tol, f"{name}: max|err|/RMS(ref) = {e:.3e} > {tol:.2e}"
    if dtype == torch.bfloat16 and np.asarray(ref).size >= 64:
        assert l2 <= 1e-2 * scale, f"{name}: relative L2 error {l2:.3e} > 1e-2"
        assert abs(slope - 1) <= 3e-3 * scale, f"{name}: slope {slope:.5f} is off 1"
    return e
