"""lr_linear_fwd_static (the entry point that allocates nothing: its scratch is a device array inside the
library) against lr_linear_fwd (scratch from the caller's workspace), through the C ABI.  Both run the
same kernels, so the results must be bit-identical, and they are also held to the oracle.  Two calls in a
row, the second on a smaller input (the array keeps the first call's contents), an fp32 call, and the
size limit."""
import pytest
import torch

import synth_inputs as si
from oracle import lowrank_oracle as orc
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LIMIT = 32 << 20    # LR_LINEAR_STATIC_SCRATCH_BYTES


def _run(T, d_in, r, d_out, dtype, seed):
    print(f"linear static T={T} d_in={d_in} r={r} d_out={d_out} {dtype}", flush=True)
    c = si.linear_case(T, d_in, r, d_out, dtype=dtype, seed=seed)
    x, wd, wu = (c[k].to(DEV) for k in ("x", "w_down", "w_up"))
    z = torch.empty((T, r), dtype=dtype, device=DEV)
    y = torch.empty((T, d_out), dtype=dtype, device=DEV)
    B.lr_linear_fwd_static(x, wd, wu, z, y)
    z0, y0 = B.lr_linear_fwd(x, wd, wu)
    torch.cuda.synchronize()
    assert torch.equal(z, z0) and torch.equal(y, y0)
    X, WD, WU = (si.f64(c[k]) for k in ("x", "w_down", "w_up"))
    z_ref, _, y_ref = orc.lr_linear_fwd(X, WD, WU, orc.ACT_SILU)
    check("z", z, z_ref, dtype)
    check("y", y, y_ref, dtype)


def test_zz_static_scratch_two_calls_second_smaller():
    _run(1031, 1024, 256, 768, torch.bfloat16, seed=3)
    _run(300, 320, 72, 264, torch.bfloat16, seed=4)      # smaller: stale contents of the first call stay behind it
    _run(77, 40, 12, 52, torch.float32, seed=5)


def test_zz_static_scratch_rejects_what_does_not_fit():
    T, r = 16400, 1024                                    # T * r * 2 bytes > 32 MiB
    assert T * r * 2 > LIMIT
    x = torch.zeros((T, 64), dtype=torch.bfloat16, device=DEV)
    wd = torch.zeros((r, 64), dtype=torch.bfloat16, device=DEV)
    wu = torch.zeros((64, r), dtype=torch.bfloat16, device=DEV)
    z = torch.empty((T, r), dtype=torch.bfloat16, device=DEV)
    y = torch.full((T, 64), 7.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.LrError, match="LR_EWORKSPACE"):
        B.lr_linear_fwd_static(x, wd, wu, z, y)
    torch.cuda.synchronize()
    assert float(y.float().min()) == 7.0                  # nothing was enqueued
    # the largest layer that fits: exactly the limit
    T = LIMIT // (r * 2)
    x = torch.zeros((T, 64), dtype=torch.bfloat16, device=DEV)
    B.lr_linear_fwd_static(x, wd, wu, z[:T], y[:T])
    torch.cuda.synchronize()
    assert float(y[:T].float().abs().max()) == 0.0
