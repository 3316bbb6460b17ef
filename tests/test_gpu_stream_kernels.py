"""GPU parity of the standalone memory-bound kernels against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import lowrank_oracle as orc
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# the last two: enough rows for the backward's row kernel to give a workgroup 128 and 192 rows (its partial
# buffer then has rows that no workgroup owns), the second with a ragged last workgroup
SHAPES = [(1, 8), (37, 72), (300, 1032), (1025, 4096), (32768, 128), (49160, 64)]


@pytest.mark.parametrize("T,d", SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rms_stat_apply_bwd(T, d, dtype):
    print(f"rmsnorm kernels T={T} d={d} {dtype}", flush=True)
    eps = 1e-5
    x = si.gaussian(3, "x", (T, d), dtype=dtype)
    gamma = si.gaussian(3, "gamma", (d,), std=0.1, mean=1.0, dtype=dtype)
    dxh = si.gaussian(3, "dxh", (T, d), dtype=dtype)
    dres = si.gaussian(3, "dres", (T, d), dtype=dtype)
    xd, gd, dxhd, dresd = (t.to(DEV) for t in (x, gamma, dxh, dres))
    stat = B.lr_rms_stat(xd)
    xh = B.lr_rmsnorm_apply(xd, gd, stat, eps)
    dx, part = B.lr_rmsnorm_bwd(xd, gd, stat, eps, dxhd, dresd)
    dx2, _ = B.lr_rmsnorm_bwd(xd, gd, stat, eps, dxhd, None)
    torch.cuda.synchronize()
    X, GAM, DXH, DRES = si.f64(x), si.f64(gamma), si.f64(dxh), si.f64(dres)
    check("stat", stat, orc.rms_stat(X), torch.float32, scale=10)
    check("xhat", xh, orc.rmsnorm_fwd(X, GAM, eps)[0], dtype)
    dx_ref, dg_ref = orc.rmsnorm_bwd(X, GAM, eps, DXH)
    check("dx+dres", dx, dx_ref + DRES, dtype)
    check("dx", dx2, dx_ref, dtype)
    check("dgamma", part.sum(0), dg_ref, torch.float32, scale=10)


@pytest.mark.parametrize("T,f", [(5, 16), (129, 344), (2048, 5504)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_act_and_swiglu(T, f, dtype):
    print(f"swiglu kernels T={T} f={f} {dtype}", flush=True)
    g = si.gaussian(4, "g", (T, f), std=2.0, dtype=dtype)
    u = si.gaussian(4, "u", (T, f), dtype=dtype)
    dm = si.gaussian(4, "dm", (T, f), dtype=dtype)
    gd, ud, dmd = (t.to(DEV) for t in (g, u, dm))
    a = B.lr_act_fwd(gd, B.LR_ACT_SILU)
    m = B.lr_swiglu_fwd(gd, ud)
    dg, du = B.lr_swiglu_bwd(gd, ud, dmd)
    torch.cuda.synchronize()
    Gm, U, DM = si.f64(g), si.f64(u), si.f64(dm)
    check("silu", a, orc.silu(Gm), dtype)
    check("m", m, orc.silu(Gm) * U, dtype)
    check("dg", dg, DM * U * orc.silu_prime(Gm), dtype)
    check("du", du, DM * orc.silu(Gm), dtype)
