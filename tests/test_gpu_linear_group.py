"""GPU parity: lr_linear_* and lr_group_* through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import lowrank_oracle as orc
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(t):
    return t.to(DEV)


LIN_CASES = [
    # T, d_in, r, d_out, dtype  (first: BASELINE config 1; others span tiles + ragged tails)
    (512, 256, 64, 256, torch.float32),
    (77, 40, 12, 52, torch.float32),
    (1, 8, 8, 8, torch.float32),
    (512, 256, 64, 256, torch.bfloat16),
    (600, 320, 72, 264, torch.bfloat16),      # nothing a multiple of the 256 / 128 / 64 tiles
    (1031, 1024, 256, 768, torch.bfloat16),   # odd T, several k slices, both tile shapes
    (3, 8, 8, 8, torch.bfloat16),
]


@pytest.mark.parametrize("T,d_in,r,d_out,dtype", LIN_CASES)
@pytest.mark.parametrize("act", [B.LR_ACT_SILU, B.LR_ACT_IDENTITY])
def test_linear_fwd_bwd(T, d_in, r, d_out, dtype, act):
    print(f"linear T={T} d_in={d_in} r={r} d_out={d_out} {dtype} act={act}", flush=True)
    c = si.linear_case(T, d_in, r, d_out, dtype=dtype, seed=0)
    x, wd, wu, dy = (_dev(c[k]) for k in ("x", "w_down", "w_up", "dy"))
    z, y = B.lr_linear_fwd(x, wd, wu, act)
    dx, dwd, dwu = B.lr_linear_bwd(x, wd, wu, z, dy, act)
    torch.cuda.synchronize()
    X, WD, WU, DY = (si.f64(c[k]) for k in ("x", "w_down", "w_up", "dy"))
    z_ref, _, y_ref = orc.lr_linear_fwd(X, WD, WU, act)
    dx_ref, dwd_ref, dwu_ref = orc.lr_linear_bwd(X, WD, WU, DY, act)
    check("z", z, z_ref, dtype)
    check("y", y, y_ref, dtype)
    check("dx", dx, dx_ref, dtype)
    check("dw_down", dwd, dwd_ref, dtype)
    check("dw_up", dwu, dwu_ref, dtype)


def test_linear_accumulate_and_empty():
    c = si.linear_case(300, 64, 16, 72, dtype=torch.float32, seed=1)
    x, wd, wu, dy = (_dev(c[k]) for k in ("x", "w_down", "w_up", "dy"))
    z, _ = B.lr_linear_fwd(x, wd, wu)
    _, dwd, dwu = B.lr_linear_bwd(x, wd, wu, z, dy)
    g = (dwd.clone(), dwu.clone())
    B.lr_linear_bwd(x, wd, wu, z, dy, grads=g)        # accumulate on top: twice the gradient
    torch.cuda.synchronize()
    assert torch.allclose(g[0], 2 * dwd, rtol=1e-6, atol=1e-6) and torch.allclose(g[1], 2 * dwu, rtol=1e-6, atol=1e-6)
    # T = 0: valid no-op
    x0 = torch.empty((0, 64), device=DEV)
    z0, y0 = B.lr_linear_fwd(x0, wd, wu)
    assert z0.shape == (0, 16) and y0.shape == (0, 72)


GRP_CASES = [
    # T, d_in, r, d_out, G, dtype
    (130, 48, 12, 40, 3, torch.float32),
    (512, 256, 64, 256, 2, torch.float32),
    (700, 512, 128, 512, 3, torch.bfloat16),     # ragged T; N = 3r = 384 (128-wide tiles + tail)
    (1024, 1024, 256, 1024, 3, torch.bfloat16),  # N = 768: 256-wide tiles
    (520, 256, 64, 344, 2, torch.bfloat16),      # d_out not a multiple of any tile
]


@pytest.mark.parametrize("T,d_in,r,d_out,G,dtype", GRP_CASES)
@pytest.mark.parametrize("norm", [B.LR_NORM_ONLINE, B.LR_NORM_TWO_PASS, B.LR_NORM_NONE, B.LR_NORM_ONLINE_GATHER])
def test_group_fwd_bwd(T, d_in, r, d_out, G, dtype, norm):
    print(f"group T={T} d_in={d_in} r={r} d_out={d_out} G={G} {dtype} norm={norm}", flush=True)
    eps = 1e-5
    c = si.group_case(T, d_in, r, d_out, G, dtype=dtype, seed=0)
    wdc, wus = si.pack_group(c)
    x, gamma, wdc, wus = _dev(c["x"]), _dev(c["gamma"]), _dev(wdc), _dev(wus)
    dy = _dev(torch.stack(c["dy"], 0).contiguous())
    z, stat, y = B.lr_group_fwd(x, gamma, eps, norm, wdc, wus)
    dx, dgamma, dwd, dwu = B.lr_group_bwd(x, gamma, eps, norm, wdc, wus, z, stat, dy)
    torch.cuda.synchronize()
    X, GAM = si.f64(c["x"]), si.f64(c["gamma"])
    WD, WU, DY = [si.f64(w) for w in c["w_down"]], [si.f64(w) for w in c["w_up"]], [si.f64(w) for w in c["dy"]]
    normed = norm != B.LR_NORM_NONE
    zs, ys, stat_ref = orc.lr_group_fwd(X, GAM, eps, WD, WU, norm=normed)
    dx_ref, dg_ref, dwd_ref, dwu_ref = orc.lr_group_bwd(X, GAM, eps, WD, WU, DY, norm=normed)
    check("z_cat", z, np.concatenate(zs, axis=1), dtype)
    check("y", y, np.stack(ys, 0), dtype)
    if normed:
        check("stat", stat, stat_ref, torch.float32, scale=10)
        check("dgamma", dgamma, dg_ref, dtype)
    check("dx", dx, dx_ref, dtype)
    check("dw_down_cat", dwd, np.concatenate(dwd_ref, axis=0), dtype)
    check("dw_up_stack", dwu, np.stack(dwu_ref, 0), dtype)


def test_group_config2_full_shape():
    """BASELINE config 2 at full size (T=16384, d=2048, r=512, G=3), online RMSNorm, bf16."""
    T, d, r, G, eps = 8 * 2048, 2048, 512, 3, 1e-5
    print("group config 2 full shape", flush=True)
    c = si.group_case(T, d, r, d, G, dtype=torch.bfloat16, seed=0)
    wdc, wus = si.pack_group(c)
    x, gamma, wdc, wus = _dev(c["x"]), _dev(c["gamma"]), _dev(wdc), _dev(wus)
    dy = _dev(torch.stack(c["dy"], 0).contiguous())
    z, stat, y = B.lr_group_fwd(x, gamma, eps, B.LR_NORM_ONLINE, wdc, wus)
    dx, dgamma, dwd, dwu = B.lr_group_bwd(x, gamma, eps, B.LR_NORM_ONLINE, wdc, wus, z, stat, dy)
    torch.cuda.synchronize()
    X, GAM = si.f64(c["x"]), si.f64(c["gamma"])
    WD, WU, DY = [si.f64(w) for w in c["w_down"]], [si.f64(w) for w in c["w_up"]], [si.f64(w) for w in c["dy"]]
    zs, ys, stat_ref = orc.lr_group_fwd(X, GAM, eps, WD, WU)
    dx_ref, dg_ref, dwd_ref, dwu_ref = orc.lr_group_bwd(X, GAM, eps, WD, WU, DY)
    dt = torch.bfloat16
    check("z_cat", z, np.concatenate(zs, axis=1), dt)
    check("y", y, np.stack(ys, 0), dt)
    check("dx", dx, dx_ref, dt)
    check("dgamma", dgamma, dg_ref, dt)
    check("dw_down_cat", dwd, np.concatenate(dwd_ref, axis=0), dt)
    check("dw_up_stack", dwu, np.stack(dwu_ref, 0), dt)


def test_bf16_weight_gradients_are_the_fp32_ones_rounded():
    """grad_dt = LR_BF16 (pure-bf16 training) differs from grad_dt = LR_F32 only by the final rounding."""
    c = si.group_case(900, 256, 64, 256, 3, dtype=torch.bfloat16, seed=5)
    wdc, wus = si.pack_group(c)
    x, gamma, wdc, wus = _dev(c["x"]), _dev(c["gamma"]), _dev(wdc), _dev(wus)
    dy = _dev(torch.stack(c["dy"], 0).contiguous())
    z, stat, y = B.lr_group_fwd(x, gamma, 1e-5, B.LR_NORM_ONLINE, wdc, wus)
    r32 = B.lr_group_bwd(x, gamma, 1e-5, B.LR_NORM_ONLINE, wdc, wus, z, stat, dy, grad_dt=B.LR_F32)
    r16 = B.lr_group_bwd(x, gamma, 1e-5, B.LR_NORM_ONLINE, wdc, wus, z, stat, dy, grad_dt=B.LR_BF16)
    torch.cuda.synchronize()
    assert torch.equal(r32[0], r16[0])
    for a32, a16 in zip(r32[1:], r16[1:]):
        assert a32.dtype == torch.float32 and a16.dtype == torch.bfloat16
        assert torch.equal(a32.to(torch.bfloat16), a16)


def test_determinism():
    """Two runs give bit-identical results (no atomics-order dependence in split-K / row stats)."""
    c = si.group_case(1000, 512, 128, 512, 3, dtype=torch.bfloat16, seed=2)
    wdc, wus = si.pack_group(c)
    x, gamma, wdc, wus = _dev(c["x"]), _dev(c["gamma"]), _dev(wdc), _dev(wus)
    dy = _dev(torch.stack(c["dy"], 0).contiguous())
    outs = []
    for _ in range(2):
        z, stat, y = B.lr_group_fwd(x, gamma, 1e-5, B.LR_NORM_ONLINE, wdc, wus)
        r = B.lr_group_bwd(x, gamma, 1e-5, B.LR_NORM_ONLINE, wdc, wus, z, stat, dy)
        torch.cuda.synchronize()
        outs.append((z, stat, y) + tuple(r))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("T,d_in,r", [(512, 256, 64), (700, 384, 256)])
def test_rank_r_activation_recomputed_equals_forward(T, d_in, r):
    """Sec. 4.4: the backward rebuilds sigma(z) from the rank-r checkpoint z alone; it must be the
    activation the forward fed into its up-projection, bit for bit.  With W_up = identity (d_out = r) the
    forward's y IS that activation (products with 1 and 0 and their fp32 sum are exact), and lr_act_fwd
    on the stored z is the kernel the backward uses to rebuild it."""
    c = si.linear_case(T, d_in, r, r, dtype=torch.bfloat16, seed=9)
    x, wd = _dev(c["x"]), _dev(c["w_down"])
    eye = torch.eye(r, dtype=torch.bfloat16, device=DEV)
    z, y = B.lr_linear_fwd(x, wd, eye, B.LR_ACT_SILU)
    a = B.lr_act_fwd(z, B.LR_ACT_SILU)
    torch.cuda.synchronize()
    assert torch.equal(y, a)
    # and it is sigma of the checkpoint as stored, rounded once
    ref = torch.nn.functional.silu(z.float()).to(torch.bfloat16)
    assert (y.float() - ref.float()).abs().max() <= 2.0 ** -7 * ref.float().abs().max()
