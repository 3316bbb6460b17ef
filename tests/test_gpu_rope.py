"""GPU parity of the rotary position embedding: lr_rope alone (forward and transposed) and the block
with the option on, through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import bf16_model as M
import synth_inputs as si
from oracle import lowrank_oracle as orc
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS = 1e-5


def _tables(S, hd=128, base=10000.0):
    cos, sin = orc.rope_tables(S, hd, base)
    to = lambda a: torch.from_numpy(a.astype(np.float32)).to(DEV)
    # the oracle sees the same fp32-rounded tables as the kernel
    return (cos.astype(np.float32).astype(np.float64), sin.astype(np.float32).astype(np.float64)), (to(cos), to(sin))


@pytest.mark.parametrize("Bn,S,H,ld_extra", [(1, 1, 1, 0), (2, 77, 3, 0), (3, 130, 2, 64)])
def test_rope_alone(Bn, S, H, ld_extra):
    print(f"rope B={Bn} S={S} H={H} ld+{ld_extra}", flush=True)
    T, d = Bn * S, H * 128
    x = si.gaussian(5, "rope_x", (T, d + ld_extra), dtype=torch.bfloat16)
    tab64, tab_dev = _tables(S)
    for inverse in (False, True):
        xd = x.clone().to(DEV)
        B.lr_rope(xd, tab_dev[0], tab_dev[1], Bn, S, H, 128, inverse=inverse)
        torch.cuda.synchronize()
        ref = orc.rope_apply(si.f64(x[:, :d]), tab64[0], tab64[1], Bn, S, H, 128, inverse=inverse)
        check(f"rope inverse={inverse}", xd[:, :d], ref, torch.bfloat16)
        if ld_extra:   # columns past the heads are not touched
            assert torch.equal(xd[:, d:].cpu(), x[:, d:])


def _unpack_grads(g, f, r):
    out = {"gamma1": g["gamma1"], "gamma2": g["gamma2"], "wd_o": g["w_dn_o"], "wu_o": g["w_up_o"],
           "wu_d": g["w_up_d"], "wd_d": g["w_dn_d"][:, :f]}
    for i, n in enumerate("qkv"):
        out["wd_" + n] = g["w_dn_qkv"][i * r:(i + 1) * r]
        out["wu_" + n] = g["w_up_qkv"][i]
    for i, n in enumerate("gu"):
        out["wd_" + n] = g["w_dn_gu"][i * r:(i + 1) * r]
        out["wu_" + n] = g["w_up_gu"][i][:f]
    return out


@pytest.mark.parametrize("Bn,S,H,f,r", [(2, 192, 2, 344, 64), (1, 300, 1, 200, 32)])
def test_block_with_rope(Bn, S, H, f, r):
    print(f"block rope B={Bn} S={S} H={H} f={f} r={r}", flush=True)
    d = 128 * H
    f_ld = si.pad_ld(f, 8)
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=41)
    tab64, tab_dev = _tables(S)
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=EPS, rope=tab_dev)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    y, ck = B.lr_block_fwd(desc, packed, x)
    dx, grads = B.lr_block_bwd(desc, packed, x, dy, ck)
    torch.cuda.synchronize()
    P = {k: si.f64(v) for k, v in case["params"].items()}
    X, DY = si.f64(case["x"]), si.f64(case["dy"])
    y_ref, c = orc.block_fwd(X, P, Bn, S, H, 128, EPS, rope=tab64)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS, rope=tab64)
    # the option matters here: without it the query-projection gradient is a different tensor altogether
    _, g_plain = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS)
    assert np.abs(g_plain["wd_q"] - g_ref["wd_q"]).max() > 0.5 * np.sqrt(np.mean(g_ref["wd_q"] ** 2))
    dt = torch.bfloat16
    bud = M.block_budget(X, P, DY, Bn, S, H, 128, EPS, y_ref, c, dx_ref, g_ref, rope=tab64)
    check("y", y, y_ref, dt, bud["y"])
    check("dx", dx, dx_ref, dt, bud["dx"])
    got = _unpack_grads(grads, f, r)
    for name, ref in g_ref.items():
        check("d" + name, got[name], ref, dt, bud["d" + name])
