"""The store-everything twin of the block (lr_block_fwd_save / lr_block_bwd_saved) against the rank-r
checkpoint path (lr_block_fwd / lr_block_bwd): Sec. 4.4's claim is that re-forwarding from x and the rank-r
pre-activations reproduces every wide activation, so both backward passes must return the same bits, and
the kept activations must equal the oracle's within the block's tolerances."""
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


@pytest.mark.parametrize("Bn,S,H,f,r,rope,Hkv", [(2, 192, 2, 344, 64, False, None), (1, 300, 1, 200, 32, False, None),
                                                 (1, 320, 4, 1376, 1024, False, None), (2, 264, 4, 512, 128, True, 2)])
def test_recomputed_equals_stored(Bn, S, H, f, r, rope, Hkv):
    d, f_ld = 128 * H, si.pad_ld(f, 8)
    dkv = d if Hkv is None else 128 * Hkv
    print(f"block saved B={Bn} S={S} H={H} f={f} r={r} rope={rope} Hkv={Hkv}", flush=True)
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=51, Hkv=Hkv)
    tabs = orc.rope_tables(S, 128) if rope else None
    tab_dev = tuple(torch.from_numpy(np.ascontiguousarray(t)).float().to(DEV) for t in tabs) if rope else None
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=EPS, rope=tab_dev, n_kv_heads=Hkv or 0)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    y0, ck0 = B.lr_block_fwd(desc, packed, x)
    dx0, g0 = B.lr_block_bwd(desc, packed, x, dy, ck0)
    y1, ck1, sv = B.lr_block_fwd_save(desc, packed, x)
    kept = {k: v.clone() for k, v in sv.items()}
    dx1, g1 = B.lr_block_bwd_saved(desc, packed, x, dy, ck1, sv)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    for k in ck0:
        assert torch.equal(ck0[k], ck1[k]), k
    assert torch.equal(dx0, dx1)
    for k in g0:
        assert torch.equal(g0[k], g1[k]), k
    for k in sv:                       # the backward only reads the kept activations
        assert torch.equal(sv[k], kept[k]), k
    # what was kept is what the oracle's forward holds
    T = Bn * S
    P = {k: si.f64(v) for k, v in case["params"].items()}
    _, c = orc.block_fwd(si.f64(case["x"]), P, Bn, S, H, 128, EPS, rope=tabs, Hkv=Hkv)
    X, DY = si.f64(case["x"]), si.f64(case["dy"])

    def one_run(jit):              # the wide intermediates of the bf16 model against the oracle's
        tr = {}
        M.block(X, P, DY, Bn, S, H, 128, EPS, rope=tabs, Hkv=Hkv, jitter=jit, trace=tr)
        return {k: M.err2(tr[k], c[ref]) for k, ref in (("q", "qr"), ("v", "v"), ("o", "o"), ("h1", "h1"), ("g", "g"),
                                                          ("u", "u"), ("m", "m"))}

    bud = M.over_realisations(one_run)
    q = sv["qkv"][:T * d].view(T, d)
    v = sv["qkv"][T * (d + dkv):].view(T, dkv)
    dt = torch.bfloat16
    check("q", q, c["qr"], dt, bud["q"])
    check("v", v, c["v"], dt, bud["v"])
    check("o", sv["o"], c["o"], dt, bud["o"])
    check("h1", sv["h1"], c["h1"], dt, bud["h1"])
    check("g", sv["gu"][0][:, :f], c["g"], dt, bud["g"])
    check("u", sv["gu"][1][:, :f], c["u"], dt, bud["u"])
    check("m", sv["m"][:, :f], c["m"], dt, bud["m"])
    e = float(np.max(np.abs(sv["lse"].cpu().double().numpy() - c["lse"])))
    assert e < 5e-3, e
