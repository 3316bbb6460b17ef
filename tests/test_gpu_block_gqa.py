"""GPU parity of the block with grouped-query attention (lr_block_desc.n_kv_heads: the K and V
up-projections narrower than Q; section "Discussion and Future Work") through the C ABI against the
fp64 oracle, element by element on small shapes: outputs, rank-r checkpoints, input gradient and every
weight gradient, with and without the rotary embedding."""
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
HD = 128


def _unpack_grads(g, d, dkv, f, r):
    wq = g["w_up_qkv"].reshape(-1, r)
    out = {"gamma1": g["gamma1"], "gamma2": g["gamma2"], "wd_o": g["w_dn_o"], "wu_o": g["w_up_o"],
           "wu_d": g["w_up_d"], "wd_d": g["w_dn_d"][:, :f],
           "wu_q": wq[:d], "wu_k": wq[d:d + dkv], "wu_v": wq[d + dkv:d + 2 * dkv]}
    for i, n in enumerate("qkv"):
        out["wd_" + n] = g["w_dn_qkv"][i * r:(i + 1) * r]
    for i, n in enumerate("gu"):
        out["wd_" + n] = g["w_dn_gu"][i * r:(i + 1) * r]
        out["wu_" + n] = g["w_up_gu"][i][:f]
    return out


CASES = [
    # Bn, S, H, Hkv, f, r, rope
    (2, 192, 4, 2, 344, 64, False),
    (1, 300, 2, 1, 200, 32, False),      # one shared key / value head, ragged S (recomputing attention backward)
    (1, 320, 8, 2, 1376, 256, True),     # rotary embedding over 8 query and 2 key heads
    (2, 264, 6, 3, 512, 128, True),
]


@pytest.mark.parametrize("Bn,S,H,Hkv,f,r,with_rope", CASES)
def test_block_gqa_parity(Bn, S, H, Hkv, f, r, with_rope):
    d, dkv, f_ld = HD * H, HD * Hkv, si.pad_ld(f, 8)
    print(f"block gqa B={Bn} S={S} H={H} Hkv={Hkv} f={f} r={r} rope={with_rope}", flush=True)
    case = si.block_case(Bn, S, d, H, HD, f, r, seed=41, Hkv=Hkv)
    rope_ref = orc.rope_tables(S, HD, 10000.0) if with_rope else None
    rope_dev = None
    if with_rope:
        rope_dev = tuple(torch.from_numpy(np.ascontiguousarray(t)).float().to(DEV) for t in rope_ref)
    desc = B.make_block_desc(Bn, S, d, H, HD, f, f_ld, r, eps=EPS, rope=rope_dev, n_kv_heads=Hkv)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    assert packed["w_up_qkv"].shape == (d + 2 * dkv, r)
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    y, ck = B.lr_block_fwd(desc, packed, x)
    dx, grads = B.lr_block_bwd(desc, packed, x, dy, ck)
    torch.cuda.synchronize()

    P = {k: si.f64(v) for k, v in case["params"].items()}
    X, DY = si.f64(case["x"]), si.f64(case["dy"])
    y_ref, c = orc.block_fwd(X, P, Bn, S, H, HD, EPS, rope=rope_ref, Hkv=Hkv)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, HD, EPS, rope=rope_ref, Hkv=Hkv)
    dt = torch.bfloat16
    bud = M.block_budget(X, P, DY, Bn, S, H, HD, EPS, y_ref, c, dx_ref, g_ref, rope=rope_ref, Hkv=Hkv)
    check("y", y, y_ref, dt, bud["y"])
    check("z_qkv", ck["z_qkv"], np.concatenate([c["z_q"], c["z_k"], c["z_v"]], 1), dt, bud["z_qkv"])
    check("z_o", ck["z_o"], c["z_o"], dt, bud["z_o"])
    check("z_gu", ck["z_gu"], np.concatenate([c["z_g"], c["z_u"]], 1), dt, bud["z_gu"])
    check("z_d", ck["z_d"], c["z_d"], dt, bud["z_d"])
    check("dx", dx, dx_ref, dt, bud["dx"])
    got = _unpack_grads(grads, d, dkv, f, r)
    for name, ref in g_ref.items():
        check("d" + name, got[name], ref, dt, bud["d" + name])


def test_block_with_as_many_kv_heads_is_the_multi_head_block():
    """n_kv_heads = n_heads and n_kv_heads = 0 run the same launches: bit-identical results."""
    Bn, S, H, f, r = 2, 192, 2, 344, 64
    d, f_ld = HD * H, si.pad_ld(f, 8)
    case = si.block_case(Bn, S, d, H, HD, f, r, seed=42)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    res = []
    for nkv in (0, H):
        desc = B.make_block_desc(Bn, S, d, H, HD, f, f_ld, r, eps=EPS, n_kv_heads=nkv)
        y, ck = B.lr_block_fwd(desc, packed, x)
        dx, g = B.lr_block_bwd(desc, packed, x, dy, ck)
        torch.cuda.synchronize()
        res.append((y, dx, g))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    for k in res[0][2]:
        assert torch.equal(res[0][2][k], res[1][2][k]), k


def test_block_rejects_kv_head_counts_that_do_not_divide():
    desc = B.make_block_desc(1, 128, 3 * HD, 3, HD, 256, 256, 32, n_kv_heads=2)
    assert B.lr_block_workspace_bytes(desc, 0) == 0 and B.lr_block_workspace_bytes(desc, 1) == 0
