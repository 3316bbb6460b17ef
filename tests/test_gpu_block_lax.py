"""GPU parity of lr_block_lax_fwd / lr_block_lax_bwd (the LaX variant: identity gate, rank-r residual
from the layer below, App. "LaX variant (residual low-rank)") through the C ABI against the fp64
oracle in oracle/lax_oracle.py, element by element on small shapes, plus a two-block stack whose
inter-layer tensors are produced and consumed by the library itself."""
import numpy as np
import pytest
import torch

import bf16_model as M
import synth_inputs as si
from oracle import lax_oracle as lax
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS = 1e-5


def _lax_budget(X, P, DY, hp, dzn, Bn, S, H, y_ref, z_ref, dx_ref, g_ref, dh_ref, Hkv=None):
    """Error of the ideal bf16 pipeline (tests/bf16_model.py) per tensor: the budget of parity.py, rule 3."""
    def one_run(jit):
        out, g, dh = M.block(X, P, DY, Bn, S, H, 128, EPS, h_prev=hp, dz_next=dzn, lax=True, Hkv=Hkv, jitter=jit)
        bud = {"y": M.err2(out["y"], y_ref), "dx": M.err2(out["dx"], dx_ref)}
        for n in lax.PROJ:
            bud["z_" + n] = M.err2(out["z_" + n], z_ref[n])
            bud["dh_prev_" + n] = M.err2(dh[n], dh_ref[n])
        bud.update({"d" + k: M.err2(g[k], g_ref[k]) for k in g_ref})
        return bud

    return M.over_realisations(one_run)

PARTS = {"qkv": ("q", "k", "v"), "o": ("o",), "gu": ("g", "u"), "d": ("d",)}


def _rank_tensors(seed, tag, T, r, std):
    """The seven [T, r] rank-r tensors of a block, bf16, keyed by projection."""
    return {n: si.gaussian(seed, f"{tag}_{n}", (T, r), std=std, dtype=torch.bfloat16) for n in lax.PROJ}


def _cat(d, dev=None):
    """Projection-keyed dict -> the ABI's four tensors (qkv and gu concatenated along the rank axis)."""
    out = {k: torch.cat([d[n] for n in names], dim=1).contiguous() for k, names in PARTS.items()}
    return {k: v.to(dev) for k, v in out.items()} if dev else out


def _split(cat, r):
    out = {}
    for k, names in PARTS.items():
        for i, n in enumerate(names):
            out[n] = cat[k][:, i * r:(i + 1) * r]
    return out


def _f64(d):
    return {k: si.f64(v) for k, v in d.items()}


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


def _setup(Bn, S, H, f, r, seed):
    d = 128 * H
    f_ld = si.pad_ld(f, 8)
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=seed)
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=EPS, act=B.LR_ACT_IDENTITY)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    return d, case, desc, packed


@pytest.mark.parametrize("Bn,S,H,f,r", [(2, 192, 2, 344, 64), (1, 300, 1, 200, 32), (1, 320, 4, 1376, 1024)])
def test_block_lax_parity(Bn, S, H, f, r):
    print(f"block lax B={Bn} S={S} H={H} f={f} r={r}", flush=True)
    d, case, desc, packed = _setup(Bn, S, H, f, r, seed=21)
    T = Bn * S
    h_prev = _rank_tensors(21, "hprev", T, r, 0.5)
    dz_next = _rank_tensors(21, "dznext", T, r, 1.0)
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    hp_dev, dzn_dev = _cat(h_prev, DEV), _cat(dz_next, DEV)
    y, ck = B.lr_block_lax_fwd(desc, packed, x, h_prev=hp_dev)
    dx, grads, dh = B.lr_block_lax_bwd(desc, packed, x, dy, ck, h_prev=hp_dev, dz_next=dzn_dev)
    torch.cuda.synchronize()

    P = {k: si.f64(v) for k, v in case["params"].items()}
    X, DY = si.f64(case["x"]), si.f64(case["dy"])
    y_ref, z_ref, _ = lax.block_fwd(X, P, _f64(h_prev), Bn, S, H, 128, EPS)
    dx_ref, g_ref, dh_ref = lax.block_bwd(X, P, _f64(h_prev), DY, _f64(dz_next), Bn, S, H, 128, EPS)
    dt = torch.bfloat16
    bud = _lax_budget(X, P, DY, _f64(h_prev), _f64(dz_next), Bn, S, H, y_ref, z_ref, dx_ref, g_ref, dh_ref)
    check("y", y, y_ref, dt, bud["y"])
    z_gpu = _split({k: ck["z_" + k] for k in PARTS}, r)
    for n in lax.PROJ:
        check("z_" + n, z_gpu[n], z_ref[n], dt, bud["z_" + n])
    check("dx", dx, dx_ref, dt, bud["dx"])
    dh_gpu = _split(dh, r)
    for n in lax.PROJ:
        check("dh_prev_" + n, dh_gpu[n], dh_ref[n], dt, bud["dh_prev_" + n])
    got = _unpack_grads(grads, f, r)
    for name, ref in g_ref.items():
        check("d" + name, got[name], ref, dt, bud["d" + name])


def test_block_lax_null_residuals_equal_the_plain_identity_block():
    """No h_prev, no dz_next, no dh_prev wanted: bit-identical to lr_block_fwd / lr_block_bwd with
    sigma = identity (absent tensors count as zeros)."""
    Bn, S, H, f, r = 2, 128, 1, 256, 32
    d, case, desc, packed = _setup(Bn, S, H, f, r, seed=22)
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    y0, ck0 = B.lr_block_fwd(desc, packed, x)
    dx0, g0 = B.lr_block_bwd(desc, packed, x, dy, ck0)
    y1, ck1 = B.lr_block_lax_fwd(desc, packed, x)
    dx1, g1, dh = B.lr_block_lax_bwd(desc, packed, x, dy, ck1, want_dh_prev=False)
    torch.cuda.synchronize()
    assert dh is None
    assert torch.equal(y0, y1) and torch.equal(dx0, dx1)
    for k in ("z_qkv", "z_o", "z_gu", "z_d"):
        assert torch.equal(ck0[k], ck1[k]), k
    for k in g0:
        assert torch.equal(g0[k], g1[k]), k


def test_block_lax_rejects_a_gated_block():
    Bn, S, H, f, r = 1, 128, 1, 256, 32
    d = 128
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=23)
    desc = B.make_block_desc(Bn, S, d, H, 128, f, si.pad_ld(f, 8), r, eps=EPS, act=B.LR_ACT_SILU)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, si.pad_ld(f, 8)).items()}
    with pytest.raises(B.LrError):
        B.lr_block_lax_fwd(desc, packed, case["x"].to(DEV))


def test_two_block_stack_through_the_library():
    """Block 2 takes block 1's checkpoints as h_prev; block 1's backward takes block 2's dh_prev as
    dz_next.  The stack's input gradient and a few of block 1's weight gradients against the oracle
    run the same way in fp64."""
    Bn, S, H, f, r = 1, 256, 2, 344, 64
    d, case1, desc, packed1 = _setup(Bn, S, H, f, r, seed=31)
    _, case2, _, packed2 = _setup(Bn, S, H, f, r, seed=32)
    x, dy = case1["x"].to(DEV), case1["dy"].to(DEV)
    y1, ck1 = B.lr_block_lax_fwd(desc, packed1, x)
    hp2 = {k: ck1["z_" + k] for k in PARTS}
    y2, ck2 = B.lr_block_lax_fwd(desc, packed2, y1, h_prev=hp2)
    dx2, g2, dh2 = B.lr_block_lax_bwd(desc, packed2, y1, dy, ck2, h_prev=hp2)
    dx1, g1, _ = B.lr_block_lax_bwd(desc, packed1, x, dx2, ck1, dz_next=dh2, want_dh_prev=False)
    torch.cuda.synchronize()

    P1 = {k: si.f64(v) for k, v in case1["params"].items()}
    P2 = {k: si.f64(v) for k, v in case2["params"].items()}
    X, DY = si.f64(case1["x"]), si.f64(case1["dy"])
    T = Bn * S
    zero = lax.zeros_h(T, d, f, r)
    y1r, z1r, _ = lax.block_fwd(X, P1, zero, Bn, S, H, 128, EPS)
    y2r, _, _ = lax.block_fwd(y1r, P2, z1r, Bn, S, H, 128, EPS)
    dx2r, g2r, dh2r = lax.block_bwd(y1r, P2, z1r, DY, zero, Bn, S, H, 128, EPS)
    dx1r, g1r, _ = lax.block_bwd(X, P1, zero, dx2r, dh2r, Bn, S, H, 128, EPS)
    dt = torch.bfloat16
    # the budget: the same two-block chain through the bf16 model (its y1, z1, dx2 and dh2 feed the next call)
    def one_run(jit):
        m1, _, _ = M.block(X, P1, DY, Bn, S, H, 128, EPS, lax=True, jitter=jit)
        z1m = {n: m1["z_" + n] for n in lax.PROJ}
        m2, _, dh2m = M.block(m1["y"], P2, DY, Bn, S, H, 128, EPS, h_prev=z1m, lax=True, jitter=jit)
        m1b, g1m, _ = M.block(X, P1, m2["dx"], Bn, S, H, 128, EPS, dz_next=dh2m, lax=True, jitter=jit)
        bud = {"y2": M.err2(m2["y"], y2r), "dx1": M.err2(m1b["dx"], dx1r)}
        bud.update({"d" + k: M.err2(g1m[k], g1r[k]) for k in g1r})
        return bud

    bud = M.over_realisations(one_run)
    check("y2", y2, y2r, dt, bud["y2"])
    check("dx1", dx1, dx1r, dt, bud["dx1"])
    got1 = _unpack_grads(g1, f, r)
    for name in ("wd_q", "wu_v", "wd_o", "wd_g", "wu_u", "wd_d", "gamma1"):
        check("d" + name, got1[name], g1r[name], dt, bud["d" + name])


def test_block_lax_with_grouped_kv_heads():
    """LaX block with 4 query and 2 key / value heads: outputs, checkpoints, dx, dh_prev and the weight
    gradients against the fp64 oracle."""
    Bn, S, H, Hkv, f, r = 2, 192, 4, 2, 344, 64
    d, dkv, f_ld = 128 * H, 128 * Hkv, si.pad_ld(f, 8)
    print(f"block lax gqa B={Bn} S={S} H={H} Hkv={Hkv} f={f} r={r}", flush=True)
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=24, Hkv=Hkv)
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=EPS, act=B.LR_ACT_IDENTITY, n_kv_heads=Hkv)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    T = Bn * S
    h_prev = _rank_tensors(24, "hprev", T, r, 0.5)
    dz_next = _rank_tensors(24, "dznext", T, r, 1.0)
    x, dy = case["x"].to(DEV), case["dy"].to(DEV)
    hp_dev, dzn_dev = _cat(h_prev, DEV), _cat(dz_next, DEV)
    y, ck = B.lr_block_lax_fwd(desc, packed, x, h_prev=hp_dev)
    dx, grads, dh = B.lr_block_lax_bwd(desc, packed, x, dy, ck, h_prev=hp_dev, dz_next=dzn_dev)
    torch.cuda.synchronize()
    P = {k: si.f64(v) for k, v in case["params"].items()}
    X, DY = si.f64(case["x"]), si.f64(case["dy"])
    y_ref, z_ref, _ = lax.block_fwd(X, P, _f64(h_prev), Bn, S, H, 128, EPS, Hkv=Hkv)
    dx_ref, g_ref, dh_ref = lax.block_bwd(X, P, _f64(h_prev), DY, _f64(dz_next), Bn, S, H, 128, EPS, Hkv=Hkv)
    dt = torch.bfloat16
    bud = _lax_budget(X, P, DY, _f64(h_prev), _f64(dz_next), Bn, S, H, y_ref, z_ref, dx_ref, g_ref, dh_ref, Hkv=Hkv)
    check("y", y, y_ref, dt, bud["y"])
    z_gpu = _split({k: ck["z_" + k] for k in PARTS}, r)
    for n in lax.PROJ:
        check("z_" + n, z_gpu[n], z_ref[n], dt, bud["z_" + n])
    check("dx", dx, dx_ref, dt, bud["dx"])
    dh_gpu = _split(dh, r)
    for n in lax.PROJ:
        check("dh_prev_" + n, dh_gpu[n], dh_ref[n], dt, bud["dh_prev_" + n])
    wq = grads["w_up_qkv"].reshape(-1, r)
    got = {"wu_q": wq[:d], "wu_k": wq[d:d + dkv], "wu_v": wq[d + dkv:], "wd_q": grads["w_dn_qkv"][:r],
           "wd_k": grads["w_dn_qkv"][r:2 * r], "wd_v": grads["w_dn_qkv"][2 * r:], "wu_o": grads["w_up_o"],
           "gamma1": grads["gamma1"], "wd_d": grads["w_dn_d"][:, :f]}
    for name, g in got.items():
        check("d" + name, g, g_ref[name], dt, bud["d" + name])
