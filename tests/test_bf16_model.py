"""The bf16 error-budget model (tests/bf16_model.py) against the fp64 oracle.

With its roundings switched off the model follows the GPU design's data flow in exact arithmetic: norm
scale folded into the weight, row scale after the product, the RMSNorm-backward statistic taken at
rank r, weight gradient of the folded weight scaled back by gamma, dgamma as a column sum over it.  It
must then agree with the plain definition (separate projections, two-pass norm, store-everything
backward) to fp64 round-off: that pins the model and the algebra the kernels are built on.  With the
roundings on, its distance to the oracle is the budget the GPU tests grant beyond the flat tolerance.
"""
import numpy as np
import pytest
import torch

import bf16_model as M
import synth_inputs as si
from oracle import gqa_oracle, lax_oracle
from oracle import lowrank_oracle as orc

EPS = 1e-5
KEYS_Z = ("z_q", "z_k", "z_v", "z_o", "z_g", "z_u", "z_d")


def _case(Bn, S, H, f, r, seed, Hkv=None):
    d = 128 * H
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=seed, Hkv=Hkv)
    P = {k: si.f64(v) for k, v in case["params"].items()}
    return d, P, si.f64(case["x"]), si.f64(case["dy"])


def _close(a, b, tol=1e-9):
    assert M.relerr(a, b) < tol, M.relerr(a, b)


@pytest.mark.parametrize("act", ["silu", "identity"])
@pytest.mark.parametrize("two_pass", [False, True])
def test_exact_model_equals_oracle(act, two_pass):
    Bn, S, H, f, r = 2, 96, 2, 200, 48
    d, P, X, DY = _case(Bn, S, H, f, r, seed=11)
    oact = orc.ACT_SILU if act == "silu" else orc.ACT_IDENTITY
    out, g, _ = M.block(X, P, DY, Bn, S, H, 128, EPS, act=act, two_pass=two_pass, rnd=M.identity)
    y_ref, c = orc.block_fwd(X, P, Bn, S, H, 128, EPS, act=oact)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS, act=oact)
    _close(out["y"], y_ref)
    _close(out["dx"], dx_ref)
    for k in KEYS_Z:
        _close(out[k], c[k])
    _close(out["s1"], orc.rms_stat(X))
    _close(out["s2"], orc.rms_stat(c["h1"]))
    assert set(g) == set(g_ref)
    for k in g_ref:
        _close(g[k], g_ref[k])


def test_exact_model_equals_oracle_rope_and_gqa():
    Bn, S, H, f, r, Hkv = 1, 80, 4, 160, 32, 2
    d, P, X, DY = _case(Bn, S, H, f, r, seed=12, Hkv=Hkv)
    rope = orc.rope_tables(S, 128)
    out, g, _ = M.block(X, P, DY, Bn, S, H, 128, EPS, rope=rope, Hkv=Hkv, rnd=M.identity)
    y_ref, c = orc.block_fwd(X, P, Bn, S, H, 128, EPS, rope=rope, Hkv=Hkv)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS, rope=rope, Hkv=Hkv)
    _close(out["y"], y_ref)
    _close(out["dx"], dx_ref)
    for k in g_ref:
        _close(g[k], g_ref[k])


def test_exact_model_equals_lax_oracle():
    Bn, S, H, f, r = 1, 64, 2, 144, 40
    d, P, X, DY = _case(Bn, S, H, f, r, seed=13)
    T = Bn * S
    rng = np.random.default_rng(5)
    hp = {n: rng.standard_normal((T, r)) * 0.5 for n in M.PROJ}
    dzn = {n: rng.standard_normal((T, r)) for n in M.PROJ}
    out, g, dh = M.block(X, P, DY, Bn, S, H, 128, EPS, h_prev=hp, dz_next=dzn, lax=True, rnd=M.identity)
    y_ref, z_ref, _ = lax_oracle.block_fwd(X, P, hp, Bn, S, H, 128, EPS)
    dx_ref, g_ref, dh_ref = lax_oracle.block_bwd(X, P, hp, DY, dzn, Bn, S, H, 128, EPS)
    _close(out["y"], y_ref)
    _close(out["dx"], dx_ref)
    for n in M.PROJ:
        _close(out["z_" + n], z_ref[n])
        _close(dh[n], dh_ref[n])
    for k in g_ref:
        _close(g[k], g_ref[k])


def test_exact_attention_model_equals_oracle():
    B, S, H, Hkv, hd = 2, 70, 4, 2, 128
    rng = np.random.default_rng(3)
    q = rng.standard_normal((B * S, H * hd))
    k = rng.standard_normal((B * S, Hkv * hd))
    v = rng.standard_normal((B * S, Hkv * hd))
    do = rng.standard_normal((B * S, H * hd))
    o, lse = M.attention_fwd(q, k, v, B, S, H, Hkv, hd, rnd=M.identity)
    o_ref, lse_ref = gqa_oracle.attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd, True)
    _close(o, o_ref)
    _close(lse, lse_ref)
    dq, dk, dv = M.attention_bwd(q, k, v, o, do, lse, B, S, H, Hkv, hd, rnd=M.identity)
    for a, b in zip((dq, dk, dv), gqa_oracle.attention_gqa_bwd(q, k, v, do, B, S, H, Hkv, hd, True)):
        _close(a, b)


def test_rounding_is_bf16_nearest_even():
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -3.0 - 2.0 ** -7, 1e-30, 0.0])
    got = M.bf16(a)
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.0 + 2.0 ** -6 and got[5] == 0.0   # ties to even
    assert got[3] == -3.0 - 2.0 ** -6 or got[3] == -3.0           # a tie: even mantissa
    t = torch.tensor(a, dtype=torch.float32).to(torch.bfloat16).double().numpy()
    assert np.array_equal(got, t)


def test_budget_of_a_small_block_is_of_the_size_of_a_few_roundings():
    """The budget is neither trivial nor a blank cheque: every tensor's modelled error lies between the
    error of one rounding of a unit Gaussian tensor and 6e-2, and the outputs behind the longest chains
    (weight gradients behind forward + backward) sit above the outputs behind the shortest (z_qkv)."""
    Bn, S, H, f, r = 2, 192, 2, 344, 64
    d, P, X, DY = _case(Bn, S, H, f, r, seed=0)
    out, g, _ = M.block(X, P, DY, Bn, S, H, 128, EPS)
    y_ref, c = orc.block_fwd(X, P, Bn, S, H, 128, EPS)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS)
    errs = {"y": M.relerr(out["y"], y_ref), "dx": M.relerr(out["dx"], dx_ref)}
    errs.update({k: M.relerr(out[k], c[k]) for k in KEYS_Z})
    errs.update({"d" + k: M.relerr(g[k], g_ref[k]) for k in g_ref})
    print({k: f"{v:.2e}" for k, v in errs.items()})
    assert all(2e-3 < v < 6e-2 for v in errs.values()), errs
    assert errs["dwd_q"] > errs["z_q"]


def test_realisations_agree_in_l2_and_scatter_in_the_maximum():
    """Why the budget bounds L2 sharply and the maximum loosely: across realisations of the rounding
    errors of the SAME ideal pipeline (softmax references jittered by a fraction of a binade) the relative
    L2 error of most tensors moves by a few percent (up to a fifth for the value-path gradients of this
    short sequence, where one probability per row carries much of the weight and is exact only when the
    reference is the row maximum), the max-norm error of a weight gradient by tens of percent."""
    Bn, S, H, f, r = 1, 300, 1, 200, 32
    d, P, X, DY = _case(Bn, S, H, f, r, seed=0)
    dx_ref, g_ref = orc.block_bwd(X, P, DY, Bn, S, H, 128, EPS)
    runs = []
    for i in range(5):
        jit = None if i == 0 else np.random.default_rng(1000 + i)
        _, g, _ = M.block(X, P, DY, Bn, S, H, 128, EPS, jitter=jit)
        runs.append({k: M.err2(g[k], g_ref[k]) for k in g_ref})
    spread_max = max(max(r[k][0] for r in runs) / min(r[k][0] for r in runs) for k in g_ref)
    spread_l2 = max(max(r[k][1] for r in runs) / min(r[k][1] for r in runs) for k in g_ref)
    print(f"largest ratio between realisations: max-norm {spread_max:.2f}, L2 {spread_l2:.3f}")
    med_l2 = float(np.median([max(r[k][1] for r in runs) / min(r[k][1] for r in runs) for k in g_ref]))
    assert med_l2 < 1.06 and spread_l2 < 1.25
    assert 1.15 < spread_max < 1.9
