"""Pins for oracle/gqa_oracle.py (grouped-query attention, the extension named in the section
"Discussion and Future Work"): nothing here re-uses its formulas.  Reduction to the multi-head oracle, equivalence with
multi-head attention on explicitly repeated key / value heads (gradients of the copies added),
softmax invariants, and central finite differences of a scalar loss."""
import numpy as np
import pytest

from oracle import gqa_oracle as gqa
from oracle import lowrank_oracle as orc


def _relerr(a, b):
    return np.max(np.abs(a - b)) / (np.sqrt(np.mean(b * b)) + 1e-300)


def _case(rng, B, S, H, Hkv, hd):
    T = B * S
    return (rng.normal(size=(T, H * hd)), rng.normal(size=(T, Hkv * hd)), rng.normal(size=(T, Hkv * hd)),
            rng.normal(size=(T, H * hd)))


def _repeat_heads(x, T, Hkv, grp, hd):
    return np.repeat(x.reshape(T, Hkv, 1, hd), grp, axis=2).reshape(T, Hkv * grp * hd)


def test_as_many_kv_heads_as_query_heads_is_multi_head_attention():
    rng = np.random.default_rng(1)
    B, S, H, hd = 2, 7, 3, 4
    q, k, v, do = _case(rng, B, S, H, H, hd)
    o, lse = gqa.attention_gqa_fwd(q, k, v, B, S, H, H, hd)
    o0, lse0 = orc.attention_fwd(q, k, v, B, S, H, hd)
    assert _relerr(o, o0) < 1e-13 and _relerr(lse, lse0) < 1e-13
    for a, b in zip(gqa.attention_gqa_bwd(q, k, v, do, B, S, H, H, hd), orc.attention_bwd(q, k, v, do, B, S, H, hd)):
        assert _relerr(a, b) < 1e-12


@pytest.mark.parametrize("H,Hkv", [(4, 2), (6, 2), (4, 1), (6, 3)])
@pytest.mark.parametrize("causal", [True, False])
def test_equals_multi_head_attention_on_repeated_kv_heads(H, Hkv, causal):
    rng = np.random.default_rng(10 * H + Hkv)
    B, S, hd = 2, 6, 4
    T, grp = B * S, H // Hkv
    q, k, v, do = _case(rng, B, S, H, Hkv, hd)
    kr, vr = _repeat_heads(k, T, Hkv, grp, hd), _repeat_heads(v, T, Hkv, grp, hd)
    o, lse = gqa.attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd, causal)
    o0, lse0 = orc.attention_fwd(q, kr, vr, B, S, H, hd, causal)
    assert _relerr(o, o0) < 1e-13 and _relerr(lse, lse0) < 1e-13
    dq, dk, dv = gqa.attention_gqa_bwd(q, k, v, do, B, S, H, Hkv, hd, causal)
    dq0, dk0, dv0 = orc.attention_bwd(q, kr, vr, do, B, S, H, hd, causal)
    assert _relerr(dq, dq0) < 1e-12
    assert _relerr(dk, dk0.reshape(T, Hkv, grp, hd).sum(axis=2).reshape(T, Hkv * hd)) < 1e-12
    assert _relerr(dv, dv0.reshape(T, Hkv, grp, hd).sum(axis=2).reshape(T, Hkv * hd)) < 1e-12
    # the sum over the group matters: one copy alone is far off
    assert _relerr(dk, dk0.reshape(T, Hkv, grp, hd)[:, :, 0].reshape(T, Hkv * hd)) > 1e-2


def test_first_token_returns_v0_and_uniform_keys_average_the_values():
    rng = np.random.default_rng(3)
    B, S, H, Hkv, hd = 1, 5, 4, 2, 4
    q, k, v, _ = _case(rng, B, S, H, Hkv, hd)
    o, lse = gqa.attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd)
    o4, v4 = o.reshape(S, H, hd), v.reshape(S, Hkv, hd)
    for h in range(H):
        assert np.allclose(o4[0, h], v4[0, h // 2], atol=1e-14)
    # all keys equal: every probability row is uniform over the visible keys, so token t returns the
    # mean of v_0..v_t of its group's value head, and lse = s + log(t + 1)
    k_same = np.tile(k.reshape(S, Hkv, hd)[:1], (S, 1, 1)).reshape(S, Hkv * hd)
    o, lse = gqa.attention_gqa_fwd(q, k_same, v, B, S, H, Hkv, hd)
    o4 = o.reshape(S, H, hd)
    for h in range(H):
        for t in range(S):
            assert np.allclose(o4[t, h], v4[:t + 1, h // 2].mean(axis=0), atol=1e-13)
            s = q.reshape(S, H, hd)[t, h] @ k_same.reshape(S, Hkv, hd)[0, h // 2] / 2.0
            assert abs(lse[0, h, t] - (s + np.log(t + 1))) < 1e-12


def test_gradients_by_finite_differences():
    rng = np.random.default_rng(4)
    B, S, H, Hkv, hd = 1, 5, 4, 2, 3
    q, k, v, do = _case(rng, B, S, H, Hkv, hd)

    def loss():
        return float(np.sum(gqa.attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd)[0] * do))

    def fd(arr, eps=1e-6):
        g = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            old = arr[idx]
            arr[idx] = old + eps
            fp = loss()
            arr[idx] = old - eps
            fm = loss()
            arr[idx] = old
            g[idx] = (fp - fm) / (2 * eps)
        return g

    dq, dk, dv = gqa.attention_gqa_bwd(q, k, v, do, B, S, H, Hkv, hd)
    assert _relerr(dq, fd(q)) < 1e-6
    assert _relerr(dk, fd(k)) < 1e-6
    assert _relerr(dv, fd(v)) < 1e-6


# ---- the block with grouped K / V projections -------------------------------------------------
def _block_params(rng, D, Dkv, F, R):
    dims = {"q": (D, D), "k": (D, Dkv), "v": (D, Dkv), "o": (D, D), "g": (D, F), "u": (D, F), "d": (F, D)}
    p = {}
    for n, (d_in, d_out) in dims.items():
        p["wd_" + n] = rng.normal(size=(R, d_in)) * d_in ** -0.5
        p["wu_" + n] = rng.normal(size=(d_out, R)) * R ** -0.5
    p["gamma1"] = 1.0 + 0.1 * rng.normal(size=(D,))
    p["gamma2"] = 1.0 + 0.1 * rng.normal(size=(D,))
    return p


@pytest.mark.parametrize("with_rope", [False, True])
def test_gqa_block_equals_the_multi_head_block_with_repeated_kv_up_projection_rows(with_rope):
    """A block with Hkv key / value heads is the multi-head block whose K and V up-projections repeat every
    head's rows H / Hkv times; the gradient of a shared row block is the sum over its copies."""
    rng = np.random.default_rng(21)
    B, S, H, Hkv, hd, F, R = 2, 5, 4, 2, 4, 6, 3
    D, Dkv, T, grp = H * hd, Hkv * hd, B * S, H // Hkv
    p = _block_params(rng, D, Dkv, F, R)
    x, dy = rng.normal(size=(T, D)), rng.normal(size=(T, D))
    rope = orc.rope_tables(S, hd, 100.0) if with_rope else None

    def rep_rows(w):      # [Hkv*hd, R] -> [H*hd, R]
        return np.repeat(w.reshape(Hkv, 1, hd, R), grp, axis=1).reshape(H * hd, R)

    def sum_rows(w):      # [H*hd, R] -> [Hkv*hd, R]
        return w.reshape(Hkv, grp, hd, R).sum(axis=1).reshape(Hkv * hd, R)

    pf = dict(p)
    pf["wu_k"], pf["wu_v"] = rep_rows(p["wu_k"]), rep_rows(p["wu_v"])
    y, _ = orc.block_fwd(x, p, B, S, H, hd, 1e-5, rope=rope, Hkv=Hkv)
    y0, _ = orc.block_fwd(x, pf, B, S, H, hd, 1e-5, rope=rope)
    assert _relerr(y, y0) < 1e-12
    dx, g = orc.block_bwd(x, p, dy, B, S, H, hd, 1e-5, rope=rope, Hkv=Hkv)
    dx0, g0 = orc.block_bwd(x, pf, dy, B, S, H, hd, 1e-5, rope=rope)
    assert _relerr(dx, dx0) < 1e-11
    for k in g:
        want = sum_rows(g0[k]) if k in ("wu_k", "wu_v") else g0[k]
        assert _relerr(g[k], want) < 1e-11, k


def test_gqa_block_gradients_by_finite_differences():
    rng = np.random.default_rng(22)
    B, S, H, Hkv, hd, F, R = 1, 4, 4, 2, 2, 5, 3
    D, Dkv, T = H * hd, Hkv * hd, B * S
    p = _block_params(rng, D, Dkv, F, R)
    x, dy = rng.normal(size=(T, D)), rng.normal(size=(T, D))

    def loss():
        return float(np.sum(orc.block_fwd(x, p, B, S, H, hd, 1e-5, Hkv=Hkv)[0] * dy))

    def fd(arr, eps=1e-6):
        g = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            old = arr[idx]
            arr[idx] = old + eps
            fp = loss()
            arr[idx] = old - eps
            fm = loss()
            arr[idx] = old
            g[idx] = (fp - fm) / (2 * eps)
        return g

    dx, g = orc.block_bwd(x, p, dy, B, S, H, hd, 1e-5, Hkv=Hkv)
    assert _relerr(dx, fd(x)) < 1e-6
    for k in ("wu_k", "wu_v", "wd_k", "wd_v", "wu_q", "wd_o", "gamma1"):
        assert _relerr(g[k], fd(p[k])) < 1e-6, k
