"""Pins for oracle/lowrank_oracle.py: things the paper and the mathematics fix, none of which
re-use the oracle's own formulas.  A dropped term, a wrong sign, a transposed operand or a
wrong index in the oracle fails at least one test here."""
import math

import numpy as np
import pytest

from golden_io import load_golden
from oracle import lowrank_oracle as orc

G = load_golden()
RNG = np.random.default_rng(12345)


# ---------------------------------------------------------------- scalar brute force helpers
def _silu_scalar(z):
    return z / (1.0 + math.exp(-z))


def _brute_linear(x, wd, wu, silu=True):
    T, d_in = x.shape
    r = wd.shape[0]
    d_out = wu.shape[0]
    z = [[0.0] * r for _ in range(T)]
    y = [[0.0] * d_out for _ in range(T)]
    for t in range(T):
        for i in range(r):
            acc = 0.0
            for j in range(d_in):
                acc += wd[i, j] * x[t, j]
            z[t][i] = acc
        for o in range(d_out):
            acc = 0.0
            for i in range(r):
                a = _silu_scalar(z[t][i]) if silu else z[t][i]
                acc += wu[o, i] * a
            y[t][o] = acc
    return np.array(z), np.array(y)


def _fd_grad(fun, arr, eps=1e-6):
    """Central finite differences of scalar fun() w.r.t. every entry of arr (in place)."""
    g = np.zeros_like(arr)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = arr[idx]
        arr[idx] = old + eps
        fp = fun()
        arr[idx] = old - eps
        fm = fun()
        arr[idx] = old
        g[idx] = (fp - fm) / (2 * eps)
    return g


def _relerr(a, b):
    return np.max(np.abs(a - b)) / (np.sqrt(np.mean(b * b)) + 1e-300)


# ---------------------------------------------------------------- sigma
def test_silu_closed_forms():
    assert orc.silu(0.0) == 0.0
    assert math.isclose(float(orc.silu(1.0)), 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-15)
    assert math.isclose(float(orc.silu_prime(0.0)), 0.5, rel_tol=1e-15)
    # SiLU(z) - SiLU(-z) = z ; large |z| limits
    z = RNG.normal(size=100) * 3
    np.testing.assert_allclose(orc.silu(z) - orc.silu(-z), z, rtol=1e-13, atol=1e-13)
    assert abs(float(orc.silu(40.0)) - 40.0) < 1e-12 and abs(float(orc.silu(-40.0))) < 1e-12
    # derivative by finite differences
    h = 1e-6
    fd = (orc.silu(z + h) - orc.silu(z - h)) / (2 * h)
    np.testing.assert_allclose(orc.silu_prime(z), fd, rtol=1e-8, atol=1e-9)


# ---------------------------------------------------------------- one bottleneck layer
def test_linear_matches_scalar_loops():
    T, d_in, r, d_out = 5, 7, 3, 6          # non-square on purpose: catches transposed operands
    x = RNG.normal(size=(T, d_in)); wd = RNG.normal(size=(r, d_in)); wu = RNG.normal(size=(d_out, r))
    for act, silu in ((orc.ACT_SILU, True), (orc.ACT_IDENTITY, False)):
        z, a, y = orc.lr_linear_fwd(x, wd, wu, act)
        zb, yb = _brute_linear(x, wd, wu, silu)
        np.testing.assert_allclose(z, zb, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(y, yb, rtol=1e-13, atol=1e-13)


def test_identity_sigma_equals_dense_product():
    """SVD variant (App. 'SVD baseline'): y = A (B x) is the dense map W = W_up W_down."""
    T, d_in, r, d_out = 9, 12, 4, 10
    x = RNG.normal(size=(T, d_in)); wd = RNG.normal(size=(r, d_in)); wu = RNG.normal(size=(d_out, r))
    W = np.zeros((d_out, d_in))
    for o in range(d_out):
        for j in range(d_in):
            W[o, j] = sum(wu[o, i] * wd[i, j] for i in range(r))
    _, _, y = orc.lr_linear_fwd(x, wd, wu, orc.ACT_IDENTITY)
    dense = np.array([[sum(W[o, j] * x[t, j] for j in range(d_in)) for o in range(d_out)] for t in range(T)])
    np.testing.assert_allclose(y, dense, rtol=1e-12, atol=1e-12)
    assert np.linalg.matrix_rank(W) == r


@pytest.mark.parametrize("act", [orc.ACT_SILU, orc.ACT_IDENTITY])
def test_linear_bwd_finite_differences(act):
    T, d_in, r, d_out = 4, 6, 3, 5
    x = RNG.normal(size=(T, d_in)); wd = RNG.normal(size=(r, d_in)); wu = RNG.normal(size=(d_out, r))
    dy = RNG.normal(size=(T, d_out))
    loss = lambda: float(np.sum(orc.lr_linear_fwd(x, wd, wu, act)[2] * dy))
    dx, dwd, dwu = orc.lr_linear_bwd(x, wd, wu, dy, act)
    assert _relerr(dx, _fd_grad(loss, x)) < 1e-7
    assert _relerr(dwd, _fd_grad(loss, wd)) < 1e-7
    assert _relerr(dwu, _fd_grad(loss, wu)) < 1e-7


# ---------------------------------------------------------------- RMSNorm (Eq. 4) and Alg. 1
def test_rmsnorm_scalar_definition_and_eps_placement():
    T, d = 4, 6
    x = RNG.normal(size=(T, d)); gamma = 1 + 0.1 * RNG.normal(size=d)
    for eps in (0.0, 1e-6, 1e-5, 0.3):
        xh, rms = orc.rmsnorm_fwd(x, gamma, eps)
        for t in range(T):
            ms = sum(x[t, j] ** 2 for j in range(d)) / d
            rt = math.sqrt(ms + eps)             # eps inside the root, after the mean
            assert math.isclose(rms[t], rt, rel_tol=1e-14)
            for j in range(d):
                assert math.isclose(xh[t, j], x[t, j] * gamma[j] / rt, rel_tol=1e-13, abs_tol=1e-15)
    # eps = 0, gamma = 1: every normalised row has mean square exactly 1; scale invariance
    xh, _ = orc.rmsnorm_fwd(x, np.ones(d), 0.0)
    np.testing.assert_allclose(np.mean(xh * xh, axis=1), 1.0, rtol=1e-13)
    xh2, _ = orc.rmsnorm_fwd(7.5 * x, np.ones(d), 0.0)
    np.testing.assert_allclose(xh, xh2, rtol=1e-13)


def test_rmsnorm_bwd_finite_differences():
    T, d = 3, 7
    x = RNG.normal(size=(T, d)); gamma = 1 + 0.1 * RNG.normal(size=d); dxh = RNG.normal(size=(T, d))
    for eps in (0.0, 1e-5, 0.2):
        loss = lambda: float(np.sum(orc.rmsnorm_fwd(x, gamma, eps)[0] * dxh))
        dx, dgamma = orc.rmsnorm_bwd(x, gamma, eps, dxh)
        assert _relerr(dx, _fd_grad(loss, x)) < 1e-7
        assert _relerr(dgamma, _fd_grad(loss, gamma)) < 1e-7


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_online_rmsnorm_shards_equal_two_pass(k):
    """Eq. 5: Alg. 1 over k shards is exactly RMSNorm followed by the full matmul."""
    T, d, r = 6, 32, 5
    x = RNG.normal(size=(T, d)) * 3; gamma = 1 + 0.1 * RNG.normal(size=d); w = RNG.normal(size=(d, r))
    for eps in (0.0, 1e-5):
        xh, _ = orc.rmsnorm_fwd(x, gamma, eps)
        ref = xh @ w
        got = orc.online_rmsnorm_sharded(x, gamma, w, k, eps)
        assert _relerr(got, ref) < 1e-13


def test_online_rmsnorm_fp32_magnitude_vs_table2():
    """Table 2 gives only magnitudes (shapes unstated): fp32 online (TP=4) vs TP=1 differs at
    the 1e-7..1e-6 level in max-abs and 1e-8..1e-7 in mean-abs for unit-scale outputs."""
    T, d, r, k, eps = 256, 1024, 256, 4, 1e-5
    rng = np.random.default_rng(7)
    x = rng.normal(size=(T, d)).astype(np.float32)
    gamma = np.ones(d, dtype=np.float32)
    w = (rng.normal(size=(d, r)) / math.sqrt(d)).astype(np.float32)
    # TP=1 baseline in fp32
    rms = np.sqrt(np.mean(x * x, axis=1, dtype=np.float32) + np.float32(eps))
    base = (x / rms[:, None] * gamma) @ w
    # Alg. 1 in fp32
    dl = d // k
    h = np.zeros((T, r), dtype=np.float32); s = np.zeros(T, dtype=np.float32)
    for i in range(k):
        xi = x[:, i * dl:(i + 1) * dl]
        sl = np.sum(xi * xi, axis=1, dtype=np.float32)
        rl = np.sqrt(sl / np.float32(dl) + np.float32(eps))
        h += ((xi / rl[:, None] * gamma[i * dl:(i + 1) * dl]) @ w[i * dl:(i + 1) * dl]) * rl[:, None]
        s += sl
    y = h / np.sqrt(s / np.float32(d) + np.float32(eps))[:, None]
    diff = np.abs(y.astype(np.float64) - base.astype(np.float64))
    assert G["table2_fp32_avg_max_abs"] / 10 < diff.max() < G["table2_fp32_avg_max_abs"] * 10
    assert G["table2_fp32_avg_mean_abs"] / 10 < diff.mean() < G["table2_fp32_avg_mean_abs"] * 10
    # and the fp64 oracle sits within fp32 round-off of both
    ref = orc.online_rmsnorm_sharded(x, gamma, w, k, eps)
    assert np.abs(ref - base).max() < 1e-5


# ---------------------------------------------------------------- grouping (Sec. 4.3)
def test_grouped_down_projection_equals_separate():
    T, d, r, dout, Gn, eps = 7, 16, 4, 10, 3, 1e-5
    x = RNG.normal(size=(T, d)); gamma = 1 + 0.1 * RNG.normal(size=d)
    wds = [RNG.normal(size=(r, d)) for _ in range(Gn)]; wus = [RNG.normal(size=(dout, r)) for _ in range(Gn)]
    zs, ys, stat = orc.lr_group_fwd(x, gamma, eps, wds, wus)
    xh, _ = orc.rmsnorm_fwd(x, gamma, eps)
    zcat = xh @ np.concatenate(wds, axis=0).T            # one GEMM on concatenated weights
    for g in range(Gn):
        np.testing.assert_allclose(zs[g], zcat[:, g * r:(g + 1) * r], rtol=1e-13, atol=1e-13)
    a = orc.silu(np.stack(zs, 0))                          # batched up-projection
    ystack = np.einsum("gtr,gor->gto", a, np.stack(wus, 0))
    for g in range(Gn):
        np.testing.assert_allclose(ys[g], ystack[g], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(stat, [sum(v * v for v in row) for row in x], rtol=1e-13)


@pytest.mark.parametrize("norm", [True, False])
def test_group_bwd_finite_differences(norm):
    T, d, r, dout, Gn, eps = 3, 6, 2, 4, 3, 1e-5
    x = RNG.normal(size=(T, d)); gamma = 1 + 0.1 * RNG.normal(size=d)
    wds = [RNG.normal(size=(r, d)) for _ in range(Gn)]; wus = [RNG.normal(size=(dout, r)) for _ in range(Gn)]
    dys = [RNG.normal(size=(T, dout)) for _ in range(Gn)]

    def loss():
        _, ys, _ = orc.lr_group_fwd(x, gamma, eps, wds, wus, norm=norm)
        return float(sum(np.sum(y * dy) for y, dy in zip(ys, dys)))

    dx, dgamma, dwd, dwu = orc.lr_group_bwd(x, gamma, eps, wds, wus, dys, norm=norm)
    assert _relerr(dx, _fd_grad(loss, x)) < 1e-7
    if norm:
        assert _relerr(dgamma, _fd_grad(loss, gamma)) < 1e-7
    else:
        assert dgamma is None
    for g in range(Gn):
        assert _relerr(dwd[g], _fd_grad(loss, wds[g])) < 1e-7
        assert _relerr(dwu[g], _fd_grad(loss, wus[g])) < 1e-7


# ---------------------------------------------------------------- attention
def _brute_attention(q, k, v, B, S, H, hd, causal):
    o = np.zeros((B * S, H * hd))
    for b in range(B):
        for h in range(H):
            for i in range(S):
                qi = q[b * S + i, h * hd:(h + 1) * hd]
                last = i if causal else S - 1
                sc = [sum(qi[c] * k[b * S + j, h * hd + c] for c in range(hd)) / math.sqrt(hd) for j in range(last + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                den = sum(e)
                for c in range(hd):
                    o[b * S + i, h * hd + c] = sum(e[j] / den * v[b * S + j, h * hd + c] for j in range(last + 1))
    return o


@pytest.mark.parametrize("causal", [True, False])
def test_attention_matches_scalar_loops(causal):
    B, S, H, hd = 2, 5, 3, 4
    q, k, v = (RNG.normal(size=(B * S, H * hd)) for _ in range(3))
    o, lse = orc.attention_fwd(q, k, v, B, S, H, hd, causal)
    np.testing.assert_allclose(o, _brute_attention(q, k, v, B, S, H, hd, causal), rtol=1e-12, atol=1e-12)


def test_attention_invariants():
    B, S, H, hd = 2, 6, 2, 4
    q, k, v = (RNG.normal(size=(B * S, H * hd)) for _ in range(3))
    o, lse, p = orc.attention_fwd(q, k, v, B, S, H, hd, True, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-13)
    assert np.all(np.triu(p, 1) == 0.0)                         # no weight on future keys
    for b in range(B):                                          # first token sees only itself
        np.testing.assert_allclose(o[b * S], v[b * S], rtol=1e-13)
    # S = 1  =>  o = v
    o1, _ = orc.attention_fwd(q[:B], k[:B], v[:B], B, 1, H, hd, True)
    np.testing.assert_allclose(o1, v[:B], rtol=1e-13)
    # changing a future token never changes earlier outputs
    k2, v2 = k.copy(), v.copy(); k2[S - 1] += 1.0; v2[S - 1] -= 2.0
    o2, _ = orc.attention_fwd(q, k2, v2, B, S, H, hd, True)
    np.testing.assert_allclose(o2[:S - 1], o[:S - 1], rtol=1e-13)
    # batch elements are independent: swapping them swaps the outputs
    sw = np.concatenate([np.arange(S, 2 * S), np.arange(S)])
    o3, _ = orc.attention_fwd(q[sw], k[sw], v[sw], B, S, H, hd, True)
    np.testing.assert_allclose(o3, o[sw], rtol=1e-13)
    # LSE definition
    s00 = (q[:S, :hd] @ k[:S, :hd].T) / math.sqrt(hd)
    for i in range(S):
        assert math.isclose(lse[0, 0, i], math.log(sum(math.exp(s00[i, j]) for j in range(i + 1))), rel_tol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_attention_bwd_finite_differences(causal):
    B, S, H, hd = 2, 4, 2, 3
    q, k, v, do = (RNG.normal(size=(B * S, H * hd)) for _ in range(4))
    loss = lambda: float(np.sum(orc.attention_fwd(q, k, v, B, S, H, hd, causal)[0] * do))
    dq, dk, dv = orc.attention_bwd(q, k, v, do, B, S, H, hd, causal)
    assert _relerr(dq, _fd_grad(loss, q)) < 1e-7
    assert _relerr(dk, _fd_grad(loss, k)) < 1e-7
    assert _relerr(dv, _fd_grad(loss, v)) < 1e-7


# ---------------------------------------------------------------- the block
def _tiny_block(seed=3, B=2, S=3, H=2, hd=4, f=12, r=4):
    rng = np.random.default_rng(seed)
    d = H * hd
    dims = {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d), "g": (d, f), "u": (d, f), "d": (f, d)}
    p = {}
    for n, (di, do) in dims.items():
        p["wd_" + n] = rng.normal(size=(r, di)) / math.sqrt(di)
        p["wu_" + n] = rng.normal(size=(do, r)) / math.sqrt(r)
    p["gamma1"] = 1 + 0.1 * rng.normal(size=d)
    p["gamma2"] = 1 + 0.1 * rng.normal(size=d)
    x = rng.normal(size=(B * S, d)); dy = rng.normal(size=(B * S, d))
    return x, dy, p, dict(B=B, S=S, H=H, hd=hd, eps=1e-5), (d, f, r)


def test_block_parameter_count_and_rank_boundaries():
    """App. 'Communication volume analysis': 11dr + 3 d_ff r parameters in the seven factored
    maps; Eq. 3: seven rank-r boundaries per block."""
    x, dy, p, kw, (d, f, r) = _tiny_block()
    n = sum(v.size for k_, v in p.items() if k_.startswith("w"))
    assert n == orc.block_param_count(d, f, r) == 11 * d * r + 3 * f * r
    _, c = orc.block_fwd(x, p, **kw)
    assert sum(c["z_" + n_].shape[1] for n_ in orc.PROJ) == 7 * r
    _, _, d7, f7, r7 = (int(v) for v in G["model_7B"])
    assert orc.block_param_count(d7, f7, r7) == 79953920


def test_block_forward_composition_by_hand():
    """Rebuild y from scalar-loop pieces (no oracle linear/attention code)."""
    x, dy, p, kw, (d, f, r) = _tiny_block()
    B, S, H, hd, eps = kw["B"], kw["S"], kw["H"], kw["hd"], kw["eps"]

    def norm(a, g):
        return np.array([[a[t, j] * g[j] / math.sqrt(sum(a[t, c] ** 2 for c in range(d)) / d + eps)
                          for j in range(d)] for t in range(a.shape[0])])

    lin = lambda a, n: _brute_linear(a, p["wd_" + n], p["wu_" + n])[1]
    xh1 = norm(x, p["gamma1"])
    o = _brute_attention(lin(xh1, "q"), lin(xh1, "k"), lin(xh1, "v"), B, S, H, hd, True)
    h1 = x + lin(o, "o")
    xh2 = norm(h1, p["gamma2"])
    g, u = lin(xh2, "g"), lin(xh2, "u")
    m = np.vectorize(_silu_scalar)(g) * u
    y_ref = h1 + lin(m, "d")
    y, _ = orc.block_fwd(x, p, **kw)
    np.testing.assert_allclose(y, y_ref, rtol=1e-11, atol=1e-12)


def test_block_bwd_finite_differences():
    x, dy, p, kw, _ = _tiny_block()
    loss = lambda: float(np.sum(orc.block_fwd(x, p, **kw)[0] * dy))
    dx, g = orc.block_bwd(x, p, dy, **kw)
    assert _relerr(dx, _fd_grad(loss, x)) < 1e-6
    for name in p:
        assert _relerr(g[name], _fd_grad(loss, p[name])) < 1e-6, name


def test_rank_r_checkpoints_suffice():
    """Sec. 4.4: re-forwarding from x and the rank-r pre-activations reproduces every wide
    activation the backward consumes."""
    x, dy, p, kw, _ = _tiny_block()
    _, c = orc.block_fwd(x, p, **kw)
    ck = {k_: c[k_] for k_ in c if k_.startswith("z_")}
    r = orc.reforward_from_checkpoints(x, p, ck, kw["B"], kw["S"], kw["H"], kw["hd"])
    for name in ("q", "k", "v", "o", "h1", "g", "u", "m"):
        np.testing.assert_allclose(r[name], c[name], rtol=1e-13, atol=1e-13)
