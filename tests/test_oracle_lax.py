"""Pins for oracle/lax_oracle.py (the LaX variant, App. "LaX variant (residual low-rank)"): nothing
here re-uses the oracle's own formulas.  Reductions to the plain block, a dense-product closed form,
central finite differences of a scalar loss for every gradient (including the two inter-layer
terms), and a two-block stack differentiated as a whole."""
import numpy as np

from oracle import lax_oracle as lax
from oracle import lowrank_oracle as orc

RNG = np.random.default_rng(2468)
EPS = 1e-5
B, S, H, HD, F, R = 1, 5, 1, 4, 6, 3
D = H * HD
T = B * S


def _params(rng):
    dims = {"q": (D, D), "k": (D, D), "v": (D, D), "o": (D, D), "g": (D, F), "u": (D, F), "d": (F, D)}
    p = {}
    for n, (d_in, d_out) in dims.items():
        p["wd_" + n] = rng.normal(size=(R, d_in)) * d_in ** -0.5
        p["wu_" + n] = rng.normal(size=(d_out, R)) * R ** -0.5
    p["gamma1"] = 1.0 + 0.1 * rng.normal(size=(D,))
    p["gamma2"] = 1.0 + 0.1 * rng.normal(size=(D,))
    return p


def _hdict(rng, scale=1.0):
    return {n: scale * rng.normal(size=(T, R)) for n in lax.PROJ}


def _fd_grad(fun, arr, eps=1e-6):
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


def test_zero_residual_is_the_identity_sigma_block():
    """h_prev = 0 and dz_next = 0: the block of lowrank_oracle.py with sigma = identity (the SVD variant)."""
    p = _params(RNG)
    x, dy = RNG.normal(size=(T, D)), RNG.normal(size=(T, D))
    zero = lax.zeros_h(T, D, F, R)
    y, z, _ = lax.block_fwd(x, p, zero, B, S, H, HD, EPS)
    y0, c0 = orc.block_fwd(x, p, B, S, H, HD, EPS, act=orc.ACT_IDENTITY)
    assert _relerr(y, y0) < 1e-13
    for n in lax.PROJ:
        assert _relerr(z[n], c0["z_" + n]) < 1e-13
    dx, g, dh = lax.block_bwd(x, p, zero, dy, zero, B, S, H, HD, EPS)
    dx0, g0 = orc.block_bwd(x, p, dy, B, S, H, HD, EPS, act=orc.ACT_IDENTITY)
    assert _relerr(dx, dx0) < 1e-12
    for k in g0:
        assert _relerr(g[k], g0[k]) < 1e-12, k


def test_one_layer_is_a_dense_product_plus_the_residual_term():
    """y = x (B A)^T + h_prev B^T, written with explicit scalar loops."""
    x = RNG.normal(size=(4, 5))
    a_, b_ = RNG.normal(size=(3, 5)), RNG.normal(size=(6, 3))
    h = RNG.normal(size=(4, 3))
    z, y = lax.lax_linear_fwd(x, a_, b_, h)
    want = np.zeros((4, 6))
    for t in range(4):
        for o in range(6):
            acc = 0.0
            for i in range(3):
                hz = h[t, i]
                for j in range(5):
                    hz += a_[i, j] * x[t, j]
                acc += b_[o, i] * hz
            want[t, o] = acc
    assert _relerr(y, want) < 1e-13
    assert _relerr(z, x @ a_.T) < 1e-13


def test_block_gradients_by_finite_differences():
    """L = sum(y * dy) + sum_n sum(z_n * dz_next_n): every gradient the backward returns."""
    rng = np.random.default_rng(77)
    p = _params(rng)
    x, dy = rng.normal(size=(T, D)), rng.normal(size=(T, D))
    h_prev, dz_next = _hdict(rng, 0.5), _hdict(rng)

    def loss():
        y, z, _ = lax.block_fwd(x, p, h_prev, B, S, H, HD, EPS)
        return float(np.sum(y * dy) + sum(np.sum(z[n] * dz_next[n]) for n in lax.PROJ))

    dx, g, dh = lax.block_bwd(x, p, h_prev, dy, dz_next, B, S, H, HD, EPS)
    assert _relerr(dx, _fd_grad(loss, x)) < 1e-6
    for k in g:
        assert _relerr(g[k], _fd_grad(loss, p[k])) < 1e-6, k
    for n in lax.PROJ:
        assert _relerr(dh[n], _fd_grad(loss, h_prev[n])) < 1e-6, n
    # the dz_next term matters: dropping it changes dx far beyond the tolerance
    dx_wo, _, _ = lax.block_bwd(x, p, h_prev, dy, lax.zeros_h(T, D, F, R), B, S, H, HD, EPS)
    assert _relerr(dx_wo, dx) > 1e-2


def test_two_block_stack_chains_through_dh_prev_and_dz_next():
    """Two blocks: the upper one takes the lower one's z as h_prev.  Backward of the stack = upper block
    (dz_next = 0), then lower block with dy = upper dx and dz_next = upper dh_prev.  Checked against
    finite differences of the whole stack w.r.t. the lower block's input and parameters."""
    rng = np.random.default_rng(99)
    p1, p2 = _params(rng), _params(rng)
    x, dy = rng.normal(size=(T, D)), rng.normal(size=(T, D))
    zero = lax.zeros_h(T, D, F, R)

    def stack():
        y1, z1, _ = lax.block_fwd(x, p1, zero, B, S, H, HD, EPS)
        y2, _, _ = lax.block_fwd(y1, p2, z1, B, S, H, HD, EPS)
        return y1, z1, y2

    def loss():
        return float(np.sum(stack()[2] * dy))

    y1, z1, _ = stack()
    dx2, g2, dh2 = lax.block_bwd(y1, p2, z1, dy, zero, B, S, H, HD, EPS)
    dx1, g1, _ = lax.block_bwd(x, p1, zero, dx2, dh2, B, S, H, HD, EPS)
    assert _relerr(dx1, _fd_grad(loss, x)) < 1e-6
    for k in ("wd_q", "wu_v", "wd_o", "wd_g", "wu_u", "wd_d", "gamma1", "gamma2"):
        assert _relerr(g1[k], _fd_grad(loss, p1[k])) < 1e-6, k
    for k in ("wu_q", "wd_d"):
        assert _relerr(g2[k], _fd_grad(loss, p2[k])) < 1e-6, k


def test_lax_block_with_grouped_kv_heads_by_finite_differences():
    """Fewer key / value heads than query heads (the K and V up-projections narrower): every gradient the
    backward returns, including the inter-layer ones, against central differences; and with as many
    key / value heads as query heads the option changes nothing."""
    rng = np.random.default_rng(123)
    Bq, Sq, Hq, Hkv, hd, Fq, Rq = 1, 4, 4, 2, 2, 5, 3
    Dq, Dkv, Tq = Hq * hd, Hkv * hd, Bq * Sq
    dims = {"q": (Dq, Dq), "k": (Dq, Dkv), "v": (Dq, Dkv), "o": (Dq, Dq), "g": (Dq, Fq), "u": (Dq, Fq), "d": (Fq, Dq)}
    p = {}
    for n, (d_in, d_out) in dims.items():
        p["wd_" + n] = rng.normal(size=(Rq, d_in)) * d_in ** -0.5
        p["wu_" + n] = rng.normal(size=(d_out, Rq)) * Rq ** -0.5
    p["gamma1"] = 1.0 + 0.1 * rng.normal(size=(Dq,))
    p["gamma2"] = 1.0 + 0.1 * rng.normal(size=(Dq,))
    x, dy = rng.normal(size=(Tq, Dq)), rng.normal(size=(Tq, Dq))
    h_prev = {n: 0.5 * rng.normal(size=(Tq, Rq)) for n in lax.PROJ}
    dz_next = {n: rng.normal(size=(Tq, Rq)) for n in lax.PROJ}

    def loss():
        y, z, _ = lax.block_fwd(x, p, h_prev, Bq, Sq, Hq, hd, EPS, Hkv=Hkv)
        return float(np.sum(y * dy) + sum(np.sum(z[n] * dz_next[n]) for n in lax.PROJ))

    dx, g, dh = lax.block_bwd(x, p, h_prev, dy, dz_next, Bq, Sq, Hq, hd, EPS, Hkv=Hkv)
    assert g["wu_k"].shape == (Dkv, Rq)
    assert _relerr(dx, _fd_grad(loss, x)) < 1e-6
    for k in ("wu_k", "wu_v", "wd_k", "wu_q", "wd_o", "gamma1"):
        assert _relerr(g[k], _fd_grad(loss, p[k])) < 1e-6, k
    for n in ("k", "v", "q", "d"):
        assert _relerr(dh[n], _fd_grad(loss, h_prev[n])) < 1e-6, n
    # Hkv = H is the plain LaX block
    p2 = _params(RNG)
    x2, dy2 = RNG.normal(size=(T, D)), RNG.normal(size=(T, D))
    hp2, dz2 = _hdict(RNG, 0.5), _hdict(RNG)
    a = lax.block_bwd(x2, p2, hp2, dy2, dz2, B, S, H, HD, EPS)
    b = lax.block_bwd(x2, p2, hp2, dy2, dz2, B, S, H, HD, EPS, Hkv=H)
    assert np.array_equal(a[0], b[0])
