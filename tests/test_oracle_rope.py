"""Pins for the rotary-embedding step of the oracle (rope_tables, rope_apply, the rope option of
block_fwd / block_bwd): properties that the rotation must have, scalar loops, finite differences."""
import math

import numpy as np

from oracle import lowrank_oracle as orc

RNG = np.random.default_rng(1357)


def _relerr(a, b):
    return np.max(np.abs(a - b)) / (np.sqrt(np.mean(b * b)) + 1e-300)


def test_rope_matches_scalar_loops_and_the_usual_angles():
    B, S, H, hd = 2, 5, 2, 8
    x = RNG.normal(size=(B * S, H * hd))
    cos, sin = orc.rope_tables(S, hd, base=100.0)
    got = orc.rope_apply(x, cos, sin, B, S, H, hd)
    want = np.zeros_like(x)
    for t in range(B * S):
        p = t % S
        for h in range(H):
            for i in range(hd // 2):
                th = p * 100.0 ** (-2.0 * i / hd)
                a, b = x[t, h * hd + i], x[t, h * hd + i + hd // 2]
                want[t, h * hd + i] = a * math.cos(th) - b * math.sin(th)
                want[t, h * hd + i + hd // 2] = b * math.cos(th) + a * math.sin(th)
    assert _relerr(got, want) < 1e-13


def test_rope_is_an_orthogonal_map_with_the_stated_inverse():
    B, S, H, hd = 1, 7, 3, 16
    x = RNG.normal(size=(B * S, H * hd))
    cos, sin = orc.rope_tables(S, hd)
    y = orc.rope_apply(x, cos, sin, B, S, H, hd)
    # lengths of every head vector are kept, position 0 is left alone, inverse undoes it
    nx = np.linalg.norm(x.reshape(B * S, H, hd), axis=-1)
    ny = np.linalg.norm(y.reshape(B * S, H, hd), axis=-1)
    assert np.max(np.abs(nx - ny)) < 1e-12
    assert np.max(np.abs(y[0] - x[0])) == 0.0
    assert _relerr(orc.rope_apply(y, cos, sin, B, S, H, hd, inverse=True), x) < 1e-13
    # <R x, z> = <x, R^T z>: the inverse is the transpose (what the backward relies on)
    z = RNG.normal(size=x.shape)
    lhs = np.sum(y * z)
    rhs = np.sum(x * orc.rope_apply(z, cos, sin, B, S, H, hd, inverse=True))
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)


def test_rotated_scores_depend_on_the_position_difference_only():
    S, hd = 12, 8
    cos, sin = orc.rope_tables(S, hd)
    q, k = RNG.normal(size=(hd,)), RNG.normal(size=(hd,))
    Q = orc.rope_apply(np.tile(q, (S, 1)), cos, sin, 1, S, 1, hd)
    K = orc.rope_apply(np.tile(k, (S, 1)), cos, sin, 1, S, 1, hd)
    sc = Q @ K.T                                 # sc[m, n] = <R_m q, R_n k>
    for m in range(3, S):
        for n in range(0, S - 3):
            if m - n >= 0 and m + 2 < S and n + 2 < S:
                assert abs(sc[m, n] - sc[m + 2, n + 2]) < 1e-12
    assert abs(sc[5, 2] - sc[5, 3]) > 1e-3       # and it does depend on it


def test_block_with_rope_gradients_by_finite_differences():
    B, S, H, hd, f, r = 1, 5, 1, 4, 6, 3
    d = H * hd
    rng = np.random.default_rng(4242)
    dims = {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d), "g": (d, f), "u": (d, f), "d": (f, d)}
    p = {}
    for n, (d_in, d_out) in dims.items():
        p["wd_" + n] = rng.normal(size=(r, d_in)) * d_in ** -0.5
        p["wu_" + n] = rng.normal(size=(d_out, r)) * r ** -0.5
    p["gamma1"] = 1.0 + 0.1 * rng.normal(size=(d,))
    p["gamma2"] = 1.0 + 0.1 * rng.normal(size=(d,))
    x, dy = rng.normal(size=(B * S, d)), rng.normal(size=(B * S, d))
    rope = orc.rope_tables(S, hd, base=50.0)

    def loss():
        return float(np.sum(orc.block_fwd(x, p, B, S, H, hd, 1e-5, rope=rope)[0] * dy))

    def fd(arr, eps=1e-6):
        g = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            fp = loss()
            arr[idx] = old - eps
            fm = loss()
            arr[idx] = old
            g[idx] = (fp - fm) / (2 * eps)
        return g

    dx, g = orc.block_bwd(x, p, dy, B, S, H, hd, 1e-5, rope=rope)
    assert _relerr(dx, fd(x)) < 1e-6
    for k in ("wd_q", "wu_q", "wd_k", "wu_k", "wu_v", "wd_o", "gamma1"):
        assert _relerr(g[k], fd(p[k])) < 1e-6, k
    # the option changes the block: without it y differs far beyond any tolerance
    y0 = orc.block_fwd(x, p, B, S, H, hd, 1e-5)[0]
    y1 = orc.block_fwd(x, p, B, S, H, hd, 1e-5, rope=rope)[0]
    assert _relerr(y1, y0) > 1e-3
