"""fp64 CPU oracle of the LaX variant of the low-rank decoder block.

TEST INFRASTRUCTURE ONLY (same rules as lowrank_oracle.py: nothing in the product path imports
this; it shares no code with the HIP path).

LaX (App. "LaX variant (residual low-rank)"): identity gate at rank r, and every bottleneck layer
adds the rank-r activation of the same projection in the previous decoder layer before its
up-projection:

    h_i = A_i x_i ,   y_i = B_i (h_i + h_{i-1}) .

In the notation used here A = W_down, B = W_up, h = z.  A block therefore takes the seven
h_{i-1} of the block below it ("h_prev", zeros for the first block) and hands its own seven h_i
to the block above.  Because h_i is used twice (by this block and by the next one), its gradient
is the sum of both uses: the backward of a block receives the next block's contribution
("dz_next", zeros for the last block) and returns its own contribution to the block below
("dh_prev").

Written as the plain definition: separate projections, two-pass RMSNorm, store-everything
backward; a matrix product is the only library primitive used as a step.

Pins (tests/test_oracle_lax.py): h_prev = 0 and dz_next = 0 reduce to the sigma = identity block of
lowrank_oracle.py; one layer equals the dense product x (B A)^T + h_prev B^T; central finite
differences for every gradient, including dh_prev and the dz_next term; a two-block stack
differentiated as a whole by finite differences agrees with the chained per-block backward.
Absolute values are "parity unpinned" by the paper (it prints no worked example).
"""
from __future__ import annotations

import numpy as np

from . import lowrank_oracle as base

F64 = np.float64
PROJ = base.PROJ


def zeros_h(T, d, f, r):
    """The seven rank-r tensors of a block, all zero: h_prev of the first block, dz_next of the last."""
    return {n: np.zeros((T, r), dtype=F64) for n in PROJ}


def lax_linear_fwd(x, w_down, w_up, h_prev):
    """x[T, d_in] -> (z[T, r] = x W_down^T, y[T, d_out] = (z + h_prev) W_up^T)."""
    x = np.asarray(x, dtype=F64)
    z = x @ np.asarray(w_down, dtype=F64).T
    y = (z + np.asarray(h_prev, dtype=F64)) @ np.asarray(w_up, dtype=F64).T
    return z, y


def lax_linear_bwd(x, w_down, w_up, h_prev, dy, dz_next):
    """Gradients of L = sum(y * dy) + sum(z * dz_next).  Returns (dx, dw_down, dw_up, dh_prev)."""
    x = np.asarray(x, dtype=F64)
    w_down = np.asarray(w_down, dtype=F64)
    w_up = np.asarray(w_up, dtype=F64)
    dy = np.asarray(dy, dtype=F64)
    z, _ = lax_linear_fwd(x, w_down, w_up, h_prev)
    a = z + np.asarray(h_prev, dtype=F64)
    dw_up = dy.T @ a
    da = dy @ w_up                      # gradient w.r.t. (z + h_prev): reaches both summands unchanged
    dz = da + np.asarray(dz_next, dtype=F64)
    dw_down = dz.T @ x
    dx = dz @ w_down
    return dx, dw_down, dw_up, da


def block_fwd(x, p, h_prev, B, S, H, hd, eps, causal=True, Hkv=None):
    """Returns (y, z, cache): z is the dict of this block's seven h_i (for the block above).
    Hkv: key / value heads of grouped-query attention (None: as many as query heads); the K and V
    up-projections then have Hkv * hd rows."""
    x = np.asarray(x, dtype=F64)
    Hkv = H if Hkv is None else Hkv
    c = {"x": x}
    z = {}
    c["xh1"], c["rms1"] = base.rmsnorm_fwd(x, p["gamma1"], eps)
    for n in ("q", "k", "v"):
        z[n], c[n] = lax_linear_fwd(c["xh1"], p["wd_" + n], p["wu_" + n], h_prev[n])
    c["o"], c["lse"] = base._attn_fwd(c["q"], c["k"], c["v"], B, S, H, Hkv, hd, causal)
    z["o"], c["attn_out"] = lax_linear_fwd(c["o"], p["wd_o"], p["wu_o"], h_prev["o"])
    c["h1"] = x + c["attn_out"]
    c["xh2"], c["rms2"] = base.rmsnorm_fwd(c["h1"], p["gamma2"], eps)
    for n in ("g", "u"):
        z[n], c[n] = lax_linear_fwd(c["xh2"], p["wd_" + n], p["wu_" + n], h_prev[n])
    c["m"] = base.silu(c["g"]) * c["u"]
    z["d"], c["mlp_out"] = lax_linear_fwd(c["m"], p["wd_d"], p["wu_d"], h_prev["d"])
    y = c["h1"] + c["mlp_out"]
    return y, z, c


def block_bwd(x, p, h_prev, dy, dz_next, B, S, H, hd, eps, causal=True, Hkv=None):
    """Gradients of L = sum(y * dy) + sum_n sum(z_n * dz_next_n).
    Returns (dx, grads, dh_prev) with dh_prev the dict of gradients w.r.t. the seven h_prev."""
    dy = np.asarray(dy, dtype=F64)
    Hkv = H if Hkv is None else Hkv
    _, _, c = block_fwd(x, p, h_prev, B, S, H, hd, eps, causal, Hkv)
    g, dh = {}, {}
    dm, g["wd_d"], g["wu_d"], dh["d"] = lax_linear_bwd(c["m"], p["wd_d"], p["wu_d"], h_prev["d"], dy, dz_next["d"])
    dh1 = dy.copy()
    dg = dm * c["u"] * base.silu_prime(c["g"])
    du = dm * base.silu(c["g"])
    dxh2 = np.zeros_like(c["xh2"])
    for n, dn in (("g", dg), ("u", du)):
        dxi, g["wd_" + n], g["wu_" + n], dh[n] = lax_linear_bwd(c["xh2"], p["wd_" + n], p["wu_" + n], h_prev[n], dn,
                                                               dz_next[n])
        dxh2 += dxi
    dh1_n, g["gamma2"] = base.rmsnorm_bwd(c["h1"], p["gamma2"], eps, dxh2)
    dh1 += dh1_n
    do, g["wd_o"], g["wu_o"], dh["o"] = lax_linear_bwd(c["o"], p["wd_o"], p["wu_o"], h_prev["o"], dh1, dz_next["o"])
    dq, dk, dv = base._attn_bwd(c["q"], c["k"], c["v"], do, B, S, H, Hkv, hd, causal)
    dxh1 = np.zeros_like(c["xh1"])
    for n, dn in (("q", dq), ("k", dk), ("v", dv)):
        dxi, g["wd_" + n], g["wu_" + n], dh[n] = lax_linear_bwd(c["xh1"], p["wd_" + n], p["wu_" + n], h_prev[n], dn,
                                                               dz_next[n])
        dxh1 += dxi
    dx_n, g["gamma1"] = base.rmsnorm_bwd(c["x"], p["gamma1"], eps, dxh1)
    dx = dh1 + dx_n
    return dx, g, dh
