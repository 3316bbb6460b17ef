"""fp64 CPU oracle of the low-rank bottleneck decoder block (forward and backward).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it exists so
that tests, the smoke check and the CPU-baseline leg of the benchmark have an independent,
slow, obviously-correct definition to compare the HIP kernels with.  It shares no code with
the HIP path and never imports it.

Everything here is the *plain definition* written out in numpy float64: separate (ungrouped)
projections, two-pass RMSNorm, attention with the full score matrix, a backward pass that
stores every activation.  The method of the paper reaches these results exactly (up to the
order of floating-point sums): Online RMSNorm is an exact re-ordering (Sec. 4.2, Eq. 5),
layer grouping is concatenation / batching of independent GEMMs (Sec. 4.3, App. "Linear
Grouping Details"), and rank-r checkpointing only changes what is stored (Sec. 4.4).  A
matrix product (`@`) is the only library primitive used as a step.

Notation follows the paper's problem statement (Sec. 2, "Low-Rank Matrix Factorization" and
"Low-Rank Activation via Auto-Encoder"): a linear map W[d_out, d_in] is replaced by
W_up[d_out, r] . sigma(W_down[r, d_in] . x).  Activations are token-major, x[T, d].

Pins (tests/test_oracle_*.py): brute-force scalar loops on tiny shapes, central finite
differences for every gradient, sigma = identity == dense product (App. "SVD baseline"),
Alg. 1 over k simulated shards == two-pass RMSNorm (Eq. 5), softmax/causality invariants,
parameter count 11dr + 3 d_ff r (App. "Communication volume analysis").
Absolute values of y and of the gradients are "parity unpinned" by the paper: it prints no
worked numeric example, so they are pinned only by those invariants.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64

ACT_IDENTITY = 0
ACT_SILU = 1


# --------------------------------------------------------------------------------------------
# sigma at rank r  (Sec. 2: B sigma(A x); the SVD variant of App. "Low-rank Training
# Algorithm" has no nonlinearity.)  Reading: sigma = SiLU elementwise on the rank-r vector.
# --------------------------------------------------------------------------------------------
def logistic(z):
    z = np.asarray(z, dtype=F64)
    return 1.0 / (1.0 + np.exp(-z))


def silu(z):
    z = np.asarray(z, dtype=F64)
    return z * logistic(z)


def silu_prime(z):
    s = logistic(z)
    return s * (1.0 + z * (1.0 - s))


def act_fwd(z, act):
    if act == ACT_IDENTITY:
        return np.asarray(z, dtype=F64).copy()
    if act == ACT_SILU:
        return silu(z)
    raise ValueError("unknown activation")


def act_prime(z, act):
    if act == ACT_IDENTITY:
        return np.ones_like(np.asarray(z, dtype=F64))
    if act == ACT_SILU:
        return silu_prime(z)
    raise ValueError("unknown activation")


# --------------------------------------------------------------------------------------------
# RMSNorm, Eq. 4: per token, reduce over the feature axis; eps inside the square root after
# the mean; gamma is per feature.
# --------------------------------------------------------------------------------------------
def rms_stat(x):
    """S[t] = sum_j x[t, j]^2  (Alg. 1 line 1 with one shard)."""
    x = np.asarray(x, dtype=F64)
    return np.sum(x * x, axis=1)


def rmsnorm_fwd(x, gamma, eps):
    x = np.asarray(x, dtype=F64)
    gamma = np.asarray(gamma, dtype=F64)
    d = x.shape[1]
    rms = np.sqrt(rms_stat(x) / d + eps)           # [T]
    xhat = x * gamma[None, :] / rms[:, None]
    return xhat, rms


def rmsnorm_bwd(x, gamma, eps, dxhat):
    """Reverse mode of Eq. 4 (the paper prints no backward; this is its derivative)."""
    x = np.asarray(x, dtype=F64)
    gamma = np.asarray(gamma, dtype=F64)
    dxhat = np.asarray(dxhat, dtype=F64)
    d = x.shape[1]
    rms = np.sqrt(rms_stat(x) / d + eps)
    n = x / rms[:, None]
    dn = dxhat * gamma[None, :]
    c = np.sum(dn * n, axis=1) / d
    dx = (dn - n * c[:, None]) / rms[:, None]
    dgamma = np.sum(dxhat * n, axis=0)
    return dx, dgamma


def online_rmsnorm_sharded(x, gamma, w, k, eps):
    """The sharded form of RMSNorm + row-split projection (Sec. 4.2, Alg. 1 / Eq. 5) over k simulated
    tensor-parallel ranks, as a check of its equivalence with the unsharded two-pass result.

    x[T, d], gamma[d], w[d, r]; rank i owns the feature slice i*d/k .. (i+1)*d/k of x and gamma and the
    matching rows of w.  Each rank normalises its slice by its own local rms, multiplies by its weight
    rows and undoes the local scale on the product; the partial products and the local sums of squares
    are then added over the ranks (the all-reduce), and the global rms computed from the summed
    statistic rescales the sum.  Returns Y[T, r].
    """
    x = np.asarray(x, dtype=F64)
    gamma = np.asarray(gamma, dtype=F64)
    w = np.asarray(w, dtype=F64)
    T, d = x.shape
    assert d % k == 0
    dl = d // k
    xs = x.reshape(T, k, dl)                                   # [token, rank, local feature]
    gs = gamma.reshape(k, dl)
    ws = w.reshape(k, dl, w.shape[1])
    s_local = np.einsum("tkj,tkj->tk", xs, xs)                 # per rank: sum of squares of its slice
    rms_local = np.sqrt(s_local / dl + eps)
    xn = xs / rms_local[:, :, None] * gs[None, :, :]           # locally normalised, scaled by gamma
    part = np.einsum("tkj,kjr->tkr", xn, ws) * rms_local[:, :, None]   # local product, local scale undone
    rms_global = np.sqrt(s_local.sum(axis=1) / d + eps)        # from the statistic summed over ranks
    return part.sum(axis=1) / rms_global[:, None]


# --------------------------------------------------------------------------------------------
# One bottleneck linear layer  y = W_up sigma(W_down x)
# --------------------------------------------------------------------------------------------
def lr_linear_fwd(x, w_down, w_up, act=ACT_SILU):
    """x[T, d_in], w_down[r, d_in], w_up[d_out, r] -> (z[T, r], a[T, r], y[T, d_out])."""
    x = np.asarray(x, dtype=F64)
    w_down = np.asarray(w_down, dtype=F64)
    w_up = np.asarray(w_up, dtype=F64)
    z = x @ w_down.T
    a = act_fwd(z, act)
    y = a @ w_up.T
    return z, a, y


def lr_linear_bwd(x, w_down, w_up, dy, act=ACT_SILU):
    """Gradients of L = sum(y * dy): returns (dx, dw_down, dw_up)."""
    x = np.asarray(x, dtype=F64)
    w_down = np.asarray(w_down, dtype=F64)
    w_up = np.asarray(w_up, dtype=F64)
    dy = np.asarray(dy, dtype=F64)
    z, a, _ = lr_linear_fwd(x, w_down, w_up, act)
    dw_up = dy.T @ a
    da = dy @ w_up
    dz = da * act_prime(z, act)
    dw_down = dz.T @ x
    dx = dz @ w_down
    return dx, dw_down, dw_up


# --------------------------------------------------------------------------------------------
# G projections that share one (optionally RMS-normalised) input: Q/K/V or gate/up.
# Written as G separate layers on purpose: the grouped GEMM of Sec. 4.3 must equal this.
# --------------------------------------------------------------------------------------------
def lr_group_fwd(x, gamma, eps, w_down_list, w_up_list, act=ACT_SILU, norm=True):
    x = np.asarray(x, dtype=F64)
    if norm:
        xin, _ = rmsnorm_fwd(x, gamma, eps)
    else:
        xin = x
    zs, ys = [], []
    for wd, wu in zip(w_down_list, w_up_list):
        z, _, y = lr_linear_fwd(xin, wd, wu, act)
        zs.append(z)
        ys.append(y)
    return zs, ys, rms_stat(x)


def lr_group_bwd(x, gamma, eps, w_down_list, w_up_list, dy_list, act=ACT_SILU, norm=True):
    """Returns (dx, dgamma or None, [dw_down_g], [dw_up_g]); dx is w.r.t. the raw x."""
    x = np.asarray(x, dtype=F64)
    if norm:
        xin, _ = rmsnorm_fwd(x, gamma, eps)
    else:
        xin = x
    dxin = np.zeros_like(xin)
    dwd, dwu = [], []
    for wd, wu, dy in zip(w_down_list, w_up_list, dy_list):
        dxi, dwdi, dwui = lr_linear_bwd(xin, wd, wu, dy, act)
        dxin += dxi
        dwd.append(dwdi)
        dwu.append(dwui)
    if norm:
        dx, dgamma = rmsnorm_bwd(x, gamma, eps, dxin)
    else:
        dx, dgamma = dxin, None
    return dx, dgamma, dwd, dwu


# --------------------------------------------------------------------------------------------
# Causal multi-head self-attention (the "sharded-safe" SDPA between the chunks, Sec. 4.2).
# q, k, v are [T, H*hd] with T = B*S, batch-major; head h owns columns h*hd .. (h+1)*hd.
# --------------------------------------------------------------------------------------------
def attention_fwd(q, k, v, B, S, H, hd, causal=True, return_probs=False):
    q = np.asarray(q, dtype=F64).reshape(B, S, H, hd)
    k = np.asarray(k, dtype=F64).reshape(B, S, H, hd)
    v = np.asarray(v, dtype=F64).reshape(B, S, H, hd)
    o = np.zeros((B, S, H, hd), dtype=F64)
    lse = np.zeros((B, H, S), dtype=F64)
    probs = np.zeros((B, H, S, S), dtype=F64) if return_probs else None
    scale = 1.0 / np.sqrt(hd)
    mask = np.tril(np.ones((S, S), dtype=bool)) if causal else np.ones((S, S), dtype=bool)
    for b in range(B):
        for h in range(H):
            s = (q[b, :, h, :] @ k[b, :, h, :].T) * scale        # [S_q, S_k]
            s = np.where(mask, s, -np.inf)
            m = np.max(s, axis=1, keepdims=True)
            e = np.exp(s - m)
            den = np.sum(e, axis=1, keepdims=True)
            p = e / den
            o[b, :, h, :] = p @ v[b, :, h, :]
            lse[b, h, :] = (m + np.log(den))[:, 0]
            if return_probs:
                probs[b, h] = p
    o = o.reshape(B * S, H * hd)
    if return_probs:
        return o, lse, probs
    return o, lse


def attention_bwd(q, k, v, do, B, S, H, hd, causal=True):
    q4 = np.asarray(q, dtype=F64).reshape(B, S, H, hd)
    k4 = np.asarray(k, dtype=F64).reshape(B, S, H, hd)
    v4 = np.asarray(v, dtype=F64).reshape(B, S, H, hd)
    do4 = np.asarray(do, dtype=F64).reshape(B, S, H, hd)
    _, _, probs = attention_fwd(q, k, v, B, S, H, hd, causal, return_probs=True)
    dq = np.zeros_like(q4)
    dk = np.zeros_like(k4)
    dv = np.zeros_like(v4)
    scale = 1.0 / np.sqrt(hd)
    for b in range(B):
        for h in range(H):
            p = probs[b, h]                                   # [S_q, S_k]
            dv[b, :, h, :] = p.T @ do4[b, :, h, :]
            dp = do4[b, :, h, :] @ v4[b, :, h, :].T
            ds = p * (dp - np.sum(dp * p, axis=1, keepdims=True))
            dq[b, :, h, :] = (ds @ k4[b, :, h, :]) * scale
            dk[b, :, h, :] = (ds.T @ q4[b, :, h, :]) * scale
    T = B * S
    return dq.reshape(T, H * hd), dk.reshape(T, H * hd), dv.reshape(T, H * hd)


# --------------------------------------------------------------------------------------------
# Rotary position embedding, an optional step of the block (LLaMA-style models, Sec. 5.2; the paper
# does not describe it, the block applies it only on request).  Convention: the "rotate half" form.
# Inside every head the pair (v[i], v[i + hd/2]), i < hd/2, of the token at position p of its sequence
# is turned by the angle theta[p, i]; the caller supplies cos(theta) and sin(theta) as [S, hd/2]
# tables.  inverse=True turns by -theta: the transpose of the rotation, which is what the backward
# applies to the gradients of the rotated q and k.
# --------------------------------------------------------------------------------------------
def rope_tables(S, hd, base=10000.0):
    """cos, sin [S, hd/2] of theta[p, i] = p * base^(-2 i / hd)  (the usual choice of angles)."""
    i = np.arange(hd // 2, dtype=F64)
    theta = np.arange(S, dtype=F64)[:, None] * base ** (-2.0 * i / hd)[None, :]
    return np.cos(theta), np.sin(theta)


def rope_apply(x, cos, sin, B, S, H, hd, inverse=False):
    """x[T, H*hd] -> rotated copy; position of row t is t mod S."""
    x4 = np.asarray(x, dtype=F64).reshape(B, S, H, hd)
    c = np.asarray(cos, dtype=F64)[None, :, None, :]
    sn = np.asarray(sin, dtype=F64)[None, :, None, :]
    if inverse:
        sn = -sn
    lo, hi = x4[..., : hd // 2], x4[..., hd // 2:]
    out = np.concatenate([lo * c - hi * sn, hi * c + lo * sn], axis=-1)
    return out.reshape(B * S, H * hd)


# --------------------------------------------------------------------------------------------
# The decoder block.  Seven projections, each factored once at rank r (App. "Communication
# volume analysis": 4 attention + 3 MLP maps, 11dr + 3 d_ff r parameters), pre-norm residual
# layout of LLaMA-2 (Sec. 5.2), SwiGLU gate at width d_ff kept in addition to sigma at rank r.
# params: dict with gamma1, wd_q, wu_q, wd_k, wu_k, wd_v, wu_v, wd_o, wu_o,
#                   gamma2, wd_g, wu_g, wd_u, wu_u, wd_d, wu_d
# --------------------------------------------------------------------------------------------
PROJ = ("q", "k", "v", "o", "g", "u", "d")


def block_param_count(d, f, r):
    """Parameters of the seven factored projections of one block."""
    return 11 * d * r + 3 * f * r


def _attn_fwd(q, k, v, B, S, H, Hkv, hd, causal):
    if Hkv == H:
        return attention_fwd(q, k, v, B, S, H, hd, causal)
    from . import gqa_oracle          # grouped-query attention (section "Discussion and Future Work")
    return gqa_oracle.attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd, causal)


def _attn_bwd(q, k, v, do, B, S, H, Hkv, hd, causal):
    if Hkv == H:
        return attention_bwd(q, k, v, do, B, S, H, hd, causal)
    from . import gqa_oracle
    return gqa_oracle.attention_gqa_bwd(q, k, v, do, B, S, H, Hkv, hd, causal)


def block_fwd(x, p, B, S, H, hd, eps, act=ACT_SILU, causal=True, rope=None, Hkv=None):
    """Returns (y, cache) where cache holds every intermediate (store-everything reference).
    rope: None, or (cos, sin) tables [S, hd/2]: q and k are rotated before the attention.
    Hkv: None (= H), or the number of key / value heads of grouped-query attention: the K and V
    up-projections then have Hkv * hd rows, nothing else changes."""
    Hkv = H if Hkv is None else Hkv
    x = np.asarray(x, dtype=F64)
    c = {"x": x}
    c["xh1"], c["rms1"] = rmsnorm_fwd(x, p["gamma1"], eps)
    for n in ("q", "k", "v"):
        c["z_" + n], c["a_" + n], c[n] = lr_linear_fwd(c["xh1"], p["wd_" + n], p["wu_" + n], act)
    c["qr"], c["kr"] = c["q"], c["k"]
    if rope is not None:
        c["qr"] = rope_apply(c["q"], rope[0], rope[1], B, S, H, hd)
        c["kr"] = rope_apply(c["k"], rope[0], rope[1], B, S, Hkv, hd)
    c["o"], c["lse"] = _attn_fwd(c["qr"], c["kr"], c["v"], B, S, H, Hkv, hd, causal)
    c["z_o"], c["a_o"], c["attn_out"] = lr_linear_fwd(c["o"], p["wd_o"], p["wu_o"], act)
    c["h1"] = x + c["attn_out"]
    c["xh2"], c["rms2"] = rmsnorm_fwd(c["h1"], p["gamma2"], eps)
    for n in ("g", "u"):
        c["z_" + n], c["a_" + n], c[n] = lr_linear_fwd(c["xh2"], p["wd_" + n], p["wu_" + n], act)
    c["m"] = silu(c["g"]) * c["u"]
    c["z_d"], c["a_d"], c["mlp_out"] = lr_linear_fwd(c["m"], p["wd_d"], p["wu_d"], act)
    y = c["h1"] + c["mlp_out"]
    return y, c


def block_bwd(x, p, dy, B, S, H, hd, eps, act=ACT_SILU, causal=True, rope=None, Hkv=None):
    """Gradients of L = sum(y * dy) w.r.t. x and every parameter.  Returns (dx, grads)."""
    dy = np.asarray(dy, dtype=F64)
    Hkv = H if Hkv is None else Hkv
    _, c = block_fwd(x, p, B, S, H, hd, eps, act, causal, rope, Hkv)
    g = {}
    # y = h1 + lr(m)
    dm, g["wd_d"], g["wu_d"] = lr_linear_bwd(c["m"], p["wd_d"], p["wu_d"], dy, act)
    dh1 = dy.copy()
    # m = SiLU(g) * u
    dg = dm * c["u"] * silu_prime(c["g"])
    du = dm * silu(c["g"])
    dxh2 = np.zeros_like(c["xh2"])
    for n, dn in (("g", dg), ("u", du)):
        dxi, g["wd_" + n], g["wu_" + n] = lr_linear_bwd(c["xh2"], p["wd_" + n], p["wu_" + n], dn, act)
        dxh2 += dxi
    dh1_n, g["gamma2"] = rmsnorm_bwd(c["h1"], p["gamma2"], eps, dxh2)
    dh1 += dh1_n
    # h1 = x + lr(o)
    do, g["wd_o"], g["wu_o"] = lr_linear_bwd(c["o"], p["wd_o"], p["wu_o"], dh1, act)
    dq, dk, dv = _attn_bwd(c["qr"], c["kr"], c["v"], do, B, S, H, Hkv, hd, causal)
    if rope is not None:                 # back through the rotations: their transposes
        dq = rope_apply(dq, rope[0], rope[1], B, S, H, hd, inverse=True)
        dk = rope_apply(dk, rope[0], rope[1], B, S, Hkv, hd, inverse=True)
    dxh1 = np.zeros_like(c["xh1"])
    for n, dn in (("q", dq), ("k", dk), ("v", dv)):
        dxi, g["wd_" + n], g["wu_" + n] = lr_linear_bwd(c["xh1"], p["wd_" + n], p["wu_" + n], dn, act)
        dxh1 += dxi
    dx_n, g["gamma1"] = rmsnorm_bwd(c["x"], p["gamma1"], eps, dxh1)
    dx = dh1 + dx_n
    return dx, g


def reforward_from_checkpoints(x, p, ckpt, B, S, H, hd, act=ACT_SILU, causal=True):
    """Re-forward that may read only x and the rank-r pre-activations z_* (Sec. 4.4): every
    d-wide or d_ff-wide activation the backward needs is rebuilt from them.  Used to pin that
    the rank-r checkpoint set is sufficient and that recomputed activations equal stored ones."""
    x = np.asarray(x, dtype=F64)
    r = {}
    for n in ("q", "k", "v"):
        r[n] = act_fwd(ckpt["z_" + n], act) @ np.asarray(p["wu_" + n], dtype=F64).T
    r["o"], _ = attention_fwd(r["q"], r["k"], r["v"], B, S, H, hd, causal)
    r["h1"] = x + act_fwd(ckpt["z_o"], act) @ np.asarray(p["wu_o"], dtype=F64).T
    for n in ("g", "u"):
        r[n] = act_fwd(ckpt["z_" + n], act) @ np.asarray(p["wu_" + n], dtype=F64).T
    r["m"] = silu(r["g"]) * r["u"]
    return r
