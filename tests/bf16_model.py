"""Error-budget model of the bf16 pipeline: what bf16 storage alone costs, tensor by tensor.

TEST INFRASTRUCTURE ONLY (it lives beside the tests, imports neither the HIP path nor the oracle).

The GPU path computes in fp32 and keeps its tensors in bf16: every tensor that a later GEMM consumes
(the rank-r activations, q / k / v, the probabilities, o, h1, g, u, m and the matching gradients) is
rounded once when it is stored.  Those roundings are part of the method's arithmetic type ("pure
bf16", App. "Low-rank Training Algorithm"), not of a kernel's quality, and their effect on an output
depends on the length of the chain in front of it and, for the max-norm metric, on the number of
elements the maximum runs over.  This module computes that effect exactly: the same data flow as the
GPU design (norm scale folded into the weight, row scale after the product, statistics at rank r,
recompute from the rank-r checkpoints), in float64, with a round-to-nearest-even to bf16 at every
place where the design stores bf16, and nowhere else.  Accumulations, statistics, softmax and the
epilogue arithmetic stay exact (the GPU does them in fp32, whose error is four orders below).

Use:
  * `rnd=identity` turns every rounding off; the model must then reproduce the oracle to fp64
    round-off (tests/test_bf16_model.py).  That pins the model's algebra (and, through it, the
    algebra of the GPU design) against the plain definition.
  * with the default rounding, `max|model - oracle| / RMS(oracle)` of a tensor is the error an ideal
    bf16 implementation of this design has; a GPU tensor may exceed the flat tolerance only up to 1.2
    times that figure (tests/parity.py), so a kernel that adds error of its own fails.

The model is deliberately not the GPU code: no tiling, no split-K, no online softmax; a matrix
product is one `@`.
"""
from __future__ import annotations

import numpy as np
import torch

F64 = np.float64
PROJ = ("q", "k", "v", "o", "g", "u", "d")


def bf16(a):
    """Round-to-nearest-even to bf16, returned as float64."""
    a = np.ascontiguousarray(np.asarray(a, dtype=F64))
    return torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def identity(a):
    return np.asarray(a, dtype=F64)


def _logistic(z):
    return 1.0 / (1.0 + np.exp(-z))


def _silu(z):
    return z * _logistic(z)


def _silu_prime(z):
    s = _logistic(z)
    return s * (1.0 + z * (1.0 - s))


def _act(z, act):
    return _silu(z) if act == "silu" else z


def _act_prime(z, act):
    return _silu_prime(z) if act == "silu" else np.ones_like(z)


def _rope(x, cos, sin, S, heads, hd, inverse=False):
    T = x.shape[0]
    x4 = x.reshape(T // S, S, heads, hd)
    c = cos[None, :, None, :]
    s = (-sin if inverse else sin)[None, :, None, :]
    lo, hi = x4[..., : hd // 2], x4[..., hd // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1).reshape(T, heads * hd)


# ------------------------------------------------------------------------------------------------
# attention: q [T, H*hd], k / v [T, Hkv*hd]; the probabilities are rounded before they multiply v (and
# dO), the scaled score gradient before it multiplies k and q; o, dq, dk, dv are rounded when stored.
# With fewer key / value heads every query head's dk / dv contribution is stored (rounded) and the
# group is summed afterwards.
# ------------------------------------------------------------------------------------------------
def attention_fwd(q, k, v, B, S, H, Hkv, hd, rnd=bf16, jitter=None):
    """jitter: None, or a numpy Generator.  The probabilities are rounded as multiples of a per-row
    reference, exp(s - reference).  An online softmax rounds them against the maximum seen so far, which
    for most rows is not the final one, so which way each probability rounds is an accident of the tile
    walk: the rounding errors have the same size but another realisation.  With a Generator every row gets
    a reference a random fraction of a binade below its maximum, which draws such another realisation."""
    q4, k4, v4 = q.reshape(B, S, H, hd), k.reshape(B, S, Hkv, hd), v.reshape(B, S, Hkv, hd)
    o = np.zeros((B, S, H, hd), dtype=F64)
    lse = np.zeros((B, H, S), dtype=F64)
    scale = 1.0 / np.sqrt(hd)
    mask = np.tril(np.ones((S, S), dtype=bool))
    grp = H // Hkv
    for b in range(B):
        for h in range(H):
            s = np.where(mask, (q4[b, :, h] @ k4[b, :, h // grp].T) * scale, -np.inf)
            m = s.max(axis=1, keepdims=True)
            p = np.exp(s - m)
            den = p.sum(axis=1, keepdims=True)
            lse[b, h] = (m + np.log(den))[:, 0]
            if jitter is not None:
                fac = 2.0 ** (-jitter.random((S, 1)))
                p, den = p * fac, den * fac
            o[b, :, h] = (rnd(p) @ v4[b, :, h // grp]) / den
    return rnd(o.reshape(B * S, H * hd)), lse


def attention_bwd(q, k, v, o, do, lse, B, S, H, Hkv, hd, rnd=bf16):
    q4, k4, v4 = q.reshape(B, S, H, hd), k.reshape(B, S, Hkv, hd), v.reshape(B, S, Hkv, hd)
    o4, do4 = o.reshape(B, S, H, hd), do.reshape(B, S, H, hd)
    dq = np.zeros((B, S, H, hd), dtype=F64)
    dk = np.zeros((B, S, Hkv, hd), dtype=F64)
    dv = np.zeros((B, S, Hkv, hd), dtype=F64)
    scale = 1.0 / np.sqrt(hd)
    mask = np.tril(np.ones((S, S), dtype=bool))
    grp = H // Hkv
    for b in range(B):
        for h in range(H):
            g = h // grp
            s = (q4[b, :, h] @ k4[b, :, g].T) * scale
            p = np.where(mask, np.exp(np.where(mask, s, 0.0) - lse[b, h][:, None]), 0.0)
            dvh = rnd(p).T @ do4[b, :, h]
            dp = do4[b, :, h] @ v4[b, :, g].T
            dsum = np.sum(do4[b, :, h] * o4[b, :, h], axis=1, keepdims=True)
            ds = rnd(p * (dp - dsum) * scale)
            dq[b, :, h] = ds @ k4[b, :, g]
            dkh = ds.T @ q4[b, :, h]
            if grp > 1:            # one stored contribution per query head, summed per group afterwards
                dkh, dvh = rnd(dkh), rnd(dvh)
            dk[b, :, g] += dkh
            dv[b, :, g] += dvh
    T = B * S
    return rnd(dq.reshape(T, H * hd)), rnd(dk.reshape(T, Hkv * hd)), rnd(dv.reshape(T, Hkv * hd))


# ------------------------------------------------------------------------------------------------
# projections
# ------------------------------------------------------------------------------------------------
def down(x, ws, gamma, stat, eps, rnd, act, h_prev=None, two_pass=False):
    """Grouped down-projection.  x [T, d] as the GEMM reads it (already rounded), ws: the members'
    W_down [r, d].  With gamma: RMSNorm with the scale folded into the weight (rounded once) and
    rsqrt(stat/d + eps) applied per row after the product; two_pass: x is normalised and rounded first.
    Returns (z, a) lists: z rounded (the checkpoint), a = sigma(z as stored) rounded (LaX: z + h_prev)."""
    d = x.shape[1]
    zs, as_ = [], []
    rho = None if gamma is None else 1.0 / np.sqrt(stat / d + eps)
    xin = x
    if gamma is not None and two_pass:
        xin = rnd(x * gamma[None, :] * rho[:, None])
    for i, w in enumerate(ws):
        if gamma is None or two_pass:
            z = rnd(xin @ w.T)
        else:
            z = rnd((x @ rnd(w * gamma[None, :]).T) * rho[:, None])
        hp = None if h_prev is None else h_prev[i]
        a = rnd(z + hp) if hp is not None else rnd(_act(z, act))
        zs.append(z)
        as_.append(a)
    return zs, as_


def up_bwd(dout, w_up, z, a, act, rnd, rho=None, dz_next=None):
    """Backward through an up-projection and sigma.  dout [T, d_out] rounded.  Returns
    (dw_up fp, dz rounded (times rho when the layer sits behind a folded norm), dz un-rounded,
    dh_prev rounded or None)."""
    dw_up = dout.T @ a
    da = dout @ w_up
    if dz_next is not None or act == "lax":
        dh_prev = rnd(da)
        dzf = da + (0.0 if dz_next is None else dz_next)
    else:
        dh_prev = None
        dzf = da * _act_prime(z, act)
    if rho is not None:
        dzf = dzf * rho[:, None]
    return dw_up, rnd(dzf), dzf, dh_prev


def norm_down_bwd(dps, dpfs, zs, ws, gamma, x, stat, eps, resid, rnd):
    """Backward of a grouped down-projection behind a folded RMSNorm.  dps: rho * dz per member
    (rounded), dpfs the same un-rounded (the row statistic is taken before rounding), zs the
    checkpoints, x [T, d] as the GEMMs read it.  Returns (dx un-rounded incl. `resid`, [dw_down], dgamma)."""
    d = x.shape[1]
    rho = 1.0 / np.sqrt(stat / d + eps)
    cdot = sum(np.sum(dpf * z, axis=1) for dpf, z in zip(dpfs, zs))
    acc = np.zeros_like(x)
    dws, dgamma = [], np.zeros(d, dtype=F64)
    for dp, w in zip(dps, ws):
        dwp = dp.T @ x                       # gradient w.r.t. (w * gamma)
        dws.append(dwp * gamma[None, :])
        dgamma += np.sum(w * dwp, axis=0)
        acc += dp @ rnd(w * gamma[None, :])
    dx = acc - (rho * cdot / d)[:, None] * x + resid
    return dx, dws, dgamma


# ------------------------------------------------------------------------------------------------
# the block
# ------------------------------------------------------------------------------------------------
def block(x, p, dy, B, S, H, hd, eps, act="silu", rope=None, Hkv=None, h_prev=None, dz_next=None, lax=False,
          two_pass=False, rnd=bf16, trace=None, jitter=None):
    """Forward and backward of the decoder block as the GPU design computes it.

    x, dy, p[...]: float64 arrays holding bf16-representable values.  lax: the LaX variant (identity
    gate, a = z + h_prev, h_prev / dz_next dicts keyed by projection, entries may be None).
    Returns (out, grads, dh_prev): out has y, dx, the seven z_*, s1, s2; grads is keyed like the
    oracle's; dh_prev is a dict (LaX) or None.  trace: optional dict that receives the wide
    intermediates (for looking at where two implementations part)."""
    Hkv = H if Hkv is None else Hkv
    T, d = x.shape
    if lax:
        act = "lax"
    hp = (lambda n: None) if h_prev is None else (lambda n: h_prev.get(n))
    dzn = (lambda n: None) if dz_next is None else (lambda n: dz_next.get(n))
    out, g = {}, {}

    # ---- forward -----------------------------------------------------------------------------------
    s1 = np.sum(x * x, axis=1)
    z_qkv, a_qkv = down(x, [p["wd_q"], p["wd_k"], p["wd_v"]], p["gamma1"], s1, eps, rnd, act,
                        [hp("q"), hp("k"), hp("v")] if lax else None, two_pass)
    q, k, v = (rnd(a @ p["wu_" + n].T) for a, n in zip(a_qkv, "qkv"))
    if rope is not None:
        q = rnd(_rope(q, rope[0], rope[1], S, H, hd))
        k = rnd(_rope(k, rope[0], rope[1], S, Hkv, hd))
    o, lse = attention_fwd(q, k, v, B, S, H, Hkv, hd, rnd, jitter)
    (z_o,), (a_o,) = down(o, [p["wd_o"]], None, None, eps, rnd, act, [hp("o")] if lax else None)
    h1f = x + a_o @ p["wu_o"].T                   # kept un-rounded for the second residual sum
    h1 = rnd(h1f)                                 # what the GEMMs read
    s2 = np.sum(h1f * h1f, axis=1)
    z_gu, a_gu = down(h1, [p["wd_g"], p["wd_u"]], p["gamma2"], s2, eps, rnd, act,
                      [hp("g"), hp("u")] if lax else None, two_pass)
    gg = rnd(a_gu[0] @ p["wu_g"].T)
    uf = a_gu[1] @ p["wu_u"].T
    m = rnd(_silu(gg) * uf)                       # the gate multiplies the un-rounded u accumulators
    uu = rnd(uf)                                  # what the backward's re-forward stores
    (z_d,), (a_d,) = down(m, [p["wd_d"]], None, None, eps, rnd, act, [hp("d")] if lax else None)
    out["y"] = rnd(h1f + a_d @ p["wu_d"].T)
    out.update({"z_q": z_qkv[0], "z_k": z_qkv[1], "z_v": z_qkv[2], "z_o": z_o, "z_g": z_gu[0], "z_u": z_gu[1],
                "z_d": z_d, "s1": s1, "s2": s2})

    # ---- backward (every wide activation above is bit-identical when rebuilt from the checkpoints) ----
    dh = {}
    rho1, rho2 = 1.0 / np.sqrt(s1 / d + eps), 1.0 / np.sqrt(s2 / d + eps)
    g["wu_d"], dz_d, _, dh["d"] = up_bwd(dy, p["wu_d"], z_d, a_d, act, rnd, None, dzn("d"))
    g["wd_d"] = dz_d.T @ m
    dm = dz_d @ p["wd_d"]
    dg = rnd(dm * uu * _silu_prime(gg))
    du = rnd(dm * _silu(gg))
    g["wu_g"], dp_g, dpf_g, dh["g"] = up_bwd(dg, p["wu_g"], z_gu[0], a_gu[0], act, rnd, rho2, dzn("g"))
    g["wu_u"], dp_u, dpf_u, dh["u"] = up_bwd(du, p["wu_u"], z_gu[1], a_gu[1], act, rnd, rho2, dzn("u"))
    dh1f, (g["wd_g"], g["wd_u"]), g["gamma2"] = norm_down_bwd(
        [dp_g, dp_u], [dpf_g, dpf_u], z_gu, [p["wd_g"], p["wd_u"]], p["gamma2"], h1, s2, eps, dy, rnd)
    dh1 = rnd(dh1f)
    g["wu_o"], dz_o, _, dh["o"] = up_bwd(dh1, p["wu_o"], z_o, a_o, act, rnd, None, dzn("o"))
    g["wd_o"] = dz_o.T @ o
    do = rnd(dz_o @ p["wd_o"])
    dq, dk, dv = attention_bwd(q, k, v, o, do, lse, B, S, H, Hkv, hd, rnd)
    if rope is not None:
        dq = rnd(_rope(dq, rope[0], rope[1], S, H, hd, inverse=True))
        dk = rnd(_rope(dk, rope[0], rope[1], S, Hkv, hd, inverse=True))
    dps, dpfs = [], []
    for n, dn, z, a in zip("qkv", (dq, dk, dv), z_qkv, a_qkv):
        g["wu_" + n], dp, dpf, dh[n] = up_bwd(dn, p["wu_" + n], z, a, act, rnd, rho1, dzn(n))
        dps.append(dp)
        dpfs.append(dpf)
    dxf, (g["wd_q"], g["wd_k"], g["wd_v"]), g["gamma1"] = norm_down_bwd(
        dps, dpfs, z_qkv, [p["wd_q"], p["wd_k"], p["wd_v"]], p["gamma1"], x, s1, eps, dh1f, rnd)
    out["dx"] = rnd(dxf)
    if trace is not None:
        trace.update(q=q, k=k, v=v, o=o, h1=h1, h1f=h1f, g=gg, u=uu, m=m, dz_d=dz_d, dg=dg, du=du, dh1=dh1, dh1f=dh1f,
                     dz_o=dz_o, do=do, dq=dq, dk=dk, dv=dv, a_d=a_d, a_o=a_o)
    return out, g, (dh if lax else None)


def relerr(got, ref):
    ref = np.asarray(ref, dtype=F64)
    rms = np.sqrt(np.mean(ref * ref))
    return float(np.max(np.abs(np.asarray(got, dtype=F64) - ref)) / (rms if rms > 0 else 1.0))


def err2(got, ref):
    """(max|got - ref| / RMS(ref), ||got - ref|| / ||ref||): the two figures a budget consists of."""
    ref = np.asarray(ref, dtype=F64)
    dif = np.asarray(got, dtype=F64) - ref
    nrm = float(np.linalg.norm(ref))
    return relerr(got, ref), float(np.linalg.norm(dif) / (nrm if nrm > 0 else 1.0))


def over_realisations(one_run, realisations=3):
    """Largest figures, key by key, of the dicts of (max-norm, L2) error pairs that one_run(jitter)
    returns: jitter None (the plain softmax) first, then seeded Generators (see attention_fwd)."""
    bud = None
    for i in range(max(1, realisations)):
        one = one_run(None if i == 0 else np.random.default_rng(1000 + i))
        bud = one if bud is None else {k: tuple(max(a, b) for a, b in zip(bud[k], one[k])) for k in bud}
    return bud


def block_budget(x, p, dy, B, S, H, hd, eps, y_ref, c_ref, dx_ref, g_ref, realisations=3, **kw):
    """Per-tensor error of the modelled bf16 pipeline against given exact results (the oracle's y, its
    cache of intermediates, dx and gradient dict): the budget of tests/parity.py, rule 3.  Keys: y, dx,
    z_<projection>, z_qkv and z_gu (concatenated as the ABI stores them), d<gradient name>; values:
    (max-norm error, relative L2 error) as err2 gives them.

    The maximum over a small tensor depends on the realisation of the rounding errors, and the GPU's
    online softmax draws another one than the plain softmax here (see attention_fwd), which every tensor
    behind the attention inherits.  The budget is therefore the largest error over `realisations` runs:
    the plain one and runs with jittered softmax references (seeded)."""
    def one_run(jit):
        out, g, _ = block(x, p, dy, B, S, H, hd, eps, jitter=jit, **kw)
        one = {"y": err2(out["y"], y_ref), "dx": err2(out["dx"], dx_ref)}
        for n in PROJ:
            one["z_" + n] = err2(out["z_" + n], c_ref["z_" + n])
        for cat, names in (("z_qkv", "qkv"), ("z_gu", "gu")):
            one[cat] = err2(np.concatenate([out["z_" + n] for n in names], 1),
                              np.concatenate([c_ref["z_" + n] for n in names], 1))
        one.update({"d" + k: err2(g[k], g_ref[k]) for k in g_ref})
        return one

    return over_realisations(one_run, realisations)


def attention_budget(q, k, v, do, B, S, H, Hkv, hd, o_ref, dq_ref, dk_ref, dv_ref, realisations=3):
    """Budget of a standalone attention forward + backward: keys o, dq, dk, dv."""
    def one_run(jit):
        om, lsem = attention_fwd(q, k, v, B, S, H, Hkv, hd, jitter=jit)
        gm = attention_bwd(q, k, v, om, do, lsem, B, S, H, Hkv, hd)
        return {"o": err2(om, o_ref), "dq": err2(gm[0], dq_ref), "dk": err2(gm[1], dk_ref),
                "dv": err2(gm[2], dv_ref)}

    return over_realisations(one_run, realisations)
