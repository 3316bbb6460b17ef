"""Seeded synthetic inputs for the low-rank decoder-block hot path.

This module only draws random numbers, rounds them to the storage dtype and lays them out in
memory.  It holds none of the method's arithmetic, so both the CPU oracle's tests and the HIP
path's tests/benchmark may use it.  Distributions follow the workloads the method is measured
on (LLaMA-2-shaped blocks, Gaussian activations, weights scaled 1/sqrt(fan_in)); synthetic
Gaussians stand in for tokenised text, whose values do not influence kernel time.

Every tensor is drawn from its own counter-based stream keyed by (seed, tensor name), so a
tensor's values do not depend on which other tensors were requested or in what order.
"""
from __future__ import annotations

import zlib

import numpy as np
import torch

PROJ = ("q", "k", "v", "o", "g", "u", "d")


def _stream(seed: int, name: str) -> np.random.Generator:
    key = np.array([np.uint64(seed), np.uint64(zlib.crc32(name.encode()))], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def gaussian(seed: int, name: str, shape, std: float = 1.0, mean: float = 0.0,
             dtype: torch.dtype = torch.float32) -> torch.Tensor:
    """N(mean, std^2) drawn in fp32 and rounded (nearest-even) to `dtype`."""
    g = _stream(seed, name)
    a = g.standard_normal(size=tuple(shape), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return torch.from_numpy(a).to(dtype)


def f64(t: torch.Tensor) -> np.ndarray:
    """Promote a stored tensor (already rounded to its storage dtype) to float64."""
    return t.detach().cpu().to(torch.float64).numpy()


# ------------------------------------------------------------------------------------------
def linear_case(T, d_in, r, d_out, dtype=torch.float32, seed=0):
    """One bottleneck layer: x ~ N(0,1), W_down ~ N(0,1/d_in), W_up ~ N(0,1/r), dy ~ N(0,1)."""
    return {
        "x": gaussian(seed, "x", (T, d_in), dtype=dtype),
        "w_down": gaussian(seed, "w_down", (r, d_in), std=d_in ** -0.5, dtype=dtype),
        "w_up": gaussian(seed, "w_up", (d_out, r), std=r ** -0.5, dtype=dtype),
        "dy": gaussian(seed, "dy", (T, d_out), dtype=dtype),
    }


def group_case(T, d_in, r, d_out, G, dtype=torch.bfloat16, seed=0):
    """G projections sharing x, with an RMSNorm scale gamma = 1 + 0.1 N(0,1)."""
    c = {
        "x": gaussian(seed, "x", (T, d_in), dtype=dtype),
        "gamma": gaussian(seed, "gamma", (d_in,), std=0.1, mean=1.0, dtype=dtype),
        "w_down": [gaussian(seed, f"w_down{g}", (r, d_in), std=d_in ** -0.5, dtype=dtype)
                   for g in range(G)],
        "w_up": [gaussian(seed, f"w_up{g}", (d_out, r), std=r ** -0.5, dtype=dtype)
                 for g in range(G)],
        "dy": [gaussian(seed, f"dy{g}", (T, d_out), dtype=dtype) for g in range(G)],
    }
    return c


def block_case(B, S, d, H, hd, f, r, dtype=torch.bfloat16, seed=0, gamma_std=0.1, Hkv=None):
    """Decoder block: seven factored projections, two norm scales, x and the upstream grad.
    Hkv: key / value heads of grouped-query attention (None: as many as query heads)."""
    assert H * hd == d
    T = B * S
    p = {}
    dkv = d if Hkv is None else Hkv * hd
    dims = {"q": (d, d), "k": (d, dkv), "v": (d, dkv), "o": (d, d), "g": (d, f), "u": (d, f), "d": (f, d)}
    for n in PROJ:
        d_in, d_out = dims[n]
        p["wd_" + n] = gaussian(seed, "wd_" + n, (r, d_in), std=d_in ** -0.5, dtype=dtype)
        p["wu_" + n] = gaussian(seed, "wu_" + n, (d_out, r), std=r ** -0.5, dtype=dtype)
    p["gamma1"] = gaussian(seed, "gamma1", (d,), std=gamma_std, mean=1.0, dtype=dtype)
    p["gamma2"] = gaussian(seed, "gamma2", (d,), std=gamma_std, mean=1.0, dtype=dtype)
    return {
        "x": gaussian(seed, "x", (T, d), dtype=dtype),
        "dy": gaussian(seed, "dy", (T, d), dtype=dtype),
        "params": p,
    }


# ------------------------------------------------------------------------------------------
# Layout helpers (no arithmetic): the grouped / stacked / padded buffers the C ABI takes.
# ------------------------------------------------------------------------------------------
def pad_ld(n: int, mult: int = 64) -> int:
    return (n + mult - 1) // mult * mult


def pack_group(case):
    """w_down_cat[G*r, d_in] (concatenated along the rank axis), w_up_stack[G, d_out, r]."""
    return torch.cat(case["w_down"], dim=0).contiguous(), torch.stack(case["w_up"], dim=0).contiguous()


def pack_block_params(p, f, f_ld):
    """Buffers in the block ABI's layout; the ffn axis is zero-padded from f to f_ld."""
    def pad_rows(w):      # [f, r] -> [f_ld, r]
        out = torch.zeros((f_ld, w.shape[1]), dtype=w.dtype)
        out[:f] = w
        return out

    def pad_cols(w):      # [r, f] -> [r, f_ld]
        out = torch.zeros((w.shape[0], f_ld), dtype=w.dtype)
        out[:, :f] = w
        return out

    return {
        "gamma1": p["gamma1"].contiguous(),
        "w_dn_qkv": torch.cat([p["wd_q"], p["wd_k"], p["wd_v"]], dim=0).contiguous(),
        # [3, d, r] stacked; with fewer key / value heads the rows of q, k, v packed one after the other
        "w_up_qkv": (torch.stack([p["wu_q"], p["wu_k"], p["wu_v"]], dim=0) if p["wu_k"].shape == p["wu_q"].shape
                     else torch.cat([p["wu_q"], p["wu_k"], p["wu_v"]], dim=0)).contiguous(),
        "w_dn_o": p["wd_o"].contiguous(),
        "w_up_o": p["wu_o"].contiguous(),
        "gamma2": p["gamma2"].contiguous(),
        "w_dn_gu": torch.cat([p["wd_g"], p["wd_u"]], dim=0).contiguous(),
        "w_up_gu": torch.stack([pad_rows(p["wu_g"]), pad_rows(p["wu_u"])], dim=0).contiguous(),
        "w_dn_d": pad_cols(p["wd_d"]).contiguous(),
        "w_up_d": p["wu_d"].contiguous(),
    }
