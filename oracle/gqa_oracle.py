"""fp64 CPU oracle of causal grouped-query attention.

TEST INFRASTRUCTURE ONLY (same rules as lowrank_oracle.py: nothing in the product path imports
this; it shares no code with the HIP path).

Grouped-query attention is an extension the paper names for its attention chunk (section
"Discussion and Future Work": only the shapes of the Q, K and V projections change): there are fewer
key / value heads than query heads, the H query heads are split into
H_kv groups of H / H_kv consecutive heads, and every head of a group attends over the same key and
value head.  Per (batch b, query head h), with g = h // (H / H_kv):

    s = q_bh k_bg^T / sqrt(hd)   (keys after the query masked out),   p = softmax_row(s),   o_bh = p v_bg .

Because a key / value head is used by several query heads, its gradient is the sum over them.

Written as the plain definition, one (batch, head) at a time; a matrix product is the only library
primitive used as a step.  Layout: q, o, do, dq [B*S, H*hd]; k, v, dk, dv [B*S, H_kv*hd]; lse [B, H, S].

Pins (tests/test_oracle_gqa.py): H_kv = H is the multi-head oracle; any H_kv equals the multi-head
oracle run on key / value tensors with every head repeated H / H_kv times, the gradients of the copies
added up; rows of the probabilities sum to one and the first token returns v_0; central finite
differences for dq, dk, dv.  Absolute values are "parity unpinned" by the paper (no worked example).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _probs(qh, kh, causal):
    """softmax over keys of qh kh^T / sqrt(hd) for one (batch, head): returns (p [S, S], lse [S])."""
    S, hd = qh.shape
    s = (qh @ kh.T) / np.sqrt(hd)
    if causal:
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    den = np.sum(e, axis=1, keepdims=True)
    return e / den, (m + np.log(den))[:, 0]


def attention_gqa_fwd(q, k, v, B, S, H, Hkv, hd, causal=True):
    assert H % Hkv == 0
    grp = H // Hkv
    q4 = np.asarray(q, dtype=F64).reshape(B, S, H, hd)
    k4 = np.asarray(k, dtype=F64).reshape(B, S, Hkv, hd)
    v4 = np.asarray(v, dtype=F64).reshape(B, S, Hkv, hd)
    o = np.zeros((B, S, H, hd), dtype=F64)
    lse = np.zeros((B, H, S), dtype=F64)
    for b in range(B):
        for h in range(H):
            g = h // grp
            p, lse[b, h] = _probs(q4[b, :, h, :], k4[b, :, g, :], causal)
            o[b, :, h, :] = p @ v4[b, :, g, :]
    return o.reshape(B * S, H * hd), lse


def attention_gqa_bwd(q, k, v, do, B, S, H, Hkv, hd, causal=True):
    """Gradients of L = sum(o * do): (dq [T, H*hd], dk [T, Hkv*hd], dv [T, Hkv*hd])."""
    assert H % Hkv == 0
    grp = H // Hkv
    q4 = np.asarray(q, dtype=F64).reshape(B, S, H, hd)
    k4 = np.asarray(k, dtype=F64).reshape(B, S, Hkv, hd)
    v4 = np.asarray(v, dtype=F64).reshape(B, S, Hkv, hd)
    do4 = np.asarray(do, dtype=F64).reshape(B, S, H, hd)
    dq = np.zeros_like(q4)
    dk = np.zeros_like(k4)
    dv = np.zeros_like(v4)
    for b in range(B):
        for h in range(H):
            g = h // grp
            p, _ = _probs(q4[b, :, h, :], k4[b, :, g, :], causal)
            dv[b, :, g, :] += p.T @ do4[b, :, h, :]
            dp = do4[b, :, h, :] @ v4[b, :, g, :].T
            ds = p * (dp - np.sum(dp * p, axis=1, keepdims=True)) / np.sqrt(hd)
            dq[b, :, h, :] = ds @ k4[b, :, g, :]
            dk[b, :, g, :] += ds.T @ q4[b, :, h, :]
    T = B * S
    return dq.reshape(T, H * hd), dk.reshape(T, Hkv * hd), dv.reshape(T, Hkv * hd)
