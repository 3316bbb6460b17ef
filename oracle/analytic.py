"""Closed forms of the paper's performance model, in plain Python floats.

TEST INFRASTRUCTURE ONLY (see lowrank_oracle.py).  These are the formulas of Sec. 3 (Eq. 1),
Sec. 4.1 (Eq. 2, Eq. 3) and the appendix tables "Per iteration communication volume" and
"Per MLP block GEMM arithmetic intensity", written out so that tests can check the roofline
numbers the benchmark reports against the values the paper states in its text.
"""
from __future__ import annotations


def gemm_flops(M, N, K):
    """FLOPs of C[M,N] = A[M,K] B[K,N]  (Sec. 3)."""
    return 2.0 * M * N * K


def gemm_arithmetic_intensity(M, N, K, bytes_per_element=2):
    """Eq. 1: FLOPs / bytes with ideal reuse (read A, read B, write C once)."""
    return gemm_flops(M, N, K) / ((M * K + K * N + M * N) * bytes_per_element)


# ---- per-block tensor-parallel communication volume per pass (Sec. 4.1) ---------------------
def vcomm_full(b, s, d):
    return 2.0 * b * s * d


def vcomm_vanilla(b, s, d, dff):
    """Eq. 2: one collective per low-rank linear."""
    return 5.0 * b * s * d + 2.0 * b * s * dff


def vcomm_btp(b, s, r):
    """Eq. 3: one collective per rank-r boundary, seven per block."""
    return 7.0 * b * s * r


# ---- data-parallel gradient volume per layer (appendix table, DP row) -----------------------
def dp_params_full(d, dff):
    return 4.0 * d * d + 3.0 * d * dff


def dp_params_lowrank(d, dff, r):
    return 11.0 * d * r + 3.0 * dff * r


# ---- per-MLP-block arithmetic intensity under the three TP designs (appendix table) ---------
# alpha = d_ff / d, beta = d / r, bs = tokens per micro-batch; forward GEMMs only.
def mlp_ai_fullrank_tp(bs, d, alpha, tp):
    return alpha * bs * d * d / (bs * d * tp + alpha * d * (d + bs))


def mlp_ai_vanilla_lowrank_tp(bs, d, alpha, beta, tp):
    num = 4.0 * bs * d * d * (1.0 + alpha)
    den = 4.0 * bs * d * beta * tp * (1.0 + alpha) + 4.0 * d * d * (1.0 + alpha) + 8.0 * bs * d
    return num / den


def mlp_ai_btp(bs, d, alpha, beta, tp):
    num = 4.0 * bs * d * d * (1.0 + alpha)
    den = 4.0 * beta * bs * d * (1.0 + alpha) + 4.0 * d * d * (1.0 + alpha) + 8.0 * bs * d * tp
    return num / den
