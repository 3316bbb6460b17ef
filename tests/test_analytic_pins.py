"""Pins oracle/analytic.py to the numbers the paper states in its running text."""
import math

from golden_io import load_golden
from oracle import analytic as an

G = load_golden()


def test_eq1_square_gemm_closed_form():
    # M = N = K = n  =>  2n^3 / (3 n^2 * bytes) = n / (1.5 * bytes)
    for n in (64, 1000, 4096):
        assert math.isclose(an.gemm_arithmetic_intensity(n, n, n, 2), n / 3.0, rel_tol=1e-12)
    # skinny limit: K -> small, A.I. -> K / bytes * (MN / (MN + K(M+N)))
    M, N, K = 16384, 4096, 128
    expect = 2 * M * N * K / ((M * K + K * N + M * N) * 2)
    assert an.gemm_arithmetic_intensity(M, N, K) == expect


def test_vcomm_ratios_match_text():
    b, s, d = 4, 4096, 4096
    full = an.vcomm_full(b, s, d)
    assert math.isclose(an.vcomm_vanilla(b, s, d, 2.5 * d) / full, G["vanilla_over_full_vcomm_dff_2p5d"])
    assert math.isclose(an.vcomm_vanilla(b, s, d, 4 * d) / full, G["vanilla_over_full_vcomm_dff_4d"])
    r = d // 4
    # "more than 5.7x": holds for both d_ff = 2.5 d and the 7B value 11008
    assert an.vcomm_vanilla(b, s, d, 2.5 * d) / an.vcomm_btp(b, s, r) > G["vanilla_over_btp_vcomm_min"]
    assert an.vcomm_vanilla(b, s, d, 2.5 * d) / an.vcomm_btp(b, s, r) < G["vanilla_over_btp_vcomm_min"] + 0.05
    assert an.vcomm_vanilla(b, s, d, 11008) / an.vcomm_btp(b, s, r) > G["vanilla_over_btp_vcomm_min"]
    assert abs(full / an.vcomm_btp(b, s, r) - G["full_over_btp_vcomm"]) < 0.005
    # Eq. 3's second form: 7r/(2d) x V_full
    assert math.isclose(an.vcomm_btp(b, s, r), 7 * r / (2 * d) * full)


def test_dp_reduction_matches_text():
    for key in ("model_1B", "model_3B", "model_7B", "model_13B", "model_30B"):
        _, _, d, dff, r = G[key]
        assert r == d / 4
        ratio = an.dp_params_full(d, dff) / an.dp_params_lowrank(d, dff, r)
        assert abs(ratio - G["dp_reduction_r_quarter"]) < 0.1, (key, ratio)


def test_mlp_ai_table_at_7b_tp4():
    _, _, d, dff, r = G["model_7B"]
    alpha, beta, bs, tp = dff / d, d / r, 4 * 4096, 4
    full = an.mlp_ai_fullrank_tp(bs, d, alpha, tp)
    van = an.mlp_ai_vanilla_lowrank_tp(bs, d, alpha, beta, tp)
    btp = an.mlp_ai_btp(bs, d, alpha, beta, tp)
    # the text rounds to one digit: "2.5x" and "0.2x"
    assert abs(btp / van - G["btp_over_vanilla_ai_7b_mlp"]) < 0.15
    assert abs(van / full - G["vanilla_over_full_ai_7b_mlp"]) < 0.05
    # vanilla and BTP do the same FLOPs; BTP moves less data, so its A.I. is higher
    assert btp > van
    # at TP = 1 the two low-rank layouts coincide
    assert math.isclose(an.mlp_ai_vanilla_lowrank_tp(bs, d, alpha, beta, 1),
                        an.mlp_ai_btp(bs, d, alpha, beta, 1), rel_tol=1e-12)


def test_mlp_ai_table_consistent_with_eq1():
    """The table's A.I. rows must equal FLOPs / (bytes from the Data Movement column)."""
    _, _, d, dff, r = G["model_7B"]
    alpha, beta, bs, tp = dff / d, d / r, 16384, 4
    flops_lr = 4 * (1 + alpha) * bs * d * d / (beta * tp)
    move_btp = 4 * d * (((1 + alpha) * (beta * bs + d) + 2 * bs * tp) / (beta * tp))
    move_van = 4 * d * ((1 + alpha) * bs + ((1 + alpha) * d + 2 * bs) / (beta * tp))
    assert math.isclose(flops_lr / move_btp, an.mlp_ai_btp(bs, d, alpha, beta, tp), rel_tol=1e-12)
    assert math.isclose(flops_lr / move_van, an.mlp_ai_vanilla_lowrank_tp(bs, d, alpha, beta, tp), rel_tol=1e-12)
    flops_full = 4 * alpha * bs * d * d / tp
    move_full = 4 * d * (bs + alpha * (d + bs) / tp)
    assert math.isclose(flops_full / move_full, an.mlp_ai_fullrank_tp(bs, d, alpha, tp), rel_tol=1e-12)
