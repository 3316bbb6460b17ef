"""The benchmark's FLOP accounting (host arithmetic only): the per-launch GEMM classes add up to the
executed GEMM FLOPs for every workload, the totals match the closed forms of the paper's parameter count
(App. "Communication volume analysis": 11dr + 3 d_ff r parameters, 2 FLOPs per parameter and token in the
forward), and the attainable figure is the MFMA peak exactly when every class sits above the machine
balance."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(bench)


def _dkv(w):
    return 8 * 128 if len(w) > 6 and w[6] == "gqa8" else None


def test_gemm_classes_add_up_for_every_workload():
    for name, w in bench.WORKLOADS.items():
        Bn, S, d, H, f, r = w[:6]
        fl = bench.block_flops(Bn, S, d, H, f, r, _dkv(w))
        cl = bench.gemm_classes(Bn, S, d, H, f, r, _dkv(w))
        assert abs(sum(c[0] for c in cl) - fl["gemm_exec"]) < 1e-9 * fl["gemm_exec"], name
        assert fl["exec"] > fl["model"] > 0, name


def test_block_7b_totals_match_the_closed_forms():
    Bn, S, d, H, f, r = bench.WORKLOADS["block-7B"][:6]
    T = Bn * S
    fl = bench.block_flops(Bn, S, d, H, f, r)
    params = 11 * d * r + 3 * f * r
    assert params == 79_953_920
    assert fl["lin_fwd"] == 2.0 * T * params
    assert abs(fl["exec"] / 1e12 - 11.62) < 0.01 and abs(fl["model"] / 1e12 - 9.78) < 0.01
    # fewer key / value heads only shrink the K and V up-projections
    g = bench.block_flops(Bn, S, d, H, f, r, 1024)
    assert fl["lin_fwd"] - g["lin_fwd"] == 2.0 * T * 2 * (d - 1024) * r
    assert g["attn_fwd"] == fl["attn_fwd"]


def test_attainable_rate_is_capped_by_the_memory_side_only_for_small_ranks():
    w = bench.WORKLOADS
    full = bench.attainable_tflops(bench.gemm_classes(*w["block-7B"][:6]))
    thin = bench.attainable_tflops(bench.gemm_classes(*w["block-7B-r128"][:6]))
    assert abs(full - bench.MFMA_BF16_PEAK_TFLOPS) < 1e-6
    assert thin < 0.5 * bench.MFMA_BF16_PEAK_TFLOPS
