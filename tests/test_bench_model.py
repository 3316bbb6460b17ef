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
    # at the full rank only three launches sit below the machine balance, all K = r products with wide
    # epilogue traffic: SwiGLU backward (reads g, u, writes dg, du) and the two residual sums that carry the
    # fp32 copy of the residual stream
    assert 0.97 * bench.MFMA_BF16_PEAK_TFLOPS < full < bench.MFMA_BF16_PEAK_TFLOPS
    below = [c for c in bench.gemm_launches(*w["block-7B"][:6]) if bench.attainable_of(c["flops"], c["bytes"]) < 2499.0]
    assert sorted(c["tag"] for c in below) == [6, 10, 11]
    assert thin < 0.5 * bench.MFMA_BF16_PEAK_TFLOPS


def test_launch_table_counts_32_launches_and_pads_only_the_ffn_axis():
    Bn, S, d, H, f, r = bench.WORKLOADS["block-1B"][:6]
    la = bench.gemm_launches(Bn, S, d, H, f, r, None, 5464)
    assert len(la) == 32
    assert sum(c["batch"] if c["tag"] == 0 and c["K"] == r and c["N"] == d else 0 for c in la) == 3 + 3 + 1
    assert {c["N"] for c in la if c["what"] == "up gate"} == {5464}
    assert all(c["flops"] == 2.0 * Bn * S * f * r for c in la if c["what"] == "up gate")
