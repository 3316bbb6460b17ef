"""Benchmark of the low-rank decoder-block hot path on one MI355X.

One "step" = lr_block_fwd + lr_block_bwd (all forward and backward rows of the hot path, with the
backward re-forwarding from the rank-r checkpoints) on one synthetic batch that is already resident
in HBM.  Prints ONE JSON line with the whole-job throughput in TFLOP/s of executed GEMM + attention
work, a roofline object for the dominant kernel class (the bf16 MFMA GEMMs, timed live with HIP
events on the stream they run on) and the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: batch, seq, d_model, heads, ffn, rank
    "block-7B": (4, 4096, 4096, 32, 11008, 1024),
    "block-1B": (8, 2048, 2048, 16, 5461, 512),
    "block-7B-r128": (4, 4096, 4096, 32, 11008, 128),
    "block-tiny": (2, 256, 256, 2, 344, 64),
}
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0


def block_flops(B, S, d, H, f, r):
    """FLOPs = 2MNK per GEMM; attention counted causal-halved.  Returns a dict of the totals."""
    T = B * S
    lin_fwd = 2.0 * T * (11 * d * r + 3 * f * r)
    attn_fwd = 2.0 * 2.0 * B * H * S * S * (d // H) / 2.0        # QK^T and PV, causal half
    model = 3.0 * lin_fwd + 3.5 * attn_fwd                       # bwd: 2x linear, 2.5x attention
    recompute_lin = 2.0 * T * r * (4 * d + 2 * f)                # six of the seven up-projections
    gemm_exec = 3.0 * lin_fwd + recompute_lin
    # attention as executed here: fwd, re-fwd, and a two-kernel backward (3 + 4 GEMM units of the 2 in fwd)
    attn_exec = attn_fwd * (1.0 + 1.0 + 3.5)
    return {"model": model, "gemm_exec": gemm_exec, "attn_exec": attn_exec, "exec": gemm_exec + attn_exec,
            "lin_fwd": lin_fwd, "attn_fwd": attn_fwd}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="block-7B", choices=list(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import synth_inputs as si
    from paper_2512_12131_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    Bn, S, d, H, f, r = WORKLOADS[args.workload]
    f_ld = si.pad_ld(f, 8)
    eps = 1e-5
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=0)
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=eps)
    params = {k: v.to(dev) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    x, dy = case["x"].to(dev), case["dy"].to(dev)
    ck = B.alloc_block_ckpt(desc, dev)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    grads = {n: torch.zeros_like(params[n], dtype=torch.float32) for n in B.PARAM_NAMES}
    ws = torch.empty(max(B.lr_block_workspace_bytes(desc, 0), B.lr_block_workspace_bytes(desc, 1)),
                     dtype=torch.uint8, device=dev)

    def step():
        B.lr_block_fwd(desc, params, x, ckpt=ck, ws=ws, y=y)
        B.lr_block_bwd(desc, params, x, dy, ck, grads=grads, accumulate=False, ws=ws, dx=dx)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / max(args.steps, 1)

    fl = block_flops(Bn, S, d, H, f, r)
    value = fl["exec"] / dt / 1e12

    # ---- roofline of the dominant kernel class: the forward grouped down-projection GEMM
    # (x[T,d] . w_dn_qkv[3r,d]^T with the online-RMSNorm epilogue), timed with HIP events on the
    # stream it is launched on, through the same entry point the block uses for it.
    T = Bn * S
    G = 3
    wdn, wup = params["w_dn_qkv"], params["w_up_qkv"]
    nb = B.lr_group_workspace_bytes(G, T, d, r, d, B.LR_BF16, 0)
    gws = torch.empty(nb, dtype=torch.uint8, device=dev)
    z = torch.empty((T, G * r), dtype=torch.bfloat16, device=dev)
    stat = torch.empty((T,), dtype=torch.float32, device=dev)
    yq = torch.empty((G, T, d), dtype=torch.bfloat16, device=dev)
    import ctypes as C
    L = B.lib()
    stream = torch.cuda.current_stream()

    def group_fwd():
        st = L.lr_group_fwd(x.data_ptr(), d, params["gamma1"].data_ptr(), eps, B.LR_NORM_ONLINE, wdn.data_ptr(),
                            wup.data_ptr(), z.data_ptr(), stat.data_ptr(), yq.data_ptr(), d, T * d, G, T, d, r, d,
                            B.LR_ACT_SILU, B.LR_BF16, gws.data_ptr(), nb, C.c_void_p(stream.cuda_stream))
        assert st == 0

    for _ in range(2):
        group_fwd()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    stream.synchronize()
    e0.record(stream)
    for _ in range(reps):
        group_fwd()
    e1.record(stream)
    e1.synchronize()
    g_ms = e0.elapsed_time(e1) / reps
    g_flops = 2.0 * T * d * (G * r) + G * 2.0 * T * r * d     # grouped down GEMM + batched up GEMM
    achieved = g_flops / (g_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "kernel": "gemm_bf16_kernel (grouped down-projection + batched up-projection of Q/K/V)",
                "ms_per_launch_pair": round(g_ms, 4)}

    out = {
        "metric": "TFLOP/s + % MFMA bf16 peak, low-rank decoder block fwd+bwd (1 MI355X)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: low-rank decoder block fwd+bwd, batch {Bn}, seq {S}, d_model {d}, "
                               f"{H} heads of 128, ffn {f}, rank {r}, rank-r checkpoint recompute",
                   "tokens": T, "executed_tflop": round(fl["exec"] / 1e12, 3),
                   "model_tflop": round(fl["model"] / 1e12, 3),
                   "frac_mfma_peak_executed": round(value / MFMA_BF16_PEAK_TFLOPS, 4),
                   "model_tflops": round(fl["model"] / dt / 1e12, 2)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        # fp64 oracle on the host cores, bounded sample: forward + backward of the same block on the
        # first `s_len` tokens of batch element 0.
        import numpy as np
        from oracle import lowrank_oracle as orc
        s_len = min(S, 256)
        P = {k: si.f64(v) for k, v in case["params"].items()}
        X0, DY0 = si.f64(case["x"][:s_len]), si.f64(case["dy"][:s_len])
        t0 = time.perf_counter()
        orc.block_fwd(X0, P, 1, s_len, H, 128, eps)
        orc.block_bwd(X0, P, DY0, 1, s_len, H, 128, eps)
        ct = time.perf_counter() - t0
        cfl = block_flops(1, s_len, d, H, f, r)
        cpu_flops = cfl["model"] + cfl["lin_fwd"] + cfl["attn_fwd"]   # block_bwd runs its own forward again
        out["cpu_baseline"] = {"value": round(cpu_flops / ct / 1e12, 4), "unit": "TFLOP/s",
                               "cores": os.cpu_count() if not os.environ.get("OMP_NUM_THREADS") else
                               int(os.environ["OMP_NUM_THREADS"]),
                               "kind": "oracle",
                               "sample": f"fp64 numpy oracle, block fwd + bwd on {s_len} tokens of batch element 0 "
                                         f"({ct:.1f} s)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
