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
    # one rank's share of the 7B block under bottleneck-aware tensor parallelism at TP = 8 (Sec. 4.1):
    # d, heads and d_ff divided by 8, the rank-r tensors whole; the all-reduces between chunks are not run
    "block-7B-btp8-shard": (4, 4096, 512, 4, 1376, 1024),
    # the other model sizes of the paper's configuration table (App. "Model configuration"; heads of
    # 128 here, the head counts follow from d_model), batch 4 x seq 4096 as in Sec. 5.1
    "block-3B": (4, 4096, 3072, 24, 8192, 768),
    "block-13B": (4, 4096, 5120, 40, 13824, 1280),
    "block-30B": (4, 4096, 8192, 64, 22016, 2048),
    # sigma = identity: the SVD-style factorisation without the rank-r non-linearity (App. "Low-rank
    # Training Algorithm")
    "block-7B-svd": (4, 4096, 4096, 32, 11008, 1024, "identity"),
    # the LaX variant (App. "LaX variant (residual low-rank)"): identity gate, every layer adds the rank-r
    # activation of the layer below before its up-projection; timed as a middle block of a stack (it
    # receives h_prev and dz_next and returns dh_prev)
    "block-7B-lax": (4, 4096, 4096, 32, 11008, 1024, "lax"),
    # rotary position embedding of q and k switched on (LLaMA-style attention; tables of the usual angles)
    "block-7B-rope": (4, 4096, 4096, 32, 11008, 1024, "rope"),
    # grouped-query attention, 8 key / value heads for 32 query heads (the extension of the section
    # "Discussion and Future Work": the K and V up-projections are 1024 wide instead of 4096)
    "block-7B-gqa8": (4, 4096, 4096, 32, 11008, 1024, "gqa8"),
}
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0
# Bytes per GEMM launch between L2 and the memory side, measured offline with rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE runs of this benchmark, each scaled by what the same counter reads for a
# plain 1 GiB copy (x2.000 and x1.000): profiles/gemm_bf16_block-7B_hbm_traffic.txt.  Counters cannot
# be read from inside this process, so workloads without such a measurement report null.
MEASURED_GEMM_TRAFFIC_BYTES = {"block-7B": 708.7e6}


def block_flops(B, S, d, H, f, r, dkv=None):
    """FLOPs = 2MNK per GEMM; attention counted causal-halved.  Returns a dict of the totals.
    dkv: width of k and v (grouped-query attention), d if None."""
    T = B * S
    dkv = d if dkv is None else dkv
    lin_fwd = 2.0 * T * (9 * d * r + 2 * dkv * r + 3 * f * r)
    attn_fwd = 2.0 * 2.0 * B * H * S * S * (d // H) / 2.0        # QK^T and PV, causal half
    model = 3.0 * lin_fwd + 3.5 * attn_fwd                       # bwd: 2x linear, 2.5x attention
    recompute_lin = 2.0 * T * r * (2 * d + 2 * dkv + 2 * f)      # six of the seven up-projections
    gemm_exec = 3.0 * lin_fwd + recompute_lin
    # attention as executed here: fwd, re-fwd, and a backward of 5 GEMM units against the 2 of the forward
    # (S, dP, dV, dK in one kernel that also leaves dS; dQ as one GEMM over it)
    attn_exec = attn_fwd * (1.0 + 1.0 + 2.5)
    return {"model": model, "gemm_exec": gemm_exec, "attn_exec": attn_exec, "exec": gemm_exec + attn_exec,
            "lin_fwd": lin_fwd, "attn_fwd": attn_fwd}


def gemm_classes(B, S, d, H, f, r, dkv=None):
    """Every GEMM launch class of one block step as (FLOPs, ideal bytes): 2MNK and one read of each
    operand plus one write of the result (bf16; weight gradients leave as fp32)."""
    T = B * S
    dkv = d if dkv is None else dkv
    out = []

    def g(M, N, K, count=1, out_bytes=2):
        out.append((count * 2.0 * M * N * K, count * (2.0 * (M * K + N * K) + out_bytes * M * N)))

    # (input width, output width, group size) of the four grouped low-rank layers: qkv, o, gate/up, down
    # members as (output width, how many)
    qkv = ((d, 3),) if dkv == d else ((d, 1), (dkv, 2))
    for d_in, members in ((d, qkv), (d, ((d, 1),)), (d, ((f, 2),)), (f, ((d, 1),))):
        G = sum(n for _, n in members)
        g(T, G * r, d_in)                 # forward: grouped down-projection
        for d_out, n in members:
            g(T, d_out, r, n)             # forward: batched up-projections
            g(T, r, d_out, n)             # backward: data gradient through the up-projections
            g(d_out, r, T, n, 4)          # backward: weight gradient of the up-projections
        g(T, d_in, G * r)                 # backward: data gradient through the down-projection
        g(G * r, d_in, T, 1, 4)           # backward: weight gradient of the down-projection
    for d_out, n in qkv + ((d, 1), (f, 2)):
        g(T, d_out, r, n)                 # re-forward from the rank-r checkpoints (all but the last layer)
    return out


def attainable_tflops(classes):
    """FLOP-weighted bound of the GEMM launches: each class at min(MFMA peak, A.I. x HBM peak)."""
    t = 0.0
    for fl, by in classes:
        bound = min(MFMA_BF16_PEAK_TFLOPS * 1e12, fl / by * HBM_PEAK_GBS * 1e9)
        t += fl / bound
    return sum(fl for fl, _ in classes) / t / 1e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="block-7B", choices=list(WORKLOADS))
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph after the warm-up and time replays of it")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the register-only MFMA rate measurement reported beside the roofline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ablation", action="store_true",
                    help="add an 'ablation' object: grouped / batched projections and the statistic taken "
                         "inside the GEMM against their separate forms (Table 3's compute rows, Sec. 5.3), "
                         "and the cost of the rank-r checkpoint recompute (Table 5), at 4096 and 16384 tokens")
    ap.add_argument("--chain-stat", action="store_true",
                    help="time the block as a middle block of a stack: the sum of squares of x arrives from the block "
                         "below (ckpt s1 pre-filled) and the one of y is emitted from the epilogue of the last GEMM")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (3 times), so that a hardware-counter "
                         "run of this command can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import synth_inputs as si
    from paper_2512_12131_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    Bn, S, d, H, f, r = WORKLOADS[args.workload][:6]
    variant = WORKLOADS[args.workload][6] if len(WORKLOADS[args.workload]) > 6 else "silu"
    act = B.LR_ACT_IDENTITY if variant in ("identity", "lax") else B.LR_ACT_SILU
    f_ld = si.pad_ld(f, 8)
    eps = 1e-5
    Hkv = 8 if variant == "gqa8" else None
    dkv = None if Hkv is None else Hkv * 128
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=0, Hkv=Hkv)
    rope = None
    if variant == "rope":
        ang = torch.arange(S, dtype=torch.float64)[:, None] * 10000.0 ** (-2.0 * torch.arange(64, dtype=torch.float64) / 128)
        rope = (torch.cos(ang).float().to(dev), torch.sin(ang).float().to(dev))
    chain = args.chain_stat
    sy = torch.empty((Bn * S,), dtype=torch.float32, device=dev) if chain else None
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=eps, act=act, rope=rope, stat_x_ready=chain, stat_y_out=sy,
                             n_kv_heads=Hkv or 0)
    params = {k: v.to(dev) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    x, dy = case["x"].to(dev), case["dy"].to(dev)
    ck = B.alloc_block_ckpt(desc, dev)
    if chain:   # what the block below would have left there
        ck["s1"].copy_(B.lr_rms_stat(x))
    y, dx = torch.empty_like(x), torch.empty_like(x)
    grads = {n: torch.zeros_like(params[n], dtype=torch.float32) for n in B.PARAM_NAMES}
    ws = torch.empty(max(B.lr_block_workspace_bytes(desc, 0), B.lr_block_workspace_bytes(desc, 1)),
                     dtype=torch.uint8, device=dev)

    if variant == "lax":
        shapes = {"qkv": 3 * r, "o": r, "gu": 2 * r, "d": r}
        h_prev = {n: si.gaussian(0, "h_prev_" + n, (Bn * S, w), std=0.5, dtype=torch.bfloat16).to(dev)
                  for n, w in shapes.items()}
        dz_next = {n: si.gaussian(0, "dz_next_" + n, (Bn * S, w), dtype=torch.bfloat16).to(dev) for n, w in shapes.items()}

        def step():
            B.lr_block_lax_fwd(desc, params, x, h_prev=h_prev, ckpt=ck, ws=ws, y=y)
            B.lr_block_lax_bwd(desc, params, x, dy, ck, h_prev=h_prev, dz_next=dz_next, grads=grads,
                               accumulate=False, ws=ws, dx=dx)
    else:
        def step():
            B.lr_block_fwd(desc, params, x, ckpt=ck, ws=ws, y=y)
            B.lr_block_bwd(desc, params, x, dy, ck, grads=grads, accumulate=False, ws=ws, dx=dx)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run = step
    if args.graph:
        # the step's launches recorded once into a HIP graph (the library only launches kernels on the
        # stream it is given), replayed per timed step: takes the host's launch cost out of small shapes
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / max(args.steps, 1)

    fl = block_flops(Bn, S, d, H, f, r, dkv)
    value = fl["exec"] / dt / 1e12

    # ---- roofline of the dominant kernel: gemm_bf16_kernel (all of the block's projection GEMMs,
    # forward, re-forward, data-gradient and weight-gradient launches).  The same K steps are run
    # again with the library's launch timer on: every GEMM launch is bracketed by HIP events on the
    # stream it runs on, and the summed intervals give the average launch duration.
    T = Bn * S
    B.lr_gemm_timer_begin(64 * max(args.steps, 1) + 64)
    for _ in range(args.steps):
        step()
    gemm_ms, gemm_launches = B.lr_gemm_timer_end()
    launches_per_step = gemm_launches / max(args.steps, 1)
    avg_launch_ms = gemm_ms / max(gemm_launches, 1)
    flops_per_launch = fl["gemm_exec"] / launches_per_step        # algorithmic FLOPs (2MNK) per launch
    achieved = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12
    classes = gemm_classes(Bn, S, d, H, f, r, dkv)
    assert abs(sum(c[0] for c in classes) - fl["gemm_exec"]) < 1e-6 * fl["gemm_exec"]
    attainable = attainable_tflops(classes)
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(args.workload), "traffic_unit": "bytes per launch (offline counters)",
                # each launch class at min(MFMA peak, arithmetic intensity x HBM peak), FLOP-weighted: what
                # the shapes of this workload allow (below the MFMA peak when the rank is small)
                "attainable": round(attainable, 1), "frac_of_attainable": round(achieved / attainable, 4),
                "kernel": "gemm_bf16_kernel (bf16 MFMA GEMM, all instantiations)",
                "launches_per_step": round(launches_per_step, 1), "avg_launch_us": round(avg_launch_ms * 1e3, 2),
                "gemm_ms_per_step": round(gemm_ms / max(args.steps, 1), 3),
                "gflop_per_launch": round(flops_per_launch / 1e9, 2)}
    # What the matrix pipes of THIS box sustain from registers alone with pseudo-random operands (no
    # memory traffic at all; the chip lowers its clock under matrix load): the ceiling an ideal GEMM
    # kernel would reach here.  `frac` above stays against the published peak.
    if not args.no_mfma_probe:
        sustained = B.lr_mfma_probe(True, 20000, 20)
        roofline["machine_sustained"] = round(sustained, 1)
        roofline["frac_of_machine_sustained"] = round(achieved / sustained, 4)

    # ---- the memory-bound kernels against the HBM peak (fp32 statistic / bf16 tensors >= 0.5 GB so that
    # the 256 MB last-level cache cannot hold them)
    def time_ms(fn, reps=5):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    Ts, fs = 32768, 11008
    g = torch.randn((Ts, fs), device=dev, dtype=torch.bfloat16)
    u = torch.randn((Ts, fs), device=dev, dtype=torch.bfloat16)
    nbytes = Ts * fs * 2
    stream_kernels = {}
    t = time_ms(lambda: B.lr_rms_stat(g))
    stream_kernels["lr_rms_stat"] = round(nbytes / t / 1e6, 1)
    t = time_ms(lambda: B.lr_swiglu_fwd(g, u))
    stream_kernels["lr_swiglu_fwd"] = round(3 * nbytes / t / 1e6, 1)
    dm = torch.randn((Ts, fs), device=dev, dtype=torch.bfloat16)
    t = time_ms(lambda: B.lr_swiglu_bwd(g, u, dm))             # reads g, u, dm; writes dg, du
    stream_kernels["lr_swiglu_bwd"] = round(5 * nbytes / t / 1e6, 1)
    del dm
    xs = g[:, :4096].contiguous()
    dxh = u[:, :4096].contiguous()
    dres = g[:, 4096:8192].contiguous()
    gam = torch.ones((4096,), device=dev, dtype=torch.bfloat16)
    st_ = B.lr_rms_stat(xs)
    t = time_ms(lambda: B.lr_rmsnorm_bwd(xs, gam, st_, eps, dxh, dres))   # reads x, dxhat, dres; writes dx
    stream_kernels["lr_rmsnorm_bwd"] = round(4 * Ts * 4096 * 2 / t / 1e6, 1)
    del g, u, xs, dxh, dres
    stream = {"unit": "GB/s", "peak": HBM_PEAK_GBS, "algorithmic_bytes_over_time": stream_kernels,
              "frac": {k: round(v / HBM_PEAK_GBS, 3) for k, v in stream_kernels.items()}}

    if args.ablation:
        out_abl = {}
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)

        def rnd(*shape, scale=1.0):
            return (torch.randn(shape, device=dev, generator=gen) * scale).to(torch.bfloat16)

        for Ta in (4096, 16384):
            xa = rnd(Ta, d)
            gam = torch.ones((d,), device=dev, dtype=torch.bfloat16)
            wd_cat = rnd(3 * r, d, scale=d ** -0.5)
            wu_st = rnd(3, d, r, scale=r ** -0.5)
            dys = rnd(3, Ta, d)
            # grouped down-projection + batched up-projections, statistic from the GEMM's A tiles
            zc, st_, ys = B.lr_group_fwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st)
            t_gf = time_ms(lambda: B.lr_group_fwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st))
            t_gb = time_ms(lambda: B.lr_group_bwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st, zc, st_, dys))
            # the same with the statistic from a separate pass over x
            t_2f = time_ms(lambda: B.lr_group_fwd(xa, gam, eps, B.LR_NORM_TWO_PASS, wd_cat, wu_st))
            # three separate low-rank layers on a pre-normalised input (norm kernels timed with them)
            stx = B.lr_rms_stat(xa)
            xh = B.lr_rmsnorm_apply(xa, gam, stx, eps)
            zs = [B.lr_linear_fwd(xh, wd_cat[i * r:(i + 1) * r], wu_st[i])[0] for i in range(3)]

            def sep_fwd():
                s_ = B.lr_rms_stat(xa)
                h_ = B.lr_rmsnorm_apply(xa, gam, s_, eps)
                for i in range(3):
                    B.lr_linear_fwd(h_, wd_cat[i * r:(i + 1) * r], wu_st[i])

            def sep_bwd():
                acc = None
                for i in range(3):
                    dxi = B.lr_linear_bwd(xh, wd_cat[i * r:(i + 1) * r], wu_st[i], zs[i], dys[i])[0]
                    acc = dxi if acc is None else acc.add_(dxi)
                B.lr_rmsnorm_bwd(xa, gam, stx, eps, acc)

            t_sf, t_sb = time_ms(sep_fwd), time_ms(sep_bwd)
            out_abl[f"T={Ta}"] = {"grouped_fwd_ms": round(t_gf, 4), "grouped_bwd_ms": round(t_gb, 4),
                                  "grouped_two_pass_stat_fwd_ms": round(t_2f, 4),
                                  "separate_fwd_ms": round(t_sf, 4), "separate_bwd_ms": round(t_sb, 4),
                                  "fwd_speedup": round(t_sf / t_gf, 3), "bwd_speedup": round(t_sb / t_gb, 3)}
            del xa, wd_cat, wu_st, dys, zc, ys, xh, zs
        # rank-r checkpointing: memory kept per block against every d- and d_ff-wide activation, and the
        # time of the re-forward it costs (forward minus the four down-projections that are not redone:
        # their outputs are the checkpoints)
        t_fwd = time_ms(lambda: B.lr_block_fwd(desc, params, x, ckpt=ck, ws=ws, y=y))
        t_bwd = time_ms(lambda: B.lr_block_bwd(desc, params, x, dy, ck, grads=grads, accumulate=False, ws=ws, dx=dx))
        kept = 7 * T * r * 2 + 2 * T * 4
        full = (T * d * 2) * 8 + (T * f * 2) * 3 + 7 * T * r * 2 * 2   # xhat1,q,k,v,o,h1,xhat2,(y) + g,u,m + z and sigma(z)
        out_abl["checkpoint"] = {"block_fwd_ms": round(t_fwd, 4), "block_bwd_ms": round(t_bwd, 4),
                                 "kept_MB": round(kept / 1e6, 1), "store_everything_MB": round(full / 1e6, 1),
                                 "delta_mem_MB": round((full - kept) / 1e6, 1)}
        ablation = out_abl
    else:
        ablation = None

    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "TFLOP/s + % MFMA bf16 peak, low-rank decoder block fwd+bwd (1 MI355X)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: low-rank decoder block fwd+bwd, batch {Bn}, seq {S}, d_model {d}, "
                               f"{H} heads of 128, ffn {f}, rank {r}, sigma {'identity' if act == B.LR_ACT_IDENTITY else 'SiLU'}"
                               f"{' + rank-r residual from the layer below (LaX)' if variant == 'lax' else ''}"
                               f"{', rotary embedding of q and k' if variant == 'rope' else ''}"
                               f"{', 8 key / value heads (grouped-query attention)' if variant == 'gqa8' else ''}, "
                               f"rank-r checkpoint recompute",
                   "launch": "hip graph replay" if args.graph else "eager",
                   "tokens": T, "executed_tflop": round(fl["exec"] / 1e12, 3),
                   "model_tflop": round(fl["model"] / 1e12, 3),
                   "frac_mfma_peak_executed": round(value / MFMA_BF16_PEAK_TFLOPS, 4),
                   "model_tflops": round(fl["model"] / dt / 1e12, 2)},
        "roofline": roofline,
        "hbm_bound_kernels": stream,
    }
    if ablation is not None:
        out["ablation"] = ablation

    if not args.no_cpu_baseline:
        # fp64 oracle on the host cores, bounded sample: forward + backward of the same block on the
        # first `s_len` tokens of batch element 0.
        import numpy as np
        from oracle import lowrank_oracle as orc
        s_len = S   # all of batch element 0: about 10 s of fp64 work at the 7B shape
        P = {k: si.f64(v) for k, v in case["params"].items()}
        X0, DY0 = si.f64(case["x"][:s_len]), si.f64(case["dy"][:s_len])
        if variant == "lax":
            from oracle import lax_oracle as lorc
            parts = {"qkv": "qkv", "o": "o", "gu": "gu", "d": "d"}
            hp, dzn = {}, {}
            for part, names in parts.items():
                for i, n in enumerate(names):
                    hp[n] = si.f64(h_prev[part][:s_len, i * r:(i + 1) * r].cpu())
                    dzn[n] = si.f64(dz_next[part][:s_len, i * r:(i + 1) * r].cpu())
        t0 = time.perf_counter()
        if variant == "lax":
            lorc.block_fwd(X0, P, hp, 1, s_len, H, 128, eps)
            lorc.block_bwd(X0, P, hp, DY0, dzn, 1, s_len, H, 128, eps)
        else:
            oact = orc.ACT_IDENTITY if act == B.LR_ACT_IDENTITY else orc.ACT_SILU
            orope = None if rope is None else (si.f64(rope[0].cpu()), si.f64(rope[1].cpu()))
            orc.block_fwd(X0, P, 1, s_len, H, 128, eps, act=oact, rope=orope, Hkv=Hkv)
            orc.block_bwd(X0, P, DY0, 1, s_len, H, 128, eps, act=oact, rope=orope, Hkv=Hkv)
        ct = time.perf_counter() - t0
        cfl = block_flops(1, s_len, d, H, f, r, dkv)
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
