"""Benchmark of the low-rank decoder-block hot path on one MI355X.

One "step" = lr_block_fwd + lr_block_bwd (all forward and backward rows of the hot path, with the
backward re-forwarding from the rank-r checkpoints) on one synthetic batch that is already resident
in HBM.  Prints ONE JSON line with the whole-job throughput in TFLOP/s (model FLOPs of the block's
forward + backward over wall time; the executed rate, which also counts the re-forward, beside it), a
roofline object for the dominant kernel class (the bf16 MFMA GEMMs, timed live with HIP events on the
stream they run on, in total and per launch class), the attention calls timed the same way, and the fp64
CPU oracle timed on a bounded sample.
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
    # the same at TP = 4, the degree the paper measures with (Sec. 5.1)
    "block-7B-btp4-shard": (4, 4096, 1024, 8, 2752, 1024),
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
MEASURED_GEMM_TRAFFIC_BYTES = {"block-7B": 733.0e6}


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


TAG_NAMES = {0: "store", 1: "down: row scale + sigma", 2: "up + residual", 3: "sigma' (+ row statistic)", 4: "RMSNorm backward",
             5: "weight gradient (k-major, split-K partials)", 6: "SwiGLU backward", 7: "SwiGLU forward", 8: "down (LaX)",
             9: "sigma' (LaX)", 10: "up + residual, fp32 copy out", 11: "up + fp32 residual", 12: "RMSNorm backward, fp32 copy out",
             13: "RMSNorm backward, fp32 residual", 32: "attention forward", 33: "attention backward"}


def gemm_launches(B, S, d, H, f, r, dkv=None, f_ld=None):
    """Every projection-GEMM launch of one block step (forward + backward with re-forward), as dicts:
    what, tag (epilogue class), M, N, K, batch as launched (ffn axis padded to f_ld), flops = 2MNK over the
    logical sizes, bytes = the traffic an ideal kernel has (each operand read once, every output written
    once, the auxiliary tiles an epilogue reads counted too; bf16 unless noted)."""
    T = B * S
    dkv = d if dkv is None else dkv
    f_ld = f if f_ld is None else f_ld
    out = []

    def g(what, tag, M, N, K, batch=1, aux=0.0, outs=None, n_log=None, k_log=None, m_log=None):
        n_l, k_l, m_l = n_log or N, k_log or K, m_log or M
        fl = batch * 2.0 * m_l * n_l * k_l
        by = batch * (2.0 * (m_l * k_l + n_l * k_l) + (2.0 * m_l * n_l if outs is None else outs)) + aux
        out.append({"what": what, "tag": tag, "M": M, "N": N, "K": K, "batch": batch, "flops": fl, "bytes": by})

    def up_qkv(what):                       # one batched launch, or q alone and {k, v} when k / v are narrower
        if dkv == d:
            g(what, 0, T, d, r, 3)
        else:
            g(what + " (q)", 0, T, d, r, 1)
            g(what + " (k, v)", 0, T, dkv, r, 2)

    def wg(what, M, N, m_log=None, n_log=None):      # weight gradient: reduces over the T tokens, fp32 result
        g(what, 5, M, N, T, 1, outs=4.0 * (m_log or M) * (n_log or N), m_log=m_log, n_log=n_log)

    Td = T * d
    # ---- forward ----
    g("fwd down q,k,v (grouped)", 1, T, 3 * r, d, outs=2 * 2.0 * T * 3 * r)          # z and sigma(z)
    up_qkv("fwd up q,k,v (batched)")
    g("fwd down o", 1, T, r, d, outs=2 * 2.0 * T * r)
    g("fwd up o + x, sum h1^2", 10, T, d, r, aux=2.0 * Td, outs=2.0 * Td + 4.0 * Td)
    g("fwd down gate,up (grouped)", 1, T, 2 * r, d, outs=2 * 2.0 * T * 2 * r)
    g("up gate", 0, T, f_ld, r, n_log=f)
    g("fwd up up-branch + SwiGLU", 7, T, f_ld, r, aux=2.0 * T * f, n_log=f)           # reads g, writes m only
    g("fwd down d", 1, T, r, f_ld, outs=2 * 2.0 * T * r, k_log=f)
    g("fwd up d + h1", 11, T, d, r, aux=4.0 * Td)
    # ---- backward ----
    wg("dW up d", d, r)
    g("dz d", 3, T, r, d, aux=2.0 * T * r)
    g("re-fwd up o + x", 2, T, d, r, aux=2.0 * Td)
    g("up gate", 0, T, f_ld, r, n_log=f)
    g("re-fwd up up-branch + SwiGLU", 7, T, f_ld, r, aux=2.0 * T * f, outs=2 * 2.0 * T * f, n_log=f)   # u and m
    wg("dW down d", r, f_ld, n_log=f)
    g("dm + SwiGLU backward", 6, T, f_ld, r, aux=2 * 2.0 * T * f, outs=2 * 2.0 * T * f, n_log=f)
    wg("dW up gate", f_ld, r, m_log=f)
    wg("dW up up-branch", f_ld, r, m_log=f)
    g("dz gate,up (batched)", 3, T, r, f_ld, 2, aux=2 * 2.0 * T * r, k_log=f)
    wg("dW down gate,up", 2 * r, d)
    g("dh1 (RMSNorm-2 backward + dy)", 12, T, d, 2 * r, aux=2 * 2.0 * Td, outs=2.0 * Td + 4.0 * Td)
    wg("dW up o", d, r)
    g("dz o", 3, T, r, d, aux=2.0 * T * r)
    up_qkv("re-fwd up q,k,v (batched)")
    wg("dW down o", r, d)
    g("dO", 0, T, d, r)
    wg("dW up q", d, r)
    wg("dW up k", dkv, r)
    wg("dW up v", dkv, r)
    if dkv == d:
        g("dz q,k,v (batched)", 3, T, r, d, 3, aux=3 * 2.0 * T * r)
    else:
        g("dz q", 3, T, r, d, 1, aux=2.0 * T * r)
        g("dz k,v (batched)", 3, T, r, dkv, 2, aux=2 * 2.0 * T * r)
    wg("dW down q,k,v", 3 * r, d)
    g("dx (RMSNorm-1 backward + dh1)", 13, T, d, 3 * r, aux=2.0 * Td + 4.0 * Td)
    return out


def gemm_classes(B, S, d, H, f, r, dkv=None):
    """(FLOPs, ideal bytes) of every projection-GEMM launch of a block step."""
    return [(c["flops"], c["bytes"]) for c in gemm_launches(B, S, d, H, f, r, dkv)]


def attainable_of(flops, nbytes):
    """min(MFMA peak, arithmetic intensity x HBM peak) in TFLOP/s."""
    return min(MFMA_BF16_PEAK_TFLOPS * 1e12, flops / nbytes * HBM_PEAK_GBS * 1e9) / 1e12


def attainable_tflops(classes):
    """FLOP-weighted bound of the GEMM launches: each class at min(MFMA peak, A.I. x HBM peak)."""
    t = sum(fl / (attainable_of(fl, by) * 1e12) for fl, by in classes)
    return sum(fl for fl, _ in classes) / t / 1e12


def per_class_report(records, launches, steps):
    """Joins the library's launch records (tag, M, N, K, batch, ms, flops) with the launch table: one line
    per distinct (tag, M, N, K, batch), with the logical FLOPs of the table (the padded ffn axis does no
    useful work), the measured average duration and the rate against the MFMA peak and against the class's
    own bound."""
    table = {}
    for c in launches:
        k = (c["tag"], c["M"], c["N"], c["K"], c["batch"])
        e = table.setdefault(k, {"what": [], "flops": 0.0, "bytes": 0.0, "n": 0})
        if c["what"] not in e["what"]:
            e["what"].append(c["what"])
        e["flops"] += c["flops"]; e["bytes"] += c["bytes"]; e["n"] += 1
    meas = {}
    for tag, M, N, K, batch, ms, fl in records:
        if tag >= 32:
            continue
        m = meas.setdefault((tag, M, N, K, batch), [0, 0.0])
        m[0] += 1; m[1] += ms
    rows = []
    for k, (n, ms) in sorted(meas.items(), key=lambda kv: -kv[1][1]):
        t = table.get(k)
        if t is None:      # a launch the table does not know (variant workloads): report it from the record alone
            fl1, by1, what = 2.0 * k[1] * k[2] * k[3] * k[4], None, ["(not in the launch table)"]
        else:
            fl1, by1, what = t["flops"] / t["n"], t["bytes"] / t["n"], t["what"]
        us = ms / n * 1e3
        tf = fl1 / (us * 1e-6) / 1e12
        row = {"class": TAG_NAMES.get(k[0], str(k[0])), "what": "; ".join(what), "tag": k[0], "M": k[1], "N": k[2],
               "K": k[3], "batch": k[4], "launches_per_step": round(n / steps, 2), "avg_us": round(us, 1),
               "ms_per_step": round(ms / steps, 3), "tflops": round(tf, 1), "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 3)}
        if by1:
            att = attainable_of(fl1, by1)
            row["attainable"] = round(att, 1)
            row["ideal_MB"] = round(by1 / 1e6, 1)
        rows.append(row)
    return rows


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
                    help="add an 'ablation' object: grouped / batched projections, fused SwiGLU and the norm "
                         "statistic against their separate forms (Table 3's compute rows, Sec. 5.3) at 4096 and "
                         "16384 tokens, and rank-r checkpointing against a backward that keeps every wide "
                         "activation (Table 5: memory saved, time added)")
    ap.add_argument("--stat-pass", action="store_true",
                    help="time the block as the bottom block of a stack: the sum of squares of x is taken by a pass "
                         "over x (Alg. 1's first step on its own) and none is emitted for y.  Default: a middle "
                         "block, whose statistic of x arrives from the epilogue of the block below (ckpt s1 "
                         "pre-filled) and which emits the one of y from the epilogue of its last GEMM")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="context only: also time the vendor library's bf16 GEMM (torch.matmul -> hipBLASLt) on the "
                         "block's projection shapes and report it beside the per-class rates; never on the product path")
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
    chain = not args.stat_pass
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
    # the same steps once more with an event between consecutive steps: the fastest single step beside the mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        run()
        marks[i + 1].record()
    torch.cuda.synchronize()
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]

    fl = block_flops(Bn, S, d, H, f, r, dkv)
    # headline: MODEL FLOPs over wall time (forward + backward of the block as defined; the re-forward from
    # the rank-r checkpoints and the second attention forward are overhead of the method, not useful work);
    # the executed-FLOPs rate is reported beside it
    value = fl["model"] / dt / 1e12
    value_exec = fl["exec"] / dt / 1e12

    # ---- roofline of the dominant kernel: gemm_bf16_kernel (all of the block's projection GEMMs,
    # forward, re-forward, data-gradient and weight-gradient launches).  The same K steps are run
    # again with the library's launch timer on: every GEMM launch is bracketed by HIP events on the
    # stream it runs on, and the summed intervals give the average launch duration.
    T = Bn * S
    B.lr_launch_timer_begin(80 * max(args.steps, 1) + 64)
    for _ in range(args.steps):
        step()
    records = B.lr_launch_timer_end()
    gemm_recs = [r for r in records if r[0] < 32]
    gemm_ms, gemm_launches_n = sum(r[5] for r in gemm_recs), len(gemm_recs)
    launches_per_step = gemm_launches_n / max(args.steps, 1)
    avg_launch_ms = gemm_ms / max(gemm_launches_n, 1)
    flops_per_launch = fl["gemm_exec"] / launches_per_step        # algorithmic FLOPs (2MNK) per launch
    achieved = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12
    launches = gemm_launches(Bn, S, d, H, f, r, dkv, f_ld)
    classes = [(c["flops"], c["bytes"]) for c in launches]
    assert abs(sum(c[0] for c in classes) - fl["gemm_exec"]) < 1e-6 * fl["gemm_exec"]
    attainable = attainable_tflops(classes)
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(args.workload), "traffic_unit": "bytes per launch (offline counters)",
                "algorithmic_bytes_per_launch": round(sum(c[1] for c in classes) / len(classes)),
                # each launch class at min(MFMA peak, arithmetic intensity x HBM peak), FLOP-weighted: what
                # the shapes of this workload allow (below the MFMA peak where an epilogue moves much data
                # or the rank is small)
                "attainable": round(attainable, 1), "frac_of_attainable": round(achieved / attainable, 4),
                "kernel": "gemm_bf16_kernel (bf16 MFMA GEMM, all instantiations)",
                "launches_per_step": round(launches_per_step, 1), "avg_launch_us": round(avg_launch_ms * 1e3, 2),
                "gemm_ms_per_step": round(gemm_ms / max(args.steps, 1), 3),
                "gflop_per_launch": round(flops_per_launch / 1e9, 2),
                "per_class": per_class_report(records, launches, max(args.steps, 1))}
    # attention beside it (not part of the GEMM figure): forward (run twice per step: forward and
    # re-forward) and backward, FLOPs causal-halved, from the same event timer
    attention = {}
    for tag, name in ((B.LR_TAG_ATTN_FWD, "fwd"), (B.LR_TAG_ATTN_BWD, "bwd")):
        rs = [r for r in records if r[0] == tag]
        if rs:
            us = sum(r[5] for r in rs) / len(rs) * 1e3
            tf = rs[0][6] / (us * 1e-6) / 1e12
            attention[name] = {"calls_per_step": round(len(rs) / max(args.steps, 1), 2), "avg_us": round(us, 1),
                               "tflops": round(tf, 1), "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 3)}
    attention["ms_per_step"] = round(sum(r[5] for r in records if r[0] >= 32) / max(args.steps, 1), 3)
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

        def group_vs_separate(Ta, G, d_out):
            """One concatenated down GEMM + one batched up launch (norm statistic inside) against G separate
            low-rank layers behind standalone norm kernels, forward and backward."""
            xa = rnd(Ta, d)
            gam = torch.ones((d,), device=dev, dtype=torch.bfloat16)
            wd_cat = rnd(G * r, d, scale=d ** -0.5)
            wu_st = rnd(G, d_out, r, scale=r ** -0.5)
            dys = rnd(G, Ta, d_out)
            zc, st_, ys = B.lr_group_fwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st)
            t_gf = time_ms(lambda: B.lr_group_fwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st))
            t_gb = time_ms(lambda: B.lr_group_bwd(xa, gam, eps, B.LR_NORM_ONLINE, wd_cat, wu_st, zc, st_, dys))
            # the same with the statistic and the normalisation as passes of their own
            t_2f = time_ms(lambda: B.lr_group_fwd(xa, gam, eps, B.LR_NORM_TWO_PASS, wd_cat, wu_st))
            # the statistic gathered from the A tiles inside the down-projection at this width (LR_NORM_ONLINE
            # takes the pass over x once the output is wider than 512 columns), and that pass alone
            t_ga = time_ms(lambda: B.lr_group_fwd(xa, gam, eps, B.LR_NORM_ONLINE_GATHER, wd_cat, wu_st))
            t_st = time_ms(lambda: B.lr_rms_stat(xa))
            stx = B.lr_rms_stat(xa)
            xh = B.lr_rmsnorm_apply(xa, gam, stx, eps)
            zs = [B.lr_linear_fwd(xh, wd_cat[i * r:(i + 1) * r], wu_st[i])[0] for i in range(G)]

            def sep_fwd():
                s_ = B.lr_rms_stat(xa)
                h_ = B.lr_rmsnorm_apply(xa, gam, s_, eps)
                for i in range(G):
                    B.lr_linear_fwd(h_, wd_cat[i * r:(i + 1) * r], wu_st[i])

            def sep_bwd():
                acc = None
                for i in range(G):
                    dxi = B.lr_linear_bwd(xh, wd_cat[i * r:(i + 1) * r], wu_st[i], zs[i], dys[i])[0]
                    acc = dxi if acc is None else acc.add_(dxi)
                B.lr_rmsnorm_bwd(xa, gam, stx, eps, acc)

            t_sf, t_sb = time_ms(sep_fwd), time_ms(sep_bwd)
            return {"grouped_fwd_ms": round(t_gf, 4), "grouped_bwd_ms": round(t_gb, 4),
                    "grouped_two_pass_norm_fwd_ms": round(t_2f, 4),
                    "grouped_fwd_statistic_gathered_in_gemm_ms": round(t_ga, 4), "statistic_pass_alone_ms": round(t_st, 4),
                    "separate_fwd_ms": round(t_sf, 4), "separate_bwd_ms": round(t_sb, 4),
                    "fwd_speedup": round(t_sf / t_gf, 3), "bwd_speedup": round(t_sb / t_gb, 3)}

        def launch_rows(Ta, recs, nsteps):
            """Table 3's compute rows taken launch by launch from the event timer of a block step at Ta tokens:
            each fused / grouped / batched launch against the separate launches it replaces (all of them
            launches this block really makes, at the same shapes)."""
            acc = {}
            for tag, M_, N_, K_, b_, ms, _ in recs:
                a = acc.setdefault((tag, M_, N_, K_, b_), [0, 0.0])
                a[0] += 1; a[1] += ms

            def us(tag, N_, K_, b_=1):
                n, ms = acc.get((tag, Ta, N_, K_, b_), (0, 0.0))
                return ms / n * 1e3 if n else None

            g = torch.randn((Ta, f_ld), device=dev, dtype=torch.bfloat16)
            u = torch.randn((Ta, f_ld), device=dev, dtype=torch.bfloat16)
            t_sf = time_ms(lambda: B.lr_swiglu_fwd(g, u)) * 1e3
            t_sb = time_ms(lambda: B.lr_swiglu_bwd(g, u, g)) * 1e3
            xs = torch.randn((Ta, d), device=dev, dtype=torch.bfloat16)
            t_stat = time_ms(lambda: B.lr_rms_stat(xs)) * 1e3
            rows = {}

            def row(name, fused, parts):
                if fused is None or any(p is None for p in parts):
                    return
                rows[name] = {"fused_us": round(fused, 1), "separate_us": round(sum(parts), 1),
                              "speedup": round(sum(parts) / fused, 3)}

            one_dn, one_up = us(1, r, d), us(0, d, r)           # a single down / up projection of the same shapes
            row("down q,k,v: one concatenated GEMM vs 3", us(1, 3 * r, d), [one_dn] * 3)
            row("down gate,up: one concatenated GEMM vs 2", us(1, 2 * r, d), [one_dn] * 2)
            row("up q,k,v: one batched launch vs 3", us(0, d, r, 3), [one_up] * 3)
            row("SwiGLU forward in the up-projection epilogue vs GEMM + streaming kernel", us(7, f_ld, r),
                [us(0, f_ld, r), t_sf])
            row("SwiGLU backward in the data-gradient epilogue vs GEMM + streaming kernel", us(6, f_ld, r),
                [us(0, f_ld, r), t_sb])
            up_plain, up_stat = us(2, d, r), us(10, d, r)
            if up_plain and up_stat:
                rows["sum of squares of h1: in the up-projection epilogue (with the fp32 copy of h1) vs a pass of its own"] = {
                    "epilogue_extra_us": round(up_stat - up_plain, 1), "separate_pass_us": round(t_stat, 1)}
            return rows

        out_abl["launches T=%d" % T] = launch_rows(T, records, max(args.steps, 1))
        for Ta in (4096, 16384):
            out_abl[f"qkv group T={Ta}"] = group_vs_separate(Ta, 3, d)
            out_abl[f"gate/up group T={Ta}"] = group_vs_separate(Ta, 2, f_ld)
        if Bn > 1 and variant == "silu":
            # the same block at one sequence (batch 1): the launch-by-launch rows where the GEMMs are smaller
            desc1 = B.make_block_desc(1, S, d, H, 128, f, f_ld, r, eps=eps, act=act)
            ck1 = B.alloc_block_ckpt(desc1, dev)
            x1, dy1, y1, dx1 = x[:S].contiguous(), dy[:S].contiguous(), torch.empty_like(x[:S]), torch.empty_like(x[:S])
            for _ in range(2):
                B.lr_block_fwd(desc1, params, x1, ckpt=ck1, ws=ws, y=y1)
                B.lr_block_bwd(desc1, params, x1, dy1, ck1, grads=grads, accumulate=False, ws=ws, dx=dx1)
            B.lr_launch_timer_begin(80 * 4 + 64)
            for _ in range(4):
                B.lr_block_fwd(desc1, params, x1, ckpt=ck1, ws=ws, y=y1)
                B.lr_block_bwd(desc1, params, x1, dy1, ck1, grads=grads, accumulate=False, ws=ws, dx=dx1)
            out_abl["launches T=%d" % S] = launch_rows(S, B.lr_launch_timer_end(), 4)
        # rank-r checkpointing against a backward that keeps every wide activation (Sec. 4.4, Table 5):
        # memory saved, time added, and their ratio
        if variant == "silu" or variant == "identity":
            sv = B.alloc_block_saved(desc, dev)
            ws2 = torch.empty(max(B.lib().lr_block_saved_workspace_bytes(desc, 0), B.lib().lr_block_saved_workspace_bytes(desc, 1)),
                              dtype=torch.uint8, device=dev)
            t_fwd = time_ms(lambda: B.lr_block_fwd(desc, params, x, ckpt=ck, ws=ws, y=y))
            t_bwd = time_ms(lambda: B.lr_block_bwd(desc, params, x, dy, ck, grads=grads, accumulate=False, ws=ws, dx=dx))
            t_fwd_s = time_ms(lambda: B.lr_block_fwd_save(desc, params, x, ckpt=ck, saved=sv, ws=ws2, y=y))
            t_bwd_s = time_ms(lambda: B.lr_block_bwd_saved(desc, params, x, dy, ck, sv, grads=grads, accumulate=False,
                                                           ws=ws2, dx=dx))
            kept = sum(v.numel() * v.element_size() for v in ck.values())
            wide = sum(v.numel() * v.element_size() for v in sv.values())
            plus = (t_fwd + t_bwd) - (t_fwd_s + t_bwd_s)
            out_abl["checkpoint"] = {"rank_r_fwd_ms": round(t_fwd, 4), "rank_r_bwd_ms": round(t_bwd, 4),
                                     "store_all_fwd_ms": round(t_fwd_s, 4), "store_all_bwd_ms": round(t_bwd_s, 4),
                                     "plus_time_ms": round(plus, 4), "plus_time_frac": round(plus / (t_fwd_s + t_bwd_s), 4),
                                     "rank_r_checkpoints_MB": round(kept / 1e6, 1),
                                     "wide_activations_MB": round(wide / 1e6, 1), "delta_mem_MB": round(wide / 1e6, 1),
                                     "eff_ckpt_MB_per_ms": round(wide / 1e6 / plus, 1) if plus > 0 else None}
            del sv, ws2
        ablation = out_abl
    else:
        ablation = None

    if args.vendor_gemm:
        # What the vendor's tuned GEMM reaches on this machine for the same products with a plain store (no fused
        # epilogue): context for the per-class figures, not a target the paper sets and not a path of this library.
        vend = []
        seen = set()
        for c in launches:
            key = (c["M"], c["N"], c["K"], c["tag"] == 5)
            if key in seen:
                continue
            seen.add(key)
            M_, N_, K_, tA = key
            if tA:     # weight gradient: both operands token-major, reduced over tokens
                a_ = torch.randn((K_, M_), device=dev, dtype=torch.bfloat16)
                b_ = torch.randn((K_, N_), device=dev, dtype=torch.bfloat16)
                fn = lambda: torch.matmul(a_.t(), b_)
            else:
                a_ = torch.randn((M_, K_), device=dev, dtype=torch.bfloat16)
                b_ = torch.randn((N_, K_), device=dev, dtype=torch.bfloat16)
                fn = lambda: torch.matmul(a_, b_.t())
            t = time_ms(fn, reps=10)
            tf = 2.0 * M_ * N_ * K_ / (t * 1e-3) / 1e12
            vend.append({"M": M_, "N": N_, "K": K_, "reduce_over_tokens": tA, "us": round(t * 1e3, 1),
                         "tflops": round(tf, 1), "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 3)})
            del a_, b_
        roofline["vendor_gemm_context"] = vend

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
        "ms_per_step": round(dt * 1e3, 4), "ms_per_step_min": round(min(step_ms), 4) if step_ms else None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: low-rank decoder block fwd+bwd, batch {Bn}, seq {S}, d_model {d}, "
                               f"{H} heads of 128, ffn {f}, rank {r}, sigma {'identity' if act == B.LR_ACT_IDENTITY else 'SiLU'}"
                               f"{' + rank-r residual from the layer below (LaX)' if variant == 'lax' else ''}"
                               f"{', rotary embedding of q and k' if variant == 'rope' else ''}"
                               f"{', 8 key / value heads (grouped-query attention)' if variant == 'gqa8' else ''}, "
                               f"rank-r checkpoint recompute",
                   "launch": "hip graph replay" if args.graph else "eager",
                   "norm1_statistic": ("handed over by the block below (stat_x_ready); this block emits the one of y from "
                                       "the epilogue of its last GEMM" if chain else
                                       "one pass over x (no GEMM of the block produces x); the one of h1 comes from the "
                                       "epilogue of the GEMM that produces h1"),
                   "tokens": T, "value_counts": "model FLOPs (2MNK of forward + backward, attention causal-halved); "
                                                "recompute not counted",
                   "model_tflop": round(fl["model"] / 1e12, 3), "executed_tflop": round(fl["exec"] / 1e12, 3),
                   "frac_mfma_peak_model": round(value / MFMA_BF16_PEAK_TFLOPS, 4),
                   "executed_tflops": round(value_exec, 2),
                   "frac_mfma_peak_executed": round(value_exec / MFMA_BF16_PEAK_TFLOPS, 4)},
        "roofline": roofline,
        "attention": attention,
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
