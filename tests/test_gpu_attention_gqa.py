"""GPU parity of causal grouped-query attention (lr_attention_gqa_fwd / _bwd through the C ABI) against
the fp64 oracle of oracle/gqa_oracle.py, element by element.  Shapes cover both backward forms (score
gradient kept and dQ as a GEMM: S a multiple of 8; the recomputing form otherwise), ragged tails against
the 128-query / 64-key / 256-row tiles, a single shared key / value head, and key / value rows wider
than their heads (a row stride the kernels must honour).  Tolerances as for the multi-head tests: the flat
bar plus the tensor's own storage rounding, and beyond that only what the bf16 model of the same data
flow shows (the probabilities are rounded before the P V product and o once more when stored; for the
first tokens of a sequence, the largest elements by far against the RMS over all tokens, both roundings
are of the size of the storage term)."""
import numpy as np
import pytest
import torch

import bf16_model as M
import synth_inputs as si
from oracle import gqa_oracle as gqa
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HD = 128

# B, S, H, Hkv, extra columns in the key / value rows
CASES = [(1, 1, 2, 1, 0), (2, 64, 4, 2, 0), (2, 192, 4, 2, 0), (1, 300, 4, 1, 0), (1, 776, 8, 2, 0), (2, 320, 6, 3, 64), (1, 1096, 2, 1, 0),
         (2, 333, 6, 2, 8)]


@pytest.mark.parametrize("Bn,S,H,Hkv,pad", CASES)
def test_attention_gqa_fwd_bwd(Bn, S, H, Hkv, pad):
    print(f"gqa attention B={Bn} S={S} H={H} Hkv={Hkv} kv row pad={pad}", flush=True)
    T, d, dkv = Bn * S, H * HD, Hkv * HD
    dt = torch.bfloat16
    q = si.gaussian(13, "q", (T, d), dtype=dt)
    k = si.gaussian(13, "k", (T, dkv), dtype=dt)
    v = si.gaussian(13, "v", (T, dkv), dtype=dt)
    do = si.gaussian(13, "do", (T, d), dtype=dt)

    def kv_dev(t):   # rows of dkv + pad elements, the heads in the first dkv columns
        buf = torch.full((T, dkv + pad), 7.0, dtype=dt, device=DEV)
        buf[:, :dkv] = t.to(DEV)
        return buf[:, :dkv]

    qd, dod = q.to(DEV), do.to(DEV)
    kd, vd = kv_dev(k), kv_dev(v)
    o, lse = B.lr_attention_gqa_fwd(qd, kd, vd, Bn, S, H, Hkv, HD)
    dq, dk, dv = B.lr_attention_gqa_bwd(qd, kd, vd, o, dod, lse, Bn, S, H, Hkv, HD)
    torch.cuda.synchronize()
    Q, K, V, DO = (si.f64(t) for t in (q, k, v, do))
    o_ref, lse_ref = gqa.attention_gqa_fwd(Q, K, V, Bn, S, H, Hkv, HD)
    dq_ref, dk_ref, dv_ref = gqa.attention_gqa_bwd(Q, K, V, DO, Bn, S, H, Hkv, HD)
    bud = M.attention_budget(Q, K, V, DO, Bn, S, H, Hkv, HD, o_ref, dq_ref, dk_ref, dv_ref)
    check("o", o, o_ref, dt, bud["o"])
    e = float(np.max(np.abs(lse.cpu().double().numpy() - lse_ref)))
    print(f"    lse max abs err {e:.3e}", flush=True)
    assert e < 2e-3
    check("dq", dq, dq_ref, dt, bud["dq"])
    check("dk", dk, dk_ref, dt, bud["dk"])
    check("dv", dv, dv_ref, dt, bud["dv"])
    # first token of every sequence attends only to itself: every query head returns its group's v_0
    grp = H // Hkv
    for b in range(Bn):
        for h in range(H):
            assert torch.equal(o[b * S, h * HD:(h + 1) * HD], vd[b * S, (h // grp) * HD:(h // grp + 1) * HD])


def test_gqa_with_all_heads_distinct_is_the_multi_head_call():
    """Hkv = H through the grouped-query entry points: bit-identical to lr_attention_fwd / _bwd."""
    Bn, S, H = 2, 264, 3
    T, d, dt = Bn * S, H * HD, torch.bfloat16
    q, k, v, do = (si.gaussian(14, n, (T, d), dtype=dt).to(DEV) for n in ("q", "k", "v", "do"))
    o0, lse0 = B.lr_attention_fwd(q, k, v, Bn, S, H, HD)
    g0 = B.lr_attention_bwd(q, k, v, o0, do, lse0, Bn, S, H, HD)
    o1, lse1 = B.lr_attention_gqa_fwd(q, k, v, Bn, S, H, H, HD)
    g1 = B.lr_attention_gqa_bwd(q, k, v, o1, do, lse1, Bn, S, H, H, HD)
    torch.cuda.synchronize()
    assert torch.equal(o0, o1) and torch.equal(lse0, lse1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)


def test_gqa_rejects_head_counts_that_do_not_divide():
    T, dt = 128, torch.bfloat16
    q = torch.zeros((T, 3 * HD), dtype=dt, device=DEV)
    kv = torch.zeros((T, 2 * HD), dtype=dt, device=DEV)
    with pytest.raises(B.LrError):
        B.lr_attention_gqa_fwd(q, kv, kv, 1, T, 3, 2, HD)


def test_attention_gqa_full_shape_sampled_group():
    """The attention shape of the 7B block with 8 key / value heads (B 4, S 4096, 32 query heads), in the
    launch configuration the benchmark times.  The oracle runs one group of one batch element (4 query
    heads over their shared key / value head: outputs of a group depend on nothing else) and is compared
    with those rows and columns of o, lse, dq, dk, dv."""
    Bn, S, H, Hkv = 4, 4096, 32, 8
    grp, T, dt = H // Hkv, Bn * S, torch.bfloat16
    print(f"gqa attention full shape B={Bn} S={S} H={H} Hkv={Hkv}, sampled group", flush=True)
    q = si.gaussian(15, "q", (T, H * HD), dtype=dt)
    k = si.gaussian(15, "k", (T, Hkv * HD), dtype=dt)
    v = si.gaussian(15, "v", (T, Hkv * HD), dtype=dt)
    do = si.gaussian(15, "do", (T, H * HD), dtype=dt)
    qd, kd, vd, dod = (t.to(DEV) for t in (q, k, v, do))
    o, lse = B.lr_attention_gqa_fwd(qd, kd, vd, Bn, S, H, Hkv, HD)
    dq, dk, dv = B.lr_attention_gqa_bwd(qd, kd, vd, o, dod, lse, Bn, S, H, Hkv, HD)
    torch.cuda.synchronize()
    b, g = 2, 5                                    # batch element, key / value head
    rows = slice(b * S, (b + 1) * S)
    qc = slice(g * grp * HD, (g + 1) * grp * HD)   # the group's query heads
    kc = slice(g * HD, (g + 1) * HD)
    Q, K, V, DO = si.f64(q[rows, qc]), si.f64(k[rows, kc]), si.f64(v[rows, kc]), si.f64(do[rows, qc])
    o_ref, lse_ref = gqa.attention_gqa_fwd(Q, K, V, 1, S, grp, 1, HD)
    dq_ref, dk_ref, dv_ref = gqa.attention_gqa_bwd(Q, K, V, DO, 1, S, grp, 1, HD)
    bud = M.attention_budget(Q, K, V, DO, 1, S, grp, 1, HD, o_ref, dq_ref, dk_ref, dv_ref, realisations=2)
    check("o", o[rows, qc], o_ref, dt, bud["o"])
    e = float(np.max(np.abs(lse[b, g * grp:(g + 1) * grp].cpu().double().numpy() - lse_ref[0])))
    print(f"    lse max abs err {e:.3e}", flush=True)
    assert e < 2e-3
    check("dq", dq[rows, qc], dq_ref, dt, bud["dq"])
    check("dk", dk[rows, kc], dk_ref, dt, bud["dk"])
    check("dv", dv[rows, kc], dv_ref, dt, bud["dv"])
