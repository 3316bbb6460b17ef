"""The block step under HIP graph capture: lr_block_fwd + lr_block_bwd recorded once into a graph (the
library launches kernels on the stream it is given and does nothing else: no allocation, no
synchronisation, no memset nodes), then replayed several times on changing inputs with eager work and
synchronisations between the replays; every replay must reproduce the eager result bit for bit."""
import pytest
import torch

import synth_inputs as si
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS = 1e-5


def _static_buffers(desc, packed, x):
    ck = B.alloc_block_ckpt(desc, x.device)
    grads = {n: torch.empty_like(packed[n], dtype=torch.float32) for n in B.PARAM_NAMES}
    ws_f = torch.empty(B.lr_block_workspace_bytes(desc, 0), dtype=torch.uint8, device=x.device)
    ws_b = torch.empty(B.lr_block_workspace_bytes(desc, 1), dtype=torch.uint8, device=x.device)
    return ck, grads, ws_f, ws_b, torch.empty_like(x), torch.empty_like(x)


@pytest.mark.parametrize("rope", [False, True])
def test_block_step_replays_from_a_graph(rope):
    Bn, S, H, f, r = 2, 320, 2, 344, 64
    d, f_ld = 128 * H, si.pad_ld(f, 8)
    print(f"graph capture of a block step B={Bn} S={S} d={d} f={f} r={r} rope={rope}", flush=True)
    case = si.block_case(Bn, S, d, H, 128, f, r, seed=5)
    tables = None
    if rope:
        pos = torch.arange(S, dtype=torch.float64)[:, None] * (10000.0 ** (-torch.arange(64, dtype=torch.float64) / 64))[None, :]
        tables = (torch.cos(pos).float().to(DEV).contiguous(), torch.sin(pos).float().to(DEV).contiguous())
    desc = B.make_block_desc(Bn, S, d, H, 128, f, f_ld, r, eps=EPS, rope=tables)
    packed = {k: v.to(DEV) for k, v in si.pack_block_params(case["params"], f, f_ld).items()}
    xs = [si.gaussian(5, f"x{i}", (Bn * S, d), std=1.0, dtype=torch.bfloat16).to(DEV) for i in range(3)]
    dys = [si.gaussian(5, f"dy{i}", (Bn * S, d), std=1.0, dtype=torch.bfloat16).to(DEV) for i in range(3)]

    # eager results (also the warm-up that sets the kernels' one-time attributes before any capture)
    eager = []
    for x, dy in zip(xs, dys):
        y, ck = B.lr_block_fwd(desc, packed, x)
        dx, g = B.lr_block_bwd(desc, packed, x, dy, ck)
        torch.cuda.synchronize()
        eager.append((y.clone(), dx.clone(), {k: v.clone() for k, v in g.items()}, ck["z_gu"].clone()))

    x_s, dy_s = torch.empty_like(xs[0]), torch.empty_like(dys[0])
    ck, grads, ws_f, ws_b, y_s, dx_s = _static_buffers(desc, packed, x_s)
    x_s.copy_(xs[0]); dy_s.copy_(dys[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.lr_block_fwd(desc, packed, x_s, ckpt=ck, ws=ws_f, y=y_s)
        B.lr_block_bwd(desc, packed, x_s, dy_s, ck, grads=grads, ws=ws_b, dx=dx_s)
    torch.cuda.synchronize()

    for rep in (0, 1, 2, 1, 0):
        x_s.copy_(xs[rep]); dy_s.copy_(dys[rep])
        for t in (y_s, dx_s, ck["z_gu"], *grads.values()):     # stale results must not pass for fresh ones
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        y_e, dx_e, g_e, zgu_e = eager[rep]
        assert torch.equal(y_s, y_e), f"y, replay of input {rep}"
        assert torch.equal(dx_s, dx_e), f"dx, replay of input {rep}"
        assert torch.equal(ck["z_gu"], zgu_e), f"z_gu, replay of input {rep}"
        for k in g_e:
            assert torch.equal(grads[k], g_e[k]), f"grad {k}, replay of input {rep}"
