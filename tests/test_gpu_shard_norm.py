"""The feature-sharded RMSNorm + down-projection of Sec. 4.2 (Alg. 1, Eq. 5) on one GPU: every simulated
tensor-parallel rank runs the library's shard-local step on its d/TP slice (local statistic, local
normalisation, product with its weight rows, local scale undone), the test adds the partial products and
the local statistics (the exchange, which this build does not run) and the global rescale finishes it.
The result must equal the unsharded definition: against the fp64 oracle (two-pass RMSNorm then matmul, and
its own sharded form), against the library's unsharded grouped down-projection, and with the final two
steps done on the host instead of the GPU."""
import numpy as np
import pytest
import torch

import bf16_model as M
import synth_inputs as si
from oracle import lowrank_oracle as orc
from parity import check
from paper_2512_12131_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS = 1e-5


def _model(X, G, Wcat, k, eps):
    """The same steps in fp64 with one rounding to bf16 wherever a rank stores bf16 (the budget)."""
    T, d = X.shape
    dl = d // k
    hs, ss = [], []
    for i in range(k):
        xi, gi, wi = X[:, i * dl:(i + 1) * dl], G[i * dl:(i + 1) * dl], Wcat[:, i * dl:(i + 1) * dl]
        s = np.sum(xi * xi, axis=1)
        rms = np.sqrt(s / dl + eps)
        xh = M.bf16(xi * gi[None, :] / rms[:, None])
        hs.append(M.bf16((xh @ wi.T) * rms[:, None]))
        ss.append(s)
    h = M.bf16(sum(hs))
    return M.bf16(h / np.sqrt(sum(ss) / d + eps)[:, None])


@pytest.mark.parametrize("T,d,r,G,k", [(300, 512, 64, 3, 2), (1031, 1024, 128, 2, 4), (2048, 4096, 1024, 3, 8),
                                       (2048, 4096, 1024, 3, 4), (64, 256, 32, 1, 1)])
def test_sharded_down_projection_equals_unsharded(T, d, r, G, k):
    print(f"shard-local norm T={T} d={d} r={r} G={G} TP={k}", flush=True)
    case = si.group_case(T, d, r, 8, G, dtype=torch.bfloat16, seed=61)
    x, gamma = case["x"].to(DEV), case["gamma"].to(DEV)
    wcat = torch.cat(case["w_down"], dim=0).to(DEV)                      # [G*r, d]
    dl = d // k
    h_sum = torch.zeros((T, G * r), dtype=torch.float32, device=DEV)
    s_sum = torch.zeros((T,), dtype=torch.float32, device=DEV)
    X, GAM, W = si.f64(case["x"]), si.f64(case["gamma"]), si.f64(torch.cat(case["w_down"], dim=0))
    for i in range(k):
        sl = slice(i * dl, (i + 1) * dl)
        h_i, s_i = B.lr_shard_down_fwd(x[:, sl], gamma[sl].contiguous(), EPS, wcat[:, sl].contiguous())
        check(f"S_local[{i}]", s_i, np.sum(X[:, sl] ** 2, axis=1), torch.float32, scale=10)
        h_sum += h_i.float()
        s_sum += s_i
    z = B.lr_online_rmsnorm_finish(h_sum.to(torch.bfloat16), s_sum, d, EPS)
    torch.cuda.synchronize()
    # the definition: RMSNorm over the full width, then the full projection (Eq. 4 and 5)
    xhat, _ = orc.rmsnorm_fwd(X, GAM, EPS)
    z_ref = xhat @ W.T
    z_sharded_ref = orc.online_rmsnorm_sharded(X, GAM, W.T, k, EPS)
    assert np.max(np.abs(z_sharded_ref - z_ref)) < 1e-9 * np.max(np.abs(z_ref))
    bud = M.err2(_model(X, GAM, W, k, EPS), z_ref)
    check("z", z, z_ref, torch.bfloat16, bud)
    # the last two steps on the host, from the GPU's partial sums
    z_host = h_sum.double().cpu().numpy() / np.sqrt(s_sum.double().cpu().numpy() / d + EPS)[:, None]
    check("z (host finish)", z_host, z_ref, torch.bfloat16, bud)
    # and the library's unsharded grouped down-projection
    wu = torch.zeros((G, 8, r), dtype=torch.bfloat16, device=DEV)
    z_un, s_un, _ = B.lr_group_fwd(x, gamma, EPS, B.LR_NORM_ONLINE, wcat, wu)
    torch.cuda.synchronize()
    check("S_global", s_sum, s_un.double().cpu().numpy(), torch.float32, scale=10)
    check("z vs unsharded GPU", z, z_un.double().cpu().numpy(), torch.bfloat16, (2 * bud[0], 2 * bud[1]))
