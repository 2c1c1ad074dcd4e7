"""GPU parity at the sizes of the workload table."""
import numpy as np
import pytest

from oracle import mavg_oracle as O
from paper_2110_00625_amd import kavg, synth
from paper_2110_00625_amd.configs import TINY, META_ONLY
from tests.util import flat_error, worst_error

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def test_tiny_workload_all_rounds():
    """Tiny: P=4, K=4, B=32, MLP 3072-64-10, fp32, 20 meta rounds, free running."""
    torch = _torch()
    w = TINY
    data = synth.make_workload_inputs(w)
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, kavg.KAVG_FP32, index_seed=w.seeds["index"])
    g.set_data(torch.from_numpy(data["X32"]).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(data["w0"])
    o = O.MAvgOracle(w.P, w.K, w.lr, w.mu, w.dims, w.B, index_seed=w.seeds["index"])
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    worst = 0.0
    for r in range(w.rounds):
        g.local_steps()
        o.local_steps()
        g.meta_update()
        o.meta_update()
        e = worst_error(g.params(), o.params(), w.dims)
        worst = max(worst, e)
        assert e < 1e-4, "round %d: %.3g" % (r, e)
    assert np.array_equal(g.indices(), o.indices())
    first, last = o.losses()[0].mean(), None
    assert np.max(np.abs(g.losses() - o.losses())) < 1e-3
    print("tiny: worst relative error over %d rounds = %.3g" % (w.rounds, worst))
    g.close()


def test_meta_only_workload_full_size_200_passes():
    """P=64 replicas of an 11.2M-parameter fp32 vector, 200 fused passes; the oracle's
    meta step is elementwise, so the full vector is compared (not a sample)."""
    torch = _torch()
    w = META_ONLY
    n, P = w.flat_n, w.P
    inp = synth.make_meta_only_inputs(P, n, seed=w.seeds["data"])
    stride = (n + 63) // 64 * 64
    wt = torch.from_numpy(inp["w_tilde"]).cuda()
    v = torch.from_numpy(inp["v"]).cuda()
    reps = torch.empty((P, stride), device="cuda")
    reps[:, :n] = torch.from_numpy(inp["replicas"]).cuda()
    wo, vo = O.meta_step(inp["w_tilde"].astype(np.float64), inp["v"].astype(np.float64),
                         inp["replicas"].astype(np.float64), w.mu)
    v1 = vo.copy()
    kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
    torch.cuda.synchronize()
    assert flat_error(wt.cpu().numpy(), wo) < 1e-6
    assert flat_error(v.cpu().numpy(), vo) < 1e-5
    for k in range(2, w.rounds + 1):
        kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
        # the oracle's later passes: all replicas equal w~ (they were just rebroadcast)
        a = wo.copy()                       # mean of P copies of w~
        vo = w.mu * vo + (a - wo)
        wo = wo + vo
    torch.cuda.synchronize()
    got = wt.cpu().numpy()
    assert flat_error(got, wo) < 1e-4
    closed = inp["w_tilde"].astype(np.float64) + v1 * (1 - w.mu ** w.rounds) / (1 - w.mu)
    assert flat_error(got, closed) < 1e-4
    assert np.array_equal(reps[P - 1, :n].cpu().numpy(), got)
