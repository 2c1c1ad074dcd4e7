"""Free-running GPU-vs-oracle error per meta round at a workload's full shape,
every learner walked by the oracle (minutes per round for the large ones, so
this is a report script, not a collected test).

  python tests/parity_report.py <workload> <rounds> [N] [--cpu-fp32] [--resync]

Prints, per learner, the replica error after the K local steps, and per round
the per-tensor and worst relative error of the global model after the meta step.

--resync starts every round of the GPU run from the oracle's state (global
model, momentum buffer, round counter), so each line is the error of one round.
--cpu-fp32 also walks a second CPU run whose only difference from the oracle
is that its matrix products accumulate in fp32 (numpy float32 matmul on the
same bf16-rounded operands) and prints how far THAT drifts from the oracle:
the yardstick for what two correct implementations of the mixed-precision
reading can agree on over many rounds.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from oracle import mavg_oracle as O                                    # noqa: E402
from paper_2110_00625_amd import kavg, synth                           # noqa: E402
from paper_2110_00625_amd.configs import WORKLOADS                     # noqa: E402
from tests.util import tensor_errors, worst_error                      # noqa: E402


def gradient_fp32_accumulate(w, dims, Xb, yb, bf16=False):
    """The oracle's minibatch gradient with every matrix product done by numpy in float32."""
    q = O.rne_bf16 if bf16 else (lambda x: x)
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    mm = lambda a, b: (f32(a) @ f32(b)).astype(np.float64)
    Ws, bs = O.unpack(w, dims)
    Wq = [(O.rna_bf16(W) if bf16 else W) for W in Ws]
    L = len(Ws)
    Zs, As = [], [Xb]
    for l in range(L):
        Z = mm(As[-1], Wq[l].T) + bs[l]
        Zs.append(Z)
        if l < L - 1:
            As.append(q(np.maximum(Z, 0.0)))
    loss, dZL = O.softmax_cross_entropy(Zs[-1], yb)
    dZ = q(dZL)
    pieces = [None] * L
    for l in range(L - 1, -1, -1):
        pieces[l] = np.concatenate([mm(dZ.T, As[l]).ravel(), dZ.sum(axis=0)])
        if l > 0:
            dZ = q(mm(dZ, Wq[l]) * (Zs[l - 1] > 0.0))
    return float(loss.mean()), np.concatenate(pieces)


def main():
    import torch
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    cpu_fp32 = "--cpu-fp32" in sys.argv
    resync = "--resync" in sys.argv
    name, rounds = args[0], int(args[1])
    w = WORKLOADS[name]
    N = int(args[2]) if len(args) > 2 else w.N
    bf = w.dtype == kavg.KAVG_BF16
    data = synth.make_workload_inputs(w, N=N)
    X = torch.from_numpy(data["Xbits"].view(np.int16) if bf else data["X32"]).cuda()
    y = torch.from_numpy(data["y"]).cuda()
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, w.dtype, index_seed=w.seeds["index"])
    g.set_data(X, y)
    g.set_params(data["w0"])
    o = O.MAvgOracle(w.P, w.K, w.lr, w.mu, w.dims, w.B, bf16=bf, index_seed=w.seeds["index"])
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    o32 = None
    if cpu_fp32:
        o32 = O.MAvgOracle(w.P, w.K, w.lr, w.mu, w.dims, w.B, bf16=bf, index_seed=w.seeds["index"])
        o32.set_data(data["X32"], data["y"])
        o32.set_params(data["w0"])
    for r in range(rounds):
        t = time.time()
        if resync:
            g.set_state(o.params().astype(np.float32), o.momentum().astype(np.float32), r)
        g.local_steps()
        for j in range(w.P):                       # learner by learner, so progress is visible
            o.local_steps(learners=[j])
            o.t0 -= w.K
            print("  round %d learner %d (%.0f s): replica error %.3g, last loss %.3f" % (
                r, j, time.time() - t, worst_error(g.replica(j), o.replica(j), w.dims),
                o.losses()[-1, j]), flush=True)
        o.t0 += w.K
        g.meta_update()
        o.meta_update()
        if o32 is not None:
            exact = O.minibatch_gradient
            O.minibatch_gradient = gradient_fp32_accumulate
            try:
                o32.local_steps()
            finally:
                O.minibatch_gradient = exact
            o32.meta_update()
            print("ROUND %d cpu fp32-accumulate run vs oracle: worst %.3g ; GPU vs that run: worst %.3g" % (
                r, worst_error(o32.params(), o.params(), w.dims), worst_error(g.params(), o32.params(), w.dims)),
                flush=True)
        errs = tensor_errors(g.params(), o.params(), w.dims)
        print("ROUND %d global model: %s worst %.3g" % (
            r, " ".join("%s=%.1e" % kv for kv in errs.items()),
            worst_error(g.params(), o.params(), w.dims)), flush=True)


if __name__ == "__main__":
    main()
