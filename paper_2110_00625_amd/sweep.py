"""K-AVG vs M-AVG sweep on a synthetic task: training-loss curves over a grid of
block momentum mu and learner count P at fixed (K, B, lr, rounds).

Looks at the qualitative statements of the paper on synthetic data:
  * mu = 0 is K-AVG (remark after Theorem 1); for small step sizes M-AVG gets to
    a given loss in fewer meta rounds (Lemma 2 compares N rounds of M-AVG with
    N / (1 - mu/2) rounds of K-AVG);
  * more learners tolerate / prefer a larger mu (Lemma 4, Section 4.2).
These are trends of upper bounds on another kind of model; the sweep reports
what happens, it does not assert anything.

Everything numerical runs in the HIP library (kavg.MAvg); this module only
loops over configurations and prints a table.

  python -m paper_2110_00625_amd.sweep --P 6 12 24 48 --mu 0 0.3 0.5 0.7 0.9
"""
import argparse
import json

import numpy as np

from . import kavg, synth


def run_one(torch, data, dims, P, K, B, lr, mu, rounds, dtype, seed, beta=0.0):
    """Mean minibatch loss (over the K steps and P learners) of every meta round."""
    bf = dtype == kavg.KAVG_BF16
    g = kavg.MAvg(P, K, lr, mu, dims, B, dtype, index_seed=seed)
    X = torch.from_numpy(data["Xbits"].view(np.int16) if bf else data["X32"]).cuda()
    g.set_data(X, torch.from_numpy(data["y"]).cuda())
    if beta > 0:
        g.set_learner_momentum(beta)
    g.set_params(data["w0"])
    curve = []
    for _ in range(rounds):
        g.local_steps()
        g.meta_update()
        curve.append(float(g.losses().mean()))
    g.close()
    return curve


def rounds_to_reach(curve, target):
    for i, v in enumerate(curve):
        if v <= target:
            return i + 1
    return None


def sweep(Ps, mus, K=4, B=32, lr=0.02, rounds=60, dims=(256, 256, 10), N=8192, bf16=False, seed=7,
          beta=0.0, quiet=False):
    import torch
    dtype = kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32
    data = synth.make_dataset(N, dims[0], dims[-1], bf16=bf16, seed_data=seed, seed_teacher=seed + 1,
                              teacher_hidden=64)
    data["w0"] = synth.he_normal_params(dims, seed + 2)
    out = {"K": K, "B": B, "lr": lr, "rounds": rounds, "dims": list(dims), "N": N, "bf16": bool(bf16),
           "learner_momentum": beta, "runs": []}
    for P in Ps:
        curves = {mu: run_one(torch, data, dims, P, K, B, lr, mu, rounds, dtype, seed + 3, beta) for mu in mus}
        base = curves[mus[0]]
        target = base[-1]                      # what the first mu (use 0 = K-AVG) reaches at the end
        for mu in mus:
            c = curves[mu]
            rec = {"P": P, "mu": mu, "final_loss": float(np.mean(c[-3:])), "best_loss": float(min(c)),
                   "rounds_to_first_mu_final": rounds_to_reach(c, target), "curve": c}
            out["runs"].append(rec)
            if not quiet:
                print("P=%3d mu=%.2f  final loss %.4f  best %.4f  rounds to reach %.4f: %s" % (
                    P, mu, rec["final_loss"], rec["best_loss"], target, rec["rounds_to_first_mu_final"]), flush=True)
    return out


def table(out):
    mus = sorted({r["mu"] for r in out["runs"]})
    Ps = sorted({r["P"] for r in out["runs"]})
    lines = ["| P \\\\ mu | " + " | ".join("%.2f" % m for m in mus) + " | best mu |", "|---|" + "---|" * (len(mus) + 1)]
    for P in Ps:
        row = {r["mu"]: r["final_loss"] for r in out["runs"] if r["P"] == P}
        finite = {m: v for m, v in row.items() if np.isfinite(v)}
        best = min(finite, key=finite.get) if finite else None
        lines.append("| %d | " % P + " | ".join("%.4f" % row[m] for m in mus) + " | %s |" % best)
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--P", type=int, nargs="+", default=[6, 12, 24, 48])
    ap.add_argument("--mu", type=float, nargs="+", default=[0.0, 0.3, 0.5, 0.7, 0.9])
    ap.add_argument("--K", type=int, default=4)
    ap.add_argument("--B", type=int, default=32)
    ap.add_argument("--lr", type=float, default=0.02)
    ap.add_argument("--rounds", type=int, default=60)
    ap.add_argument("--dims", type=int, nargs="+", default=[256, 256, 10])
    ap.add_argument("--N", type=int, default=8192)
    ap.add_argument("--bf16", action="store_true")
    ap.add_argument("--learner-momentum", type=float, default=0.0)
    ap.add_argument("--json", default=None, help="write curves and summary to this file")
    a = ap.parse_args()
    out = sweep(a.P, a.mu, a.K, a.B, a.lr, a.rounds, tuple(a.dims), a.N, a.bf16, beta=a.learner_momentum)
    print()
    print("final training loss (mean of the last 3 rounds), K=%d B=%d lr=%g, %d rounds:" % (a.K, a.B, a.lr, a.rounds))
    print(table(out))
    if a.json:
        with open(a.json, "w") as f:
            json.dump(out, f)


if __name__ == "__main__":
    main()
