#!/usr/bin/env python3
"""Side-by-side runs of Top-k (mu = 0) and RegTop-k on the HIP path.

    python -m paper_2501_05633_amd.demo toy
    python -m paper_2501_05633_amd.demo linreg [--S 0.6] [--mu 1.0] [--iters 2500] [--N 20] [--J 100]

`toy` replays the paper's two-worker logistic example ("Motivational Toy
Example"): Top-1 keeps sending the cancelling first entries and the model does
not move for about 100 iterations, RegTop-1 damps them after the first round.
`linreg` is the paper's linear-regression experiment as a closed loop (sparsified
round, then theta <- theta - eta * g): it prints the optimality gap
|theta - theta*| of the unsparsified run, Top-k, RegTop-k and the genie-aided
global Top-k, and how many of
the J entries all workers agree on (kept by all or dropped by all).
Everything the method computes runs in the library's kernels; torch only
produces the local gradients.
"""
from __future__ import annotations

import argparse
import math

import torch

from . import binding, workloads


def toy(iters: int = 120, mu: float = 1.0, eta: float = 0.9, device="cuda:0"):
    xs = torch.tensor([[100.0, 1.0], [-100.0, 1.0]], device=device)
    out = {}
    for name, m in (("Top-1", 0.0), ("RegTop-1", mu)):
        r = binding.RegTopk(2, 2, 1, m, device=device)
        theta = torch.tensor([0.0, 1.0], device=device)
        agg, first_move, risks = None, None, []
        for t in range(iters):
            z = torch.exp(-(xs @ theta))
            g = (-(z / (1 + z))[:, None] * xs).contiguous()
            risks.append(float(torch.log1p(z).mean()))
            idx, _, agg = r.step(g, agg)
            agg = agg.clone()
            if first_move is None and bool((agg != 0).any()):
                first_move = t
            binding.sgd_update(theta, agg, eta)
        r.close()
        out[name] = (first_move, risks)
        print("%-8s first non-zero aggregate at iteration %s; empirical risk after 1/10/100 iterations: %.4f %.4f %.4f"
              % (name, first_move, risks[1], risks[10], risks[min(100, iters - 1)]))
    return out


def linreg(S: float, mu: float, iters: int, N: int, J: int, device="cuda:0", every: int = 250, quiet=False,
           lowdim_seed=None):
    if lowdim_seed is None:
        wl = workloads.PaperLinReg(device, N=N, J=J, D=5 * J)
    else:           # the low-dimensional study of the appendix: sigma^2 = 1, gradient without the 2/D_n
        wl = workloads.PaperLinReg(device, N=N, J=J, D=5 * J, sigma2=1.0, normalised=False,
                                   seed=workloads.BASE_SEED + 200 + lowdim_seed)
    k = max(1, int(round(S * J)))
    runs = {"dense": (0.0, J), "Top-k": (0.0, k), "RegTop-k": (mu, k), "global Top-k": (None, k)}
    res = {}
    for name, (m, kk) in runs.items():
        r = binding.RegTopk(N, J, kk, 0.0 if m is None else m, device=device)
        theta = torch.zeros(J, device=device)
        agg, gaps, agree = None, [], []
        for t in range(iters):
            g = wl.grads(theta)
            _, _, agg = r.step_global(g) if m is None else r.step(g, agg)
            agg = agg.clone()
            binding.sgd_update(theta, agg, wl.eta)
            if t % every == every - 1 or t == iters - 1:
                ov = r.mask_overlap()
                gaps.append((t + 1, wl.gap(theta)))
                agree.append(int(ov[0] + ov[N]))
        r.close()
        res[name] = (gaps, agree)
    if not quiet:
        print("linear regression N=%d J=%d D_n=%d eta=%g S=%.2f (k=%d) mu=%g" % (N, J, 5 * J, wl.eta, S, k, mu))
        print("%8s %14s %14s %14s %14s   entries all workers agree on (Top-k / RegTop-k)" % (
            "iter", "gap dense", "gap Top-k", "gap RegTop-k", "gap global"))
        for i, (t, gd) in enumerate(res["dense"][0]):
            print("%8d %14.3e %14.3e %14.3e %14.3e   %d / %d" % (
                t, gd, res["Top-k"][0][i][1], res["RegTop-k"][0][i][1], res["global Top-k"][0][i][1],
                res["Top-k"][1][i], res["RegTop-k"][1][i]))
    return res


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("toy")
    t.add_argument("--iters", type=int, default=120)
    t.add_argument("--mu", type=float, default=1.0)
    l = sub.add_parser("linreg")
    l.add_argument("--S", type=float, default=0.6)
    l.add_argument("--mu", type=float, default=1.0)
    l.add_argument("--iters", type=int, default=2500)
    l.add_argument("--N", type=int, default=20)
    l.add_argument("--J", type=int, default=100)
    l.add_argument("--every", type=int, default=250, help="print the gaps every so many iterations")
    l.add_argument("--lowdim", type=int, default=None, metavar="SEED",
                   help="the appendix's low-dimensional study (use with --N 2 --J 4 --iters 60 --every 10): "
                        "sigma^2 = 1 and the gradient X^T(X theta - y) without the factor 2/D_n")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("demo: no GPU (the method runs only as HIP kernels)")
    if args.cmd == "toy":
        toy(args.iters, args.mu)
    else:
        linreg(args.S, args.mu, args.iters, args.N, args.J, every=args.every, lowdim_seed=args.lowdim)


if __name__ == "__main__":
    main()
