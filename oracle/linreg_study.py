"""The paper's N = 20 linear-regression experiment run on the CPU oracle alone
(section "Linear Regression Problem": figures "Optimality gap vs number of
iterations", "Homogeneity vs heterogeneity", "Optimality gap vs sparsity").

TEST INFRASTRUCTURE: imports only ``oracle.oracle`` and numpy.  ``run`` plays
the closed loop theta <- theta - eta * g for one (S, mu) point and returns the
optimality gap |theta - theta*| averaged over the last 50 iterations;
``python -m oracle.linreg_study`` sweeps mu over a logarithmic grid for the
sparsity factors of the figures and prints the tables quoted in the design
document.  The data generator follows the section's recipe: rows x ~ N(0, I_J),
ground truth t_n ~ N(u_n, h^2 I_J) with u_n ~ N(U, sigma^2), labels
y_n = X_n t_n + e_n, e_n ~ N(0, eps^2 I); local loss |X_n theta - y_n|^2 / D_n.
"""
from __future__ import annotations

import collections
import sys
import time

import numpy as np

N, J, D = 20, 100, 500          # workers, model size, data points per worker (the section's values)


def make_problem(seed, sigma2=5.0, h2=1.0, eps2=0.5, homogeneous=False):
    """Returns (A [N,J,J], b [N,J], theta_star): X_n^T X_n, X_n^T y_n and the closed-form optimum."""
    rng = np.random.default_rng(1000 + seed)
    X = rng.standard_normal((N, D, J))
    u = rng.normal(0.0, np.sqrt(sigma2), N)
    t = u[:, None] + np.sqrt(h2) * rng.standard_normal((N, J))
    if homogeneous:             # identical ground truths and no label noise
        t = np.repeat(t[:1], N, axis=0)
        eps2 = 0.0
    y = np.einsum("ndj,nj->nd", X, t) + np.sqrt(eps2) * rng.standard_normal((N, D))
    A = np.einsum("ndj,ndk->njk", X, X)
    b = np.einsum("ndj,nd->nj", X, y)
    star = np.linalg.solve(A.sum(0), b.sum(0))
    return A, b, star


def run(seed, S, mu, step_factor=None, homogeneous=False, sigma2=5.0, T=2500):
    """Gap after T iterations (mean over the last 50).  ``step_factor=None``: the
    gradient of the section's local loss, (2/D) X^T (X theta - y), at eta = 1e-2.
    A number f: the gradient without the factor 2/D, with eta scaled so that
    eta * (largest curvature) is f times that of the first case."""
    from oracle import oracle
    A, b, star = make_problem(seed, sigma2=sigma2, homogeneous=homogeneous)
    if step_factor is None:
        sc, eta = 2.0 / D, 1e-2
    else:
        sc, eta = 1.0, 1e-2 * (2.0 / D) * float(step_factor)
    k = int(round(S * J))
    o = oracle.Oracle(N, J, k, mu)
    theta = np.zeros(J, dtype=np.float32)
    agg = None
    A32 = (sc * A).astype(np.float32)
    b32 = (sc * b).astype(np.float32)
    gaps = []
    for it in range(T):
        g = np.einsum("njk,k->nj", A32, theta) - b32
        _, _, agg = o.step(g, agg)
        theta = oracle.sgd_update(theta, agg, eta)
        if it >= T - 50:
            gaps.append(np.linalg.norm(theta.astype(np.float64) - star))
    o.close()
    return float(np.mean(gaps))


def _job(args):
    return args, run(*args)


def main():
    from multiprocessing import Pool
    mus = [0.0] + [float(x) for x in np.round(10.0 ** np.arange(-3, 2.01, 1 / 3), 5)]
    jobs = []
    for seed in range(3):
        for S in (0.4, 0.5, 0.6, 0.9, 1.0):
            for mu in (mus if S < 1.0 else [0.0]):
                jobs.append((seed, S, mu, None, False, 5.0))
    for seed in range(2):
        for S in (0.6, 0.9):
            for mu in mus:
                for f in (10.0, 50.0):
                    jobs.append((seed, S, mu, f, False, 5.0))
        for mu in mus:
            jobs.append((seed, 0.6, mu, None, True, 5.0))
            jobs.append((seed, 0.6, mu, None, False, 2.0))
    t0 = time.time()
    res = collections.defaultdict(list)
    with Pool(6) as p:
        for (seed, S, mu, f, hom, s2), gap in p.imap_unordered(_job, jobs, chunksize=2):
            res[(f, hom, s2, S, mu)].append(gap)
    print("%d runs in %.0f s" % (len(jobs), time.time() - t0))
    for title, key in (("heterogeneous (sigma^2 = 5), section's gradient, eta = 1e-2", (None, False, 5.0)),
                       ("gradient without 2/D, step factor 10", (10.0, False, 5.0)),
                       ("gradient without 2/D, step factor 50", (50.0, False, 5.0)),
                       ("homogeneous", (None, True, 5.0)),
                       ("heterogeneous (sigma^2 = 2)", (None, False, 2.0))):
        Ss = sorted({k[3] for k in res if k[:3] == key})
        print("== " + title + "   (mean gap over the seeds; mu = 0 is plain Top-k, S = 1 no sparsification)")
        print("mu       " + " ".join("S=%.1f    " % S for S in Ss))
        for mu in mus:
            cells = []
            for S in Ss:
                v = res.get(key + (S, mu))
                cells.append("%.2e " % (sum(v) / len(v)) if v else "   -     ")
            print("%-8g " % mu + " ".join(cells))


if __name__ == "__main__":
    sys.exit(main())
