"""DeTAG against the two baselines of the paper's Experiments section, and the
spectral-gap sweep of its second experiment, on synthetic non-identical shards:

    python -m paper_2006_08085_amd.compare_algorithms [--steps-quadratic 200]

First table: D-PSGD, DSGT (K = 1, eta = 0) and DeTAG on the least-squares
workload (8 workers on a ring, worker i's targets shifted by i) and on the
diagonal quadratic (16 workers on a ring, worker i's optimum shifted by i/16):
consensus distance ||X - 1 xbar^T||_F^2 and distance of the worker mean to the
optimum of the average objective after the run.  Second table: 16 workers on a
ring with the slack matrix W_kappa = kappa*W0 + (1-kappa)*I, kappa in
{1, 0.1, 0.05, 0.01}: consensus distance after 20 steps for D-PSGD, DSGT and
DeTAG with Theorem 3's phase length and Algorithm 3's momentum.
Everything runs through the library's entry points; one JSON line per table row.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

import paper_2006_08085_amd as D
from paper_2006_08085_amd import algorithms as ALG
from workloads import CONFIGS, generate as gen


def _lstsq(dev, T):
    cfg = CONFIGS[1]
    n, d, m, K = cfg.n, cfg.d, cfg.extra["m"], cfg.K
    A, b = gen.lstsq_problem(n, m, d, seed=cfg.seed, shift=cfg.extra["offset_shift"])
    Ad, bd = torch.from_numpy(A).to(dev), torch.from_numpy(b).to(dev)
    ctx = D.detag_create(D.Topology.ring(), n, d, d)
    # optimum of the average objective reachable from x0 = 0: the minimum-norm least-squares solution
    As, bs = A.reshape(n * m, d).astype(np.float64), b.reshape(n * m).astype(np.float64)
    xstar = np.linalg.lstsq(As, bs, rcond=None)[0]
    # D-PSGD diverges at the tracking methods' step size on this problem; 0.02 is the largest of {0.05, 0.02, 0.01} that converges
    lrs = {"dpsgd": 0.02, "dsgt": cfg.lr, "detag": cfg.lr}
    for alg in ("dpsgd", "dsgt", "detag"):
        X = D.new_matrix(n, d, d, device=dev)
        log = ALG.run(ctx, alg, lambda t, Xc, G: ctx.grad_lstsq(Xc, Ad, bd, G), X, lrs[alg], T, K=K, record_every=T)
        xbar = ctx.mean(X)[:d].double().cpu().numpy()
        yield {"workload": f"least squares, ring of {n}, d={d}, T={T}", "algorithm": alg, "K": K if alg == "detag" else 1,
               "lr": lrs[alg], "consensus_distance": log["consensus"][-1],
               "mean_to_optimum": float(np.linalg.norm(xbar - xstar) / np.linalg.norm(xstar))}


def _quadratic(dev, T, kappa=1.0, K=None, algorithms=("dpsgd", "dsgt", "detag")):
    cfg = CONFIGS[2]
    n, d, alpha, sigma = cfg.n, cfg.d, cfg.lr, cfg.sigma
    ld = D.padded_ld(d)
    h, b = gen.quadratic_problem(n, d, seed=cfg.seed, b_mean="i/n")
    hd = torch.zeros(ld); hd[:d] = torch.from_numpy(h); hd = hd.to(dev)
    bd = torch.zeros(n, ld); bd[:, :d] = torch.from_numpy(b); bd = bd.to(dev)
    ctx = D.detag_create(D.Topology.ring(kappa=kappa), n, d, ld)
    K = ctx.phase_length() if K is None else K                      # Theorem 3's phase length unless given
    xstar = b.astype(np.float64).mean(axis=0)                       # optimum of the average objective, column by column
    fast = h > 0.1                                                  # columns that converge within the run (alpha*h*T >> 1)
    for alg in algorithms:
        X = D.new_matrix(n, d, ld, device=dev)
        grad = lambda t, Xc, G: ctx.grad_quadratic_diag(Xc, hd, bd, G, sigma=sigma, seed=cfg.seed, step=t)
        log = ALG.run(ctx, alg, grad, X, alpha, T, K=K, record_every=T)
        xbar = ctx.mean(X)[:d].double().cpu().numpy()
        yield {"workload": f"diagonal quadratic, ring of {n}, kappa={kappa}, d={d}, T={T}, sigma={sigma}", "algorithm": alg,
               "K": K if alg == "detag" else 1, "eta": ctx.spectrum()["eta"] if alg == "detag" else 0.0, "lr": alpha,
               "consensus_distance": log["consensus"][-1],
               "mean_to_optimum_fast_columns": float(np.sqrt(np.mean((xbar[fast] - xstar[fast]) ** 2)))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps-lstsq", type=int, default=50)
    ap.add_argument("--steps-quadratic", type=int, default=200)
    ap.add_argument("--steps-sweep", type=int, default=20)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    for row in _lstsq(dev, args.steps_lstsq):
        print(json.dumps(row))
    for row in _quadratic(dev, args.steps_quadratic, K=CONFIGS[2].K):
        print(json.dumps(row))
    for kappa in (1.0, 0.1, 0.05, 0.01):
        for row in _quadratic(dev, args.steps_sweep, kappa=kappa):
            print(json.dumps(row))


if __name__ == "__main__":
    main()
