"""TEST INFRASTRUCTURE ONLY — accelerated gossip, gradient tracking and one
DeTAG phase, in fp64, in the paper's order and notation.

State matrices are n x d, row i = worker i (the paper writes them d x n with
workers as columns; the gossip equation sums z_j * W[j, i] over neighbours j,
so with workers as rows one gossip step is W^T Z).
"""
from __future__ import annotations

import numpy as np

from .topology import neighbour_lists


def _gossip_once(Z: np.ndarray, nbrs) -> np.ndarray:
    """One gossip step (gossip equation, "Protocol Layer"):
    out_i = sum over j in N_i and j = i of Z_j * W[j, i]."""
    out = np.zeros_like(Z)
    for i, lst in enumerate(nbrs):
        for j, w in lst:
            out[i] += w * Z[j]
    return out


def accelerated_gossip(Z0: np.ndarray, W: np.ndarray, K: int, eta: float) -> np.ndarray:
    """K steps of accelerated gossip (Algorithm 3), every worker at once:
    z_{-1} = z_0;  z_{r+1} = (1+eta) * gossip(z_r) - eta * z_{r-1}."""
    nbrs = neighbour_lists(W)
    prev = np.array(Z0, dtype=np.float64)
    cur = prev.copy()
    for _ in range(K):
        new = (1.0 + eta) * _gossip_once(cur, nbrs) - eta * prev
        prev, cur = cur, new
    return cur


def tracking_update(Y, G_new, G_old) -> np.ndarray:
    """y <- y + g_(k) - g_(k-1)  (Algorithm 2, end-of-phase tracker update)."""
    return np.asarray(Y, np.float64) + np.asarray(G_new, np.float64) - np.asarray(G_old, np.float64)


def detag_step(X, Y, G_new, G_old, W, alpha: float, K: int, eta: float, variant: str = "atc"):
    """One DeTAG phase with phase length K, for all workers.

    "atc"  — the matrix form of the update analysed in the proof of Theorem 3:
             Y+ = M(Y + G_new - G_old),  X+ = M(X - alpha*Y),  M = K-step AG.
    "alg2" — Algorithm 2 as printed: gossip the model copy and the tracker for
             the K iterations of the phase, then x <- x~ - alpha*y with the
             gossiped tracker, then add the gradient difference to it.
    Returns (X+, Y+).  The caller then takes G_old <- G_new (Algorithm 2).
    """
    X = np.asarray(X, np.float64)
    Y = np.asarray(Y, np.float64)
    if variant == "atc":
        Xn = accelerated_gossip(X - alpha * Y, W, K, eta)
        Yn = accelerated_gossip(tracking_update(Y, G_new, G_old), W, K, eta)
    elif variant == "alg2":
        Xg = accelerated_gossip(X, W, K, eta)
        Yg = accelerated_gossip(Y, W, K, eta)
        Xn = Xg - alpha * Yg
        Yn = tracking_update(Yg, G_new, G_old)
    else:
        raise ValueError(variant)
    return Xn, Yn


def dpsgd_step(X, G, W, alpha: float) -> np.ndarray:
    """D-PSGD, the baseline of the Experiments section: one gossip step of the
    models minus the local gradient step, X+ = W^T X - alpha*G."""
    X = np.asarray(X, np.float64)
    return _gossip_once(X, neighbour_lists(W)) - alpha * np.asarray(G, np.float64)


def worker_mean(X) -> np.ndarray:
    """x_hat = (1/n) sum_i x_i  (output line of Algorithm 2)."""
    X = np.asarray(X, np.float64)
    return X.sum(axis=0) / X.shape[0]


def consensus_error(X) -> float:
    """|| X - 1 x_bar^T ||_F^2, the consensus distance the proof of Theorem 3
    bounds."""
    X = np.asarray(X, np.float64)
    dev = X - worker_mean(X)[None, :]
    return float((dev * dev).sum())
