"""TEST INFRASTRUCTURE ONLY — gossip matrices, their spectrum, and eta (fp64).

Follows the paper's definition of the gossip matrix class W_n ("Protocol
Layer": doubly stochastic, non-zero only on edges of the graph and the
diagonal), of the general second-largest eigenvalue lambda = max(|l2|, |ln|)
given there, and of eta in Algorithm 3.
"""
from __future__ import annotations

import numpy as np


def _degrees(n: int, edges) -> np.ndarray:
    deg = np.zeros(n, dtype=np.int64)
    for a, b in edges:
        deg[a] += 1
        deg[b] += 1
    return deg


def mixing_matrix(n: int, edges, weights: str = "uniform") -> np.ndarray:
    """Dense symmetric n x n gossip matrix on an undirected simple graph.

    "uniform": every edge and every self-loop weighs 1/(deg+1); this is
    doubly stochastic only on a regular graph, anything else is rejected.
    "metropolis": edge {i,j} weighs 1/(1+max(deg_i,deg_j)) and the diagonal
    takes what is left of the row.  The paper names a "Metropolis method"
    (Experiments) without printing it; this is the reading taken here.  On a
    regular graph both rules give the same matrix.
    """
    W = np.zeros((n, n), dtype=np.float64)
    if n == 1:
        W[0, 0] = 1.0
        return W
    deg = _degrees(n, edges)
    if weights == "uniform":
        if not np.all(deg == deg[0]):
            raise ValueError("uniform weights need a regular graph")
        w = 1.0 / (deg[0] + 1.0)
        for a, b in edges:
            W[a, b] = W[b, a] = w
        for i in range(n):
            W[i, i] = w
    elif weights == "metropolis":
        for a, b in edges:
            W[a, b] = W[b, a] = 1.0 / (1.0 + max(deg[a], deg[b]))
        for i in range(n):
            W[i, i] = 1.0 - (W[i].sum() - W[i, i])
    else:
        raise ValueError(weights)
    return W


def slack(W0: np.ndarray, kappa: float) -> np.ndarray:
    """Slack matrix W_kappa = kappa*W0 + (1-kappa)*I (Experiments, second
    experiment): shrinks the spectral gap by the factor kappa."""
    return kappa * W0 + (1.0 - kappa) * np.eye(W0.shape[0])


def check_gossip_matrix(W: np.ndarray, edges=None, tol: float = 1e-9) -> None:
    """Membership in the class W_n: rows and columns sum to one, entries are
    non-negative, and (if an edge list is given) W_ij != 0 only on edges or
    the diagonal."""
    n = W.shape[0]
    if np.abs(W.sum(axis=0) - 1.0).max() > tol or np.abs(W.sum(axis=1) - 1.0).max() > tol:
        raise ValueError("not doubly stochastic")
    if W.min() < 0:
        raise ValueError("negative weight")
    if edges is not None:
        allowed = np.eye(n, dtype=bool)
        for a, b in edges:
            allowed[a, b] = allowed[b, a] = True
        if np.any((W != 0) & ~allowed):
            raise ValueError("weight off the graph")


def spectrum(W: np.ndarray):
    """(lambda_2, lambda_n, lambda) of a symmetric gossip matrix, where
    lambda_i is the i-th largest eigenvalue and lambda = max(|l2|, |ln|)
    ("Protocol Layer").  n = 1 has no second eigenvalue: all three are 0."""
    n = W.shape[0]
    if n == 1:
        return 0.0, 0.0, 0.0
    if np.abs(W - W.T).max() > 1e-12:
        raise ValueError("spectrum() needs a symmetric W")
    ev = np.sort(np.linalg.eigvalsh(W))[::-1]
    l2, ln = float(ev[1]), float(ev[-1])
    return l2, ln, max(abs(l2), abs(ln))


def eta_from_lambda(lam: float) -> float:
    """eta = (1 - sqrt(1-lambda^2)) / (1 + sqrt(1-lambda^2))  (Algorithm 3)."""
    s = np.sqrt(1.0 - lam * lam)
    return float((1.0 - s) / (1.0 + s))


def phase_length(lam: float, n: int, outer_ratio: float = 0.0) -> int:
    """Phase length suggested by Theorem 3: R = max(log(n)/2, log(r)/2) / sqrt(1 - lambda), with
    r = varsigma_0^2 T / (Delta L) (pass 0 to leave that term out), rounded up and at least 1."""
    lead = 0.5 * np.log(n)
    if outer_ratio > 0.0:
        lead = max(lead, 0.5 * np.log(outer_ratio))
    return max(1, int(np.ceil(lead / np.sqrt(1.0 - lam))))


def neighbour_lists(W: np.ndarray):
    """For every worker i the list of (j, W[j, i]) with W[j, i] != 0, self
    included — the terms of the sum in the gossip equation, which reads
    column i of W."""
    n = W.shape[0]
    return [[(j, float(W[j, i])) for j in range(n) if W[j, i] != 0.0] for i in range(n)]
