"""TEST ORACLE - whole training runs (plain loops over oracle.gossip steps).

DeTAG (Algorithm 2 with Algorithm 3 as the gossip), and the two baselines of
the Experiments section: DSGT, which the paper identifies with phase length 1
and eta = 0, and D-PSGD.  fp64 throughout.  Test infrastructure only.
"""
from __future__ import annotations

import numpy as np

from .gossip import consensus_error, detag_step, dpsgd_step


def run(algorithm: str, grad, X0, W, alpha: float, T: int, K: int = 1, eta: float = 0.0, variant: str = "atc",
        record_every: int = 0):
    """grad(t, X) -> n x d gradient matrix at step t.  Starts from X0 with
    Y = 0 and G_old = 0 (initial condition of Algorithm 2).
    Returns (X, Y, log) with log = {"step": [...], "consensus": [...]}; Y is None for D-PSGD."""
    X = np.array(X0, np.float64)
    Y = np.zeros_like(X)
    G_old = np.zeros_like(X)
    if algorithm == "dsgt":
        K, eta = 1, 0.0
    elif algorithm not in ("detag", "dpsgd"):
        raise ValueError(algorithm)
    log = {"step": [], "consensus": []}
    for t in range(T):
        G_new = np.asarray(grad(t, X), np.float64)
        if algorithm == "dpsgd":
            X = dpsgd_step(X, G_new, W, alpha)
        else:
            X, Y = detag_step(X, Y, G_new, G_old, W, alpha, K, eta, variant)
            G_old = G_new
        if record_every and (t + 1) % record_every == 0:
            log["step"].append(t + 1)
            log["consensus"].append(consensus_error(X))
    return X, (None if algorithm == "dpsgd" else Y), log
