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


def by_phase(grad, X0, W, alpha: float, T: int, R, eta, B: int = 1, scale: float = 1.0):
    """Algorithm 2 iteration by iteration, as printed.  Iteration t belongs to phase k and is step r of it.
    Every iteration performs one step of accelerated gossip (Algorithm 3's recursion, restarted with
    z_{-1} = z_0 at r = 0) on the model replica Xt and on the tracker Y, and B gradient queries at the
    phase-start model X_k, each added (times `scale`) to the gradient buffer g(k).  The last iteration of a
    phase sets X = Xt - alpha*Y with the gossiped tracker, then Y += g(k) - g(k-1), hands the buffer over
    and copies X into Xt.  T counts iterations; an unfinished last phase leaves X at the last phase end.

    grad(t, q, X) -> n x d gradient of query q (0 <= q < B) of iteration t at X.
    R: phase length, an int or a function k -> R_k (the dynamic phase length of the paper's
    "Techniques of Running DeTAG"); eta: a float or a function k -> eta_k.
    `scale` = 1 is the printed sum of the R*B gradients; 1/(R*B) their average, which is what the proof of
    Theorem 3 analyses.
    Returns (X, Y, phases) with phases the number of completed phases."""
    Wt = np.asarray(W, np.float64).T
    X = np.array(X0, np.float64)
    Xt = X.copy()
    Y = np.zeros_like(X)
    G_k = np.zeros_like(X)
    G_km1 = np.zeros_like(X)
    phase_len = R if callable(R) else (lambda k: R)
    phase_eta = eta if callable(eta) else (lambda k: eta)
    k, r = 0, 0
    Rk, ek = int(phase_len(0)), float(phase_eta(0))
    for t in range(T):
        if r == 0:
            Xt_prev, Y_prev = Xt, Y                  # z_{-1} = z_0
        Xt, Xt_prev = (1.0 + ek) * (Wt @ Xt) - ek * Xt_prev, Xt
        Y, Y_prev = (1.0 + ek) * (Wt @ Y) - ek * Y_prev, Y
        for q in range(B):
            G_k = G_k + scale * np.asarray(grad(t, q, X), np.float64)
        if r == Rk - 1:
            X = Xt - alpha * Y
            Y = Y + G_k - G_km1
            G_km1, G_k = G_k, np.zeros_like(X)
            Xt = X.copy()
            k, r = k + 1, 0
            Rk, ek = int(phase_len(k)), float(phase_eta(k))
        else:
            r += 1
    return X, Y, k
