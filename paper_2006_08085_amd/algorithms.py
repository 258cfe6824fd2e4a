"""Training loops over the C entry points: DeTAG and the two baselines the
paper's Experiments section compares it with.  Each loop only sequences
library calls (gradient query, phase, diagnostics); all arithmetic runs in the
kernels.

  detag : Algorithm 2 with phase length K and Algorithm 3's accelerated gossip
  dsgt  : the same with K = 1 and eta = 0 (gradient tracking with plain gossip,
          which the paper's discussion of DeTAG names as that special case)
  dpsgd : X <- W^T X - alpha*G, no tracker (Experiments section baseline)
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

from .binding import Context, DETAG_VARIANT_ATC
from .memory import new_matrix

ALGORITHMS = ("detag", "dsgt", "dpsgd")


def run(ctx: Context, algorithm: str, grad: Callable, X, alpha: float, T: int, K: int = 1, eta: float = -1.0,
        variant: int = DETAG_VARIANT_ATC, record_every: int = 0, Y=None) -> Dict[str, List[float]]:
    """Run T steps in place on X (n x ld device matrix of the context's state type).

    grad(t, X, G) must fill the fp32 n x ld device matrix G with every worker's
    stochastic gradient at its own row of X for step t.
    Y (tracker) is created as zeros unless given; together with a zero first
    G_old that is the initial condition of Algorithm 2.
    With record_every > 0 the consensus distance ||X - 1 xbar^T||_F^2 is read
    back every that many steps (one host synchronisation each time).
    Returns {"step": [...], "consensus": [...]}; the tracker is left in Y if given.
    """
    if algorithm not in ALGORITHMS:
        raise ValueError(f"algorithm must be one of {ALGORITHMS}")
    if algorithm == "dsgt":
        K, eta = 1, 0.0
    n, d, ld, dev = ctx.n, ctx.d, ctx.ld, X.device
    G_new, G_old = new_matrix(n, d, ld, device=dev), new_matrix(n, d, ld, device=dev)
    if Y is None and algorithm != "dpsgd":
        Y = new_matrix(n, d, ld, dtype=X.dtype, device=dev)
    log: Dict[str, List[float]] = {"step": [], "consensus": []}
    for t in range(T):
        grad(t, X, G_new)
        if algorithm == "dpsgd":
            ctx.dpsgd_step(X, G_new, alpha)
        else:
            ctx.step(X, Y, G_new, G_old, alpha, K, eta, variant)
            G_new, G_old = G_old, G_new
        if record_every and (t + 1) % record_every == 0:
            log["step"].append(t + 1)
            log["consensus"].append(float(ctx.consensus_error(X).item()))
    return log
