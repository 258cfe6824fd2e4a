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

from .binding import Context, Factors, DETAG_VARIANT_ATC
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


class ByPhase:
    """Algorithm 2 at the granularity it is printed in, on two HIP streams.

    Every iteration enqueues one step of accelerated gossip of the model replica and of the tracker on a
    communication stream, and B gradient queries at the phase-start model, each added to the gradient
    buffer, on the caller's current stream; the two streams meet at the end of a phase for the tracker and
    model update.  Nothing in a phase's gossip depends on that phase's gradients (they enter at the phase
    end), which is what lets the two run side by side - the paper's overlap of communication with
    computation, on one GPU.

    granularity = "iteration": one detag_gossip_round per matrix per iteration (2R launches a phase).
    granularity = "phase": the R steps of a phase as one on-chip K-round call per matrix, issued at the
    phase's first iteration (same arithmetic up to rounding order; needs has_fused()).
    overlap = False puts everything on the current stream.

    grad(t, q, X, g) must fill the fp32 n x ld device matrix g with every worker's gradient for query q of
    iteration t at its own row of X (the phase-start model; X is not modified during a phase).
    """

    def __init__(self, ctx: Context, X, alpha: float, grad: Callable, B: int = 1, scale: float = 1.0,
                 overlap: bool = True, granularity: str = "iteration"):
        import torch
        if granularity not in ("iteration", "phase"):
            raise ValueError("granularity must be 'iteration' or 'phase'")
        self.ctx, self.X, self.alpha, self.grad, self.B, self.scale = ctx, X, alpha, grad, B, scale
        self.granularity = granularity
        n, d, ld, dev = ctx.n, ctx.d, ctx.ld, X.device
        mk = lambda dt: new_matrix(n, d, ld, dtype=dt, device=dev)
        # z_r and z_{r-1} of the replica and of the tracker; a step writes over z_{r-1}
        self.xt = [X.clone(), mk(X.dtype)]
        self.y = [mk(X.dtype), mk(X.dtype)]
        self.G_k, self.G_km1, self.g = mk(torch.float32), mk(torch.float32), mk(torch.float32)
        self.comm = torch.cuda.Stream(dev) if overlap else None   # None: everything on the current stream
        self.t = 0           # iterations done
        self.k = 0           # phases done
        self.r = 0           # step within the current phase

    @property
    def Y(self):
        """The tracker (valid between phases)."""
        return self.y[0]

    def iteration(self, R: int, eta: float = -1.0):
        """One iteration of a phase of length R (the same R for all iterations of one phase)."""
        import torch
        ctx, r = self.ctx, self.r
        main = torch.cuda.current_stream(self.X.device)
        comm = self.comm if self.comm is not None else main
        if r == 0 and comm is not main:
            comm.wait_stream(main)                     # the last phase end produced Xt and Y
        with torch.cuda.stream(comm):
            if self.granularity == "phase":
                if r == 0:
                    ctx.gossip_accel(self.xt[0], R, eta)
                    ctx.gossip_accel(self.y[0], R, eta)
            else:
                for z in (self.xt, self.y):
                    ctx.gossip_round(z[0], z[0] if r == 0 else z[1], z[1], eta)
                    z[0], z[1] = z[1], z[0]
        for q in range(self.B):
            self.grad(self.t, q, self.X, self.g)
            ctx.accumulate(self.G_k, self.g, self.scale)
        self.t += 1
        self.r += 1
        if self.r == R:
            if comm is not main:
                main.wait_stream(comm)
            ctx.phase_end(self.X, self.xt[0], self.y[0], self.G_k, self.G_km1, self.alpha)
            self.G_k, self.G_km1 = self.G_km1, self.G_k
            self.r = 0
            self.k += 1

    def phase(self, R: int, eta: float = -1.0):
        if self.r != 0:
            raise RuntimeError("a phase is in progress")
        for _ in range(R):
            self.iteration(R, eta)

    def capture_two_phases(self, R: int, eta: float = -1.0):
        """Record two consecutive phases of length R into a HIP graph (two, because the gradient buffers and,
        for odd R, the gossip buffers change roles every phase and are back where they started after two).
        The graph fixes every pointer and scalar argument: grad must take whatever changes between
        iterations (batch indices, noise) from device buffers the caller refreshes between replays, and it is
        called here with the iteration numbers of the recorded phases.  Run at least two phases eagerly first
        so that every scratch buffer the library allocates on first use exists.  Returns the graph; call
        replay_two_phases(graph) to run it."""
        import torch
        if self.r != 0:
            raise RuntimeError("a phase is in progress")
        t0, k0 = self.t, self.k
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.phase(R, eta)
            self.phase(R, eta)
        self.t, self.k = t0, k0          # recording executes nothing
        self._graph_R = R
        return graph

    def replay_two_phases(self, graph):
        graph.replay()
        self.t += 2 * self._graph_R
        self.k += 2


def run_by_phase(ctx: Context, grad: Callable, X, alpha: float, T: int, R, eta=-1.0, B: int = 1,
                 scale: float = 1.0, overlap: bool = True, granularity: str = "iteration") -> ByPhase:
    """T iterations of Algorithm 2 in place on X.  R and eta are numbers or functions of the phase index
    (a phase length that starts at 1 - DSGT - and grows is the dynamic schedule the paper's supplementary
    material suggests).  An unfinished last phase leaves X at the last phase end.  Returns the ByPhase
    object (its .Y is the tracker, .k the number of completed phases)."""
    bp = ByPhase(ctx, X, alpha, grad, B=B, scale=scale, overlap=overlap, granularity=granularity)
    phase_len = R if callable(R) else (lambda k: R)
    phase_eta = eta if callable(eta) else (lambda k: eta)
    while bp.t < T:
        Rk, ek = int(phase_len(bp.k)), float(phase_eta(bp.k))
        for _ in range(min(Rk, T - bp.t)):
            bp.iteration(Rk, ek)
    return bp


def run_defacto(ctx: Context, factors: Factors, grad: Callable, X, alpha: float, T: int, B: int = 1,
                granularity: str = "iteration") -> int:
    """T iterations of Algorithm 1 (DeFacto) in place on X.  A round is 2R iterations, R = factors.R: R
    iterations of B gradient queries each at the round-start model, added to the gradient buffer; R iterations
    that multiply the model copy by the factors of the exact average consensus, one per iteration; then
    x <- copy - alpha * g / R.  grad(t, q, X, g) as in ByPhase.  An unfinished round leaves X at the last round
    end.  granularity = "round" issues the R communication iterations of a round as one
    detag_average_consensus call at the first of them (on chip for up to 256 workers).
    Returns the number of completed rounds."""
    if granularity not in ("iteration", "round"):
        raise ValueError("granularity must be 'iteration' or 'round'")
    import torch
    n, d, ld, dev, R = ctx.n, ctx.d, ctx.ld, X.device, factors.R
    G = new_matrix(n, d, ld, device=dev)
    g = new_matrix(n, d, ld, device=dev)
    xt = [X.clone(), new_matrix(n, d, ld, dtype=X.dtype, device=dev)]
    rounds = 0
    for t in range(T):
        r = t % (2 * R) if R else 0
        if r < R:
            for q in range(B):
                grad(t, q, X, g)
                ctx.accumulate(G, g, 1.0)
        elif granularity == "round":
            if r == R:
                factors.average(xt[0])
        else:
            factors.apply(r - R, xt[0], xt[1])
            xt[0], xt[1] = xt[1], xt[0]
        if r == 2 * R - 1:
            ctx.defacto_update(X, xt[0], G, alpha / R)
            rounds += 1
    return rounds
