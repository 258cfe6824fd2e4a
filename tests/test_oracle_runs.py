"""Pins for oracle/runs.py and the two baselines (D-PSGD, DSGT): closed-form
fixed points on quadratics, and the qualitative ordering the Experiments
section reports on non-identically distributed shards."""
import numpy as np
import pytest

from oracle import gossip as G
from oracle import objectives as O
from oracle import runs as R
from oracle import topology as T
from workloads import generate as gen


def _asym(n=5):
    P = np.roll(np.eye(n), 1, axis=1)
    return 0.5 * np.eye(n) + 0.5 * P


def test_dpsgd_fixed_point_closed_form():
    """f_i(x) = h/2 (x - b_i)^2 per column: the D-PSGD map X -> W^T X - alpha*h*(X - b) is affine with fixed
    point x* = alpha*h (I - W^T + alpha*h I)^-1 b.  An asymmetric W tells W^T from W, the offsets the sign of
    the gradient step."""
    n, d, alpha = 5, 3, 0.2
    W = _asym(n)
    h = np.array([1.0, 0.5, 2.0])
    b = gen.state(n, d, 7).astype(np.float64)
    X, _, _ = R.run("dpsgd", lambda t, X: O.grad_quadratic_diag(X, h, b), np.zeros((n, d)), W, alpha, 600)
    for c in range(d):
        xs = alpha * h[c] * np.linalg.solve(np.eye(n) - W.T + alpha * h[c] * np.eye(n), b[:, c])
        assert np.allclose(X[:, c], xs, atol=1e-12)
        wrong = alpha * h[c] * np.linalg.solve(np.eye(n) - W + alpha * h[c] * np.eye(n), b[:, c])
        assert not np.allclose(xs, wrong, atol=1e-3)
    # the fixed point is not a consensus: the workers disagree for good
    assert G.consensus_error(X) > 1e-2
    # ... while its worker mean is right only because h is shared: mean(x*) = mean(b)
    assert np.allclose(X.mean(0), b.mean(0), atol=1e-12)


def test_dpsgd_mean_is_biased_with_heterogeneous_curvature():
    """Per-worker curvature h_i: the optimum of the average objective is sum(h_i b_i)/sum(h_i); the tracking
    methods reach it, D-PSGD with a constant step does not (its bias is what the Experiments section shows as
    a stalled loss)."""
    n, d, alpha = 8, 2, 0.1
    W = T.mixing_matrix(n, gen.edges_ring(n))
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    rng = np.random.default_rng(3)
    h = rng.uniform(0.2, 2.0, size=(n, d))
    b = rng.standard_normal((n, d)) + np.arange(n)[:, None]
    xopt = (h * b).sum(0) / h.sum(0)
    grad = lambda t, X: O.grad_quadratic_diag(X, h, b)
    Xp, _, _ = R.run("dpsgd", grad, np.zeros((n, d)), W, alpha, 4000)
    Xs, _, _ = R.run("dsgt", grad, np.zeros((n, d)), W, alpha, 4000)
    Xd, _, _ = R.run("detag", grad, np.zeros((n, d)), W, alpha, 1500, K=3, eta=eta)
    assert np.allclose(Xs, xopt[None], atol=1e-9)
    assert np.allclose(Xd, xopt[None], atol=1e-9)
    assert np.abs(Xp.mean(0) - xopt).max() > 1e-2


def test_run_is_the_step_loop():
    """runs.run sequences gradient, step and the G_old hand-over exactly as a hand-written loop does, and DSGT
    is the phase with K = 1, eta = 0."""
    n, d, alpha, K = 6, 4, 0.1, 3
    W = T.mixing_matrix(n, gen.edges_ring(n))
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    h, b = np.linspace(0.5, 1.5, d), gen.state(n, d, 5).astype(np.float64)
    grad = lambda t, X: O.grad_quadratic_diag(X, h, b) + 0.01 * (t + 1)
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Go = np.zeros((n, d))
    for t in range(7):
        Gn = grad(t, X)
        X, Y = G.detag_step(X, Y, Gn, Go, W, alpha, K, eta)
        Go = Gn
    Xr, Yr, log = R.run("detag", grad, np.zeros((n, d)), W, alpha, 7, K=K, eta=eta, record_every=7)
    assert np.array_equal(X, Xr) and np.array_equal(Y, Yr)
    assert log["step"] == [7] and log["consensus"][0] == G.consensus_error(X)
    Xa, Ya, _ = R.run("dsgt", grad, np.zeros((n, d)), W, alpha, 7, K=5, eta=0.9)
    Xb, Yb, _ = R.run("detag", grad, np.zeros((n, d)), W, alpha, 7, K=1, eta=0.0)
    assert np.array_equal(Xa, Xb) and np.array_equal(Ya, Yb)


def test_first_workload_ordering_of_the_three_algorithms():
    """n=8 ring least squares with offsets growing with the worker index (non-identical shards), lr 0.05, 50
    steps: DeTAG (K=4) ends with a far smaller consensus distance than DSGT, and D-PSGD with the largest; the
    loss at the worker mean orders the same way between D-PSGD and the tracking methods."""
    from workloads import CONFIGS
    cfg = CONFIGS[1]
    n, m, d = cfg.n, cfg.extra["m"], 256                      # same recipe, fewer columns to stay quick
    A, b = gen.lstsq_problem(n, m, d, seed=cfg.seed, shift=cfg.extra["offset_shift"])
    W = T.mixing_matrix(n, gen.edges_ring(n))
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    grad = lambda t, X: O.grad_lstsq(X, A, b)
    out = {a: R.run(a, grad, np.zeros((n, d)), W, cfg.lr, cfg.T, K=cfg.K, eta=eta) for a in ("detag", "dsgt", "dpsgd")}
    ce = {a: G.consensus_error(out[a][0]) for a in out}
    assert ce["detag"] < 1e-3 * ce["dsgt"]
    assert ce["dsgt"] < 1e-2 * ce["dpsgd"]
    loss = lambda x: 0.5 * np.mean([np.sum((A[i].astype(np.float64) @ x - b[i]) ** 2) for i in range(n)])
    assert loss(out["detag"][0].mean(0)) < loss(out["dpsgd"][0].mean(0))


def _golden_hyper(golden_dir):
    import os
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "paper_detag_hyperparameters.txt"))
            if ln.strip() and not ln.startswith("#")]
    return {float(k): (float(e), int(r)) for k, e, r in rows}


def test_spectral_gap_sweep_on_the_quadratic(golden_dir):
    """Second experiment of the paper on the synthetic quadratic: ring-16, W_kappa, lr 0.5.  With Algorithm 3's
    eta and Theorem 3's phase length DeTAG holds its consensus distance (within a small factor) at every kappa (the number of
    rounds per phase grows as 1/sqrt(gap)); DSGT and D-PSGD get worse as the gap closes; DeTAG with the
    (eta, R) pairs the paper tuned sits between; at kappa = 1 that pair is (0, 1), i.e. DSGT itself."""
    from oracle import noise as ON
    from workloads import CONFIGS
    cfg = CONFIGS[2]
    n, d, T_steps = cfg.n, 600, 40
    h, b = gen.quadratic_problem(n, d, seed=cfg.seed, b_mean="i/n")
    noise = [ON.normal_noise(cfg.seed, t, n, np.arange(d)) for t in range(T_steps)]
    grad = lambda t, X: O.grad_quadratic_diag(X, h, b, noise[t], cfg.sigma)
    W0 = T.mixing_matrix(n, gen.edges_ring(n))
    tuned = _golden_hyper(golden_dir)
    ce = {}
    for kappa in (1.0, 0.1, 0.05, 0.01):
        W = T.slack(W0, kappa)
        lam = T.spectrum(W)[2]
        settings = {"dpsgd": ("dpsgd", 1, 0.0), "dsgt": ("dsgt", 1, 0.0),
                    "tuned": ("detag", tuned[kappa][1], tuned[kappa][0]),
                    "theory": ("detag", T.phase_length(lam, n), T.eta_from_lambda(lam))}
        for name, (alg, K, eta) in settings.items():
            X, _, _ = R.run(alg, grad, np.zeros((n, d)), W, cfg.lr, T_steps, K=K, eta=eta)
            ce[kappa, name] = G.consensus_error(X)
        assert ce[kappa, "theory"] < 1e-2 * ce[kappa, "dsgt"]
        assert ce[kappa, "tuned"] <= ce[kappa, "dsgt"] < ce[kappa, "dpsgd"]
    assert ce[1.0, "tuned"] == ce[1.0, "dsgt"]
    theory = [ce[k, "theory"] for k in (1.0, 0.1, 0.05, 0.01)]
    assert max(theory) < 5 * min(theory)                      # flat to a small factor, against > 20x for DSGT
    for name in ("dsgt", "dpsgd"):
        seq = [ce[k, name] for k in (1.0, 0.1, 0.05, 0.01)]
        assert all(a < b_ for a, b_ in zip(seq, seq[1:]))
    assert ce[0.01, "dsgt"] > 20 * ce[1.0, "dsgt"]


def test_by_phase_form_is_the_phase_form_with_summed_queries():
    """Algorithm 2 run iteration by iteration (one gossip step and B gradient queries per iteration) ends every
    phase exactly where the phase-at-a-time step lands when it is given the sum of that phase's R*B gradients
    - two separately written routes through the same algorithm (this one uses dense W^T products and explicit
    recursion state, the other the neighbour lists)."""
    n, d, alpha, Rlen, B = 6, 5, 0.07, 3, 2
    W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)          # asymmetric
    eta = 0.3
    h, b = np.linspace(0.5, 1.5, d), gen.state(n, d, 5).astype(np.float64)
    rng = np.random.default_rng(0)
    noise = rng.standard_normal((4 * Rlen, B, n, d))
    g = lambda t, q, X: O.grad_quadratic_diag(X, h, b) + 0.1 * noise[t, q]
    Xb, Yb, phases = R.by_phase(g, np.zeros((n, d)), W, alpha, 4 * Rlen, Rlen, eta, B=B)
    assert phases == 4
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Go = np.zeros((n, d))
    for k in range(4):
        Gn = sum(g(k * Rlen + r, q, X) for r in range(Rlen) for q in range(B))
        X, Y = G.detag_step(X, Y, Gn, Go, W, alpha, Rlen, eta, "alg2")
        Go = Gn
    assert np.allclose(Xb, X, atol=1e-13) and np.allclose(Yb, Y, atol=1e-13)
    # the tracker's mean is the mean of the last completed buffer; iterations of an unfinished phase change nothing
    assert np.allclose(Yb.mean(0), Go.mean(0), atol=1e-13)
    Xc, _, ph = R.by_phase(g, np.zeros((n, d)), W, alpha, 4 * Rlen - 1, Rlen, eta, B=B)
    Xd, _, _ = R.by_phase(g, np.zeros((n, d)), W, alpha, 3 * Rlen, Rlen, eta, B=B)
    assert ph == 3 and np.array_equal(Xc, Xd)


def test_dynamic_phase_length_starts_as_dsgt():
    """Phase length 1 with eta = 0 for the first phases is DSGT (in the printed, gossip-then-correct order);
    afterwards the longer phases take over from that state."""
    n, d, alpha = 6, 4, 0.1
    W = T.mixing_matrix(n, gen.edges_ring(n))
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    h, b = np.linspace(0.5, 1.5, d), gen.state(n, d, 5).astype(np.float64)
    g = lambda t, q, X: O.grad_quadratic_diag(X, h, b)
    sched_R = lambda k: 1 if k < 5 else 3
    sched_eta = lambda k: 0.0 if k < 5 else eta
    Xa, Ya, ph = R.by_phase(g, np.zeros((n, d)), W, alpha, 5 + 3 * 4, sched_R, sched_eta)
    assert ph == 9
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Go = np.zeros((n, d))
    for k in range(9):
        Rk = sched_R(k)
        Gn = Rk * g(0, 0, X)
        X, Y = G.detag_step(X, Y, Gn, Go, W, alpha, Rk, sched_eta(k), "alg2")
        Go = Gn
    assert np.allclose(Xa, X, atol=1e-13) and np.allclose(Ya, Y, atol=1e-13)
