"""Pins for oracle/gossip.py: invariants the paper states, brute-force dense
evaluation on tiny n, the exact per-eigendirection contraction, special cases,
and closed-form behaviour on quadratics."""
import numpy as np
import pytest

from oracle import gossip as G
from oracle import objectives as O
from oracle import topology as T
from workloads import generate as gen


def _ring(n):
    return T.mixing_matrix(n, gen.edges_ring(n))


def _asym(n=5):
    P = np.roll(np.eye(n), 1, axis=1)            # cyclic permutation, P[i, i+1] = 1
    return 0.5 * np.eye(n) + 0.5 * P             # doubly stochastic, not symmetric


def _poly(mu, K, eta):
    """p_K(mu): the scalar the K-step recursion multiplies an eigen-direction by."""
    prev = np.ones_like(mu)
    cur = np.ones_like(mu)
    for _ in range(K):
        prev, cur = cur, (1 + eta) * mu * cur - eta * prev
    return cur


# ---- accelerated gossip ---------------------------------------------------
@pytest.mark.parametrize("K", [0, 1, 2, 5, 9])
@pytest.mark.parametrize("eta", [0.0, 0.25, 0.7])
def test_mean_is_preserved(K, eta):
    """W doubly stochastic => M(X) 1/n = X 1/n (property of accelerated
    gossip stated in the proof of Theorem 3)."""
    for W in (_ring(7), _asym(5), T.mixing_matrix(64, gen.edges_torus(8, 8))):
        Z = gen.state(W.shape[0], 13, seed=K).astype(np.float64)
        out = G.accelerated_gossip(Z, W, K, eta)
        assert np.allclose(out.mean(0), Z.mean(0), rtol=0, atol=1e-13)


@pytest.mark.parametrize("n", [3, 4, 5, 8])
@pytest.mark.parametrize("K", [1, 2, 3, 6])
def test_equals_dense_recursion(n, K):
    """Explicit dense evaluation of z_{r+1} = (1+eta) W^T z_r - eta z_{r-1}."""
    eta = 0.37
    for W in (_ring(n), _asym(n)):
        Z = gen.state(n, 6, seed=n * 10 + K).astype(np.float64)
        prev, cur = Z.copy(), Z.copy()
        for _ in range(K):
            prev, cur = cur, (1 + eta) * (W.T @ cur) - eta * prev
        assert np.allclose(G.accelerated_gossip(Z, W, K, eta), cur, rtol=0, atol=1e-13)


def test_transpose_matters_on_asymmetric_W():
    """z_i <- sum_j z_j W[j,i] reads column i of W: with workers as rows the
    operator is W^T Z, and an asymmetric W tells it from W Z."""
    W = _asym(5)
    Z = gen.state(5, 4, seed=1).astype(np.float64)
    one = G.accelerated_gossip(Z, W, 1, 0.0)
    assert np.allclose(one, W.T @ Z, atol=1e-14)
    assert not np.allclose(one, W @ Z, atol=1e-3)
    # worker 1 averages itself with worker 0 (W[0,1] = 1/2), not with worker 2
    assert np.allclose(one[1], 0.5 * Z[1] + 0.5 * Z[0], atol=1e-14)


@pytest.mark.parametrize("n,K", [(8, 4), (16, 6), (32, 8)])
def test_eigendirection_polynomial_and_exact_contraction(n, K):
    """Symmetric W: on the eigenvector of eigenvalue mu the K-step operator
    multiplies by p_K(mu), p_{r+1} = (1+eta) mu p_r - eta p_{r-1}, p_0=p_{-1}=1."""
    W = _ring(n)
    _, _, lam = T.spectrum(W)
    eta = T.eta_from_lambda(lam)
    mu, V = np.linalg.eigh(W)
    out = G.accelerated_gossip(V, W, K, eta)           # columns of V are eigenvectors
    assert np.allclose(out, V * _poly(mu, K, eta)[None, :], atol=1e-12)
    # p_K(1) = 1 (the consensus direction is untouched)
    assert _poly(np.array([1.0]), K, eta)[0] == pytest.approx(1.0, abs=1e-14)
    # consensus-error contraction equals max_{mu != 1} |p_K(mu)| on the worst direction
    factor = np.abs(_poly(mu[:-1], K, eta)).max()
    Z = gen.state(n, 200, seed=5).astype(np.float64)
    before = G.consensus_error(Z) ** 0.5
    after = G.consensus_error(G.accelerated_gossip(Z, W, K, eta)) ** 0.5
    assert after <= factor * before * (1 + 1e-12)
    worst = V[:, [int(np.argmax(np.abs(_poly(mu[:-1], K, eta))))]]
    got = G.consensus_error(G.accelerated_gossip(worst, W, K, eta)) ** 0.5 / G.consensus_error(worst) ** 0.5
    assert got == pytest.approx(factor, rel=1e-10)
    # acceleration beats plain gossip with the same number of rounds
    assert factor < lam ** K


def test_exact_contraction_values_for_the_workloads():
    # ring-8, K=4 and 8x8 torus, K=8: values of max|p_K(mu)| worked out from the recursion
    W = _ring(8)
    lam = T.spectrum(W)[2]
    eta = T.eta_from_lambda(lam)
    mu = np.linalg.eigvalsh(W)[:-1]
    assert np.abs(_poly(mu, 4, eta)).max() == pytest.approx(0.193776, abs=2e-6)
    W = T.mixing_matrix(64, gen.edges_torus(8, 8))
    lam = T.spectrum(W)[2]
    eta = T.eta_from_lambda(lam)
    mu = np.linalg.eigvalsh(W)[:-1]
    assert np.abs(_poly(mu, 8, eta)).max() == pytest.approx(0.071117, abs=2e-6)


def test_asymptotic_rate_is_sqrt_eta():
    """Long-K contraction per round tends to sqrt(eta) = lambda/(1+sqrt(1-lambda^2)),
    which is at most 1 - sqrt(1-lambda): the square-root dependence on the
    spectral gap that Theorem 3 rests on."""
    W = _ring(32)
    lam = T.spectrum(W)[2]
    eta = T.eta_from_lambda(lam)
    Z = gen.state(32, 50, seed=2).astype(np.float64)
    e1 = G.consensus_error(G.accelerated_gossip(Z, W, 60, eta)) ** 0.5
    e2 = G.consensus_error(G.accelerated_gossip(Z, W, 120, eta)) ** 0.5
    rate = (e2 / e1) ** (1 / 60)        # includes a (1+cK) factor: 2^(1/60) at most
    assert rate == pytest.approx(np.sqrt(eta), rel=2e-2)
    assert np.sqrt(eta) <= 1 - np.sqrt(1 - lam) + 1e-15
    assert rate < lam                                   # plain gossip contracts at lambda per round


def test_special_cases():
    W = _ring(6)
    Z = gen.state(6, 9, seed=3).astype(np.float64)
    assert np.array_equal(G.accelerated_gossip(Z, W, 0, 0.4), Z)                  # K=0: identity
    assert np.allclose(G.accelerated_gossip(Z, W, 1, 0.0), W.T @ Z, atol=1e-14)   # one plain gossip step
    assert np.allclose(G.accelerated_gossip(Z, W, 4, 0.0),
                       np.linalg.matrix_power(W.T, 4) @ Z, atol=1e-13)            # eta=0: (W^T)^K
    # first accelerated round uses z_{-1} = z_0
    assert np.allclose(G.accelerated_gossip(Z, W, 1, 0.3), 1.3 * (W.T @ Z) - 0.3 * Z, atol=1e-14)
    # consensus is a fixed point for any eta
    C = np.tile(Z[:1], (6, 1))
    assert np.allclose(G.accelerated_gossip(C, W, 5, 0.6), C, atol=1e-13)


# ---- one DeTAG phase -------------------------------------------------------
@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_tracker_and_mean_iterate_identities(variant):
    """Proof of Theorem 3: mean(Y) equals the mean of the last absorbed
    gradients, and mean(X_{k+1}) = mean(X_k) - alpha * mean(Y_k), for any W,
    K, eta."""
    n, d, alpha, K = 8, 11, 0.05, 3
    W = _ring(n)
    eta = 0.3
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for k in range(6):
        Gnew = gen.gaussian(n, d, seed=9, step=k).astype(np.float64) + X   # any gradients
        Xn, Yn = G.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta, variant)
        assert np.allclose(Xn.mean(0), X.mean(0) - alpha * Y.mean(0), atol=1e-13)
        assert np.allclose(Yn.mean(0), Gnew.mean(0), atol=1e-13)
        X, Y, Gold = Xn, Yn, Gnew


def test_variants_share_the_model_update_and_differ_in_the_tracker():
    """M is linear, so M(X - alpha Y) = M(X) - alpha M(Y): both forms give the
    same X+ from the same state; the trackers differ by M(dG) - dG."""
    n, d, alpha, K, eta = 6, 7, 0.1, 4, 0.45
    W = _ring(n)
    X, Y = gen.state(n, d, 1).astype(np.float64), gen.state(n, d, 2).astype(np.float64)
    Gn, Go = gen.state(n, d, 3).astype(np.float64), gen.state(n, d, 4).astype(np.float64)
    Xa, Ya = G.detag_step(X, Y, Gn, Go, W, alpha, K, eta, "atc")
    Xb, Yb = G.detag_step(X, Y, Gn, Go, W, alpha, K, eta, "alg2")
    assert np.allclose(Xa, Xb, atol=1e-13)
    assert np.allclose(Ya - Yb, G.accelerated_gossip(Gn - Go, W, K, eta) - (Gn - Go), atol=1e-13)


def test_dsgt_special_case():
    """Phase length 1 and eta = 0 is gradient tracking with plain gossip."""
    n, d, alpha = 5, 4, 0.2
    W = _asym(n)
    X, Y = gen.state(n, d, 1).astype(np.float64), gen.state(n, d, 2).astype(np.float64)
    Gn, Go = gen.state(n, d, 3).astype(np.float64), gen.state(n, d, 4).astype(np.float64)
    Xn, Yn = G.detag_step(X, Y, Gn, Go, W, alpha, 1, 0.0, "atc")
    assert np.allclose(Xn, W.T @ (X - alpha * Y), atol=1e-14)
    assert np.allclose(Yn, W.T @ (Y + Gn - Go), atol=1e-14)


@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_quadratic_mean_follows_delayed_scalar_recurrence(variant):
    """Shared diagonal curvature h: the worker mean of column c obeys
    e_{k+1} = e_k - alpha*h_c*e_{k-1} with e = mean(x_c) - mean_i(b_ic) and
    e_0 = e_1 = -mean(b), whatever the topology (mean identities above plus a
    gradient that is affine in x)."""
    n, d, alpha, K = 8, 5, 0.5, 4
    W = _ring(n)
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    h, b = gen.quadratic_problem(n, d, seed=4)
    h = h.astype(np.float64); b = b.astype(np.float64)
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    e_prev = e = -b.mean(0)
    for k in range(12):
        assert np.allclose(X.mean(0) - b.mean(0), e, atol=1e-12)
        Gnew = O.grad_quadratic_diag(X, h, b)
        X, Y = G.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta, variant)
        Gold = Gnew
        e_prev, e = e, (e if k == 0 else e - alpha * h * e_prev)


def test_quadratic_run_converges_to_the_closed_form_optimum():
    n, d, alpha, K = 8, 6, 0.5, 4
    W = _ring(n)
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    rng = np.random.default_rng(0)
    h = rng.uniform(0.3, 1.0, size=d)
    b = rng.standard_normal((n, d)) + np.arange(n)[:, None]
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for _ in range(300):
        Gnew = O.grad_quadratic_diag(X, h, b)
        X, Y = G.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta)
        Gold = Gnew
    assert np.allclose(G.worker_mean(X), b.mean(0), atol=1e-10)     # x* = mean_i b_i
    assert G.consensus_error(X) < 1e-18                            # and every worker agrees


def test_lstsq_run_converges_to_minimum_norm_solution():
    """Under-determined stacked system, x0 = 0: iterates stay in the row space
    of the stacked A, so the limit is pinv(A) b."""
    n, m, d = 4, 3, 24
    A, b = gen.lstsq_problem(n, m, d, seed=1, shift=1.5)
    A = A.astype(np.float64); b = b.astype(np.float64)
    W = _ring(n)
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for _ in range(4000):
        Gnew = O.grad_lstsq(X, A, b)
        X, Y = G.detag_step(X, Y, Gnew, Gold, W, 0.05, 4, eta)
        Gold = Gnew
    xstar = np.linalg.pinv(A.reshape(n * m, d)) @ b.reshape(-1)
    assert np.allclose(G.worker_mean(X), xstar, atol=1e-8)


def test_dpsgd_stalls_where_detag_converges():
    """Non-iid offsets: D-PSGD with a constant step keeps a consensus error
    of the order of the step size, DeTAG drives it to zero (qualitative claim
    of the first experiment)."""
    n, d, alpha = 8, 4, 0.2
    W = _ring(n)
    eta = T.eta_from_lambda(T.spectrum(W)[2])
    h = np.ones(d)
    b = np.arange(n, dtype=np.float64)[:, None] * np.ones((1, d))
    Xd = np.zeros((n, d))
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for _ in range(400):
        Xd = G.dpsgd_step(Xd, O.grad_quadratic_diag(Xd, h, b), W, alpha)
        Gnew = O.grad_quadratic_diag(X, h, b)
        X, Y = G.detag_step(X, Y, Gnew, Gold, W, alpha, 4, eta)
        Gold = Gnew
    assert G.consensus_error(X) < 1e-20
    assert G.consensus_error(Xd) > 1e-2


# ---- diagnostics -----------------------------------------------------------
def test_diagnostics_definitions():
    X = np.array([[1.0, 2.0], [3.0, 6.0], [5.0, 1.0]])
    assert np.allclose(G.worker_mean(X), [3.0, 3.0])
    assert G.consensus_error(X) == pytest.approx(4 + 0 + 4 + 1 + 9 + 4)
    assert G.consensus_error(np.ones((4, 3))) == 0.0
