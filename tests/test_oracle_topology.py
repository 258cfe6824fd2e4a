"""Pins for oracle/topology.py: closed-form spectra, the paper's linear-graph
eigenvalue, the slack-matrix gap and the printed ring-16 gaps."""
import os

import numpy as np
import pytest

from oracle import topology as T
from workloads import generate as gen


def _ring_lambda2(n):
    return (1 + 2 * np.cos(2 * np.pi / n)) / 3


@pytest.mark.parametrize("n", [3, 8, 16, 32, 33])
def test_ring_spectrum_closed_form(n):
    W = T.mixing_matrix(n, gen.edges_ring(n), "uniform")
    T.check_gossip_matrix(W, gen.edges_ring(n))
    l2, ln, lam = T.spectrum(W)
    mu = np.sort((1 + 2 * np.cos(2 * np.pi * np.arange(n) / n)) / 3)[::-1]
    assert l2 == pytest.approx(mu[1], abs=1e-13)
    assert ln == pytest.approx(mu[-1], abs=1e-13)
    assert lam == pytest.approx(max(abs(mu[1]), abs(mu[-1])), abs=1e-13)


def test_torus_spectrum_closed_form():
    W = T.mixing_matrix(64, gen.edges_torus(8, 8), "uniform")
    T.check_gossip_matrix(W, gen.edges_torus(8, 8))
    assert np.count_nonzero(W[0]) == 5 and W[0, 0] == pytest.approx(0.2)
    a = np.arange(8)
    mu = (1 + 2 * np.cos(2 * np.pi * a[:, None] / 8) + 2 * np.cos(2 * np.pi * a[None, :] / 8)) / 5
    mu = np.sort(mu.ravel())[::-1]
    l2, ln, lam = T.spectrum(W)
    assert l2 == pytest.approx(mu[1], abs=1e-13)       # (1 + 2cos(pi/4) + 2)/5 = 0.88284...
    assert l2 == pytest.approx((3 + np.sqrt(2)) / 5, abs=1e-13)
    assert ln == pytest.approx(-0.6, abs=1e-13)
    assert lam == pytest.approx(l2)


@pytest.mark.parametrize("n", [2, 5, 7, 12])
def test_linear_graph_lambda_is_cos_pi_over_n(n):
    """Corollary 1 uses a gossip matrix on the linear graph whose second
    largest eigenvalue is cos(pi/n): off-diagonals 1/2, the two end
    self-loops 1/2."""
    W = np.zeros((n, n))
    for i in range(n - 1):
        W[i, i + 1] = W[i + 1, i] = 0.5
    W[0, 0] = W[-1, -1] = 0.5
    T.check_gossip_matrix(W, gen.edges_path(n))
    l2, ln, lam = T.spectrum(W)
    assert l2 == pytest.approx(np.cos(np.pi / n), abs=1e-13)
    assert lam == pytest.approx(np.cos(np.pi / n), abs=1e-13)


def test_lambda_takes_the_negative_end_when_it_dominates():
    # triangle-free bipartite-like case: ring-4 with weight 1/3 has eigenvalues 1, 1/3, 1/3, -1/3;
    # a lazy-free even ring (self weight 0) has lambda_n = -1 -> lambda = 1.
    W = np.zeros((4, 4))
    for i in range(4):
        W[i, (i + 1) % 4] = W[i, (i - 1) % 4] = 0.5
    l2, ln, lam = T.spectrum(W)
    assert ln == pytest.approx(-1.0) and lam == pytest.approx(1.0) and l2 == pytest.approx(0.0, abs=1e-13)


@pytest.mark.parametrize("kappa", [1.0, 0.1, 0.05, 0.01])
def test_slack_matrix_scales_gap(kappa):
    W0 = T.mixing_matrix(16, gen.edges_ring(16), "uniform")
    gap0 = 1 - T.spectrum(W0)[0]
    Wk = T.slack(W0, kappa)
    T.check_gossip_matrix(Wk, gen.edges_ring(16))
    assert 1 - T.spectrum(Wk)[0] == pytest.approx(kappa * gap0, rel=1e-10)


def test_printed_ring16_gaps(golden_dir):
    """The captions of the second experiment print 1-lambda for four kappas.
    Their ratios must equal kappa (what slack() does); the absolute value at
    kappa=1 is reproduced, to the one digit printed, by a ring with neighbour
    weight 1/4 (self 1/2) — and not by 1/3, which the workloads here use."""
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "paper_ring16_spectral_gaps.txt"))
            if ln.strip() and not ln.startswith("#")]
    printed = {float(k): float(g) for k, g in rows}
    W0 = np.zeros((16, 16))
    for i in range(16):
        W0[i, (i + 1) % 16] = W0[i, (i - 1) % 16] = 0.25
        W0[i, i] = 0.5
    for kappa, gap in printed.items():
        got = 1 - T.spectrum(T.slack(W0, kappa))[2]
        assert float(f"{got:.0e}") == pytest.approx(gap, rel=1e-12), (kappa, got)
        assert printed[kappa] / printed[1.0] == pytest.approx(kappa, rel=1e-12)
    third = 1 - T.spectrum(T.mixing_matrix(16, gen.edges_ring(16)))[2]
    assert float(f"{third:.0e}") == pytest.approx(5e-2)


def test_phase_length_meets_the_condition_the_proof_needs():
    """The proof of Theorem 3 needs R >= log(n) / (2 sqrt(1-lambda)), which it shows is enough for
    (1 - sqrt(1-lambda))^R <= n^(-1/2); the suggested R must satisfy both, be minimal for the first, and
    scale as 1/sqrt(gap) under the slack construction (gap -> kappa*gap)."""
    for n in (8, 16, 64, 256):
        for lam in (0.0, 0.5, 0.9, 0.99, 0.9999):
            R = T.phase_length(lam, n)
            need = np.log(n) / (2 * np.sqrt(1 - lam))
            assert R >= need and R - 1 < max(need, 1)
            assert (1 - np.sqrt(1 - lam)) ** R <= n ** -0.5 + 1e-15
    W0 = T.mixing_matrix(16, gen.edges_ring(16))
    R1 = T.phase_length(T.spectrum(W0)[2], 16)
    R100 = T.phase_length(T.spectrum(T.slack(W0, 0.01))[2], 16)
    assert R1 == 7 and abs(R100 / R1 - 10) < 1.5
    # the outer-variance term: r = e^8 gives log(r)/2 = 4 > log(16)/2
    assert T.phase_length(0.75, 16, np.exp(8.0)) == 8
    assert T.phase_length(0.75, 16, 1.0) == T.phase_length(0.75, 16) == 3     # log(16)/2 / 0.5 = 2.77


def test_eta_formula():
    # eta = ((1-s)/(1+s)), s = sqrt(1-lambda^2); equivalently sqrt(eta) = lambda/(1+s)
    for lam in [0.0, 0.3, 0.804738, 0.99]:
        s = np.sqrt(1 - lam * lam)
        eta = T.eta_from_lambda(lam)
        assert np.sqrt(eta) == pytest.approx(lam / (1 + s), abs=1e-14)
        assert 0 <= eta < 1
    assert T.eta_from_lambda(0.0) == 0.0
    # values for the ring-8 and 8x8-torus workloads
    assert T.eta_from_lambda(_ring_lambda2(8)) == pytest.approx(0.254996, abs=5e-7)
    assert T.eta_from_lambda((3 + np.sqrt(2)) / 5) == pytest.approx(0.360851, abs=5e-7)


def test_metropolis_equals_uniform_on_regular_and_is_doubly_stochastic_on_irregular():
    e = gen.edges_random_regular(24, 4, seed=3)
    assert np.allclose(T.mixing_matrix(24, e, "uniform"), T.mixing_matrix(24, e, "metropolis"), rtol=0, atol=1e-15)
    star_plus = np.array([(0, 1), (0, 2), (0, 3), (1, 2), (3, 4)])
    W = T.mixing_matrix(5, star_plus, "metropolis")
    T.check_gossip_matrix(W, star_plus)
    assert W[0, 1] == pytest.approx(0.25) and W[3, 4] == pytest.approx(1 / 3)
    assert np.allclose(W, W.T)
    with pytest.raises(ValueError):
        T.mixing_matrix(5, star_plus, "uniform")


def test_random_regular_generator_is_simple_regular_connected():
    n = 256
    e = gen.edges_random_regular(n, 4, seed=0)
    assert len(e) == 2 * n and len({tuple(x) for x in e}) == len(e)
    deg = np.bincount(e.ravel(), minlength=n)
    assert np.all(deg == 4)
    W = T.mixing_matrix(n, e, "metropolis")
    l2, ln, lam = T.spectrum(W)
    assert lam < 1 - 1e-3            # connected: a single eigenvalue 1
    assert np.array_equal(e, gen.edges_random_regular(n, 4, seed=0))


def test_check_rejects_bad_matrices():
    W = T.mixing_matrix(6, gen.edges_ring(6))
    bad = W.copy(); bad[0, 0] += 0.1
    with pytest.raises(ValueError):
        T.check_gossip_matrix(bad)
    off = W.copy(); off[0, 3] = off[3, 0] = 0.1; off[0, 0] -= 0.1; off[3, 3] -= 0.1
    T.check_gossip_matrix(off)                       # still doubly stochastic
    with pytest.raises(ValueError):
        T.check_gossip_matrix(off, gen.edges_ring(6))   # but not on the graph
    neg = np.array([[1.5, -0.5], [-0.5, 1.5]])       # rows and columns sum to one, entries are not in [0, 1]
    with pytest.raises(ValueError):
        T.check_gossip_matrix(neg)


def test_neighbour_lists_read_columns():
    W = np.array([[0.5, 0.5, 0.0], [0.0, 0.5, 0.5], [0.5, 0.0, 0.5]])  # asymmetric, doubly stochastic
    nb = T.neighbour_lists(W)
    assert nb[0] == [(0, 0.5), (2, 0.5)]    # column 0 of W: rows 0 and 2
    assert nb[1] == [(0, 0.5), (1, 0.5)]
