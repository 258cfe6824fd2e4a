"""Pins for oracle/consensus.py: Lemma 1 (the factors multiply to 11^T/n, respect the graph, and there are
between D and 2D of them), and DeFacto's equivalence to centralized SGD."""
import numpy as np
import pytest

from oracle import consensus as C
from oracle import objectives as O
from workloads import generate as gen


def _diameter_and_ecc(n, edges, root):
    A = np.zeros((n, n), bool)
    for a, b in edges:
        A[a, b] = A[b, a] = True
    dist = np.full((n, n), np.inf)
    np.fill_diagonal(dist, 0)
    dist[A] = 1
    for k in range(n):
        dist = np.minimum(dist, dist[:, [k]] + dist[[k], :])
    return int(dist.max()), int(dist[root].max()), A


def _graphs():
    rng = np.random.default_rng(5)
    tree = [(i, int(rng.integers(0, i))) for i in range(1, 23)]            # a random tree on 23 nodes
    return [("ring16", 16, gen.edges_ring(16), 0), ("ring7", 7, gen.edges_ring(7), 3),
            ("torus4x8", 32, gen.edges_torus(4, 8), 5), ("path9", 9, gen.edges_path(9), 0),
            ("path9mid", 9, gen.edges_path(9), 4), ("tree23", 23, tree, 0),
            ("rr40", 40, gen.edges_random_regular(40, 4, seed=2), 7), ("pair", 2, [(0, 1)], 1)]


@pytest.mark.parametrize("name,n,edges,root", _graphs())
def test_lemma_1(name, n, edges, root):
    F = C.gather_propagate_factors(n, edges, root)
    D, ecc, adj = _diameter_and_ecc(n, edges, root)
    assert len(F) == 2 * ecc and D <= len(F) <= 2 * D                       # R in {D, ..., 2D}
    P = np.eye(n)
    for A in F:
        off = A.copy()
        np.fill_diagonal(off, 0)
        assert not np.any(off[~adj] != 0), "a factor uses an edge the graph does not have"
        P = A @ P
    assert np.allclose(P, np.full((n, n), 1.0 / n), rtol=0, atol=1e-15)     # A_{R-1} ... A_0 = 11^T/n
    X = gen.state(n, 6, seed=1).astype(np.float64)
    assert np.allclose(C.average_consensus(X, F), np.tile(X.mean(0), (n, 1)), atol=1e-14)


def test_defacto_round_is_exact_averaging_plus_the_local_step():
    """A round of Algorithm 1 is X <- (11^T/n) X - alpha * G / R with G the workers' own accumulated gradients
    at X (the averaging is exact, not approximate); for a gradient that is affine with a shared slope, the
    worker mean therefore follows centralized SGD on the average objective with the summed batches."""
    n, d, alpha, B = 9, 5, 0.1, 2
    edges = gen.edges_path(n)
    F = C.gather_propagate_factors(n, edges, 4)
    R = len(F)
    h, b = np.linspace(0.5, 1.5, d), gen.state(n, d, 5).astype(np.float64)
    rng = np.random.default_rng(0)
    noise = rng.standard_normal((8 * R, B, n, d))
    g = lambda t, q, X: O.grad_quadratic_diag(X, h, b) + 0.1 * noise[t, q]
    X0 = gen.state(n, d, 8).astype(np.float64)                  # workers start apart
    X, rounds = C.defacto(g, X0, F, alpha, 3 * 2 * R, B)
    assert rounds == 3
    Xe, xbar = X0.copy(), X0.mean(0)
    for k in range(3):
        tot = sum(g(k * 2 * R + r, q, Xe) for r in range(R) for q in range(B))
        mean_noise = sum(0.1 * noise[k * 2 * R + r, q].mean(0) for r in range(R) for q in range(B))
        Xe = np.tile(Xe.mean(0), (n, 1)) - alpha * tot / R
        xbar = xbar - alpha * (R * B * h * (xbar - b.mean(0)) + mean_noise) / R     # centralized SGD on the mean
    assert np.allclose(X, Xe, atol=1e-13)
    assert np.allclose(X.mean(0), xbar, atol=1e-13)
    # an unfinished round changes nothing
    X2, r2 = C.defacto(g, X0, F, alpha, 3 * 2 * R + R + 1, B)
    assert r2 == 3 and np.array_equal(X2, X)
