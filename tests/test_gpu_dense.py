"""Parity of DETAG_PATH_DENSE -- the K rounds of Algorithm 3 as one product with the matrix polynomial p_K(W^T) on
the matrix cores -- against the oracle, which takes the K rounds one after the other."""
import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from oracle import gossip as OG
from oracle import objectives as OO
from oracle import topology as OT
from tests.util import TOL_BF16, TOL_F32, amax, rel_err
from workloads import generate as gen

pytestmark = pytest.mark.gpu

from tests.gpu_util import DEV, SENTINEL, _built, padding_ok, to_dev, to_host  # noqa: F401,E402


def _graph(n, graph):
    if graph == "asym":
        W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)
        return D.Topology.from_dense(W), W, 0.3
    if graph == "ring":
        W = OT.mixing_matrix(n, gen.edges_ring(n))
        return D.Topology.ring(), W, (OT.eta_from_lambda(OT.spectrum(W)[2]) if n > 1 else 0.0)
    if graph == "torus88":
        W = OT.mixing_matrix(64, gen.edges_torus(8, 8))
        return D.Topology.torus(8, 8), W, OT.eta_from_lambda(OT.spectrum(W)[2])
    if graph == "star":                                         # a hub with n-1 neighbours: no on-chip round kernel
        e = np.array([(0, j) for j in range(1, n)])
    else:
        e = gen.edges_random_regular(n, 4, seed=n)
    W = OT.mixing_matrix(n, e, "metropolis")
    return D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), W, OT.eta_from_lambda(OT.spectrum(W)[2])


CASES = [(5, "asym"), (1, "ring"), (2, "ring"), (17, "ring"), (33, "ring"), (64, "torus88"), (20, "star"), (100, "rr"),
         (130, "rr"), (256, "rr")]


@pytest.mark.parametrize("n,graph", CASES)
@pytest.mark.parametrize("K", [1, 5, 16])
def test_dense_gossip_and_step_f32(n, graph, K):
    d, ld = 150, 160               # two full 64-column tiles and a ragged one
    topo, W, eta = _graph(n, graph)
    ctx = D.detag_create(topo, n, d, ld)
    ctx.set_path(D.DETAG_PATH_DENSE)
    alpha = 0.05
    Z = gen.state(n, d, seed=K)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K, eta)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(Z, W, K, eta), amax(Z)) < TOL_F32
    assert padding_ok(Zd, d)
    X, Y, Gn, Go = (gen.state(n, d, s) for s in (1, 2, 3, 4))
    for variant, vcode in (("atc", D.DETAG_VARIANT_ATC), ("alg2", D.DETAG_VARIANT_ALG2)):
        Xd, Yd, Gnd, God = (to_dev(a, ld) for a in (X, Y, Gn, Go))
        ctx.step(Xd, Yd, Gnd, God, alpha, K, eta, vcode)
        Xr, Yr = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
        S = amax(X, Y, Gn, Go)
        assert rel_err(to_host(Xd, d), Xr, S) < TOL_F32
        assert rel_err(to_host(Yd, d), Yr, S) < TOL_F32
        assert padding_ok(Xd, d) and padding_ok(Yd, d)
        assert np.array_equal(to_host(Gnd, d), Gn.astype(np.float32)) and np.array_equal(to_host(God, d), Go.astype(np.float32))


@pytest.mark.parametrize("n,graph", [(12, "rr"), (64, "torus88"), (256, "rr")])
@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_dense_step_bf16_state(n, graph, variant):
    d, ld, K, alpha = 200, 256, 8, 0.05
    topo, W, eta = _graph(n, graph)
    ctx = D.detag_create(topo, n, d, ld, D.DETAG_BF16)
    ctx.set_path(D.DETAG_PATH_DENSE)
    X, Y = (OO.round_bf16(gen.state(n, d, s)) for s in (1, 2))
    Gn, Go = (gen.state(n, d, s) for s in (3, 4))
    Xd, Yd = (to_dev(a, ld, torch.bfloat16) for a in (X, Y))
    Gnd, God = (to_dev(a, ld) for a in (Gn, Go))
    ctx.step(Xd, Yd, Gnd, God, alpha, K, eta, D.DETAG_VARIANT_ATC if variant == "atc" else D.DETAG_VARIANT_ALG2)
    Xr, Yr = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
    S = amax(X, Y, Gn, Go)
    assert rel_err(to_host(Xd, d), Xr, S) < TOL_BF16
    assert rel_err(to_host(Yd, d), Yr, S) < TOL_BF16
    assert padding_ok(Xd, d) and padding_ok(Yd, d)
    Zd = to_dev(X, ld, torch.bfloat16)
    ctx.gossip_accel(Zd, K, eta)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(X, W, K, eta), amax(X)) < TOL_BF16


def test_dense_long_K_near_one_eta():
    """The slack ring of the spectral-gap sweep (kappa = 0.01) at its phase length: the polynomial is
    evaluated in fp64 on the host, so the error does not grow with K as it does round by round."""
    n, d, ld = 16, 300, 320
    W = OT.slack(OT.mixing_matrix(n, gen.edges_ring(n)), 0.01)
    ctx = D.detag_create(D.Topology.ring(kappa=0.01), n, d, ld)
    ctx.set_path(D.DETAG_PATH_DENSE)
    eta = OT.eta_from_lambda(OT.spectrum(W)[2])
    K = ctx.phase_length()
    assert K > 40 and eta > 0.9
    Z = gen.state(n, d, seed=3)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K)
    assert np.abs(to_host(Zd, d) - OG.accelerated_gossip(Z, W, K, eta)).max() < 2e-6 * amax(Z)


def test_dense_polynomial_cache_and_mean():
    """More (K, eta) pairs than the context keeps polynomials for, then the first again; equal values across the
    workers stay put and the worker mean is kept."""
    n, d, ld = 100, 130, 160
    topo, W, eta = _graph(n, "rr")
    ctx = D.detag_create(topo, n, d, ld)
    ctx.set_path(D.DETAG_PATH_DENSE)
    Z = gen.state(n, d, seed=9)
    for K, e in [(3, eta), (4, eta), (5, eta), (3, 0.0), (6, eta), (7, 0.1), (3, eta)]:
        Zd = to_dev(Z, ld)
        ctx.gossip_accel(Zd, K, e)
        out = to_host(Zd, d)
        assert rel_err(out, OG.accelerated_gossip(Z, W, K, e), amax(Z)) < TOL_F32
        assert np.abs(out.mean(0) - Z.mean(0)).max() < 2e-6 * amax(Z)
    C = np.tile(gen.state(1, d, seed=2), (n, 1))
    Cd = to_dev(C, ld)
    ctx.gossip_accel(Cd, 9)
    assert np.abs(to_host(Cd, d) - C).max() < 1e-6 * amax(C)


def test_dense_path_is_refused_above_256_workers():
    ctx = D.detag_create(D.Topology.ring(), 300, 64, 64)
    with pytest.raises(D.DetagError) as ei:
        ctx.set_path(D.DETAG_PATH_DENSE)
    assert ei.value.status == D.DETAG_EUNSUPPORTED


def test_config5_shape_bf16_short_run_dense():
    """The 256-worker workload (random 4-regular graph, Metropolis weights, bf16 X/Y, K=16) on the dense path,
    d reduced to 4,096 + 37 columns and 3 steps; the oracle rounds X and Y to bf16 after every step."""
    from workloads import CONFIGS
    cfg = CONFIGS[5]
    n, K, alpha = cfg.n, cfg.K, cfg.lr
    d, T = 4096 + 37, 3
    ld = D.padded_ld(d)
    e = gen.edges_random_regular(n, 4, seed=cfg.seed)
    W = OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), n, d, ld, D.DETAG_BF16)
    ctx.set_path(D.DETAG_PATH_DENSE)
    eta = ctx.spectrum()["eta"]
    h, b = gen.quadratic_problem(n, d, seed=cfg.seed, b_std=cfg.extra["b_std"])
    hd = torch.zeros(ld); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    bd = to_dev(b, ld)
    Xd, Yd = (D.new_matrix(n, d, ld, dtype=torch.bfloat16) for _ in range(2))
    Ga, Gb = D.new_matrix(n, d, ld), D.new_matrix(n, d, ld)
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for t in range(T):
        ctx.grad_quadratic_diag(Xd, hd, bd, Ga)
        ctx.step(Xd, Yd, Ga, Gb, alpha, K)
        Ga, Gb = Gb, Ga
        Gnew = OO.grad_quadratic_diag(X, h, b)
        Xn, Yn = OG.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta)
        if t == 0:
            S1 = amax(X, Y, Gnew, Gold)
            assert rel_err(to_host(Xd, d), Xn, S1) < TOL_BF16
            assert rel_err(to_host(Yd, d), Yn, S1) < TOL_BF16
        X, Y, Gold = OO.round_bf16(Xn).astype(np.float64), OO.round_bf16(Yn).astype(np.float64), Gnew
    S = amax(X, Y, Gold)
    assert rel_err(to_host(Xd, d), X, S, floor=1.0) < TOL_BF16
    assert rel_err(to_host(Yd, d), Y, S, floor=1.0) < TOL_BF16
