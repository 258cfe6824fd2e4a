"""Host-side tests of the C-ABI library (no GPU needed): it loads, exports every
declared symbol, builds the gossip matrices the oracle builds, computes the
same spectrum, and rejects bad input with a status instead of crashing."""
import math
import os
import re

import numpy as np
import pytest

import paper_2006_08085_amd as D
from oracle import topology as T
from workloads import generate as gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(D.LIB_PATH):
        from paper_2006_08085_amd.build import build
        build(verbose=False)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "detag.h")).read()
    declared = set(re.findall(r"\b(detag_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    L = D.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"libdetag.so does not export {name}"
    assert declared == set(D.EXPORTS)
    assert D.detag_version().startswith("detag-gfx950")


@pytest.mark.parametrize("n", [1, 2, 3, 8, 16, 32, 33])
def test_ring_matches_oracle(n):
    ctx = D.detag_create(D.Topology.ring(), n, 16)
    W = T.mixing_matrix(n, gen.edges_ring(n))
    assert np.allclose(ctx.dense_W(), W, rtol=0, atol=1e-15)
    l2, ln, lam = T.spectrum(W)
    s = ctx.spectrum()
    assert s["lambda2"] == pytest.approx(l2, abs=1e-12)
    assert s["lambdan"] == pytest.approx(ln, abs=1e-12)
    assert s["lam"] == pytest.approx(lam, abs=1e-12)
    assert s["eta"] == pytest.approx(T.eta_from_lambda(lam), abs=1e-12)


def test_torus_and_kappa_match_oracle():
    for kappa in (1.0, 0.1):
        ctx = D.detag_create(D.Topology.torus(8, 8, kappa=kappa), 64, 16)
        W = T.slack(T.mixing_matrix(64, gen.edges_torus(8, 8)), kappa)
        assert np.allclose(ctx.dense_W(), W, rtol=0, atol=1e-15)
        s = ctx.spectrum()
        l2, ln, lam = T.spectrum(W)
        assert (s["lambda2"], s["lambdan"], s["lam"]) == pytest.approx((l2, ln, lam), abs=1e-12)
        assert s["eta"] == pytest.approx(T.eta_from_lambda(lam), abs=1e-12)
        assert ctx.has_fused()
    assert D.detag_create(D.Topology.random_regular(4, 1), 300, 16).has_fused() is False   # n > 256: per-round only


def test_edge_list_with_metropolis_weights_matches_oracle():
    e = gen.edges_random_regular(256, 4, seed=0)
    ctx = D.detag_create(D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), 256, 8)
    W = T.mixing_matrix(256, e, "metropolis")
    assert np.allclose(ctx.dense_W(), W, rtol=0, atol=1e-15)
    assert ctx.spectrum()["lam"] == pytest.approx(T.spectrum(W)[2], abs=1e-12)
    irregular = np.array([(0, 1), (0, 2), (0, 3), (1, 2), (3, 4)])
    ctx = D.detag_create(D.Topology.from_edges(irregular, D.DETAG_W_METROPOLIS), 5, 8)
    W = T.mixing_matrix(5, irregular, "metropolis")
    assert np.allclose(ctx.dense_W(), W, rtol=0, atol=1e-15)
    assert ctx.spectrum()["eta"] == pytest.approx(T.eta_from_lambda(T.spectrum(W)[2]), abs=1e-12)
    with pytest.raises(D.DetagError) as ei:
        D.detag_create(D.Topology.from_edges(irregular, D.DETAG_W_UNIFORM), 5, 8)
    assert ei.value.status == D.DETAG_EINVAL


def test_library_random_regular_graph_is_valid_by_the_oracles_checks():
    """The library's own generator: the oracle receives the CSR as data and
    re-validates it independently (4-regular, simple, symmetric, doubly
    stochastic, connected) and recomputes lambda and eta."""
    ctx = D.detag_create(D.Topology.random_regular(4, seed=7), 256, 8)
    W = ctx.dense_W()
    T.check_gossip_matrix(W)
    assert np.array_equal(W, W.T)
    off = W - np.diag(np.diag(W))
    assert np.all((off != 0).sum(0) == 4) and np.allclose(off[off != 0], 0.2) and np.allclose(np.diag(W), 0.2)
    l2, ln, lam = T.spectrum(W)
    assert lam < 1 - 1e-3
    s = ctx.spectrum()
    assert (s["lambda2"], s["lambdan"], s["lam"]) == pytest.approx((l2, ln, lam), abs=1e-12)
    assert s["eta"] == pytest.approx(T.eta_from_lambda(lam), abs=1e-12)
    again = D.detag_create(D.Topology.random_regular(4, seed=7), 256, 8).dense_W()
    other = D.detag_create(D.Topology.random_regular(4, seed=8), 256, 8).dense_W()
    assert np.array_equal(W, again) and not np.array_equal(W, other)


def test_linear_graph_lambda_through_csr():
    n = 9
    W = np.zeros((n, n))
    for i in range(n - 1):
        W[i, i + 1] = W[i + 1, i] = 0.5
    W[0, 0] = W[-1, -1] = 0.5
    ctx = D.detag_create(D.Topology.from_dense(W), n, 4)
    assert ctx.spectrum()["lam"] == pytest.approx(math.cos(math.pi / n), abs=1e-12)   # Corollary 1
    assert np.array_equal(ctx.dense_W(), W)


def test_phase_length_of_theorem_3():
    """Host-side formula: same integer as the oracle's, the outer-variance term takes over when it is the
    larger one, and an asymmetric W (no stored lambda) is an error, not a guess."""
    for kappa in (1.0, 0.1, 0.05, 0.01):
        ctx = D.detag_create(D.Topology.ring(kappa=kappa), 16, 8)
        lam = ctx.spectrum()["lam"]
        assert ctx.phase_length() == T.phase_length(lam, 16)
        assert ctx.phase_length(1e6) == T.phase_length(lam, 16, 1e6) > ctx.phase_length()
        assert ctx.phase_length(2.0) == ctx.phase_length()          # log(2)/2 < log(16)/2
    assert D.detag_create(D.Topology.ring(), 1, 8).phase_length() == 1
    P = np.roll(np.eye(5), 1, axis=1)
    with pytest.raises(D.DetagError) as ei:
        D.detag_create(D.Topology.from_dense(0.5 * np.eye(5) + 0.5 * P), 5, 4).phase_length()
    assert ei.value.status == D.DETAG_EINVAL


def test_consensus_factors_on_the_host():
    """The library's average-consensus factors (built without a GPU) against the oracle's construction and
    against Lemma 1 itself: same matrices, product 11^T/n, graph sparsity, R = 2 * eccentricity of the root."""
    from oracle import consensus as OC
    cases = [(D.Topology.ring(), 16, gen.edges_ring(16), 0), (D.Topology.torus(4, 8), 32, gen.edges_torus(4, 8), 5),
             (D.Topology.from_edges(gen.edges_path(9), D.DETAG_W_METROPOLIS), 9, gen.edges_path(9), 4)]
    for topo, n, edges, root in cases:
        ctx = D.detag_create(topo, n, 8)
        f = D.Factors(ctx, root)
        ref = OC.gather_propagate_factors(n, edges, root)
        assert f.R == len(ref)
        P = np.eye(n)
        for r in range(f.R):
            A = f.dense(r)
            assert np.array_equal(A, ref[r])
            P = A @ P
        assert np.allclose(P, 1.0 / n, rtol=0, atol=1e-15)
        f.close()
    ctx = D.detag_create(D.Topology.ring(), 8, 8)
    with pytest.raises(D.DetagError):
        D.Factors(ctx, 8)
    with pytest.raises(D.DetagError):
        D.Factors(ctx, -1)
    one = D.Factors(D.detag_create(D.Topology.ring(), 1, 8), 0)
    assert one.R == 0


def _run_program(prog, Z):
    """The operations of detag_factors_get_program carried out as its description says, in fp64."""
    tile = Z.copy()
    f32 = lambda w: float(np.array([w], np.uint32).view(np.float32)[0])
    for batch in prog:
        reads = [(tile[int(op[0]) // 256].copy(), tile[int(op[1]) // 256].copy()) for op in batch]
        acc, sums = np.zeros(Z.shape[1]), []
        for j, (op, (x0, x1)) in enumerate(zip(batch, reads)):
            for mask in (op[3], op[6], op[7]):
                assert mask in (0, 0xFFFFFFFF)
            acc = acc if (j > 0 and op[3]) else np.zeros(Z.shape[1])
            if op[6]:
                acc = acc + f32(op[4]) * x0
            if op[7]:
                acc = acc + f32(op[5]) * x1
            sums.append(acc)
        for op, a in zip(batch, sums):
            assert int(op[2]) % 256 == 0
            tile[int(op[2]) // 256] = a
    return tile


def test_consensus_program_on_the_host():
    """What the one-launch form of the average consensus executes, interpreted on the CPU, against the factors
    applied one after the other (and so against Lemma 1): rings, tori, a path, stars, random regular graphs up to
    256 workers, several roots; and the cases it has to decline."""
    rng = np.random.default_rng(11)
    cases = [(D.Topology.ring(), 16, 0), (D.Topology.ring(), 31, 7), (D.Topology.torus(8, 8), 64, 0),
             (D.Topology.torus(4, 8), 32, 13), (D.Topology.from_edges(gen.edges_path(9), D.DETAG_W_METROPOLIS), 9, 4),
             (D.Topology.from_edges(np.array([[0, i] for i in range(1, 8)]), D.DETAG_W_METROPOLIS), 8, 0),
             (D.Topology.from_edges(np.array([[0, i] for i in range(1, 8)]), D.DETAG_W_METROPOLIS), 8, 3),
             (D.Topology.from_edges(gen.edges_random_regular(64, 4, 3), D.DETAG_W_METROPOLIS), 64, 9),
             (D.Topology.from_edges(gen.edges_random_regular(256, 4, 5), D.DETAG_W_METROPOLIS), 256, 100),
             (D.Topology.ring(), 2, 1), (D.Topology.ring(), 3, 0)]
    for topo, n, root in cases:
        ctx = D.detag_create(topo, n, 8)
        f = D.Factors(ctx, root)
        prog = f.program()
        assert prog.shape[0] > 0 and prog.shape[0] % 2 == 0, (n, root)
        Z = rng.standard_normal((n, 5))
        ref = Z.copy()
        changed = 0
        for r in range(f.R):
            A = f.dense(r)
            changed += int(np.sum(np.any(A != np.eye(n), axis=1)))
            ref = A @ ref
        got = _run_program(prog, Z)
        assert np.allclose(ref, Z.mean(0), rtol=0, atol=1e-14)
        assert np.abs(got - ref).max() < 1e-6, (n, root)          # the program's weights are fp32
        assert prog.shape[0] * 4 < 2 * changed + 8                # no more operations than changed rows call for
        # an entry far from the others must not leak through an absent term: the masks, not the weights, drop it
        Zbig = Z.copy(); Zbig[root, 0] = 1e30
        assert np.all(np.isfinite(_run_program(prog, Zbig)))
    # more than 8 terms in a factor row (a star's centre with 12 leaves) and more than 256 workers are declined
    star = D.Topology.from_edges(np.array([[0, i] for i in range(1, 13)]), D.DETAG_W_METROPOLIS)
    assert D.Factors(D.detag_create(star, 13, 8), 0).program().shape[0] == 0
    assert D.Factors(D.detag_create(D.Topology.ring(), 300, 8), 0).program().shape[0] == 0
    assert D.Factors(D.detag_create(D.Topology.ring(), 1, 8), 0).program().shape[0] == 0


def test_consensus_program_on_random_graphs():
    """The same check on seeded random connected graphs of bounded degree (a random spanning tree plus extra edges),
    random roots: whenever the library offers a program it reproduces the factor sequence, and it offers one exactly
    when no factor row has more than 8 terms."""
    rng = np.random.default_rng(2024)
    offered = declined = 0
    for trial in range(40):
        n = int(rng.integers(2, 70))
        max_deg = int(rng.integers(3, 12))
        deg = np.zeros(n, int)
        edges = set()
        hub = trial % 5 == 0 and n >= 12                        # every fifth graph has a node with 10 neighbours
        for v in range(1, n):                                   # random tree: attach v to an earlier node with room
            cand = [u for u in range(v) if deg[u] < max_deg]
            u = 0 if hub and v <= 10 else int(rng.choice(cand))
            edges.add((u, v)); deg[u] += 1; deg[v] += 1
        for _ in range(n):                                      # a few extra edges
            a, b = sorted(int(x) for x in rng.integers(0, n, 2))
            if a != b and (a, b) not in edges and deg[a] < max_deg and deg[b] < max_deg:
                edges.add((a, b)); deg[a] += 1; deg[b] += 1
        topo = D.Topology.from_edges(np.array(sorted(edges)), D.DETAG_W_METROPOLIS)
        ctx = D.detag_create(topo, n, 8)
        root = 0 if hub else int(rng.integers(0, n))
        f = D.Factors(ctx, root)
        widest = max(int(np.count_nonzero(f.dense(r), axis=1).max()) for r in range(f.R))
        prog = f.program()
        if widest > 8:
            assert prog.shape[0] == 0
            declined += 1
            continue
        offered += 1
        assert prog.shape[0] > 0
        Z = rng.standard_normal((n, 3))
        ref = Z.copy()
        for r in range(f.R):
            ref = f.dense(r) @ ref
        assert np.allclose(ref, Z.mean(0), rtol=0, atol=1e-13)
        assert np.abs(_run_program(prog, Z) - ref).max() < 1e-6, (trial, n, root)
    assert offered >= 10 and declined >= 3                      # the sweep reaches both outcomes


def test_gossip_polynomial_on_the_host():
    """detag_get_gossip_polynomial against the oracle's Algorithm 3 run on the identity, and against what the
    paper says about it: P 1 = 1 and 1^T P = 1^T (the worker mean is kept), K = 0 gives I, eta = 0 gives (W^T)^K,
    and on a symmetric W its singular values are |p_K(mu)| over W's eigenvalues mu."""
    from oracle import gossip as OG
    cases = [(D.Topology.ring(), 8, T.mixing_matrix(8, gen.edges_ring(8))),
             (D.Topology.torus(8, 8), 64, T.mixing_matrix(64, gen.edges_torus(8, 8))),
             (D.Topology.from_edges(gen.edges_random_regular(40, 4, 2), D.DETAG_W_METROPOLIS), 40,
              T.mixing_matrix(40, gen.edges_random_regular(40, 4, 2), "metropolis"))]
    for topo, n, W in cases:
        ctx = D.detag_create(topo, n, 8)
        eta = T.eta_from_lambda(T.spectrum(W)[2])
        for K in (0, 1, 2, 7, 16):
            P = ctx.gossip_polynomial(K)
            ref = OG.accelerated_gossip(np.eye(n), W, K, eta)
            assert np.abs(P - ref).max() < 1e-13
            assert np.abs(P.sum(0) - 1).max() < 1e-13 and np.abs(P.sum(1) - 1).max() < 1e-13
            mu = np.linalg.eigvalsh(W)
            pk_prev, pk = np.ones_like(mu), np.ones_like(mu)
            for _ in range(K):
                pk_prev, pk = pk, (1 + eta) * mu * pk - eta * pk_prev
            assert np.allclose(np.linalg.svd(P, compute_uv=False), np.sort(np.abs(pk))[::-1], rtol=0, atol=1e-12)
        assert np.array_equal(ctx.gossip_polynomial(0), np.eye(n))
        assert np.abs(ctx.gossip_polynomial(3, 0.0) - np.linalg.matrix_power(W.T, 3)).max() < 1e-14
    asym = 0.5 * np.eye(5) + 0.5 * np.roll(np.eye(5), 1, axis=1)
    ctx = D.detag_create(D.Topology.from_dense(asym), 5, 8)
    assert np.abs(ctx.gossip_polynomial(4, 0.2) - OG.accelerated_gossip(np.eye(5), asym, 4, 0.2)).max() < 1e-14
    with pytest.raises(D.DetagError):
        ctx.gossip_polynomial(4)          # no stored eta for an asymmetric W
    with pytest.raises(D.DetagError):
        ctx.gossip_polynomial(-1, 0.2)


def test_asymmetric_W_is_accepted_without_eta():
    P = np.roll(np.eye(5), 1, axis=1)
    W = 0.5 * np.eye(5) + 0.5 * P
    ctx = D.detag_create(D.Topology.from_dense(W), 5, 4)
    assert np.array_equal(ctx.dense_W(), W)
    s = ctx.spectrum()
    assert all(math.isnan(s[k]) for k in ("lambda2", "lambdan", "lam", "eta"))


def test_rejections():
    def status(topo, n=6, d=4, ld=None, dtype=D.DETAG_F32):
        with pytest.raises(D.DetagError) as ei:
            D.detag_create(topo, n, d, ld, dtype)
        assert ei.value.message
        return ei.value.status

    W = T.mixing_matrix(6, gen.edges_ring(6))
    bad = W.copy(); bad[0, 0] += 1e-6
    assert status(D.Topology.from_dense(bad)) == D.DETAG_ENOT_DOUBLY_STOCHASTIC
    neg = W.copy(); neg[0, 1] = neg[1, 0] = -0.1; neg[0, 0] += 0.1 + 1 / 3; neg[1, 1] += 0.1 + 1 / 3
    assert status(D.Topology.from_dense(neg)) == D.DETAG_ENOT_DOUBLY_STOCHASTIC
    two = np.kron(np.eye(2), T.mixing_matrix(3, gen.edges_ring(3)))
    assert status(D.Topology.from_dense(two)) == D.DETAG_EDISCONNECTED
    periodic = np.zeros((4, 4))
    for i in range(4):
        periodic[i, (i + 1) % 4] = periodic[i, (i - 1) % 4] = 0.5
    assert status(D.Topology.from_dense(periodic), n=4) == D.DETAG_EDISCONNECTED   # lambda_n = -1
    assert status(D.Topology.ring(), n=0) == D.DETAG_EINVAL
    assert status(D.Topology.ring(), d=0) == D.DETAG_EINVAL
    assert status(D.Topology.ring(), d=8, ld=7) == D.DETAG_EINVAL
    assert status(D.Topology.ring(kappa=0.0)) == D.DETAG_EINVAL
    assert status(D.Topology.ring(kappa=1.5)) == D.DETAG_EINVAL
    assert status(D.Topology.torus(2, 2)) == D.DETAG_EINVAL            # rows*cols != n
    assert status(D.Topology.random_regular(3, 0)) == D.DETAG_EINVAL   # odd degree
    assert status(D.Topology.from_edges(np.array([(0, 1), (1, 0)]))) == D.DETAG_EINVAL   # repeated edge
    assert status(D.Topology.from_edges(np.array([(0, 9)]))) == D.DETAG_EINVAL
    assert status(D.Topology(kind=99)) == D.DETAG_EINVAL
    assert status(D.Topology.ring(), dtype=5) == D.DETAG_EINVAL


def test_fused_availability_and_path_selection():
    ring8 = D.detag_create(D.Topology.ring(), 8, 4)
    assert ring8.has_fused()
    ring8.set_path(D.DETAG_PATH_FUSED)
    ring8.set_path(D.DETAG_PATH_PER_ROUND)
    ring7 = D.detag_create(D.Topology.ring(), 7, 4)
    if not ring7.has_fused():
        with pytest.raises(D.DetagError) as ei:
            ring7.set_path(D.DETAG_PATH_FUSED)
        assert ei.value.status == D.DETAG_EUNSUPPORTED
    with pytest.raises(D.DetagError):
        ring8.set_path(17)


def test_device_calls_fail_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    ctx = D.detag_create(D.Topology.ring(), 8, 16)
    import ctypes as C
    st = D.lib().detag_gossip_accel(ctx._h, C.c_void_p(4096), 2, -1.0, None)
    assert st == D.DETAG_EHIP
    assert b"GPU" in D.lib().detag_last_error(ctx._h)


def test_which_kernel_a_topology_gets():
    """The kernel family is a function of (topology, n, path); the families differ in cost by integer factors
    (see detag_get_kernel in detag.h), so the table is pinned."""
    REG, LDS, PER, DENSE = D.DETAG_KERNEL_REGISTER_TILE, D.DETAG_KERNEL_LDS_TILE, D.DETAG_KERNEL_PER_ROUND, D.DETAG_KERNEL_DENSE
    ring = {1: LDS, 2: LDS, 3: LDS, 4: REG, 5: LDS, 7: LDS, 8: REG, 12: REG, 16: REG, 20: LDS, 24: REG, 32: REG, 33: LDS,
            48: REG, 64: REG,
            65: LDS, 128: LDS, 256: LDS, 257: PER}
    for n, want in ring.items():
        assert D.detag_create(D.Topology.ring(), n, 16).kernel() == want, ("ring", n)
    torus = {(4, 4): REG, (4, 8): REG, (8, 8): REG, (8, 4): LDS, (2, 8): LDS, (3, 5): LDS, (16, 16): LDS, (16, 17): PER}
    for (r, c), want in torus.items():
        assert D.detag_create(D.Topology.torus(r, c), r * c, 16).kernel() == want, ("torus", r, c)
    assert D.detag_create(D.Topology.ring(kappa=0.3), 16, 16).kernel() == REG          # the slack matrix keeps the pattern
    assert D.detag_create(D.Topology.random_regular(4, 0), 256, 16).kernel() == LDS
    assert D.detag_create(D.Topology.random_regular(4, 0), 300, 16).kernel() == PER
    star = np.array([(0, j) for j in range(1, 14)])                                     # hub with 13 neighbours
    assert D.detag_create(D.Topology.from_edges(star), 14, 16).kernel() == PER
    ring16_as_edges = D.detag_create(D.Topology.from_edges(gen.edges_ring(16), D.DETAG_W_UNIFORM), 16, 16)
    assert ring16_as_edges.kernel() in (REG, LDS)                                       # the same W given as an edge list
    ctx = D.detag_create(D.Topology.ring(), 8, 16)
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    assert ctx.kernel() == PER
    ctx.set_path(D.DETAG_PATH_DENSE)
    assert ctx.kernel() == DENSE
    ctx.set_path(D.DETAG_PATH_AUTO)
    assert ctx.kernel() == REG


def test_more_rejections_and_degenerate_sizes():
    import ctypes as C
    L = D.lib()
    h = C.c_void_p()
    topo = D.Topology.ring()._as_struct()
    assert L.detag_create(None, 4, 4, 4, D.DETAG_F32, C.byref(h)) == D.DETAG_EINVAL          # NULL topology
    assert L.detag_create(C.byref(topo), 4, 4, 4, D.DETAG_F32, None) == D.DETAG_EINVAL       # NULL out
    assert L.detag_last_error(None)
    csr = D.Topology.from_dense(T.mixing_matrix(4, gen.edges_ring(4)))
    for field in ("rowptr", "colidx", "vals"):                                               # CSR with a missing array
        t = D.Topology(D.DETAG_TOPO_CSR, rowptr=csr.rowptr, colidx=csr.colidx, vals=csr.vals)
        setattr(t, field, None)
        with pytest.raises(D.DetagError) as ei:
            D.detag_create(t, 4, 4)
        assert ei.value.status == D.DETAG_EINVAL
    bad_ptr = D.Topology(D.DETAG_TOPO_CSR, rowptr=np.array([0, 3, 2, 9, 12], np.int32), colidx=csr.colidx, vals=csr.vals)
    bad_col = D.Topology(D.DETAG_TOPO_CSR, rowptr=csr.rowptr, colidx=np.where(csr.colidx == 3, 7, csr.colidx).astype(np.int32), vals=csr.vals)
    nan_val = D.Topology(D.DETAG_TOPO_CSR, rowptr=csr.rowptr, colidx=csr.colidx, vals=np.where(np.arange(len(csr.vals)) == 1, np.nan, csr.vals))
    for t in (bad_ptr, bad_col, nan_val, D.Topology.ring(kappa=float("nan")), D.Topology.torus(0, 4), D.Topology.torus(-2, -2),
              D.Topology.random_regular(4, 0, weights=7)):
        with pytest.raises(D.DetagError) as ei:
            D.detag_create(t, 4, 4)
        assert ei.value.status in (D.DETAG_EINVAL, D.DETAG_ENOT_DOUBLY_STOCHASTIC), ei.value
    with pytest.raises(D.DetagError):
        D.detag_create(D.Topology.random_regular(4, 0), 4, 4)                                # n <= degree
    # degenerate sizes are accepted: one worker (W = [1], eta = 0), two workers
    one = D.detag_create(D.Topology.ring(), 1, 3)
    assert one.dense_W().tolist() == [[1.0]] and one.spectrum()["eta"] == 0.0 and one.phase_length() == 1
    two = D.detag_create(D.Topology.ring(), 2, 3)
    assert np.allclose(two.dense_W(), [[0.5, 0.5], [0.5, 0.5]]) and two.spectrum()["lam"] == pytest.approx(0.0, abs=1e-15)
    R = C.c_int32()
    assert L.detag_get_phase_length(two._h, float("nan"), C.byref(R)) == D.DETAG_EINVAL
    assert L.detag_get_phase_length(two._h, 0.0, None) == D.DETAG_EINVAL
    P = np.empty((2, 2))
    assert L.detag_get_gossip_polynomial(two._h, 3, float("nan"), P.ctypes.data_as(C.POINTER(C.c_double))) == D.DETAG_EINVAL
    assert L.detag_get_gossip_polynomial(two._h, -1, 0.1, P.ctypes.data_as(C.POINTER(C.c_double))) == D.DETAG_EINVAL
    assert L.detag_get_gossip_polynomial(two._h, 0, 0.1, P.ctypes.data_as(C.POINTER(C.c_double))) == D.DETAG_OK and np.array_equal(P, np.eye(2))
    k = C.c_int32()
    assert L.detag_get_kernel(None, C.byref(k)) == D.DETAG_EINVAL and L.detag_get_kernel(two._h, None) == D.DETAG_EINVAL
    with pytest.raises(D.DetagError):
        D.Factors(two, root=5)                                                               # root outside the graph


@pytest.mark.parametrize("seed", range(6))
def test_random_graphs_build_and_agree_with_the_oracle(seed):
    """Random connected graphs of random size and degree, Metropolis weights: the library's W, spectrum and the
    factor sequence of the exact average against the oracle's."""
    from oracle import consensus as OC
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 40))
    e = {(i, i + 1) for i in range(n - 1)}
    for _ in range(int(rng.integers(0, 3 * n))):
        a, b = sorted(rng.integers(0, n, 2).tolist())
        if a != b:
            e.add((a, b))
    e = np.array(sorted(e), dtype=np.int64).reshape(-1, 2)
    if len(e) == 0:
        pytest.skip("no edge")
    ctx = D.detag_create(D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), n, 8)
    W = T.mixing_matrix(n, e, "metropolis")
    assert np.allclose(ctx.dense_W(), W, rtol=0, atol=1e-15)
    assert ctx.spectrum()["lam"] == pytest.approx(T.spectrum(W)[2], abs=1e-11)
    root = int(rng.integers(0, n))
    f = D.Factors(ctx, root)
    ref = OC.gather_propagate_factors(n, e, root)
    assert f.R == len(ref)
    prod = np.eye(n)
    for r in range(f.R):
        assert np.allclose(f.dense(r), ref[r], rtol=0, atol=1e-15)
        prod = f.dense(r) @ prod
    assert np.allclose(prod, np.full((n, n), 1.0 / n), atol=1e-12)


def test_bench_refuses_more_than_one_gpu():
    """The library has no cross-GPU code: the benchmark says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
