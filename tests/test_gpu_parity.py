"""Parity of the HIP path (through the C ABI) against the fp64 oracle, element by
element, on the same seeded inputs.  Bar: max relative error (tests/util.py)
1e-5 for fp32 state, 2e-2 for bf16 state; padding columns must stay untouched.
"""
import os

import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from oracle import gossip as OG
from oracle import noise as ON
from oracle import objectives as OO
from oracle import topology as OT
from tests.util import TOL_BF16, TOL_F32, amax, rel_err
from workloads import generate as gen

pytestmark = pytest.mark.gpu

from tests.gpu_util import DEV, SENTINEL, _built, make_ctx, padding_ok, to_dev, to_host  # noqa: F401


def eta_for(W):
    return OT.eta_from_lambda(OT.spectrum(W)[2]) if np.allclose(W, W.T) else 0.3


# ---------------------------------------------------------------------------
# accelerated gossip
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind,n", [("asym", 5), ("ring", 5), ("ring", 7), ("rr", 12), ("ring", 2), ("ring", 1)])
@pytest.mark.parametrize("K", [0, 1, 2, 3, 4, 5, 8])
def test_gossip_per_round_matches_oracle(kind, n, K):
    d, ld = 1029, 1032          # two vector blocks and a ragged tail; pitch a multiple of 4
    ctx, W = make_ctx(kind, n, d, ld)
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    eta = eta_for(W)
    Z = gen.state(n, d, seed=K + 1)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K, eta)
    ref = OG.accelerated_gossip(Z, W, K, eta)
    assert rel_err(to_host(Zd, d), ref, amax(Z)) < TOL_F32
    assert padding_ok(Zd, d)


def test_gossip_per_round_unaligned_pitch_uses_scalar_path():
    n, d, ld, K = 6, 515, 517, 5     # odd pitch: no 16-byte row alignment
    ctx, W = make_ctx("ring", n, d, ld)
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    eta = eta_for(W)
    Z = gen.state(n, d, seed=3)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K)             # eta < 0: the context's own eta
    assert ctx.spectrum()["eta"] == pytest.approx(eta, abs=1e-12)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(Z, W, K, eta), amax(Z)) < TOL_F32
    assert padding_ok(Zd, d)


@pytest.mark.parametrize("kind,n", [("ring", 4), ("ring", 8), ("ring", 12), ("ring", 16), ("ring", 24), ("ring", 32),
                                    ("ring", 48), ("ring", 64),
                                    ("torus44", 16), ("torus48", 32), ("torus88", 64), ("ring_slack", 16)])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 7, 8])
def test_gossip_fused_matches_oracle(kind, n, K):
    d, ld = 777, 777              # three full 256-column tiles and a ragged one, odd pitch
    ctx, W = make_ctx(kind, n, d, ld)
    assert ctx.has_fused()
    ctx.set_path(D.DETAG_PATH_FUSED)
    eta = eta_for(W)
    Z = gen.state(n, d, seed=K)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K, eta)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(Z, W, K, eta), amax(Z)) < TOL_F32
    assert padding_ok(Zd, d)


def test_gossip_preserves_worker_mean_and_contracts():
    n, d, ld, K = 64, 4096, 4096, 8
    ctx, W = make_ctx("torus88", n, d, ld)
    Z = gen.state(n, d, seed=11)
    Zd = to_dev(Z, ld)
    before = ctx.consensus_error(Zd).item()
    mean0 = ctx.mean(Zd).cpu().numpy().astype(np.float64)
    ctx.gossip_accel(Zd, K)
    after = ctx.consensus_error(Zd).item()
    mean1 = ctx.mean(Zd).cpu().numpy().astype(np.float64)
    assert np.abs(mean1 - mean0).max() < 1e-6
    assert mean0 == pytest.approx(OG.worker_mean(Z), abs=1e-7)
    assert before == pytest.approx(OG.consensus_error(Z), rel=1e-6)
    # exact contraction bound: max_{mu != 1} |p_K(mu)| for the 8x8 torus at K=8 is 0.071117
    assert (after / before) ** 0.5 <= 0.071117 * (1 + 1e-4)
    eta = ctx.spectrum()["eta"]
    assert after == pytest.approx(OG.consensus_error(OG.accelerated_gossip(Z, W, K, eta)), rel=1e-4)


# ---------------------------------------------------------------------------
# tracking, phase update, D-PSGD
# ---------------------------------------------------------------------------
def test_track_matches_oracle():
    n, d, ld = 7, 1000, 1024
    ctx, _ = make_ctx("ring", n, d, ld)
    Y, Gn, Go = gen.state(n, d, 1), gen.state(n, d, 2), gen.state(n, d, 3)
    Yd, Gnd, God = to_dev(Y, ld), to_dev(Gn, ld), to_dev(Go, ld)
    ctx.track(Yd, Gnd, God)
    assert rel_err(to_host(Yd, d), OG.tracking_update(Y, Gn, Go)) < TOL_F32
    assert padding_ok(Yd, d)


STEP_CASES = [("ring", 12, D.DETAG_PATH_FUSED), ("ring", 24, D.DETAG_PATH_FUSED), ("ring", 48, D.DETAG_PATH_FUSED),
              ("ring", 24, D.DETAG_PATH_PER_ROUND),
              ("ring", 8, D.DETAG_PATH_FUSED), ("ring", 8, D.DETAG_PATH_PER_ROUND),
              ("ring", 16, D.DETAG_PATH_FUSED), ("ring", 32, D.DETAG_PATH_FUSED),
              ("torus88", 64, D.DETAG_PATH_FUSED), ("torus88", 64, D.DETAG_PATH_PER_ROUND),
              ("torus48", 32, D.DETAG_PATH_FUSED), ("asym", 5, D.DETAG_PATH_PER_ROUND),
              ("rr", 12, D.DETAG_PATH_AUTO), ("ring", 7, D.DETAG_PATH_AUTO)]


@pytest.mark.parametrize("kind,n,path", STEP_CASES)
@pytest.mark.parametrize("variant", ["atc", "alg2"])
@pytest.mark.parametrize("K", [0, 1, 4, 5])
def test_step_matches_oracle(kind, n, path, variant, K):
    d, ld = 600, 640
    ctx, W = make_ctx(kind, n, d, ld)
    ctx.set_path(path)
    eta, alpha = eta_for(W), 0.05
    X, Y, Gn, Go = (gen.state(n, d, s) for s in (1, 2, 3, 4))
    Xd, Yd, Gnd, God = (to_dev(a, ld) for a in (X, Y, Gn, Go))
    ctx.step(Xd, Yd, Gnd, God, alpha, K, eta, D.DETAG_VARIANT_ATC if variant == "atc" else D.DETAG_VARIANT_ALG2)
    Xr, Yr = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
    S = amax(X, Y, Gn, Go)
    assert rel_err(to_host(Xd, d), Xr, S) < TOL_F32
    assert rel_err(to_host(Yd, d), Yr, S) < TOL_F32
    assert np.array_equal(to_host(Gnd, d), Gn.astype(np.float64))     # inputs untouched
    assert np.array_equal(to_host(God, d), Go.astype(np.float64))
    assert padding_ok(Xd, d) and padding_ok(Yd, d)


def test_dpsgd_step_matches_oracle():
    n, d, ld = 8, 900, 960
    ctx, W = make_ctx("ring", n, d, ld)
    X, Gr = gen.state(n, d, 1), gen.state(n, d, 2)
    Xd, Gd = to_dev(X, ld), to_dev(Gr, ld)
    ctx.dpsgd_step(Xd, Gd, 0.1)
    assert rel_err(to_host(Xd, d), OG.dpsgd_step(X, Gr, W, 0.1)) < TOL_F32
    assert padding_ok(Xd, d)


# ---------------------------------------------------------------------------
# diagnostics
# ---------------------------------------------------------------------------
def test_mean_and_consensus_error_match_oracle():
    n, d, ld = 16, 5000, 5056
    ctx, _ = make_ctx("ring", n, d, ld)
    X = gen.state(n, d, seed=5) + 3.0
    Xd = to_dev(X, ld)
    assert rel_err(ctx.mean(Xd).cpu().numpy()[None, :], OG.worker_mean(X)[None, :]) < TOL_F32
    ce = ctx.consensus_error(Xd).item()
    assert ce == pytest.approx(OG.consensus_error(X), rel=1e-10)
    assert ctx.consensus_error(Xd).item() == ce                    # deterministic reduction
    near = np.tile(X[:1], (n, 1)); near[3, 7] += 1e-3               # workers agree except one entry
    got = ctx.consensus_error(to_dev(near, ld)).item()
    assert got == pytest.approx(OG.consensus_error(near.astype(np.float32)), rel=1e-6)


# ---------------------------------------------------------------------------
# gradients
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("ld", [1003, 1024])
def test_grad_quadratic_with_noise_array(ld):
    n, d = 6, 1003
    ctx, _ = make_ctx("ring", n, d, ld)
    h, b = gen.quadratic_problem(n, d, seed=2)
    X, z = gen.state(n, d, 1), gen.gaussian(n, d, seed=2, step=0)
    hd = torch.zeros(ld); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    Xd, bd, zd, Gd = to_dev(X, ld), to_dev(b, ld), to_dev(z, ld), to_dev(np.zeros((n, d)), ld)
    ctx.grad_quadratic_diag(Xd, hd, bd, Gd, noise=zd, sigma=0.1)
    assert rel_err(to_host(Gd, d), OO.grad_quadratic_diag(X, h, b, z, 0.1)) < TOL_F32
    assert padding_ok(Gd, d)
    # per-worker curvature, no noise
    hw = (np.tile(h, (n, 1)) * np.arange(1, n + 1)[:, None]).astype(np.float32)
    ctx.grad_quadratic_diag(Xd, to_dev(hw, ld), bd, Gd)
    assert rel_err(to_host(Gd, d), OO.grad_quadratic_diag(X, hw, b)) < TOL_F32


def test_grad_quadratic_counter_noise_matches_oracle_generator():
    """In-kernel Philox-4x32-10 + Box-Muller against the oracle's own
    implementation of the same published generator.  The uniforms are
    bit-identical; the fp32 log/sin/cos differ from fp64 by a few ulp of the
    normal, so the noise itself is compared at 2e-6 absolute (|z| < 5.8) and the
    gradient at the fp32 bar."""
    n, d, ld, sigma, seed, step = 5, 4099, 4100, 0.1, 1234567890123, 17
    ctx, _ = make_ctx("ring", n, d, ld)
    h, b = gen.quadratic_problem(n, d, seed=2)
    X = gen.state(n, d, 1)
    hd = torch.zeros(ld); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    Xd, bd, Gd = to_dev(X, ld), to_dev(b, ld), to_dev(np.zeros((n, d)), ld)
    ctx.grad_quadratic_diag(Xd, hd, bd, Gd, sigma=sigma, seed=seed, step=step)
    z = ON.normal_noise(seed, step, n, np.arange(d))
    ref = OO.grad_quadratic_diag(X, h, b, z, sigma)
    got = to_host(Gd, d)
    assert rel_err(got, ref) < TOL_F32
    clean = OO.grad_quadratic_diag(X, h, b)
    assert np.abs((got - clean) / sigma - z).max() < 2e-5     # limited by fp32 cancellation in got - clean
    ctx.grad_quadratic_diag(Xd, hd, bd, Gd, sigma=sigma, seed=seed, step=step + 1)
    assert np.abs(to_host(Gd, d) - got).max() > 1e-3          # a new step draws new noise
    assert padding_ok(Gd, d)


def test_grad_lstsq_matches_oracle():
    n, m, d, ld = 8, 64, 1024, 1024
    ctx, _ = make_ctx("ring", n, d, ld)
    A, b = gen.lstsq_problem(n, m, d, seed=0, shift=3.5)
    X = gen.state(n, d, 1)
    Xd, Gd = to_dev(X, ld), to_dev(np.zeros((n, d)), ld)
    ctx.grad_lstsq(Xd, torch.from_numpy(A).to(DEV), torch.from_numpy(b).to(DEV), Gd)
    assert rel_err(to_host(Gd, d), OO.grad_lstsq(X, A, b)) < TOL_F32


# ---------------------------------------------------------------------------
# bf16 state
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind,n,path", [("ring", 16, D.DETAG_PATH_FUSED), ("ring", 16, D.DETAG_PATH_PER_ROUND),
                                         ("rr", 12, D.DETAG_PATH_AUTO), ("torus88", 64, D.DETAG_PATH_FUSED)])
@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_bf16_state_step(kind, n, path, variant):
    """Inputs are the bf16-rounded values; the oracle works in fp64 with no
    intermediate rounding; the bf16 result must land within 2e-2."""
    d, ld, K, alpha = 700, 704, 6, 0.05
    ctx, W = make_ctx(kind, n, d, ld, D.DETAG_BF16)
    ctx.set_path(path)
    eta = eta_for(W)
    X, Y = OO.round_bf16(gen.state(n, d, 1)), OO.round_bf16(gen.state(n, d, 2))
    Gn, Go = gen.state(n, d, 3), gen.state(n, d, 4)
    Xd, Yd = to_dev(X, ld, torch.bfloat16), to_dev(Y, ld, torch.bfloat16)
    assert np.array_equal(to_host(Xd, d), X.astype(np.float64))       # already representable
    Gnd, God = to_dev(Gn, ld), to_dev(Go, ld)
    ctx.step(Xd, Yd, Gnd, God, alpha, K, eta, D.DETAG_VARIANT_ATC if variant == "atc" else D.DETAG_VARIANT_ALG2)
    Xr, Yr = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
    S = amax(X, Y, Gn, Go)
    assert rel_err(to_host(Xd, d), Xr, S) < TOL_BF16
    assert rel_err(to_host(Yd, d), Yr, S) < TOL_BF16
    assert padding_ok(Xd, d) and padding_ok(Yd, d)
    # every path computes in fp32 (on chip, or in widened scratch on the per-round path) and rounds once
    # at the end: the stored value is the RNE rounding of the fp32 result, so it is within half a bf16 ulp
    # (2^-9 relative) of the oracle, up to fp32 noise
    assert rel_err(to_host(Xd, d), Xr) < 2.0 ** -8
    assert rel_err(to_host(Yd, d), Yr) < 2.0 ** -8


def test_bf16_gossip_and_diagnostics():
    n, d, ld, K = 32, 1000, 1024, 8
    ctx, W = make_ctx("ring", n, d, ld, D.DETAG_BF16)
    Z = OO.round_bf16(gen.state(n, d, 1))
    Zd = to_dev(Z, ld, torch.bfloat16)
    assert ctx.consensus_error(Zd).item() == pytest.approx(OG.consensus_error(Z), rel=1e-10)
    ctx.gossip_accel(Zd, K)
    ref = OG.accelerated_gossip(Z, W, K, ctx.spectrum()["eta"])
    assert rel_err(to_host(Zd, d), ref, amax(Z)) < TOL_BF16


# ---------------------------------------------------------------------------
# whole runs
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("path", [D.DETAG_PATH_FUSED, D.DETAG_PATH_PER_ROUND])
def test_config1_full_run_matches_oracle(path):
    """n=8 ring, d=1024, least squares, x0=0, lr=0.05, K=4, T=50: the whole
    trajectory (gradient + phase, 50 times) against the oracle."""
    from workloads import CONFIGS
    cfg = CONFIGS[1]
    n, d, m, K, T, alpha = cfg.n, cfg.d, cfg.extra["m"], cfg.K, cfg.T, cfg.lr
    A, b = gen.lstsq_problem(n, m, d, seed=cfg.seed, shift=cfg.extra["offset_shift"])
    ctx, W = make_ctx("ring", n, d, d)
    ctx.set_path(path)
    eta = ctx.spectrum()["eta"]
    assert eta == pytest.approx(eta_for(W), abs=1e-12)
    Ad, bd = torch.from_numpy(A).to(DEV), torch.from_numpy(b).to(DEV)
    Xd, Yd = D.new_matrix(n, d, d), D.new_matrix(n, d, d)
    Ga, Gb = D.new_matrix(n, d, d), D.new_matrix(n, d, d)       # G_new / G_old, swapped every step
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for _ in range(T):
        ctx.grad_lstsq(Xd, Ad, bd, Ga)
        ctx.step(Xd, Yd, Ga, Gb, alpha, K)
        Ga, Gb = Gb, Ga
        Gnew = OO.grad_lstsq(X, A, b)
        X, Y = OG.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta)
        Gold = Gnew
    S = amax(X, Y, Gold)                      # whole run: normwise (see tests/util.py)
    assert rel_err(to_host(Xd, d), X, S, floor=1.0) < TOL_F32
    assert rel_err(to_host(Yd, d), Y, S, floor=1.0) < TOL_F32
    # invariants of the proof of Theorem 3 hold on the device state too
    assert np.abs(to_host(Yd, d).mean(0) - Gold.mean(0)).max() < 1e-5
    xhat = ctx.mean(Xd).cpu().numpy()
    assert rel_err(xhat[None], OG.worker_mean(X)[None], S, floor=1.0) < TOL_F32
    # T=50 is far from converged; the loss has dropped a lot from f(0)
    f = lambda x: 0.5 * np.mean([np.sum((A[i].astype(np.float64) @ x - b[i]) ** 2) for i in range(n)])
    assert f(xhat.astype(np.float64)) < 0.1 * f(np.zeros(d))


def test_config2_shape_short_run_matches_oracle():
    """n=16 ring, d=272,474 (full size), diagonal quadratic with in-kernel
    counter noise sigma=0.1, K=6, lr=0.5; 4 steps instead of 200 so the oracle
    finishes in seconds."""
    from workloads import CONFIGS
    cfg = CONFIGS[2]
    n, d, K, alpha, sigma, T = cfg.n, cfg.d, cfg.K, cfg.lr, cfg.sigma, 4
    ld = D.padded_ld(d)
    h, b = gen.quadratic_problem(n, d, seed=cfg.seed, b_mean="i/n")
    ctx, W = make_ctx("ring", n, d, ld)
    eta = ctx.spectrum()["eta"]
    hd = torch.zeros(ld); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    bd = to_dev(b, ld)
    Xd, Yd, Ga, Gb = (D.new_matrix(n, d, ld) for _ in range(4))
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    cols = np.arange(d)
    for t in range(T):
        ctx.grad_quadratic_diag(Xd, hd, bd, Ga, sigma=sigma, seed=cfg.seed, step=t)
        ctx.step(Xd, Yd, Ga, Gb, alpha, K)
        Ga, Gb = Gb, Ga
        Gnew = OO.grad_quadratic_diag(X, h, b, ON.normal_noise(cfg.seed, t, n, cols), sigma)
        X, Y = OG.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta)
        Gold = Gnew
    S = amax(X, Y, Gold)                      # whole run: normwise (see tests/util.py)
    assert rel_err(to_host(Xd, d), X, S, floor=1.0) < TOL_F32
    assert rel_err(to_host(Yd, d), Y, S, floor=1.0) < TOL_F32


def test_errors_are_statuses_not_crashes():
    ctx, _ = make_ctx("ring", 8, 100, 128)
    Z = D.new_matrix(8, 100, 128)
    with pytest.raises(D.DetagError) as ei:
        ctx.gossip_accel(Z, -1)
    assert ei.value.status == D.DETAG_EINVAL
    with pytest.raises(D.DetagError):
        ctx.gossip_accel(Z, 2, eta=1.0)
    with pytest.raises(D.DetagError):
        ctx.step(Z, Z, Z, Z, 0.1, 2)                  # overlapping buffers
    actx, _ = make_ctx("asym", 5, 100, 128)
    with pytest.raises(D.DetagError) as ei:
        actx.gossip_accel(D.new_matrix(5, 100, 128), 2)    # no stored eta for an asymmetric W
    assert ei.value.status == D.DETAG_EINVAL
    with pytest.raises(ValueError):
        ctx.gossip_accel(torch.zeros(8, 64, device=DEV), 2)   # wrong pitch is caught by the binding


# ---------------------------------------------------------------------------
# on-chip kernel for arbitrary W (n <= 256)
# ---------------------------------------------------------------------------
def _irregular_edges(n, seed, max_deg=8):
    rng = np.random.default_rng(seed)
    e = {(i, i + 1) for i in range(n - 1)}                     # a path keeps it connected
    deg = np.zeros(n, int); deg[0] = deg[-1] = 1; deg[1:-1] = 2
    while len(e) < 2 * n:
        a, b = sorted(rng.integers(0, n, 2).tolist())
        if a != b and (a, b) not in e and deg[a] < max_deg and deg[b] < max_deg:
            e.add((a, b)); deg[a] += 1; deg[b] += 1
    return np.array(sorted(e), dtype=np.int64)


def test_wide_rows_fall_back_to_the_per_round_path():
    n, d, ld, K = 14, 100, 128, 3                               # a star: the hub has 13 neighbours, more than the on-chip kernel's 8
    e = np.array([(0, j) for j in range(1, n)])
    W = OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), n, d, ld)
    assert not ctx.has_fused()
    with pytest.raises(D.DetagError) as ei:
        ctx.set_path(D.DETAG_PATH_FUSED)
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    Z = gen.state(n, d, seed=1)
    Zd = to_dev(Z, ld)
    ctx.gossip_accel(Zd, K)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(Z, W, K, eta_for(W)), amax(Z)) < TOL_F32


@pytest.mark.parametrize("n,graph", [(5, "asym"), (12, "rr"), (61, "irregular"), (100, "irregular"), (130, "rr"), (256, "rr"),
                                     (1, "ring"), (2, "ring"), (3, "ring"), (17, "ring"),    # degenerate and odd rings
                                     # worker counts at and just past a full set of row slots (16 wavefronts x 1, 2, 4, 8 rows)
                                     (16, "rr"), (33, "irregular"), (64, "rr"), (128, "rr"), (129, "irregular")])
@pytest.mark.parametrize("K", [1, 2, 5, 16])
def test_generic_fused_gossip_and_step(n, graph, K):
    d, ld = 150, 160               # two full 64-column tiles and a ragged one
    if graph == "asym":
        W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)
        topo = D.Topology.from_dense(W)
    elif graph == "ring":          # n = 1: W = [1]; n = 2: one edge; sizes the register-resident kernels do not cover
        topo, W = D.Topology.ring(), OT.mixing_matrix(n, gen.edges_ring(n))
    else:
        e = gen.edges_random_regular(n, 4, seed=n) if graph == "rr" else _irregular_edges(n, seed=n)
        topo, W = D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(topo, n, d, ld)
    assert ctx.has_fused()
    ctx.set_path(D.DETAG_PATH_FUSED)
    eta, alpha = eta_for(W), 0.05
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


def test_config5_shape_bf16_short_run():
    """n=256 random 4-regular graph with Metropolis weights, bf16 X/Y, K=16, lr=0.5,
    heterogeneous offsets b ~ N(0,4); d reduced to 4,096 columns and 3 steps so
    the oracle finishes in seconds (columns are independent).  The oracle rounds
    X and Y to bf16 after every step, as the stored state is."""
    from workloads import CONFIGS
    cfg = CONFIGS[5]
    n, K, alpha = cfg.n, cfg.K, cfg.lr
    d, T = 4096 + 37, 3
    ld = D.padded_ld(d)
    e = gen.edges_random_regular(n, 4, seed=cfg.seed)
    W = OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), n, d, ld, D.DETAG_BF16)
    eta = ctx.spectrum()["eta"]
    assert eta == pytest.approx(eta_for(W), abs=1e-12)
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
        if t == 0:      # one step from identical inputs, no intermediate rounding in the oracle
            S1 = amax(X, Y, Gnew, Gold)
            assert rel_err(to_host(Xd, d), Xn, S1) < TOL_BF16
            assert rel_err(to_host(Yd, d), Yn, S1) < TOL_BF16
        X, Y, Gold = OO.round_bf16(Xn).astype(np.float64), OO.round_bf16(Yn).astype(np.float64), Gnew
    S = amax(X, Y, Gold)
    assert rel_err(to_host(Xd, d), X, S, floor=1.0) < TOL_BF16
    assert rel_err(to_host(Yd, d), Y, S, floor=1.0) < TOL_BF16


# ---------------------------------------------------------------------------
# gradient query + phase in one kernel
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind,n", [("ring", 8), ("ring", 12), ("ring", 16), ("ring", 24), ("ring", 48), ("torus48", 32),
                                    ("torus88", 64), ("ring", 64)])
@pytest.mark.parametrize("sigma", [0.0, 0.1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_step_quadratic_matches_oracle_and_the_two_separate_calls(kind, n, sigma, dtype, variant):
    d, ld, K, alpha, seed = 777, 832, 5, 0.5, 99
    bf = dtype == "bf16"
    var = D.DETAG_VARIANT_ATC if variant == "atc" else D.DETAG_VARIANT_ALG2
    tdt = torch.bfloat16 if bf else torch.float32
    ctx, W = make_ctx(kind, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    eta = eta_for(W)
    h, b = gen.quadratic_problem(n, d, seed=3)
    X, Y, Go = gen.state(n, d, 1), gen.state(n, d, 2), gen.state(n, d, 3)
    if bf:
        X, Y = OO.round_bf16(X), OO.round_bf16(Y)
    hd = torch.full((ld,), SENTINEL); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    bd = to_dev(b, ld)
    cols = np.arange(d)
    # fused
    Xf, Yf, Gf = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld)
    # separate calls
    Xs, Ys, Gos, Gns = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld), to_dev(np.zeros((n, d)), ld)
    Xr, Yr, Gor = X.astype(np.float64), Y.astype(np.float64), Go.astype(np.float64)
    for t in range(2):
        ctx.step_quadratic(Xf, Yf, Gf, hd, bd, alpha, K, sigma=sigma, seed=seed, step=t, variant=var)
        ctx.grad_quadratic_diag(Xs, hd, bd, Gns, sigma=sigma, seed=seed, step=t)
        ctx.step(Xs, Ys, Gns, Gos, alpha, K, variant=var)
        Gos, Gns = Gns, Gos
        noise = ON.normal_noise(seed, t, n, cols) if sigma else None
        Gn = OO.grad_quadratic_diag(Xr, h, b, noise, sigma)
        if t == 0:
            S = amax(Xr, Yr, Gn, Gor)
            Xn, Yn = OG.detag_step(Xr, Yr, Gn, Gor, W, alpha, K, eta, variant)
            tol = TOL_BF16 if bf else TOL_F32
            assert rel_err(to_host(Gf, d), Gn, S) < TOL_F32
            assert rel_err(to_host(Xf, d), Xn, S) < tol
            assert rel_err(to_host(Yf, d), Yn, S) < tol
        # same arithmetic as the two separate kernels: bit-identical state and gradient, both steps
        torch.cuda.synchronize()
        assert torch.equal(Xf, Xs) and torch.equal(Yf, Ys) and torch.equal(Gf, Gos)
        Xr, Yr, Gor = to_host(Xf, d), to_host(Yf, d), to_host(Gf, d)
    assert padding_ok(Xf, d) and padding_ok(Yf, d) and padding_ok(Gf, d)


def test_step_quadratic_unsupported_cases_are_statuses():
    n = 12
    full = [(i, j) for i in range(n) for j in range(i + 1, n)]         # 11 neighbours per worker: no on-chip kernel
    ctx = D.detag_create(D.Topology.from_edges(full, D.DETAG_W_METROPOLIS), n, 100, 128)
    assert not ctx.has_fused()
    X, Y, Gm, b = (D.new_matrix(n, 100, 128) for _ in range(4))
    h = torch.ones(128, device=DEV)
    with pytest.raises(D.DetagError) as ei:
        ctx.step_quadratic(X, Y, Gm, h, b, 0.1, 4)
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    ctx1, _ = make_ctx("rr", 12, 100, 128)                            # LDS-resident family: ATC only
    with pytest.raises(D.DetagError) as ei:
        ctx1.step_quadratic(X, Y, Gm, h, b, 0.1, 4, variant=D.DETAG_VARIANT_ALG2)
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    ctx1.set_path(D.DETAG_PATH_PER_ROUND)
    with pytest.raises(D.DetagError) as ei:
        ctx1.step_quadratic(X, Y, Gm, h, b, 0.1, 4)
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    ctx2, _ = make_ctx("ring", 8, 100, 128)
    X, Y, Gm, b = (D.new_matrix(8, 100, 128) for _ in range(4))
    with pytest.raises(D.DetagError) as ei:
        ctx2.step_quadratic(X, Y, Gm, h, b, 0.1, 0)
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    with pytest.raises(D.DetagError) as ei:
        ctx2.step_quadratic(X, X, Gm, h, b, 0.1, 2)
    assert ei.value.status == D.DETAG_EINVAL
    with pytest.raises(D.DetagError) as ei:
        ctx2.step_quadratic(X, Y, Gm, h, b, 0.1, 2, variant=7)
    assert ei.value.status == D.DETAG_EINVAL


@pytest.mark.parametrize("n,graph", [(5, "asym"), (12, "rr"), (17, "ring"), (33, "irregular"), (61, "irregular"),
                                     (100, "irregular"), (128, "rr"), (256, "rr")])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("hkind", ["shared", "per_worker"])
def test_step_quadratic_on_lds_resident_contexts(n, graph, dtype, hkind):
    """Gradient query + ATC phase in one kernel for an arbitrary sparse W (every count of row slots per wavefront):
    two steps against the oracle and bit for bit against detag_grad_quadratic_diag + detag_step."""
    d, ld, K, alpha, sigma, seed = 150, 160, 5, 0.4, 0.1, 11           # two full 64-column tiles and a ragged one
    bf = dtype == "bf16"
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    if graph == "asym":
        W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)
        topo = D.Topology.from_dense(W)
    elif graph == "ring":
        topo, W = D.Topology.ring(), OT.mixing_matrix(n, gen.edges_ring(n))
    else:
        e = gen.edges_random_regular(n, 4, seed=n) if graph == "rr" else _irregular_edges(n, seed=n)
        topo, W = D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(topo, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    assert ctx.kernel() == D.DETAG_KERNEL_LDS_TILE
    eta = 0.3 if graph == "asym" else eta_for(W)
    h1, b = gen.quadratic_problem(n, d, seed=3)
    if hkind == "per_worker":
        h = np.exp(np.random.default_rng(5).uniform(np.log(1e-3), 0.0, size=(n, d))).astype(np.float32)
        hd = to_dev(h, ld)
    else:
        h = h1
        hd = torch.full((ld,), SENTINEL); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    X, Y, Go = gen.state(n, d, 1), gen.state(n, d, 2), gen.state(n, d, 3)
    if bf:
        X, Y = OO.round_bf16(X), OO.round_bf16(Y)
    bd = to_dev(b, ld)
    cols = np.arange(d)
    Xf, Yf, Gf = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld)
    Xs, Ys, Gos, Gns = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld), to_dev(np.zeros((n, d)), ld)
    Xr, Yr, Gor = X.astype(np.float64), Y.astype(np.float64), Go.astype(np.float64)
    for t in range(2):
        ctx.step_quadratic(Xf, Yf, Gf, hd, bd, alpha, K, sigma=sigma, seed=seed, step=t, eta=eta)
        ctx.grad_quadratic_diag(Xs, hd, bd, Gns, sigma=sigma, seed=seed, step=t)
        ctx.step(Xs, Ys, Gns, Gos, alpha, K, eta)
        Gos, Gns = Gns, Gos
        Gn = OO.grad_quadratic_diag(Xr, h, b, ON.normal_noise(seed, t, n, cols), sigma)
        if t == 0:
            S = amax(Xr, Yr, Gn, Gor)
            Xn, Yn = OG.detag_step(Xr, Yr, Gn, Gor, W, alpha, K, eta)
            assert rel_err(to_host(Gf, d), Gn, S) < TOL_F32
            assert rel_err(to_host(Xf, d), Xn, S) < tol
            assert rel_err(to_host(Yf, d), Yn, S) < tol
        torch.cuda.synchronize()
        assert torch.equal(Xf, Xs) and torch.equal(Yf, Ys) and torch.equal(Gf, Gos)
        Xr, Yr, Gor = to_host(Xf, d), to_host(Yf, d), to_host(Gf, d)
    assert padding_ok(Xf, d) and padding_ok(Yf, d) and padding_ok(Gf, d)


# ---------------------------------------------------------------------------
# one gossip round with the neighbour tile staged in LDS (n <= 256, matrices of 128 MiB and more)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,graph", [(5, "asym"), (17, "ring"), (61, "irregular"), (64, "torus88"), (256, "rr")])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pad", [0, 5])          # pitch a multiple of 64, and an odd pitch
def test_one_round_with_lds_staged_tile(n, graph, dtype, pad):
    d = 64 * 256 + 37                            # 257 column tiles, the last one ragged
    bf = dtype == "bf16"
    # the launcher takes this kernel from 128 MiB per matrix on (n * pitch * element size): a wide pitch gets a
    # narrow matrix there, so that the oracle's work stays small
    ld = D.padded_ld(max(d, -(-(128 << 20) // (n * (2 if bf else 4))))) + pad
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    if graph == "asym":
        W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)
        topo = D.Topology.from_dense(W)
    elif graph == "ring":
        topo, W = D.Topology.ring(), OT.mixing_matrix(n, gen.edges_ring(n))
    elif graph == "torus88":
        topo, W = D.Topology.torus(8, 8), OT.mixing_matrix(n, gen.edges_torus(8, 8))
    else:
        e = gen.edges_random_regular(n, 4, seed=n) if graph == "rr" else _irregular_edges(n, seed=n)
        topo, W = D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), OT.mixing_matrix(n, e, "metropolis")
    ctx = D.detag_create(topo, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    rnd = OO.round_bf16 if bf else (lambda a: a)
    cur, prev, G = rnd(gen.state(n, d, 1)), rnd(gen.state(n, d, 2)), gen.state(n, d, 3)
    eta, alpha = 0.3, 0.05
    want = (1 + eta) * (W.T @ cur.astype(np.float64)) - eta * prev.astype(np.float64)
    # out distinct from both inputs, and out written over z_{r-1}
    cd, pd, od = to_dev(cur, ld, tdt), to_dev(prev, ld, tdt), to_dev(np.zeros((n, d)), ld, tdt)
    ctx.gossip_round(cd, pd, od, eta)
    assert rel_err(to_host(od, d), want, amax(cur, prev)) < tol and padding_ok(od, d)
    ctx.gossip_round(cd, pd, pd, eta)
    torch.cuda.synchronize()
    assert torch.equal(pd, od) and padding_ok(pd, d)
    assert np.array_equal(to_host(cd, d), cur.astype(np.float64))          # z_r is only read
    # the D-PSGD step on the per-round path takes the same kernel with the gradient in place of z_{r-1}
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    xd, gd = to_dev(cur, ld, tdt), to_dev(G, ld)
    ctx.dpsgd_step(xd, gd, alpha)
    assert rel_err(to_host(xd, d), OG.dpsgd_step(cur, G, W, alpha), amax(cur, G)) < tol and padding_ok(xd, d)
    # K rounds through the per-round path land where the on-chip kernels land
    K = 3
    zd = to_dev(cur, ld, tdt)
    ctx.gossip_accel(zd, K, eta)
    assert rel_err(to_host(zd, d), OG.accelerated_gossip(cur, W, K, eta), amax(cur)) < tol and padding_ok(zd, d)


@pytest.mark.parametrize("kind,n", [("ring", 12), ("ring", 16), ("ring", 48), ("torus88", 64)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("variant", ["atc", "alg2"])
def test_step_quadratic_with_per_worker_curvature(kind, n, dtype, variant):
    """h as an n x ld matrix (every worker its own curvature): against the oracle and bit for bit against
    detag_grad_quadratic_diag + detag_step on the same inputs."""
    d, ld, K, alpha, sigma, seed = 700, 704, 4, 0.4, 0.1, 7
    bf = dtype == "bf16"
    var = D.DETAG_VARIANT_ATC if variant == "atc" else D.DETAG_VARIANT_ALG2
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    ctx, W = make_ctx(kind, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    eta = eta_for(W)
    _, b = gen.quadratic_problem(n, d, seed=3)
    h = np.exp(np.random.default_rng(5).uniform(np.log(1e-3), 0.0, size=(n, d))).astype(np.float32)
    X, Y, Go = gen.state(n, d, 1), gen.state(n, d, 2), gen.state(n, d, 3)
    if bf:
        X, Y = OO.round_bf16(X), OO.round_bf16(Y)
    hd, bd = to_dev(h, ld), to_dev(b, ld)
    Xf, Yf, Gf = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld)
    Xs, Ys, Gos, Gns = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld), to_dev(np.zeros((n, d)), ld)
    ctx.step_quadratic(Xf, Yf, Gf, hd, bd, alpha, K, sigma=sigma, seed=seed, step=2, variant=var)
    ctx.grad_quadratic_diag(Xs, hd, bd, Gns, sigma=sigma, seed=seed, step=2)
    ctx.step(Xs, Ys, Gns, Gos, alpha, K, variant=var)
    Gn = OO.grad_quadratic_diag(X, h, b, ON.normal_noise(seed, 2, n, np.arange(d)), sigma)
    Xn, Yn = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
    S = amax(X, Y, Gn, Go)
    assert rel_err(to_host(Gf, d), Gn, S) < TOL_F32
    assert rel_err(to_host(Xf, d), Xn, S) < tol and rel_err(to_host(Yf, d), Yn, S) < tol
    torch.cuda.synchronize()
    assert torch.equal(Xf, Xs) and torch.equal(Yf, Ys) and torch.equal(Gf, Gns)
    assert padding_ok(Xf, d) and padding_ok(Yf, d) and padding_ok(Gf, d) and padding_ok(hd, d)


# ---------------------------------------------------------------------------
# matrices narrower than one vector, one wavefront or one tile
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind,n", [("ring", 8), ("torus88", 64), ("rr", 12), ("asym", 5)])
@pytest.mark.parametrize("path", [D.DETAG_PATH_AUTO, D.DETAG_PATH_PER_ROUND])
@pytest.mark.parametrize("d,ld", [(1, 1), (3, 3), (3, 64), (63, 63), (65, 128)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_very_narrow_matrices(kind, n, path, d, ld, dtype):
    """d = 1, 3, 63, 65 columns with the pitch equal to d (odd: no vector access is aligned) and padded: every
    entry point of the step against the oracle, padding untouched."""
    bf = dtype == "bf16"
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    ctx, W = make_ctx(kind, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    ctx.set_path(path)
    eta, alpha, K, sigma, seed = eta_for(W), 0.3, 3, 0.1, 5
    rnd = OO.round_bf16 if bf else (lambda a: a)
    X, Y, Gn, Go = rnd(gen.state(n, d, 1)), rnd(gen.state(n, d, 2)), gen.state(n, d, 3), gen.state(n, d, 4)
    S = amax(X, Y, Gn, Go)
    # gossip alone
    Zd = to_dev(X, ld, tdt)
    ctx.gossip_accel(Zd, K, eta)
    assert rel_err(to_host(Zd, d), OG.accelerated_gossip(X, W, K, eta), amax(X)) < tol and padding_ok(Zd, d)
    # phase, both variants
    for variant, vcode in (("atc", D.DETAG_VARIANT_ATC), ("alg2", D.DETAG_VARIANT_ALG2)):
        Xd, Yd, Gnd, God = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Gn, ld), to_dev(Go, ld)
        ctx.step(Xd, Yd, Gnd, God, alpha, K, eta, vcode)
        Xr, Yr = OG.detag_step(X, Y, Gn, Go, W, alpha, K, eta, variant)
        assert rel_err(to_host(Xd, d), Xr, S) < tol and rel_err(to_host(Yd, d), Yr, S) < tol
        assert padding_ok(Xd, d) and padding_ok(Yd, d)
    # D-PSGD step, worker mean, consensus distance
    Xd, Gd = to_dev(X, ld, tdt), to_dev(Gn, ld)
    ctx.dpsgd_step(Xd, Gd, alpha)
    assert rel_err(to_host(Xd, d), OG.dpsgd_step(X, Gn, W, alpha), S) < tol and padding_ok(Xd, d)
    Xd = to_dev(X, ld, tdt)
    assert np.abs(ctx.mean(Xd).cpu().numpy()[:d] - X.astype(np.float64).mean(axis=0)).max() < 1e-6 * amax(X)
    ce = float(ctx.consensus_error(Xd).item())
    ref = float(((X.astype(np.float64) - X.astype(np.float64).mean(axis=0)) ** 2).sum())
    assert abs(ce - ref) <= 1e-10 * max(ref, 1.0)
    # gradient query, alone and fused with the phase where the context has an on-chip kernel
    h, b = gen.quadratic_problem(n, d, seed=3)
    hd = torch.full((max(ld, 4),), SENTINEL); hd[:d] = torch.from_numpy(h); hd = hd.to(DEV)
    bd, cols = to_dev(b, ld), np.arange(d)
    Gref = OO.grad_quadratic_diag(X.astype(np.float64), h, b, ON.normal_noise(seed, 1, n, cols), sigma)
    Xd, Gd = to_dev(X, ld, tdt), to_dev(np.zeros((n, d)), ld)
    ctx.grad_quadratic_diag(Xd, hd, bd, Gd, sigma=sigma, seed=seed, step=1)
    S2 = amax(X, Gref, Go)
    assert rel_err(to_host(Gd, d), Gref, S2) < TOL_F32 and padding_ok(Gd, d)
    if path == D.DETAG_PATH_AUTO and ctx.has_fused():
        Xd, Yd, Gd = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(Go, ld)
        ctx.step_quadratic(Xd, Yd, Gd, hd, bd, alpha, K, sigma=sigma, seed=seed, step=1, eta=eta)
        Xr, Yr = OG.detag_step(X, Y, Gref, Go, W, alpha, K, eta)
        S3 = amax(X, Y, Gref, Go)
        assert rel_err(to_host(Gd, d), Gref, S3) < TOL_F32
        assert rel_err(to_host(Xd, d), Xr, S3) < tol and rel_err(to_host(Yd, d), Yr, S3) < tol
        assert padding_ok(Xd, d) and padding_ok(Yd, d) and padding_ok(Gd, d)
