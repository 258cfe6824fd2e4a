"""Algorithm 2 iteration by iteration: the three entry points it adds
(detag_gossip_round, detag_accumulate, detag_phase_end), the two-stream
driver, the dynamic phase length, and a recorded HIP graph of two phases, all
against the oracle's iteration-by-iteration form."""
import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from oracle import gossip as OG
from oracle import objectives as OO
from oracle import runs as OR
from oracle import topology as OT
from paper_2006_08085_amd import algorithms as ALG
from tests.gpu_util import DEV, _built, make_ctx, padding_ok, to_dev, to_host  # noqa: F401
from tests.util import TOL_BF16, TOL_F32, amax, rel_err
from workloads import CONFIGS, generate as gen

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,n", [("asym", 5), ("ring", 16), ("rr", 12)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gossip_round_is_one_step_of_algorithm_3(kind, n, dtype):
    bf = dtype == "bf16"
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    d, ld, eta = 1029, 1032, 0.35
    ctx, W = make_ctx(kind, n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    Zc, Zp = gen.state(n, d, 1), gen.state(n, d, 2)
    if bf:
        Zc, Zp = OO.round_bf16(Zc), OO.round_bf16(Zp)
    want = (1 + eta) * (W.T @ Zc.astype(np.float64)) - eta * Zp.astype(np.float64)
    Zcd, Zpd, Zod = to_dev(Zc, ld, tdt), to_dev(Zp, ld, tdt), to_dev(np.zeros((n, d)), ld, tdt)
    ctx.gossip_round(Zcd, Zpd, Zod, eta)
    assert rel_err(to_host(Zod, d), want, amax(Zc, Zp)) < tol
    assert padding_ok(Zod, d)
    ctx.gossip_round(Zcd, Zpd, Zpd, eta)                       # in place over the previous iterate
    assert np.array_equal(to_host(Zpd, d), to_host(Zod, d))
    first = (1 + eta) * (W.T @ Zc.astype(np.float64)) - eta * Zc.astype(np.float64)
    ctx.gossip_round(Zcd, Zcd, Zod, eta)                       # first step of a phase: z_{-1} = z_0
    assert rel_err(to_host(Zod, d), first, amax(Zc)) < tol
    with pytest.raises(D.DetagError):
        ctx.gossip_round(Zcd, Zpd, Zcd, eta)                   # output over the current iterate


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("separate_replica", [True, False])
def test_accumulate_and_phase_end(dtype, separate_replica):
    bf = dtype == "bf16"
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    n, d, ld, alpha = 7, 1300, 1344, 0.2
    ctx, _ = make_ctx("ring", n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    Xt, Y = gen.state(n, d, 1), gen.state(n, d, 2)
    if bf:
        Xt, Y = OO.round_bf16(Xt), OO.round_bf16(Y)
    Gk, Gm, g = gen.state(n, d, 3), gen.state(n, d, 4), gen.state(n, d, 5)
    Gkd, Gmd, gd = to_dev(Gk, ld), to_dev(Gm, ld), to_dev(g, ld)
    ctx.accumulate(Gkd, gd, 0.25)
    Gk2 = Gk.astype(np.float64) + 0.25 * g
    assert rel_err(to_host(Gkd, d), Gk2, amax(Gk, g)) < TOL_F32 and padding_ok(Gkd, d)
    Xtd, Yd = to_dev(Xt, ld, tdt), to_dev(Y, ld, tdt)
    Xd = to_dev(np.zeros((n, d)), ld, tdt) if separate_replica else Xtd
    ctx.phase_end(Xd, Xtd, Yd, Gkd, Gmd, alpha)
    Xw = Xt.astype(np.float64) - alpha * Y
    Yw = Y.astype(np.float64) + to_host(Gkd, d) - Gm
    assert rel_err(to_host(Xd, d), Xw, amax(Xt, Y)) < tol
    assert rel_err(to_host(Yd, d), Yw, amax(Y, Gk2, Gm)) < tol
    assert np.array_equal(to_host(Xtd, d), to_host(Xd, d))     # the replica is the new model
    assert np.all(to_host(Gmd, d) == 0.0)                      # cleared for the next phase
    assert all(padding_ok(t, d) for t in (Xd, Xtd, Yd, Gmd))
    with pytest.raises(D.DetagError):
        ctx.phase_end(Xd, Xtd, Yd, Gkd, Gkd, alpha)


def _lstsq_setup():
    cfg = CONFIGS[1]
    n, d, m = cfg.n, cfg.d, cfg.extra["m"]
    A, b = gen.lstsq_problem(n, m, d, seed=cfg.seed, shift=cfg.extra["offset_shift"])
    ctx, W = make_ctx("ring", n, d, d)
    return cfg, n, d, A, b, ctx, W, torch.from_numpy(A).to(DEV), torch.from_numpy(b).to(DEV)


@pytest.mark.parametrize("granularity", ["iteration", "phase"])
@pytest.mark.parametrize("overlap", [True, False])
def test_by_phase_run_matches_oracle(granularity, overlap):
    """First workload (least squares, n=8 ring), phase length 4, two gradient queries per iteration averaged
    over the phase, 6 phases and 2 iterations of an unfinished seventh."""
    cfg, n, d, A, b, ctx, W, Ad, bd = _lstsq_setup()
    R, B, T = cfg.K, 2, 6 * cfg.K + 2
    eta = ctx.spectrum()["eta"]
    scale = 1.0 / (R * B)
    # query q of iteration t: the least-squares gradient plus a known per-query offset, so that the
    # accumulation order and count are visible in the result
    off = gen.state(n, d, 9)
    offd = to_dev(off, d)

    def grad_dev(t, q, X, g):
        ctx.grad_lstsq(X, Ad, bd, g)
        ctx.accumulate(g, offd, 0.01 * ((t + 2 * q) % 5))

    grad_ref = lambda t, q, X: OO.grad_lstsq(X, A, b) + 0.01 * ((t + 2 * q) % 5) * off
    Xd = D.new_matrix(n, d, d)
    bp = ALG.run_by_phase(ctx, grad_dev, Xd, cfg.lr, T, R, eta, B=B, scale=scale, overlap=overlap,
                          granularity=granularity)
    torch.cuda.synchronize()
    Xr, _, phases = OR.by_phase(grad_ref, np.zeros((n, d)), W, cfg.lr, T, R, eta, B=B, scale=scale)
    assert bp.k == phases == 6
    assert rel_err(to_host(Xd, d), Xr, amax(Xr, b), floor=1.0) < TOL_F32          # whole run: normwise
    # ... and the finished phases are the phase-at-a-time entry point fed the averaged gradients
    Xr6, Yr6, _ = OR.by_phase(grad_ref, np.zeros((n, d)), W, cfg.lr, 6 * R, R, eta, B=B, scale=scale)
    assert np.array_equal(Xr6, Xr)


def test_two_streams_give_the_same_bits_as_one():
    cfg, n, d, A, b, ctx, W, Ad, bd = _lstsq_setup()
    out = []
    for overlap in (False, True):
        Xd = D.new_matrix(n, d, d)
        bp = ALG.run_by_phase(ctx, lambda t, q, X, g: ctx.grad_lstsq(X, Ad, bd, g), Xd, cfg.lr, 5 * cfg.K, cfg.K,
                              overlap=overlap)
        torch.cuda.synchronize()
        out.append((Xd.cpu().numpy().copy(), bp.Y.cpu().numpy().copy()))
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])


def test_dynamic_phase_length():
    """Phase length 1 with eta = 0 (DSGT) for the first 5 phases, then length 3 with Algorithm 3's eta."""
    cfg, n, d, A, b, ctx, W, Ad, bd = _lstsq_setup()
    eta = ctx.spectrum()["eta"]
    sched_R = lambda k: 1 if k < 5 else 3
    sched_eta = lambda k: 0.0 if k < 5 else eta
    T = 5 + 3 * 6
    Xd = D.new_matrix(n, d, d)
    bp = ALG.run_by_phase(ctx, lambda t, q, X, g: ctx.grad_lstsq(X, Ad, bd, g), Xd, cfg.lr, T, sched_R, sched_eta)
    torch.cuda.synchronize()
    Xr, Yr, phases = OR.by_phase(lambda t, q, X: OO.grad_lstsq(X, A, b), np.zeros((n, d)), W, cfg.lr, T, sched_R,
                                 sched_eta)
    assert bp.k == phases == 11
    S = amax(Xr, Yr, b)
    assert rel_err(to_host(Xd, d), Xr, S, floor=1.0) < TOL_F32
    assert rel_err(to_host(bp.Y, d), Yr, S, floor=1.0) < TOL_F32


@pytest.mark.parametrize("R", [3, 4])
def test_recorded_graph_of_two_phases_replays_like_eager(R):
    """A HIP graph of two phases, replayed three times with eager work and synchronisations in between, gives
    the bits of an eager run of the same eight phases (odd and even phase length: the gossip buffers swap
    roles differently)."""
    cfg, n, d, A, b, ctx, W, Ad, bd = _lstsq_setup()
    grad = lambda t, q, X, g: ctx.grad_lstsq(X, Ad, bd, g)
    Xe = D.new_matrix(n, d, d)
    be = ALG.run_by_phase(ctx, grad, Xe, cfg.lr, 8 * R, R)
    torch.cuda.synchronize()
    Xg = D.new_matrix(n, d, d)
    bg = ALG.ByPhase(ctx, Xg, cfg.lr, grad)
    bg.phase(R), bg.phase(R)                                     # eager: allocates every scratch buffer
    torch.cuda.synchronize()
    graph = bg.capture_two_phases(R)
    for rep in range(3):
        bg.replay_two_phases(graph)
        torch.cuda.synchronize()
        junk = torch.randn(1000, device=DEV).sum().item()        # unrelated eager work between replays
        assert np.isfinite(junk)
        Xchk = D.new_matrix(n, d, d)
        ALG.run_by_phase(ctx, grad, Xchk, cfg.lr, (4 + 2 * rep) * R, R)
        torch.cuda.synchronize()
        assert np.array_equal(Xg.cpu().numpy(), Xchk.cpu().numpy()), rep
    assert bg.k == be.k == 8
    assert np.array_equal(Xg.cpu().numpy(), Xe.cpu().numpy())
    assert np.array_equal(bg.Y.cpu().numpy(), be.Y.cpu().numpy())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_odd_pitch_takes_the_scalar_paths(dtype):
    """Pitch 517: no row is 16-byte (or, for bf16, 8-byte) aligned, so every streaming kernel runs its
    one-element-per-lane form: the gossip step, the accumulation, the phase end, the per-round phase (with its
    widening and narrowing copies for bf16), a consensus factor and the DeFacto update."""
    from oracle import consensus as OC
    bf = dtype == "bf16"
    tdt, tol = (torch.bfloat16, TOL_BF16) if bf else (torch.float32, TOL_F32)
    n, d, ld, eta, alpha, K = 6, 515, 517, 0.3, 0.1, 3
    ctx, W = make_ctx("ring", n, d, ld, D.DETAG_BF16 if bf else D.DETAG_F32)
    rnd = (lambda a: OO.round_bf16(a)) if bf else (lambda a: a)
    X, Y = rnd(gen.state(n, d, 1)), rnd(gen.state(n, d, 2))
    Gk, Gm = gen.state(n, d, 3), gen.state(n, d, 4)
    # one gossip step
    Xd, Yd, Od = to_dev(X, ld, tdt), to_dev(Y, ld, tdt), to_dev(np.zeros((n, d)), ld, tdt)
    ctx.gossip_round(Xd, Yd, Od, eta)
    want = (1 + eta) * (W.T @ X.astype(np.float64)) - eta * Y.astype(np.float64)
    assert rel_err(to_host(Od, d), want, amax(X, Y)) < tol and padding_ok(Od, d)
    # accumulation and phase end
    Gkd, Gmd = to_dev(Gk, ld), to_dev(Gm, ld)
    ctx.accumulate(Gkd, Gmd, 0.5)
    Gk2 = Gk.astype(np.float64) + 0.5 * Gm
    assert rel_err(to_host(Gkd, d), Gk2, amax(Gk, Gm)) < TOL_F32 and padding_ok(Gkd, d)
    ctx.phase_end(Od, Xd, Yd, Gkd, Gmd, alpha)
    assert rel_err(to_host(Od, d), X.astype(np.float64) - alpha * Y, amax(X, Y)) < tol
    assert rel_err(to_host(Yd, d), Y.astype(np.float64) + to_host(Gkd, d) - Gm, amax(Y, Gk2, Gm)) < tol
    assert all(padding_ok(t, d) for t in (Od, Xd, Yd, Gmd))
    # the per-round phase
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    Xd, Yd = to_dev(X, ld, tdt), to_dev(Y, ld, tdt)
    ctx.step(Xd, Yd, to_dev(Gk, ld), to_dev(Gm, ld), alpha, K, eta)
    Xr, Yr = OG.detag_step(X, Y, Gk, Gm, W, alpha, K, eta)
    S = amax(X, Y, Gk, Gm)
    assert rel_err(to_host(Xd, d), Xr, S) < tol and rel_err(to_host(Yd, d), Yr, S) < tol
    assert padding_ok(Xd, d) and padding_ok(Yd, d)
    # a consensus factor and the DeFacto update
    f = D.Factors(ctx, 2)
    ref = OC.gather_propagate_factors(n, gen.edges_ring(n), 2)
    Zd, Od = to_dev(X, ld, tdt), to_dev(np.zeros((n, d)), ld, tdt)
    f.apply(0, Zd, Od)
    assert rel_err(to_host(Od, d), ref[0] @ X.astype(np.float64), 2 * amax(X)) < tol and padding_ok(Od, d)
    Gd = to_dev(Gk, ld)
    held = to_host(Od, d)
    ctx.defacto_update(Zd, Od, Gd, 0.25)
    assert rel_err(to_host(Zd, d), held - 0.25 * Gk, amax(held, Gk)) < tol
    assert np.array_equal(to_host(Od, d), to_host(Zd, d)) and np.all(to_host(Gd, d) == 0.0)
    assert padding_ok(Zd, d) and padding_ok(Gd, d)


def test_capture_refuses_to_allocate_and_works_after_reserve():
    """Under HIP graph capture an entry point that would have to allocate its scratch returns a status and
    enqueues nothing; after detag_reserve_* the same calls record, and the replayed graph (three times, with
    eager work in between) gives the bits of the eager calls."""
    n, d, ld, K = 8, 700, 704, 3
    ctx, W = make_ctx("ring", n, d, ld)
    ctx.set_path(D.DETAG_PATH_PER_ROUND)
    Z = gen.state(n, d, seed=5)
    m = 16
    A = torch.from_numpy(gen.lstsq_problem(n, m, d, seed=1, shift=0.0)[0]).to(DEV)
    bb = torch.from_numpy(gen.lstsq_problem(n, m, d, seed=1, shift=0.0)[1]).to(DEV)
    Zd, Gd = to_dev(Z, ld), D.new_matrix(n, d, ld)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            with pytest.raises(D.DetagError) as e1:
                ctx.gossip_accel(Zd, K)                          # per-round scratch does not exist yet
            with pytest.raises(D.DetagError) as e2:
                ctx.grad_lstsq(Zd, A, bb, Gd)                    # nor the residual scratch
            Gd.zero_()                                           # so that the recording holds some node
    assert e1.value.status == D.DETAG_EINVAL and "detag_reserve_gossip" in e1.value.message
    assert e2.value.status == D.DETAG_EINVAL and "detag_reserve_gradient" in e2.value.message
    torch.cuda.synchronize()
    assert np.array_equal(to_host(Zd, d), Z.astype(np.float64))  # nothing ran
    ctx.reserve_gossip(D.DETAG_PATH_PER_ROUND)
    ctx.reserve_gradient(m=m)
    with pytest.raises(D.DetagError):
        ctx.reserve_gossip(D.DETAG_PATH_FUSED)                   # owns nothing to reserve
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph2, stream=side):
            ctx.gossip_accel(Zd, K)
            ctx.grad_lstsq(Zd, A, bb, Gd)
    Ze, Ge = to_dev(Z, ld), D.new_matrix(n, d, ld)
    for rep in range(3):
        graph2.replay()
        ctx.gossip_accel(Ze, K)
        ctx.grad_lstsq(Ze, A, bb, Ge)
        torch.cuda.synchronize()
        assert np.isfinite(torch.randn(100, device=DEV).sum().item())
        assert torch.equal(Zd, Ze) and torch.equal(Gd, Ge), rep
    eta = OT.eta_from_lambda(OT.spectrum(W)[2])
    ref = Z
    for _ in range(3):
        ref = OG.accelerated_gossip(ref, W, K, eta)
    assert rel_err(to_host(Zd, d), ref, amax(Z), floor=1.0) < TOL_F32
    # the dense path: the polynomial of an unseen (K, eta) is refused under capture, accepted once reserved
    ctx.set_path(D.DETAG_PATH_DENSE)
    graph3 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph3, stream=side):
            with pytest.raises(D.DetagError) as e3:
                ctx.gossip_accel(Zd, 5)
            Gd.zero_()
    assert "detag_reserve_gossip" in e3.value.message
    ctx.reserve_gossip(D.DETAG_PATH_DENSE, 5)
    Z1, Z2 = to_dev(Z, ld), to_dev(Z, ld)
    graph4 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph4, stream=side):
            ctx.gossip_accel(Z1, 5)
    graph4.replay()
    ctx.gossip_accel(Z2, 5)
    torch.cuda.synchronize()
    assert torch.equal(Z1, Z2)
