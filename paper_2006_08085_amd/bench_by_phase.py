"""Time per phase of Algorithm 2 run iteration by iteration, on the two small
workloads whose step is bound by launches rather than by HBM:

    python -m paper_2006_08085_amd.bench_by_phase [--phases 200]

Compared: the phase-at-a-time entry point (gradient, then detag_step), the
iteration-by-iteration form on one stream, on two streams (gossip beside the
gradient queries), with the phase's gossip as one on-chip call, and as a
recorded HIP graph of two phases.  Prints one JSON line per workload.
"""
from __future__ import annotations

import argparse
import json
import time

import torch

import paper_2006_08085_amd as D
from paper_2006_08085_amd import algorithms as ALG
from workloads import CONFIGS, generate as gen


def _time_phases(run_phase, phases, per_call=1):
    for _ in range(4):
        run_phase()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(phases // per_call):
        run_phase()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (phases // per_call * per_call) * 1e6


def _workload(cfg_id, dev):
    cfg = CONFIGS[cfg_id]
    n, d = cfg.n, cfg.d
    ld = D.padded_ld(d)
    ctx = D.detag_create(D.Topology.ring(), n, d, ld)
    if cfg.objective == "lstsq":
        A, b = gen.lstsq_problem(n, cfg.extra["m"], d, seed=cfg.seed, shift=cfg.extra["offset_shift"])
        Ad, bd = torch.from_numpy(A).to(dev), torch.from_numpy(b).to(dev)
        if ld != d:
            Ap = torch.zeros(n, A.shape[1], ld, device=dev); Ap[:, :, :d] = Ad; Ad = Ap
        grad = lambda t, q, X, g: ctx.grad_lstsq(X, Ad, bd, g)
    else:
        F, C, S, B = (cfg.extra[k] for k in ("F", "C", "S", "B"))
        feats, labels = gen.softmax_problem(n, S, F, C, cfg.seed)
        fd = torch.from_numpy(feats).to(torch.bfloat16).to(dev)
        lab = torch.from_numpy(labels).to(dev)
        idx = torch.from_numpy(gen.batch_indices(n, S, B, seed=cfg.seed, step=0)).to(dev)   # refreshed by the caller in real use
        grad = lambda t, q, X, g: ctx.grad_softmax_bf16(X, fd, lab, idx, C, g)
    return cfg, ctx, grad


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--phases", type=int, default=200)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    for cfg_id in (1, 3):
        cfg, ctx, grad = _workload(cfg_id, dev)
        n, d, ld, R, alpha = cfg.n, cfg.d, ctx.ld, cfg.K, cfg.lr
        out = {"workload": f"config {cfg_id}: n={n} ring, d={d}, {cfg.objective}, phase length R={R}, one gradient "
                           f"query per iteration (R per phase) unless the name says otherwise",
               "unit": "us per phase", "phases": args.phases}
        # phase at a time: one gradient query, then the fused phase (printed order of Algorithm 2)
        X, Y = D.new_matrix(n, d, ld, device=dev), D.new_matrix(n, d, ld, device=dev)
        Ga, Gb = D.new_matrix(n, d, ld, device=dev), D.new_matrix(n, d, ld, device=dev)

        def phase_call():
            grad(0, 0, X, Ga)
            ctx.step(X, Y, Ga, Gb, alpha, R, -1.0, D.DETAG_VARIANT_ALG2)
        out["phase_at_a_time_1_query"] = _time_phases(phase_call, args.phases)
        g = D.new_matrix(n, d, ld, device=dev)

        def phase_call_R():               # the same R gradient queries as the iteration-by-iteration runs below
            Ga.zero_()
            for r in range(R):
                grad(r, 0, X, g)
                ctx.accumulate(Ga, g, 1.0 / R)
            ctx.step(X, Y, Ga, Gb, alpha, R, -1.0, D.DETAG_VARIANT_ALG2)
        out["phase_at_a_time_R_queries"] = _time_phases(phase_call_R, args.phases)
        for name, kw in (("iterations_one_stream", dict(overlap=False)), ("iterations_two_streams", dict(overlap=True)),
                         ("phase_gossip_two_streams", dict(overlap=True, granularity="phase"))):
            bp = ALG.ByPhase(ctx, D.new_matrix(n, d, ld, device=dev), alpha, grad, scale=1.0 / R, **kw)
            out[name] = _time_phases(lambda: bp.phase(R), args.phases)
        bp = ALG.ByPhase(ctx, D.new_matrix(n, d, ld, device=dev), alpha, grad, scale=1.0 / R, overlap=True)
        bp.phase(R), bp.phase(R)
        torch.cuda.synchronize()
        graph = bp.capture_two_phases(R)
        out["iterations_two_streams_graph"] = _time_phases(lambda: bp.replay_two_phases(graph), args.phases, per_call=2)
        print(json.dumps(out), flush=True)
        ctx.close()


if __name__ == "__main__":
    main()
