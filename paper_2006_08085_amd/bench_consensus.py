"""Time of the exact average consensus (Lemma 1; spanning-tree gather and
propagate factors) on the benchmark's state matrix, beside K rounds of
accelerated gossip on the same matrix:

    python -m paper_2006_08085_amd.bench_consensus [--reps 10]

Compared: the factor sequence applied one factor per launch
(detag_factor_apply, R launches), the whole sequence in one launch
(detag_average_consensus), and detag_gossip_accel with K = 8 and K = 16.
Prints one JSON line; GB/s counts 8 B per element (the state read and written
once) per factor for the first form and per call for the others.
"""
from __future__ import annotations

import argparse
import json

import torch

import paper_2006_08085_amd as D
from workloads import CONFIGS


def _ms(fn, reps, stream):
    for _ in range(3):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = CONFIGS[4]
    n, d = cfg.n, cfg.d
    ld = D.padded_ld(d)
    rows, cols = cfg.torus_shape
    ctx = D.detag_create(D.Topology.torus(rows, cols), n, d, ld)
    f = D.Factors(ctx, 0)
    stream = torch.cuda.current_stream()
    Z = torch.randn(n, ld, device=dev)
    Z[:, d:] = 0
    mean = Z[:, :d].double().mean(0)
    T = torch.empty_like(Z)
    state = [Z, T]

    def factor_by_factor():
        for r in range(f.R):
            f.apply(r, state[0], state[1])
            state.reverse()

    t_steps = _ms(factor_by_factor, args.reps, stream)
    err_steps = float((state[0][:, :d].double() - mean).abs().max())
    Z2 = torch.randn(n, ld, device=dev)
    Z2[:, d:] = 0
    mean2 = Z2[:, :d].double().mean(0)
    t_one = _ms(lambda: f.average(Z2), args.reps, stream)
    err_one = float((Z2[:, :d].double() - mean2).abs().max())
    t_k8 = _ms(lambda: ctx.gossip_accel(Z2, 8), args.reps, stream)
    t_k16 = _ms(lambda: ctx.gossip_accel(Z2, 16), args.reps, stream)
    gbs = lambda ms, passes=1: 8.0 * n * d * passes / ms / 1e6
    print(json.dumps({
        "workload": f"config 4: n={n}, {rows}x{cols} torus, d={d} fp32; R={f.R} factors",
        "reps": args.reps,
        "factor_by_factor_ms": t_steps, "factor_by_factor_GBps": gbs(t_steps, f.R),
        "one_launch_ms": t_one, "one_launch_GBps": gbs(t_one),
        "gossip_accel_K8_ms": t_k8, "gossip_accel_K16_ms": t_k16,
        "max_abs_distance_from_mean": {"factor_by_factor": err_steps, "one_launch": err_one},
    }))


if __name__ == "__main__":
    main()
