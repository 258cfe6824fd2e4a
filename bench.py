#!/usr/bin/env python3
"""Benchmark of the DeTAG hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4]

One step = one pass of the whole hot path over all n workers: the local
stochastic gradient (diagonal quadratic + in-kernel Gaussian noise), then one
DeTAG phase (tracking update, model update and K rounds of accelerated gossip
of X and Y).  The workload is the n=64, 8x8-torus, d=11,173,962 fp32
configuration; inputs are synthetic, seeded, and resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
PHASE_BYTES_PER_ELEMENT = 24   # detag_step, fp32: read X, Y, G_new, G_old; write X, Y (independent of K)
FUSED_BYTES_PER_ELEMENT = 28   # detag_step_quadratic, fp32: read X, Y, G, b; write X, Y, G
DPSGD_BYTES_PER_ELEMENT = 12   # detag_dpsgd_step, fp32: read X, G; write X


def measured_traffic(fused: bool):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3
    counter summary (profiles/*_traffic.json), or None if the kernel sources have
    changed since those counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "fused_quadratic_traffic.json" if fused else "fused_step_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    csrc = os.path.join(ROOT, "paper_2006_08085_amd", "csrc")
    src = b"".join(open(os.path.join(csrc, f), "rb").read() for f in rec["sources"])
    if hashlib.sha256(src).hexdigest() != rec.get("source_sha256"):
        return None
    return rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]


def cpu_baseline(cfg, sample_cols: int, W):
    """The fp64 oracle, as it stands, on the first `sample_cols` columns of the
    same workload (columns are independent for this objective), one step."""
    import numpy as np
    from oracle import gossip as OG, noise as ON, objectives as OO, topology as OT
    from workloads import generate as gen
    n, K = cfg.n, cfg.K
    OT.check_gossip_matrix(W)                 # W is data for the oracle (rebuilt from the library's CSR): re-validated
    eta = OT.eta_from_lambda(OT.spectrum(W)[2])
    h, b = gen.quadratic_problem(n, sample_cols, seed=cfg.seed, b_mean=cfg.extra["b_mean"], b_std=cfg.extra["b_std"])
    X, Y, Gold = gen.state(n, sample_cols, 11), gen.state(n, sample_cols, 12), gen.state(n, sample_cols, 13)
    t0 = time.perf_counter()
    z = ON.normal_noise(cfg.seed, 0, n, np.arange(sample_cols))
    Gnew = OO.grad_quadratic_diag(X, h, b, z, cfg.sigma)
    OG.detag_step(X, Y, Gnew, Gold, W, cfg.lr, K, eta)
    dt = time.perf_counter() - t0
    return {"value": n * sample_cols * K / dt, "unit": "worker-param-gossip-rounds/s", "cores": 1,
            "kind": "oracle",
            "sample": f"1 step on the first {sample_cols} of {cfg.d} columns, all {n} workers, numpy fp64, "
                      f"{dt:.1f} s; host has {os.cpu_count()} cpus"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, choices=[2, 4, 5],
                    help="4 (default) is the headline workload; 2 and 5 are the other quadratic workloads "
                         "(5: n=256 random 4-regular graph, bf16 state, K=16, runs as gradient kernel + phase kernel)")
    ap.add_argument("--cpu-sample-cols", type=int, default=2_097_152)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unfused", action="store_true",
                    help="run the step as two kernels (detag_grad_quadratic_diag, then detag_step) instead of "
                         "the single detag_step_quadratic kernel")
    ap.add_argument("--algorithm", default="detag", choices=["detag", "dsgt", "dpsgd"],
                    help="detag (default, the headline line); dsgt = the same kernels with K=1, eta=0; dpsgd = "
                         "detag_grad_quadratic_diag + detag_dpsgd_step.  The two baselines of the paper's "
                         "Experiments section, timed on the same workload")
    ap.add_argument("--dense", action="store_true",
                    help="run detag_step on DETAG_PATH_DENSE (the K rounds as one matrix-core product with the "
                         "polynomial p_K(W^T)); for the unfused step only, i.e. --config 5 or --unfused")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain device copies of one n x ld fp32 matrix (a kernel of known "
                         "traffic, for scaling profiler byte counters); untimed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (it has no cross-GPU code); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2006_08085_amd as D
    from workloads import CONFIGS, generate as gen

    if not os.path.exists(D.LIB_PATH):
        from paper_2006_08085_amd.build import build
        build(verbose=False)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = CONFIGS[args.config]
    n, d, K, alpha, sigma = cfg.n, cfg.d, cfg.K, cfg.lr, cfg.sigma
    alg = args.algorithm
    eta = -1.0                      # Algorithm 3's formula from the context's lambda
    if alg != "detag":
        K, eta = 1, 0.0             # one plain gossip round per step
    ld = D.padded_ld(d)
    bf16 = cfg.state_dtype == "bf16"
    sdt = torch.bfloat16 if bf16 else torch.float32
    if cfg.topology == "torus":
        topo, tname = D.Topology.torus(*cfg.torus_shape), "8x8 torus"
    elif cfg.topology == "random_regular":
        topo, tname = D.Topology.random_regular(cfg.degree, cfg.seed), f"random {cfg.degree}-regular graph, Metropolis weights"
    else:
        topo, tname = D.Topology.ring(), "ring"
    ctx = D.detag_create(topo, n, d, ld, D.DETAG_BF16 if bf16 else D.DETAG_F32)
    assert ctx.has_fused()
    structured = cfg.topology != "random_regular"     # the register-resident kernels cover ring and torus
    sb = 2 if bf16 else 4                             # bytes per state element

    # inputs, generated on the device and resident before anything is timed
    b = gen.device_normal(n, d, ld, cfg.seed, 1, dev, std=cfg.extra["b_std"])
    h = gen.device_log_uniform(d, ld, cfg.seed, 2, dev, cfg.extra["h_lo"], cfg.extra["h_hi"])
    X, Y = D.new_matrix(n, d, ld, dtype=sdt, device=dev), D.new_matrix(n, d, ld, dtype=sdt, device=dev)
    Ga, Gb = D.new_matrix(n, d, ld, device=dev), D.new_matrix(n, d, ld, device=dev)

    state = {"t": 0, "Ga": Ga, "Gb": Gb}
    fused = not args.unfused and alg != "dpsgd" and structured
    if args.dense:
        if fused or alg == "dpsgd":
            print("bench.py: --dense applies to the two-kernel step (--config 5, or --unfused)", file=sys.stderr)
            sys.exit(2)
        ctx.set_path(D.DETAG_PATH_DENSE)

    def one_step(ev=None):
        if alg == "dpsgd":
            ctx.grad_quadratic_diag(X, h, b, state["Ga"], sigma=sigma, seed=cfg.seed, step=state["t"])
            if ev is not None:
                ev[0].record()
            ctx.dpsgd_step(X, state["Ga"], alpha)
            if ev is not None:
                ev[1].record()
        elif fused:   # gradient query + phase in one kernel; Ga is the single gradient matrix, updated in place
            if ev is not None:
                ev[0].record()
            ctx.step_quadratic(X, Y, state["Ga"], h, b, alpha, K, sigma=sigma, seed=cfg.seed, step=state["t"],
                               eta=eta)
            if ev is not None:
                ev[1].record()
        else:
            ctx.grad_quadratic_diag(X, h, b, state["Ga"], sigma=sigma, seed=cfg.seed, step=state["t"])
            if ev is not None:
                ev[0].record()
            ctx.step(X, Y, state["Ga"], state["Gb"], alpha, K, eta)
            if ev is not None:
                ev[1].record()
            state["Ga"], state["Gb"] = state["Gb"], state["Ga"]
        state["t"] += 1

    for _ in range(args.warmup):
        one_step()
    if args.calibrate_copy:
        scratch = torch.empty_like(Ga)
        for _ in range(3):
            scratch.copy_(b)          # reads n*ld*4 bytes, writes n*ld*4 bytes
        del scratch
    torch.cuda.synchronize()

    # kernels are launched on torch's current stream, so torch events bracket them
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(evs[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    phase_ms = sum(a.elapsed_time(b_) for a, b_ in evs) / args.steps
    # algorithmic bytes per element: state read and written once each, gradient-side arrays fp32
    bpe = (2 * sb + 4) if alg == "dpsgd" else (4 * sb + 12) if fused else (4 * sb + 8)
    assert bf16 or bpe == (DPSGD_BYTES_PER_ELEMENT if alg == "dpsgd" else FUSED_BYTES_PER_ELEMENT if fused
                           else PHASE_BYTES_PER_ELEMENT)
    achieved = bpe * n * d / (phase_ms * 1e-3) / 1e9
    xbar = ctx.mean(X)
    finite = bool(torch.isfinite(xbar[:d]).all().item())

    out = {
        "metric": "worker-param-gossip-rounds/s (n*d*K/s)",
        "value": n * d * K / (dt / args.steps),
        "unit": "worker-param-gossip-rounds/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",      # arithmetic is fp32 on chip whatever the storage of X and Y
        "config": {"workload": f"config {args.config}: n={n} workers, "
                               f"{tname}, d={d} {'bf16 X and Y, fp32 gradients' if bf16 else 'fp32'} (ld={ld}), "
                               f"K={K} accelerated-gossip rounds of X and Y per step, diagonal quadratic + "
                               f"N(0,{sigma}^2) counter-based noise, lr={alpha}",
                   "algorithm": alg,
                   "step": "detag_grad_quadratic_diag + detag_dpsgd_step" if alg == "dpsgd"
                           else "detag_step_quadratic (gradient query + ATC phase, one kernel)" if fused
                           else "detag_grad_quadratic_diag + detag_step (ATC, one product with p_K(W^T))" if args.dense
                           else "detag_grad_quadratic_diag + detag_step (ATC, fused K rounds)",
                   "matrix_rounds_per_s": 2 * n * d * K / (dt / args.steps),   # X and Y counted separately
                   "finite": finite},
        "roofline": {"bound": "hbm",
                     "kernel": ("fused_structured_kernel, D-PSGD mode" if structured else "gossip_round_kernel")
                               + " (detag_dpsgd_step)" if alg == "dpsgd"
                               else "fused_quadratic_kernel (detag_step_quadratic)" if fused
                               else "dense_phase_kernel (detag_step)" if args.dense
                               else ("fused_structured_kernel" if structured else "fused_generic_kernel") + " (detag_step)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(fused) if args.config == 4 and alg == "detag" else None, "kernel_ms": phase_ms,
                     "algorithmic_bytes_per_launch": bpe * n * d,
                     **({"note": "bound by the latency of its staging loads and by instruction issue, not yet by HBM "
                                 "or the matrix cores"} if args.dense else {} if structured
                        else {"note": "this kernel keeps all rows of a tile in LDS and is bound by "
                                      "LDS bandwidth and VALU issue, not by HBM"})},
    }
    if not args.no_cpu_baseline and alg == "detag":
        out["cpu_baseline"] = cpu_baseline(cfg, min(args.cpu_sample_cols, d), ctx.dense_W())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
