#!/usr/bin/env python3
"""Benchmark of the DeTAG hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4]
                    [--what step|gossip|stream|diag] [--path auto|per_round] [--unfused] [--dense]

One step = one pass of the whole hot path over all n workers: the local
stochastic gradient (diagonal quadratic + in-kernel Gaussian noise), then one
DeTAG phase (tracking update, model update and K rounds of accelerated gossip
of X and Y).  The workload is the n=64, 8x8-torus, d=11,173,962 fp32
configuration; inputs are synthetic, seeded, and resident in HBM before the
timed region.  Prints ONE JSON line.

--what selects what one timed "step" is (default: the whole hot path, above):
  gossip  one detag_gossip_accel call on X (K rounds of Algorithm 3 alone)
  stream  the tracking and model update without gossip (detag_step with K = 0): a plain elementwise pass over
          the same six streams, the streaming reference for the phase kernel's 24 bytes per element
  diag    the two diagnostics, detag_mean and detag_consensus_error
--path per_round runs the gossip with one launch per round (the CSR kernel) instead of the K-round kernels.
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
LDS_PEAK_GBS = 256 * 128 * 2.4  # 256 compute units x 128 B per clock x 2.4 GHz = 78,643 GB/s
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


def _oracle_step(cfg, W, eta, cols_lo: int, cols_hi: int, seed_shift: int):
    """One oracle step (noise, gradient, phase) on columns [cols_lo, cols_hi) of the workload."""
    import numpy as np
    from oracle import gossip as OG, noise as ON, objectives as OO
    from workloads import generate as gen
    n, m = cfg.n, cols_hi - cols_lo
    h, b = gen.quadratic_problem(n, m, seed=cfg.seed + seed_shift, b_mean=cfg.extra["b_mean"], b_std=cfg.extra["b_std"])
    X, Y, Gold = (gen.state(n, m, 11 + k + 3 * seed_shift) for k in range(3))
    t0 = time.perf_counter()
    z = ON.normal_noise(cfg.seed, 0, n, np.arange(cols_lo, cols_hi))
    Gnew = OO.grad_quadratic_diag(X, h, b, z, cfg.sigma)
    OG.detag_step(X, Y, Gnew, Gold, W, cfg.lr, cfg.K, eta)
    return time.perf_counter() - t0


def cpu_baseline(cfg, sample_cols: int, W):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload, one step.  Columns are independent
    for this objective, so the oracle's work is exactly linear in the number of columns: the rate measured on the
    sample is the rate of the full width (stated as extrapolated in the line).  Two legs: one thread, and one
    thread per host core over disjoint column ranges (numpy releases the interpreter lock inside its loops)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import topology as OT
    n, K = cfg.n, cfg.K
    OT.check_gossip_matrix(W)                 # W is data for the oracle (rebuilt from the library's CSR): re-validated
    eta = OT.eta_from_lambda(OT.spectrum(W)[2])
    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)))
    single_cols = max(1, sample_cols // 2)
    dt1 = _oracle_step(cfg, W, eta, 0, single_cols, 0)
    per = max(1, sample_cols // 8)            # columns per thread
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(lambda k: _oracle_step(cfg, W, eta, k * per, (k + 1) * per, k + 1), range(cores)))
    dtp = time.perf_counter() - t0
    return {"value": n * per * cores * K / dtp, "unit": "worker-param-gossip-rounds/s", "cores": cores,
            "kind": "oracle",
            "single_core_value": n * single_cols * K / dt1,
            "sample": f"numpy fp64 oracle, 1 step, all {n} workers; rate extrapolated from a column sample "
                      f"(work is linear in columns): {cores} threads x {per} columns in {dtp:.1f} s "
                      f"(value), 1 thread x {single_cols} columns in {dt1:.1f} s (single_core_value); "
                      f"full width is {cfg.d} columns; host has {os.cpu_count()} cpus"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, choices=[2, 4, 5],
                    help="4 (default) is the headline workload; 2 and 5 are the other quadratic workloads "
                         "(5: n=256 random 4-regular graph, bf16 state, K=16, on the LDS-resident kernels)")
    ap.add_argument("--what", default="step", choices=["step", "gossip", "stream", "diag"],
                    help="what one timed step is: the whole hot path (default), detag_gossip_accel alone, the "
                         "elementwise update without gossip (K = 0), or the two diagnostics")
    ap.add_argument("--path", default="auto", choices=["auto", "per_round"],
                    help="per_round: one launch per gossip round (the CSR kernel) instead of the K-round kernels; "
                         "implies --unfused for --what step")
    ap.add_argument("--cpu-sample-cols", type=int, default=2_097_152)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unfused", action="store_true",
                    help="run the step as two kernels (detag_grad_quadratic_diag, then detag_step) instead of "
                         "the single detag_step_quadratic kernel")
    ap.add_argument("--algorithm", default="detag", choices=["detag", "dsgt", "dpsgd"],
                    help="detag (default, the headline line); dsgt = the same kernels with K=1, eta=0; dpsgd = "
                         "detag_grad_quadratic_diag + detag_dpsgd_step.  The two baselines of the paper's "
                         "Experiments section, timed on the same workload")
    ap.add_argument("--variant", default="atc", choices=["atc", "alg2"],
                    help="phase update: atc (default; gradients enter before the gossip, the form the proof of "
                         "Theorem 3 analyses) or alg2 (Algorithm 2 as printed: gossip first)")
    ap.add_argument("--dense", action="store_true",
                    help="run detag_step on DETAG_PATH_DENSE (the K rounds as one matrix-core product with the "
                         "polynomial p_K(W^T)); implies --unfused")
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
    alg, what = args.algorithm, args.what
    per_round = args.path == "per_round"
    variant = D.DETAG_VARIANT_ALG2 if args.variant == "alg2" else D.DETAG_VARIANT_ATC
    VN = "ALG2" if args.variant == "alg2" else "ATC"
    if args.variant != "atc" and (what != "step" or alg == "dpsgd"):
        print("bench.py: --variant applies to --what step of detag and dsgt", file=sys.stderr)
        sys.exit(2)
    if what != "step" and (alg != "detag" or args.dense or args.unfused):
        print("bench.py: --algorithm, --dense and --unfused apply to --what step", file=sys.stderr)
        sys.exit(2)
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
    if per_round:
        ctx.set_path(D.DETAG_PATH_PER_ROUND)

    # inputs, generated on the device and resident before anything is timed
    b = gen.device_normal(n, d, ld, cfg.seed, 1, dev, std=cfg.extra["b_std"])
    h = gen.device_log_uniform(d, ld, cfg.seed, 2, dev, cfg.extra["h_lo"], cfg.extra["h_hi"])
    X, Y = D.new_matrix(n, d, ld, dtype=sdt, device=dev), D.new_matrix(n, d, ld, dtype=sdt, device=dev)
    Ga, Gb = D.new_matrix(n, d, ld, device=dev), D.new_matrix(n, d, ld, device=dev)
    xbar_out = torch.empty(ld, dtype=torch.float32, device=dev)
    ce_out = torch.zeros(1, dtype=torch.float64, device=dev)

    state = {"t": 0, "Ga": Ga, "Gb": Gb}
    # one kernel for gradient query + phase: both variants on ring and torus, ATC for any other on-chip context
    fused = what == "step" and not args.unfused and not per_round and alg != "dpsgd" and not args.dense and \
        (structured or args.variant == "atc")
    if args.dense:
        if fused or alg == "dpsgd" or per_round:
            print("bench.py: --dense applies to the two-kernel step of detag and dsgt, timed as launches", file=sys.stderr)
            sys.exit(2)
        ctx.set_path(D.DETAG_PATH_DENSE)
    if what != "step":                                # a non-trivial state for the partial paths
        X.copy_(gen.device_normal(n, d, ld, cfg.seed, 3, dev).to(sdt))
        Y.copy_(gen.device_normal(n, d, ld, cfg.seed, 4, dev).to(sdt))

    # one_step records ev[0] / ev[1] around the launches the roofline figure is about
    def one_step(ev=None):
        rec = (lambda k: ev[k].record()) if ev is not None else (lambda k: None)
        if what == "gossip":
            rec(0)
            ctx.gossip_accel(X, K, eta)
            rec(1)
        elif what == "stream":
            rec(0)
            ctx.step(X, Y, state["Ga"], state["Gb"], alpha, 0, eta)
            rec(1)
        elif what == "diag":
            rec(0)
            ctx.mean(X, xbar_out)
            rec(1)
            ctx.consensus_error(X, ce_out)
            rec(2)
        elif alg == "dpsgd":
            ctx.grad_quadratic_diag(X, h, b, state["Ga"], sigma=sigma, seed=cfg.seed, step=state["t"])
            rec(0)
            ctx.dpsgd_step(X, state["Ga"], alpha)
            rec(1)
        elif fused:   # gradient query + phase in one kernel; Ga is the single gradient matrix, updated in place
            rec(0)
            ctx.step_quadratic(X, Y, state["Ga"], h, b, alpha, K, sigma=sigma, seed=cfg.seed, step=state["t"],
                               eta=eta, variant=variant)
            rec(1)
        else:
            ctx.grad_quadratic_diag(X, h, b, state["Ga"], sigma=sigma, seed=cfg.seed, step=state["t"])
            rec(0)
            ctx.step(X, Y, state["Ga"], state["Gb"], alpha, K, eta, variant)
            rec(1)
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
    nev = 3 if what == "diag" else 2
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(evs[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    phase_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    E = n * d
    rounds_bytes = 4 * (3 * K - 1)      # per matrix, one launch per round: first round reads 1 and writes 1, the rest read 2, write 1
    note = None
    # the launcher's rule for one round per launch: the fp32 working matrix decides (bf16 state is widened first)
    big = n <= 256 and n * ld * 4 >= (128 << 20)
    round_kernel = "structured_round_kernel" if structured else "gossip_round_tile_kernel" if big \
        else "gossip_round_kernel"
    # algorithmic bytes per element of what the two events bracket: state read and written once each by the
    # K-round kernels; one launch per round moves every round through HBM (fp32 scratch whatever the state type)
    if what == "gossip":
        bpe = rounds_bytes if per_round else 2 * sb
        kernel = ("%s x%d" % (round_kernel, K)) if per_round else \
            ("fused_structured_kernel, gossip mode" if structured else "fused_generic_kernel, gossip mode")
        kernel += " (detag_gossip_accel)"
    elif what == "stream":
        bpe = 4 * sb + 8
        kernel = "elementwise_kernel (detag_step, K = 0)"
    elif what == "diag":
        bpe = sb
        kernel = "mean_kernel (detag_mean)"
    elif alg == "dpsgd":
        bpe = 2 * sb + 4
        staged = n <= 256 and n * ld * sb >= (128 << 20)      # the launcher's rule for the LDS-staged round kernel
        kernel = (("fused_structured_kernel, D-PSGD mode" if structured and not per_round else
                   "gossip_round_tile_kernel, in place" if staged else "copy + gossip_round_kernel")
                  + " (detag_dpsgd_step)")
    elif fused:
        bpe = 4 * sb + 12
        kernel = ("fused_generic_quadratic_kernel" if not structured else "fused_quadratic_alg2_kernel"
                  if args.variant == "alg2" else "fused_quadratic_kernel") + " (detag_step_quadratic)"
        if not structured:
            note = "this kernel keeps all rows of a tile in LDS and is bound by LDS bandwidth and VALU issue, not by HBM"
    elif per_round:
        bpe = 24 + 2 * rounds_bytes
        kernel = "elementwise_kernel + %s x%d (detag_step, one launch per round)" % (
            round_kernel, 2 * K)
        note = "sum over the launches of one detag_step call; every round crosses HBM"
    else:
        bpe = 4 * sb + 8
        kernel = ("dense_phase_kernel" if args.dense else "fused_structured_kernel" if structured
                  else "fused_generic_kernel") + " (detag_step)"
        if args.dense:
            note = "bound by the latency of its staging loads and by instruction issue, not yet by HBM or the matrix cores"
        elif not structured:
            note = "this kernel keeps all rows of a tile in LDS and is bound by LDS bandwidth and VALU issue, not by HBM"
    if not bf16 and what == "step" and not per_round:
        assert bpe == (DPSGD_BYTES_PER_ELEMENT if alg == "dpsgd" else FUSED_BYTES_PER_ELEMENT if fused
                       else PHASE_BYTES_PER_ELEMENT)
    achieved = bpe * E / (phase_ms * 1e-3) / 1e9
    xbar = ctx.mean(X)
    finite = bool(torch.isfinite(xbar[:d]).all().item())

    step_name = {"gossip": "detag_gossip_accel on X", "stream": "detag_step with K = 0 (tracking and model update only)",
                 "diag": "detag_mean + detag_consensus_error"}.get(what) or (
        "detag_grad_quadratic_diag + detag_dpsgd_step" if alg == "dpsgd"
        else "detag_step_quadratic (gradient query + %s phase, one kernel)" % VN if fused
        else "detag_grad_quadratic_diag + detag_step (%s, one product with p_K(W^T))" % VN if args.dense
        else "detag_grad_quadratic_diag + detag_step (%s, one launch per gossip round)" % VN if per_round
        else "detag_grad_quadratic_diag + detag_step (%s, fused K rounds)" % VN)
    if what in ("step", "gossip"):
        metric, unit, value = "worker-param-gossip-rounds/s (n*d*K/s)", "worker-param-gossip-rounds/s", E * K / (dt / args.steps)
    else:
        metric, unit, value = "state elements per second (n*d/s)", "elements/s", E / (dt / args.steps)
    traffic, traffic_source = None, None
    if args.config == 4 and alg == "detag" and what == "step" and not per_round and not args.dense \
            and args.variant == "atc":
        traffic = measured_traffic(fused)
        traffic_source = ("stored: profiles/%s (rocprofv3 FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size), "
                          "valid while the kernel sources hash to the recorded value"
                          % ("fused_quadratic_traffic.json" if fused else "fused_step_traffic.json")) if traffic else None
    out = {
        "metric": metric, "value": value, "unit": unit,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",      # arithmetic is fp32 on chip whatever the storage of X and Y
        "config": {"workload": f"config {args.config}: n={n} workers, "
                               f"{tname}, d={d} {'bf16 X and Y, fp32 gradients' if bf16 else 'fp32'} (ld={ld}), "
                               f"K={K} accelerated-gossip rounds of X and Y per step, diagonal quadratic + "
                               f"N(0,{sigma}^2) counter-based noise, lr={alpha}",
                   "algorithm": alg, "what": what, "step": step_name,
                   "matrix_rounds_per_s": 2 * E * K / (dt / args.steps) if what == "step" else None,
                   "finite": finite},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "bar": 0.70,      # the fraction of peak asked of the gossip+tracking kernels on this workload
                     "traffic": traffic, "traffic_source": traffic_source, "kernel_ms": phase_ms,
                     "algorithmic_bytes_per_launch": bpe * E,
                     **({"note": note} if note else {})},
    }
    if what == "step" and alg == "detag" and not structured and not args.dense and not per_round:
        # the K rounds of the kernel for arbitrary W run out of LDS: per output and round it reads the neighbours'
        # values (table width: the degree rounded up to 2, 4 or 8) and writes its own, 4 bytes each, for X and for Y
        width = 2 if cfg.degree <= 2 else 4 if cfg.degree <= 4 else 8
        lds_bytes = (width + 1) * 4 * E * K * 2
        lds_rate = lds_bytes / (phase_ms * 1e-3) / 1e9
        out["roofline"].update({"bound": "lds", "achieved": lds_rate, "peak": LDS_PEAK_GBS, "frac": lds_rate / LDS_PEAK_GBS,
                                "lds_bytes_per_launch": lds_bytes, "hbm_achieved": achieved, "hbm_peak": HBM_PEAK_GBS,
                                "hbm_frac": achieved / HBM_PEAK_GBS,
                                "note": "the rounds run out of LDS: achieved/peak are LDS bytes over the whole kernel "
                                        "against 256 CUs x 128 B/clk x 2.4 GHz; hbm_* give the HBM side of the same launch"})
        out["roofline"].pop("bar", None)
    if what == "diag":
        ce_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
        out["roofline"]["consensus_error_ms"] = ce_ms      # two kernels; the second pass over a column comes from cache
        out["roofline"]["consensus_error_GBps"] = sb * E / (ce_ms * 1e-3) / 1e9
    if not args.no_cpu_baseline and alg == "detag" and what == "step" and not per_round:
        out["cpu_baseline"] = cpu_baseline(cfg, min(args.cpu_sample_cols, d), ctx.dense_W())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
