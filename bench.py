#!/usr/bin/env python3
"""Benchmark of the lattice hot path on one MI355X.

Workload: the wordpiece-scale denominator (B=16, T=500, V=256, bigram context,
C=257 states, dense float32 weights [16,500,257,257] ~ 2*N(0,1), 2.114 GB),
the configuration the headline metric is quoted on.  One step = one
log-semiring forward+backward over the whole batch (shortest distance D and
the arc marginals of Eq. 1 written as the gradient tensor), inputs and outputs
resident in HBM.  value = arcs/s with arcs = sum_b len[b]*C*(V+1).

Also timed (reported under "extra", not part of `value`): the full globally
normalised loss (forward+backward plus the numerator on the intersected
lattice and its scatter), the tropical shortest path with backpointers, and
the shortest distance alone.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is
single-GPU by design.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
BYTES_PER_ARC = 12.0           # forward reads w (4), backward reads w (4) and writes gamma (4)

# HBM traffic per forward+backward launch measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); see
# profiles/cluster2_kernel_B16_T500_V256.md: 4.344 GB fetched + 2.260 GB written.
MEASURED_TRAFFIC_BYTES = 6.581e9


def time_region(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


def cpu_baseline(cfg, arcs):
    """The float64 oracle, as it stands, on the same workload (forward, backward, marginals)."""
    import oracle
    oracle.build()
    cores = oracle.max_threads()
    t0 = time.perf_counter()
    alpha, D = oracle.forward(cfg["w"], cfg["lengths"], 1)
    beta = oracle.backward(cfg["w"], cfg["lengths"], 1)
    gamma = oracle.posteriors(cfg["w"], cfg["lengths"], 1, alpha, beta, D)
    dt = time.perf_counter() - t0
    del gamma
    return {"value": arcs / dt, "unit": "arcs/s", "cores": cores, "kind": "oracle",
            "sample": "the full workload (B=%d, T=%d, V=%d): float64 forward + backward + marginals, "
                      "OpenMP over batch items, %.2f s" % (cfg["B"], cfg["T"], cfg["V"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run plain device copies of the weight tensor (known size) so that a "
                         "rocprofv3 --pmc run can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--generation", type=int, default=0,
                    help="cooperating-workgroup kernel generation (0 = the library's choice)")
    ap.add_argument("--B", type=int, default=16)
    ap.add_argument("--T", type=int, default=500)
    ap.add_argument("--V", type=int, default=256)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (items are independent recursions; "
              "sharding would be over the batch with no collectives). --gpus %d refused." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2304_13134_amd import binding as lb
    from paper_2304_13134_amd import workloads

    lb.load_library()                      # fails loudly if the HIP library is missing
    if args.generation:
        lb.set_option(lb.OPT_CLUSTER_GENERATION, args.generation)
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    full = (args.B, args.T, args.V) == (16, 500, 256)
    cfg = workloads.config(3, B=args.B, T=args.T, V=args.V)      # config 2's lattice + references
    if not full:
        cfg = workloads.config(3, B=args.B, T=args.T, V=args.V,
                               Umax=max(1, args.T // 4), u_lo=1, u_hi=max(1, args.T // 4))
    arcs = float(np.sum(cfg["lengths"].astype(np.int64)) * cfg["C"] * (cfg["V"] + 1))
    w = torch.from_numpy(cfg["w"]).cuda()
    lengths = torch.from_numpy(cfg["lengths"]).cuda()
    refs = torch.from_numpy(cfg["refs"]).cuda()
    ulen = torch.from_numpy(cfg["ref_lengths"]).cuda()
    dw = torch.empty_like(w)
    torch.cuda.synchronize()

    def step():
        lb.last_arc_posteriors(w, lengths, order=1, dw=dw)

    if args.pmc_calibration:
        for _ in range(3):
            dw.copy_(w)                 # reads and writes w.numel() * 4 bytes
        torch.cuda.synchronize()

    ms, wall_ms = time_region(step, args.steps, args.warmup)
    value = arcs / (ms * 1e-3)
    achieved = BYTES_PER_ARC * arcs / (ms * 1e-3) / 1e9

    extra = {}
    if not args.no_extra:
        def loss_step():
            lb.last_arc_posteriors(w, lengths, order=1, dw=dw)
            lb.last_intersect_reference(w, lengths, refs, ulen, order=1, dw=dw, scale=-1.0, accumulate=True)
        k = max(3, args.steps // 4)
        extra["full_loss_ms"], _ = time_region(loss_step, k, 1)
        extra["shortest_path_ms"], _ = time_region(lambda: lb.last_shortest_path(w, lengths, order=1), k, 1)
        extra["shortest_distance_log_ms"], _ = time_region(lambda: lb.last_shortest_distance(w, lengths, order=1), k, 1)
        # the trigram lattice with on-the-fly weights (B=4, T=1000, V=64, hidden 512)
        c4 = workloads.config(4)

        def bf16(bits):
            return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)
        se = lb.SharedEmb(bf16(c4["f"]), bf16(c4["e"]), bf16(c4["W"]))
        len4 = torch.from_numpy(c4["lengths"]).cuda()
        _, g4 = lb.last_arc_posteriors(se, len4, order=2)
        extra["fused_trigram_shortest_distance_ms"], _ = time_region(
            lambda: lb.last_shortest_distance(se, len4, order=2), 3, 1)
        extra["fused_trigram_fwd_bwd_ms"], _ = time_region(
            lambda: lb.last_arc_posteriors(se, len4, order=2, dw=g4), 3, 1)
        arcs4 = float(np.sum(c4["lengths"].astype(np.int64)) * c4["C"] * (c4["V"] + 1))
        extra["fused_trigram_arcs_per_s_fwd_bwd"] = arcs4 / (extra["fused_trigram_fwd_bwd_ms"] * 1e-3)
        # matrix-core work of one forward+backward: the weights three times (forward, beta pass, dW pass)
        # plus the two gradient contractions, 2*H flops per arc each
        extra["fused_trigram_tflops"] = 5 * 2.0 * 512 * arcs4 / (extra["fused_trigram_fwd_bwd_ms"] * 1e-3) / 1e12
        del se, g4
        extra["wall_ms_per_step"] = wall_ms
        wt, cx = lb.dense_weights(w), lb.context(cfg["V"], 1)
        extra["kernel_variant"] = lb.last_kernel_variant(wt, cx, lb.OP_ARC_POSTERIORS)

    out = {
        "metric": "lattice arcs/sec (fwd+bwd, log semiring) and achieved HBM GB/s vs peak",
        "value": value, "unit": "arcs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "wordpiece-scale denominator: B=%d T=%d V=%d bigram C=%d, dense fp32 "
                               "weights ~ 2*N(0,1), forward+backward arc marginals"
                               % (cfg["B"], cfg["T"], cfg["V"], cfg["C"]),
                   "B": cfg["B"], "T": cfg["T"], "V": cfg["V"], "C": cfg["C"], "arcs": arcs},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES if full else None,
                     "kernel": "cluster2_kernel<true, false, true> (+ the 5 us tag-clear kernel of the same call)",
                     "algorithmic_bytes_per_launch": BYTES_PER_ARC * arcs},
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        del dw
        out["cpu_baseline"] = cpu_baseline(cfg, arcs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
