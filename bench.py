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
lattice and its scatter), the tropical shortest path with backpointers, the
shortest distance alone, the locally normalised log-likelihood, the trigram
lattice with on-the-fly weights, and -- under "ceilings" -- a plain read sweep
and a plain copy of the same weight tensor, the streaming yardstick of this
GPU that the forward+backward time is held against.

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

# HBM traffic of one forward+backward launch at B=16, T=500, V=256, from two rocprofv3 --pmc runs of
# this script (FETCH_SIZE, then WRITE_SIZE, per dispatch), each scaled by what the same counter reads
# for the plain copy of the weight tensor that --pmc-calibration adds; the runs and their arithmetic
# are in profiles/cluster3_kernel_B16_T500_V256.md.
MEASURED_FETCH_BYTES = 4.350e9
MEASURED_WRITE_BYTES = 2.263e9
HEADLINE_KERNEL = "cluster3_kernel<true, false, 3> (+ the 3 us tag-clear kernel of the same call)"


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


def cpu_baseline(cfg):
    """The float64 oracle, as it stands, on the same workload (forward, backward, marginals): all
    host threads on the whole batch, and one thread on the first four items."""
    import numpy as np
    import oracle
    oracle.build()
    cores = oracle.max_threads()

    def run(w, lengths):
        t0 = time.perf_counter()
        alpha, D = oracle.forward(w, lengths, 1)
        beta = oracle.backward(w, lengths, 1)
        gamma = oracle.posteriors(w, lengths, 1, alpha, beta, D)
        dt = time.perf_counter() - t0
        del gamma
        return float(np.sum(lengths.astype(np.int64)) * cfg["C"] * (cfg["V"] + 1)) / dt, dt

    all_rate, all_dt = run(cfg["w"], cfg["lengths"])
    n1 = min(4, cfg["B"])
    oracle.set_threads(1)
    one_rate, one_dt = run(cfg["w"][:n1], cfg["lengths"][:n1])
    oracle.set_threads(cores)
    return {"value": all_rate, "unit": "arcs/s", "cores": cores, "kind": "oracle",
            "sample": "the full workload (B=%d, T=%d, V=%d): float64 forward + backward + marginals, "
                      "OpenMP over batch items, %.2f s" % (cfg["B"], cfg["T"], cfg["V"], all_dt),
            "single_thread": {"value": one_rate, "unit": "arcs/s", "cores": 1,
                              "sample": "the first %d items of the same workload, %.2f s" % (n1, one_dt)}}


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
    ap.add_argument("--option", action="append", default=[], metavar="N=VALUE",
                    help="set process-wide option N of the library (numbers of last_option_t in "
                         "include/last.h), e.g. 2=0 for the one-workgroup shortest-path kernels")
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
    for kv in args.option:
        k, v = kv.split("=")
        lb.set_option(int(k), int(v))
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
    st = torch.full((cfg["B"],), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def step():
        lb.last_arc_posteriors(w, lengths, order=1, dw=dw, item_status=st)

    if args.pmc_calibration:
        for _ in range(3):              # probe_copy_kernel: reads and writes w.numel() * 4 bytes
            lb.last_probe_bandwidth(lb.PROBE_COPY, w, dw)
        torch.cuda.synchronize()

    ms, wall_ms = time_region(step, args.steps, args.warmup)
    lb.check_item_status(st)            # a timed-out or out-of-range item would void the number
    value = arcs / (ms * 1e-3)
    achieved = BYTES_PER_ARC * arcs / (ms * 1e-3) / 1e9

    # what this GPU streams when nothing else happens, on the same tensor: one read sweep, one copy
    wbytes = float(w.numel() * 4)
    k = max(5, args.steps // 2)
    read_ms, _ = time_region(lambda: lb.last_probe_bandwidth(lb.PROBE_READ, w, dw), k, 2)
    copy_ms, _ = time_region(lambda: lb.last_probe_bandwidth(lb.PROBE_COPY, w, dw), k, 2)
    ceilings = {}
    if cfg["C"] == 257:
        # the kernel's two read patterns without its arithmetic (rows per wavefront / column blocks per workgroup)
        rows_ms, _ = time_region(lambda: lb.last_probe_bandwidth(lb.PROBE_READ_ROWS, w, dw), k, 2)
        cols_ms, _ = time_region(lambda: lb.last_probe_bandwidth(lb.PROBE_READ_COLUMNS, w, dw), k, 2)
        ceilings.update({"read_rows_pattern_GBs": wbytes / rows_ms / 1e6,
                         "read_column_blocks_pattern_GBs": wbytes / cols_ms / 1e6})
    ceilings.update({"read_sweep_ms": read_ms, "read_sweep_GBs": wbytes / read_ms / 1e6,
                "copy_ms": copy_ms, "copy_GBs": 2 * wbytes / copy_ms / 1e6,
                # forward+backward = one read-only pass + one read-and-write pass over the weights
                "read_plus_copy_ms": read_ms + copy_ms,
                "frac_of_read_plus_copy": (read_ms + copy_ms) / ms})

    extra = {}
    # every call timed by itself as well: median and minimum (the headline figure is the mean of the
    # whole timed region above)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    each = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    extra["ms_per_step_median"] = each[len(each) // 2]
    extra["ms_per_step_min"] = each[0]
    if not args.no_extra:
        def loss_step():
            lb.last_arc_posteriors(w, lengths, order=1, dw=dw)
            lb.last_intersect_reference(w, lengths, refs, ulen, order=1, dw=dw, scale=-1.0, accumulate=True)
        k = max(3, args.steps // 4)
        extra["full_loss_two_calls_ms"], _ = time_region(loss_step, k, 1)
        extra["full_loss_ms"], _ = time_region(
            lambda: lb.last_globally_normalized_loss(w, lengths, refs, ulen, order=1, dw=dw, item_status=st), k, 1)
        lb.check_item_status(st)
        extra["numerator_cost_ms"] = extra["full_loss_ms"] - ms
        extra["shortest_path_ms"], _ = time_region(lambda: lb.last_shortest_path(w, lengths, order=1), k, 1)
        extra["shortest_distance_log_ms"], _ = time_region(lambda: lb.last_shortest_distance(w, lengths, order=1), k, 1)
        extra["local_log_likelihood_and_gradient_ms"], _ = time_region(
            lambda: lb.last_local_log_likelihood(w, lengths, refs, ulen, order=1, dw=dw), k, 1)
        lb.check_item_status()
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
        # the forward kernel with the weights of one frame at a time instead of two (the default)
        frames_default = lb.set_option(lb.OPT_FUSED_FRAMES_PER_TILE, 1)
        extra["fused_trigram_shortest_distance_ms_one_frame_per_tile"], _ = time_region(
            lambda: lb.last_shortest_distance(se, len4, order=2), 3, 1)
        lb.set_option(lb.OPT_FUSED_FRAMES_PER_TILE, frames_default)
        extra["fused_frames_per_tile"] = frames_default
        # forward+backward with the marginals rebuilt for dW (a third evaluation of the weights) instead of kept
        keep_default = lb.set_option(lb.OPT_FUSED_KEEP_MARGINALS, 0)
        extra["fused_trigram_fwd_bwd_ms_marginals_recomputed"], _ = time_region(
            lambda: lb.last_arc_posteriors(se, len4, order=2, dw=g4), 3, 1)
        lb.set_option(lb.OPT_FUSED_KEEP_MARGINALS, keep_default)
        extra["fused_keep_marginals"] = keep_default
        arcs4 = float(np.sum(c4["lengths"].astype(np.int64)) * c4["C"] * (c4["V"] + 1))
        extra["fused_trigram_arcs_per_s_fwd_bwd"] = arcs4 / (extra["fused_trigram_fwd_bwd_ms"] * 1e-3)
        # matrix-core work of one forward+backward: the weights twice (forward, beta pass; the dW pass
        # takes the marginals the beta pass kept) plus the two gradient contractions, 2*H flops per arc each
        extra["fused_trigram_tflops"] = 4 * 2.0 * 512 * arcs4 / (extra["fused_trigram_fwd_bwd_ms"] * 1e-3) / 1e12
        del se, g4
        # the shape of the paper's own benchmark (Table 2: 32 labels, 1057 states, 512 hidden units,
        # batch 16, 1024 frames, 256 output labels): one training step of the globally normalised loss =
        # denominator forward-backward + numerator, gradients to f, e, W.  The paper's Table 3 times
        # this step on other hardware (context, not a target).
        c5 = workloads.config(5)
        se5 = lb.SharedEmb(bf16(c5["f"]), bf16(c5["e"]), bf16(c5["W"]))
        len5 = torch.from_numpy(c5["lengths"]).cuda()
        refs5, ulen5 = torch.from_numpy(c5["refs"]).cuda(), torch.from_numpy(c5["ref_lengths"]).cuda()
        _, g5 = lb.last_arc_posteriors(se5, len5, order=2)

        def table2_step():
            lb.last_globally_normalized_loss(se5, len5, refs5, ulen5, order=2, dw=g5)
        extra["table2_training_step_ms"], _ = time_region(table2_step, 3, 1)
        lb.check_item_status()
        extra["table2_numerator_ms"], _ = time_region(
            lambda: lb.last_intersect_reference(se5, len5, refs5, ulen5, order=2, dw=g5, scale=-1.0,
                                                accumulate=True), 3, 1)
        arcs5 = float(np.sum(c5["lengths"].astype(np.int64)) * c5["C"] * (c5["V"] + 1))
        extra["table2_arcs_per_s"] = arcs5 / (extra["table2_training_step_ms"] * 1e-3)
        del se5, g5
        # the small batch denominator (B=8, T<=200, V=32): 7 MB of weights, latency bound; time only
        c1 = workloads.config(1)
        w1, len1 = torch.from_numpy(c1["w"]).cuda(), torch.from_numpy(c1["lengths"]).cuda()
        g1 = torch.empty_like(w1)
        extra["config1_forward_backward_ms"], _ = time_region(
            lambda: lb.last_arc_posteriors(w1, len1, order=1, dw=g1), 10, 2)
        lb.check_item_status()
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
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_FETCH_BYTES + MEASURED_WRITE_BYTES if full and not args.generation else None,
                     "counter_GBs": (MEASURED_FETCH_BYTES + MEASURED_WRITE_BYTES) / (ms * 1e-3) / 1e9
                                    if full and not args.generation else None,
                     "kernel": HEADLINE_KERNEL if full and not args.generation else None,
                     "algorithmic_bytes_per_launch": BYTES_PER_ARC * arcs},
        "ceilings": ceilings,
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        del dw
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
