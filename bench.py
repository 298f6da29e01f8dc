"""Throughput of the full relay distillation step on one MI355X.

A step = pbd_distill_step: cast x, teacher relay T_1..T_B (each block once, activations kept in
HBM), then for every student block forward, MSE loss + gradient, backward and the SGD-momentum
update.  Prints ONE JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA
# fp32 vector FMA without packed instructions (this build must compile them out): 256 CUs x 4 SIMDs
# x 16 lanes x 2 flop x 2.4 GHz; the published 157.3 TFLOP/s counts the packed form
PEAK_FP32_VALU_TFLOPS = 78.6
LR_ALPHA = 0.005          # learning rate of the architecture parameters in the arch / two_round modes

# HBM bytes per launch (mean over a kernel class's launches in one step) from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this script, each scaled by what the same counter reads for a
# 256 MiB copy (fetch x2.000, write x1.000).  Counters cannot be read from inside the process: the
# figures are CARRIED from the counter runs whose commands and full tables are in the named file
# under profiles/ (the record says so under roofline.traffic_source), and apply only to the workload
# and the kernel build they were measured on.
HBM_TRAFFIC_PER_LAUNCH = {
    "resnet50_x1.5": ("profiles/resnet50_x1.5_step_hbm_traffic.md", {
        "bn_bwd_apply_nt": 529362959, "bn_bwd_apply": 109015272, "bn_bwd_reduce_nt": 316315223, "bn_bwd_reduce": 68903370,
        "bn_bwd_reduce_add_nt": 783209493, "bn_bwd_reduce_add_mse_nt": 961371582,
        "wgrad_128x128": 305611219, "wgrad_192x256": 237289843, "wgrad_256x256": 218329889,
        "igemm_fwd_256x192x64_store": 233869020, "igemm_dgrad_256x192x64_store": 166897786,
        "igemm_fwd_256x256x64_affine": 111665417, "igemm_fwd_256x256x64_store": 212692777,
    }),
}

# Batch of the oracle's timed step per configuration: the direct-loop CPU oracle at the full batch of the
# 224 x 224 configurations would take many minutes, so it is timed at a reduced batch on the same graph and
# image size (its samples/s do not depend on the batch to first order: every loop is linear in it).
CPU_BASELINE_BATCH = {"tiny_cnn": 8, "vgg16_dsconv": 256, "mbv2_mbconv_k5e4": 8, "mbv2_supernet": 2, "resnet50_x1.5": 2}

CONV_PREFIXES = ("igemm_", "wgrad_")
# the bandwidth-bound families: normalisation, depthwise, joins, pooling, loss, update, casts, partial sums
EW_PREFIXES = ("bn_", "dw_", "join_", "maxpool_", "mse_", "sgd_", "cast_", "sum_partials", "splitk_", "transpose_", "mix_")


def family_fractions(prof, steps):
    """The two halves of the metric besides samples/s: the convolutions (implicit GEMM forward / backward-data
    and backward-weight launches) as a time-weighted TFLOP/s against the bf16 MFMA peak, and the bandwidth-bound
    families (normalisation, depthwise, joins, pooling, loss, update) as GB/s of algorithmic bytes against the
    HBM peak.  Convolutions are given three ways: all launches, those whose own arithmetic intensity is above
    the MFMA ridge (the matrix-core-bound ones, which the 50 % target is about) and those below it (bandwidth-
    bound 1x1 layers and stems, as GB/s)."""
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    acc = {k: dict(ms=0.0, bytes=0.0, flops=0.0, n=0) for k in ("conv", "conv_hi", "conv_lo", "ew")}
    for p in prof:
        keys = []
        if p["name"].startswith(CONV_PREFIXES):
            keys = ["conv", "conv_hi" if p["bytes"] and p["flops"] / p["bytes"] >= ridge else "conv_lo"]
        elif p["name"].startswith(EW_PREFIXES):
            keys = ["ew"]
        for k in keys:
            a = acc[k]
            a["ms"] += p["ms"]; a["bytes"] += p["bytes"]; a["flops"] += p["flops"]; a["n"] += 1

    def tf(a):
        return a["flops"] / (a["ms"] * 1e-3) / 1e12 if a["ms"] else 0.0

    def gb(a):
        return a["bytes"] / (a["ms"] * 1e-3) / 1e9 if a["ms"] else 0.0

    def conv_entry(a):
        return dict(ms_per_step=round(a["ms"] / steps, 4), launches_per_step=a["n"] // steps,
                    TFLOPs=round(tf(a), 2), frac_of_mfma_peak=round(tf(a) / PEAK_BF16_TFLOPS, 4),
                    GBs=round(gb(a), 1), frac_of_hbm_peak=round(gb(a) / PEAK_HBM_GBS, 4))
    conv = conv_entry(acc["conv"])
    conv["above_ridge"] = conv_entry(acc["conv_hi"])
    conv["below_ridge"] = conv_entry(acc["conv_lo"])
    e = acc["ew"]
    ew = dict(ms_per_step=round(e["ms"] / steps, 4), launches_per_step=e["n"] // steps, GBs=round(gb(e), 1),
              frac_of_hbm_peak=round(gb(e) / PEAK_HBM_GBS, 4))
    return conv, ew


def roofline_from_profile(prof, steps):
    """Aggregate the library's per-launch HIP-event timings by kernel class; report the class that
    takes the most time against the roofline that bounds it."""
    ridge_mfma = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    ridge_alu = PEAK_FP32_VALU_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)

    def bound_of(p):
        # contractions (implicit GEMM, weight gradient) run on the matrix cores; depthwise kernels do
        # their multiply-adds on the vector ALUs; everything else only moves bytes.  A launch counts
        # against the compute peak only when its own arithmetic intensity lies above the ridge.
        ai = p["flops"] / p["bytes"] if p["bytes"] else 0.0
        if p["name"].startswith(("igemm_", "wgrad_")) and ai >= ridge_mfma:
            return "mfma"
        if p["name"].startswith("dw_") and ai >= ridge_alu:
            return "alu"
        return "hbm"

    agg, groups = {}, {}
    for p in prof:
        a = agg.setdefault(p["name"], dict(ms=0.0, bytes=0.0, flops=0.0, n=0))
        a["ms"] += p["ms"]; a["bytes"] += p["bytes"]; a["flops"] += p["flops"]; a["n"] += 1
        g = groups.setdefault((p["name"], bound_of(p)), dict(ms=0.0, bytes=0.0, flops=0.0, n=0))
        g["ms"] += p["ms"]; g["bytes"] += p["bytes"]; g["flops"] += p["flops"]; g["n"] += 1
    # the kernel class with the most time; of its launches, those on the side of the ridge where most
    # of that time is spent
    name = max(agg.items(), key=lambda kv: kv[1]["ms"])[0]
    bound, a = max(((k[1], v) for k, v in groups.items() if k[0] == name), key=lambda kv: kv[1]["ms"])
    avg_s = a["ms"] / a["n"] * 1e-3
    if bound == "mfma":
        achieved, peak, unit = a["flops"] / a["n"] / avg_s / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
    elif bound == "alu":
        achieved, peak, unit = a["flops"] / a["n"] / avg_s / 1e12, PEAK_FP32_VALU_TFLOPS, "TFLOP/s"
    else:
        achieved, peak, unit = a["bytes"] / a["n"] / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
    classes = {k: dict(ms_per_step=round(v["ms"] / steps, 4), launches_per_step=v["n"] // steps,
                       gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] else 0.0,
                       tflops=round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] else 0.0)
               for k, v in sorted(agg.items(), key=lambda kv: -kv[1]["ms"])}
    # the whole step against its algorithmic work: every profiled launch's bytes and flops, once
    totals = dict(algorithmic_bytes=round(sum(v["bytes"] for v in agg.values()) / steps),
                  algorithmic_flops=round(sum(v["flops"] for v in agg.values()) / steps),
                  launches=sum(v["n"] for v in agg.values()) // steps,
                  kernel_ms=round(sum(v["ms"] for v in agg.values()) / steps, 4))
    return dict(bound=bound, achieved=round(achieved, 2), peak=peak, unit=unit, frac=round(achieved / peak, 4),
                traffic=None, kernel=name, avg_launch_us=round(avg_s * 1e6, 2),
                launches_per_step=a["n"] // steps, class_launches_per_step=agg[name]["n"] // steps), classes, totals


def measure_peaks(torch):
    """Achievable rates on this machine, for context beside the datasheet peaks: a device-to-device copy
    (read + write bytes over time) and a large bf16 GEMM through the vendor library."""
    def timed(fn, reps):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    src = torch.ones(2**28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    t_copy = timed(lambda: dst.copy_(src), 20)
    del src, dst
    a = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda:0")
    b = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda:0")
    t_mm = timed(lambda: torch.matmul(a, b), 10)
    return {"copy_GBs": round(2 * 2**30 / t_copy / 1e9, 1), "matmul_bf16_TFLOPs": round(2 * 8192**3 / t_mm / 1e12, 1)}


def cpu_baseline(wl):
    """The oracle as it stands (fp32 instance, OpenMP), timed on the host cores on the same graph and image
    size; at the full batch where that takes seconds, else at the reduced batch of CPU_BASELINE_BATCH."""
    from oracle import pbd_oracle as orc
    from paper_2301_12443_amd import workloads as W
    batch = min(wl.batch, CPU_BASELINE_BATCH.get(wl.name, wl.batch))
    words, pool = W.pack(wl)
    o = orc.Oracle(words, pool, batch, precision=32, momentum=wl.momentum)
    for net, b, j, slot, arr in W.iter_params(wl):
        o.set_param(net, b, j, slot, arr)
    x = W.make_input(wl, batch=batch)
    o.relay_step(x, wl.lr)                      # first-touch
    t0 = time.time()
    n = 2
    for _ in range(n):
        o.relay_step(x, wl.lr)
    dt = (time.time() - t0) / n
    what = f"full batch {batch}" if batch == wl.batch else f"batch {batch} of the configured {wl.batch} (same graph, same {wl.in_shape[1]} x {wl.in_shape[2]} images)"
    return dict(value=round(batch / dt, 2), unit="samples/s", cores=orc.num_threads(), kind="oracle",
                sample=f"fp32 oracle relay_step, {what}, mean of {n} steps after 1 warm-up, {dt:.2f} s per step")


W_NAMES = ("tiny_cnn", "vgg16_dsconv", "mbv2_mbconv_k5e4", "mbv2_supernet", "resnet50_x1.5")


def tune_pipeline_order(d, x, wl, torch, tries=None):
    """Untimed, before the warm-up: the B+1 branches of the pipelined step are independent, so the order in
    which they are captured changes no result, only how the replayed graph shares the hardware queues.  A few
    orders (each student block first, the students in reverse, the teacher first) are timed over `tries`
    steps each and the fastest is kept.  tries=None: as many steps as fit in about 0.3 s, between 5 and 20."""
    B = wl.B
    base = list(range(B))
    cands = [base + [B]] + [[b] + [v for v in base if v != b] + [B] for b in range(1, B)]
    cands += [base[::-1] + [B], [B] + base[::-1], [B] + base]
    best = None
    for order in cands:
        d.set_pipeline_order(order)
        t0 = time.perf_counter()
        for _ in range(3):
            d.pipeline_step(x, wl.lr)
        d.pipeline_flush()
        torch.cuda.synchronize()
        if tries is None:       # (the first three steps include the capture: an upper bound of the step time)
            tries = max(5, min(20, int(0.3 / max((time.perf_counter() - t0) / 3, 1e-6))))
        t0 = time.perf_counter()
        for _ in range(tries):
            d.pipeline_step(x, wl.lr)
        d.pipeline_flush()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if best is None or dt < best[0]:
            best = (dt, order)
    d.set_pipeline_order(best[1])
    return best[1]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="resnet50_x1.5", choices=sorted(W_NAMES),
                    help="workload; the default is the largest single-GPU configuration (ResNet-50 -> x1.5 inner widths, "
                         "batch 256, 224 x 224, bf16)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["pipelined", "relay", "redundant", "arch", "two_round"], default="pipelined",
                    help="pipelined: pbd_pipeline_step, the whole step with the teacher's relay of batch k+1 running "
                         "beside the students' training on batch k (Sec. IV-A, IV-B); the timed region starts and "
                         "ends with an empty pipeline (K calls and the flush: K teacher passes, K student passes).  "
                         "relay: pbd_distill_step, one whole step at a time (same results bit for bit; faster on the "
                         "two largest configurations, whose kernels fill the chip by themselves).  redundant: the baseline's teacher "
                         "schedule on the same kernels (before block i, T_1..T_i are run again from the input, "
                         "Sec. III), for the relay-vs-redundant ratio; never the headline value.  arch: "
                         "pbd_distill_arch_step, the architecture round of a supernet student (Sec. VI-A).  two_round: "
                         "the NAS step, architecture round then weight round on the same batch")
    ap.add_argument("--no-tune", action="store_true",
                    help="pipelined mode: keep the default capture order of the graph's branches instead of timing "
                         "a few orders before the warm-up and keeping the fastest (any order computes the same bits)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch the step's kernels one by one (for rocprofv3 --pmc runs)")
    ap.add_argument("--counter-run", action="store_true",
                    help="for rocprofv3 --pmc runs, where every dispatch is serialised: no one-step-at-a-time timing, "
                         "one event-timed step instead of 20, and a progress line on stderr after every phase")
    ap.add_argument("--classes", action="store_true", help="also print the per-kernel-class table to stderr")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure what this box reaches on a plain 1 GiB device copy and on a library "
                         "bf16 GEMM (8192^3, torch.matmul), reported under \"calibration\" next to the datasheet peaks")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run a plain device-to-device copy of this many MiB (a kernel of known "
                         "traffic to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU relay step only: run with --gpus 1 "
              "(this build has no multi-GPU path)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2301_12443_amd import pbd, workloads as W
    wl = W.CONFIGS[args.config]()
    d = pbd.Distiller(wl, no_graph=args.no_graph)
    d.bind("cuda:0")
    d.load_params()
    x = torch.from_numpy(W.make_input(wl)).cuda()       # resident in HBM before the timed region

    def step():
        if args.mode == "pipelined":
            d.pipeline_step(x, wl.lr)
        elif args.mode == "relay":
            d.distill_step(x, wl.lr)
        elif args.mode == "arch":
            d.distill_arch_step(x, LR_ALPHA)
        elif args.mode == "two_round":
            d.distill_arch_step(x, LR_ALPHA)
            d.distill_step(x, wl.lr)
        else:
            for i in range(1, wl.B + 1):
                d.teacher_prefix(x, i)
                d.student_step(i, wl.lr)

    def progress(what):
        if args.counter_run:
            print(f"[bench] {what}", file=sys.stderr, flush=True)

    progress("set up")
    order = None
    if args.mode == "pipelined" and not args.no_tune and not args.no_graph:
        order = tune_pipeline_order(d, x, wl, torch)
    for _ in range(args.warmup):
        step()
    d.pipeline_flush()                  # (nothing to do outside the pipelined mode)
    torch.cuda.synchronize()
    progress("warm-up done")
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
        if args.counter_run:
            torch.cuda.synchronize()
            progress(f"step {k + 1} of {args.steps}")
    d.pipeline_flush()                  # the students' pass on the last batch belongs to the K steps
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    losses = d.losses.cpu().numpy()
    assert all(l == l and l > 0 for l in losses), losses

    # One step at a time: median over pbd_distill_step calls, each bracketed by two HIP events recorded on the
    # library's own stream (the stream its kernels run on), beside the mean of the pipelined steps above.
    one_step = None
    if args.mode in ("pipelined", "relay") and not args.counter_run:
        nev = max(20, min(args.steps, 50))
        for _ in range(3):
            d.distill_step(x, wl.lr)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nev)]
        for e0, e1 in evs:
            e0.record(d._stream)
            d.distill_step(x, wl.lr)
            e1.record(d._stream)
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        med = ms[len(ms) // 2]
        one_step = dict(call="pbd_distill_step", timed_calls=nev, median_ms=round(med, 4), min_ms=round(ms[0], 4),
                        samples_per_s=round(wl.batch / (med * 1e-3), 1), timer="HIP events on the library's stream")

    # per-kernel timings with HIP events on the library's stream (separate, profiled steps)
    psteps = 1 if args.counter_run else 20
    d.set_profile(True); d.reset_profile()
    for _ in range(psteps):
        if args.mode in ("arch", "two_round"):
            d.distill_arch_step(x, LR_ALPHA)
        if args.mode != "arch":
            d.distill_step(x, wl.lr)
    prof = d.get_profile()
    d.set_profile(False)
    progress("event-timed step done")
    roof, classes, totals = roofline_from_profile(prof, psteps)
    conv, elementwise = family_fractions(prof, psteps)
    src, table = HBM_TRAFFIC_PER_LAUNCH.get(args.config, (None, {}))
    if roof["kernel"] in table and roof["launches_per_step"] == roof["class_launches_per_step"]:
        roof["traffic"] = table[roof["kernel"]]          # counters were averaged over the whole class
        roof["traffic_source"] = f"carried from the rocprofv3 --pmc runs recorded in {src}, not measured in this run"
    if args.classes:
        for k, v in classes.items():
            print(f"{k:24s} {v}", file=sys.stderr)

    if args.calibrate_copy:
        src = torch.ones(args.calibrate_copy * 2**20 // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    rec = {
        "metric": {"pipelined": "distillation samples/sec/GPU (full relay step) + % MFMA peak on convs",
                   "relay": "distillation samples/sec/GPU (full relay step, one step at a time)",
                   "redundant": "distillation samples/sec/GPU (teacher re-run per block, no relay; direct launches)",
                   "arch": "distillation samples/sec/GPU (relay + architecture round only)",
                   "two_round": "distillation samples/sec/GPU (NAS step: relay + architecture round, relay + weight round)"}[args.mode],
        "value": round(wl.batch * args.steps / dt, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.precision == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {wl.batch}, input {wl.in_shape}, {wl.B} blocks, "
                               + {"arch": "teacher relay + student fwd/MSE/bwd to the mix ops/alpha update",
                                  "two_round": "architecture round (alpha) then weight round, one relay each"}.get(
                                      args.mode, "teacher relay + student fwd/MSE/bwd/SGD-momentum")
                               + ("; steps pipelined over batches (teacher of batch k+1 beside the students of batch k), "
                                  "timed from an empty pipeline to an empty pipeline" if args.mode == "pipelined" else ""),
                   "lr": wl.lr, **({"pipeline_order": order} if order else {})},
        "roofline": roof,
        # the metric's second half: convolutions against the bf16 MFMA peak, and the bandwidth-bound
        # families against the HBM peak (time-weighted over the profiled steps' launches)
        "conv": conv,
        "elementwise": elementwise,
    }
    if one_step:
        rec["one_step"] = one_step
    # step level: unfused algorithmic bytes and flops of one step over the measured step time (how far
    # the whole step is from moving its tensors once at the HBM peak / doing its MACs at the MFMA peak)
    step_s = dt / args.steps
    rec["step_level"] = dict(totals, GBs=round(totals["algorithmic_bytes"] / step_s / 1e9, 1),
                             TFLOPs=round(totals["algorithmic_flops"] / step_s / 1e12, 2),
                             hbm_frac=round(totals["algorithmic_bytes"] / step_s / 1e9 / PEAK_HBM_GBS, 4),
                             mfma_frac=round(totals["algorithmic_flops"] / step_s / 1e12 / PEAK_BF16_TFLOPS, 4))
    if args.peaks:
        rec["calibration"] = measure_peaks(torch)
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
