#!/usr/bin/env python3
"""Benchmark of the ASGD mini-batch K-Means hot path on one MI355X.

A "step" is one pass of the whole path (assignment, gradient, merge, update, send) over the
synthetic streaming workload: one epoch of N = 1e8 fp32 samples, d = 10, k = 10, W = 1024
workers, b = 1000, exchange every 8 mini-batches, deterministic mode.  The samples are
resident in HBM before the timed region starts.  Prints ONE JSON line.

--config 2, 3 or 4 times the other workloads the same way (one epoch per step): the wider one
(k = d = 100), the 100 GB one, and the contraction-bound one (k = 1024, d = 128), whose roofline
is the fp32 matrix-core peak instead of the HBM bandwidth.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MATRIX_PEAK_TFLOPS = 157.3 # MI355X published dense fp32 matrix (and packed vector) rate
KERNEL_NAMES = {1: "generic_steps_kernel", 2: "small_steps_kernel", 3: "mfma_steps_kernel"}


def traffic_from_profile(kernel_name, workload_name):
    """HBM bytes per EPOCH measured with rocprofv3 counters (committed summary: bytes per launch and the epochs a
    launch of the profiled command covered), or None."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.txt" % (kernel_name, workload_name))
    try:
        text = open(path).read()
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
        e = re.search(r"^epochs_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
        return float(m.group(1)) / (float(e.group(1)) if e else 1.0) if m else None
    except OSError:
        return None


def cpu_baseline(wl, X):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload: about 15 s of
    its work.  The sample is the first steps of the run, all W workers; if an epoch is shorter than that, the
    run simply goes on into further epochs; if the rows those steps touch would not fit the host (100 GB
    workload), the prefix that fits 8 GB is run several times."""
    from oracle import asgd_oracle
    asgd_oracle.build()
    cores = min(asgd_oracle.threads(), 16)
    asgd_oracle.set_threads(cores)
    est_rate = cores * 2.0e9 / (wl.k * wl.d)              # rough samples/s of the fp64 oracle, to size the sample
    want = 15.0 * est_rate                                # samples
    steps = int(max(1, want / (wl.W * wl.b)))
    if wl.E >= 1:
        steps = max(steps, 2 * wl.E + 1)                  # at least two communication rounds
    rows = min(steps, wl.S) * wl.b                        # rows per worker those steps touch
    max_rows = int(8e9 / (wl.W * wl.d * 4))
    reps = 1
    if rows > max_rows:
        steps = max(1, max_rows // wl.b)
        rows = steps * wl.b
        reps = int(max(1, round(want / (steps * wl.W * wl.b))))
    # shard by shard (the oracle sees W shards of `rows` rows; a run longer than that wraps like an epoch does)
    Xc = X[:wl.W * wl.H].view(wl.W, wl.H, wl.d)[:, :rows, :].contiguous().cpu().numpy().reshape(wl.W * rows, wl.d)
    dt = 0.0
    for _ in range(reps):
        o = asgd_oracle.OracleASGD(Xc, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
        t0 = time.perf_counter()
        o.run_steps(steps)
        dt += time.perf_counter() - t0
    n = reps * steps * wl.W * wl.b
    return {"value": n / dt, "unit": "samples/s", "cores": cores, "nproc": os.cpu_count(), "kind": "oracle",
            "sample": "%d x the first %d steps (an epoch has %d) of the same workload, all %d workers: %d samples in "
                      "%.1f s, fp64, %d OpenMP threads over workers" % (reps, steps, wl.S, wl.W, n, dt, cores)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = streaming workload of the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", type=int, default=0)
    ap.add_argument("--mode", choices=("deterministic", "free", "silent"), default="deterministic",
                    help="deterministic: seeded schedule, reproducible (the metric); free: free-running exchange with "
                         "the paper's races; silent: no exchange at all (E = 0), for the merge-overhead column")
    ap.add_argument("--buffers", type=int, default=1,
                    help="external buffers per worker = recipients per message (Eq. 3 / Eq. 6); 1 is the metric's")
    ap.add_argument("--parts", type=int, default=1,
                    help="partial messages: a copy carries one of P parts of the centroid rows (Sec. 4.4); 1 is the metric's")
    ap.add_argument("--mini-batch", type=int, default=0,
                    help="override the workload's mini-batch size b (sensitivity runs; the workload name gets a suffix)")
    ap.add_argument("--quant-error", action="store_true", help="also report Eq. 8 of worker 0 after the timed epochs")
    ap.add_argument("--plain-launch", action="store_true",
                    help="start the single-launch kernel with a plain launch instead of a cooperative one "
                         "(same kernel, same grid); needed under rocprofv3, whose tool library crashes at "
                         "process exit after cooperative launches")
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed device time spent on the same epochs before the warmup steps, until the clocks of a "
                         "freshly woken device have settled (the first few dozen launches of a process run up to 10 %% "
                         "slower); reported in the JSON line; 0 switches it off")
    ap.add_argument("--epochs-per-call", type=int, default=10,
                    help="epochs (= steps of this benchmark) handed to the library in one asgd_run_epochs call; where "
                         "the library runs a call as ONE launch (streaming kernel, matrix-core kernel with two "
                         "workgroups per CU) the start and the tail of a launch are then paid once per call, not once "
                         "per epoch.  1: one call, one host synchronisation per epoch")
    ap.add_argument("--no-exchange-overhead", action="store_true",
                    help="skip the two extra timed runs (free-running, silent) behind the exchange_overhead object")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the sample array (known size: N*d*4 bytes read and "
                         "written), so that a counter profile of this command can be scaled")
    args = ap.parse_args()
    if args.steps < 1 or args.warmup < 0:
        sys.exit("bench.py: --steps must be at least 1 and --warmup at least 0")
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (all workers share one MI355X); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no HIP device visible; there is no CPU fallback for the product path")
    from paper_1505_04956_amd import binding as B
    from paper_1505_04956_amd import workloads

    wl = workloads.CONFIGS[args.config]
    if args.parts > 1 and args.config in (2, 4):
        sys.exit("bench.py: partial messages are not measured on the matrix-core workloads: the library limits that "
                 "combination to the sizes its tests cover (an unexplained device fault in the one batch of such runs)")
    if args.mini_batch > 0 and args.mini_batch != wl.b:
        wl = wl.scaled(b=args.mini_batch, name="%s_b%d" % (wl.name, args.mini_batch))
    torch.cuda.set_device(0)
    X = workloads.generate_device(wl, device="cuda:0")
    torch.cuda.synchronize()

    if args.calibrate_copy:
        Y = torch.empty_like(X)
        torch.mul(X, 1.0, out=Y)      # an elementwise kernel: reads N*d*4 bytes, writes N*d*4 bytes
        torch.cuda.synchronize()
        del Y
    def context(mode):
        c = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=(0 if mode == "silent" else wl.E), seed=wl.schedule_seed,
                   mode=(B.MODE_FREE_RUNNING if mode == "free" else B.MODE_DETERMINISTIC), tune=args.tune,
                   cooperative=not args.plain_launch, buffers=args.buffers, parts=args.parts)
        c.load_shards(X)
        return c

    per_call = max(1, args.epochs_per_call)

    def run(c, epochs):
        """`epochs` epochs in calls of `per_call` (the last one may be shorter); kernel time and epochs of every call."""
        calls = []
        while epochs > 0:
            n = min(per_call, epochs)
            c.run_epochs(n)                   # returns after the device has finished
            calls.append((c.last_run_ms(), n))
            epochs -= n
        return calls

    def timed(c, steps):
        """`steps` epochs; wall time over all of them and (kernel ms, epochs) of each library call."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        calls = run(c, steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, calls

    g = context(args.mode)
    settle_epochs, settle_ms = 0, 0.0
    while settle_ms < args.settle_ms and settle_epochs < 10000:
        for ms, n in run(g, per_call):
            settle_ms += ms
            settle_epochs += n
    run(g, args.warmup)
    elapsed, calls = timed(g, args.steps)
    st = g.stats()

    samples = wl.processed_per_epoch
    value = args.steps * samples / elapsed
    avg_kernel_ms = sum(ms for ms, n in calls) / sum(n for ms, n in calls)       # per epoch
    last_call_epochs = calls[-1][1]
    algo_bytes = samples * wl.d * 4            # one read of every processed sample
    algo_flops = samples * (2.0 * wl.k * wl.d + wl.k + wl.d)   # expanded-form scores, compares, accumulation
    kname = KERNEL_NAMES.get(int(st.kernel), "?")
    if int(st.kernel) == B.KERNEL_MFMA:
        achieved = algo_flops / (avg_kernel_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": FP32_MATRIX_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / FP32_MATRIX_PEAK_TFLOPS, "algorithmic_flops_per_step": algo_flops,
                    "hbm_GBps": algo_bytes / (avg_kernel_ms * 1e-3) / 1e9}
    else:
        achieved = algo_bytes / (avg_kernel_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBPS, "algorithmic_bytes_per_launch": algo_bytes}
    # per epoch: kernel_ms and the algorithmic bytes / flops above; the launches of the last library call and its epochs
    # say how many epochs one launch covers (traffic is per launch of the profiled command, see profiles/)
    epochs_per_launch = last_call_epochs / max(1, int(st.launches))
    per_epoch_traffic = traffic_from_profile(kname, wl.name)
    roofline.update({"traffic": None if per_epoch_traffic is None else per_epoch_traffic * epochs_per_launch,
                     "kernel": kname, "kernel_ms": avg_kernel_ms, "launches": int(st.launches),
                     "epochs_per_launch": epochs_per_launch, "kernel_ms_per_launch": avg_kernel_ms * epochs_per_launch,
                     "kernel_ms_per_call": [round(ms, 4) for ms, n in calls][:8]})
    if "algorithmic_bytes_per_launch" in roofline:
        roofline["algorithmic_bytes_per_launch"] = algo_bytes * epochs_per_launch
    else:
        roofline["algorithmic_flops_per_launch"] = algo_flops * epochs_per_launch
    out = {
        "metric": "samples/sec (assign+grad+update+merge) and % of peak HBM GB/s, 1 MI355X",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "d": wl.d, "k": wl.k, "W": wl.W, "b": wl.b, "lr": wl.lr,
                   "exchange_every": (0 if args.mode == "silent" else wl.E), "epochs_per_step": 1, "mode": args.mode,
                   "buffers": args.buffers, "parts": args.parts,
                   "samples_per_step": samples, "kernel": int(st.kernel), "epochs_per_call": per_call,
                   "launches_per_step": int(st.launches) / last_call_epochs},
        "roofline": roofline,
        "stats": {"messages_sent": int(st.sent), "messages_received": int(st.received),
                  "messages_accepted": int(st.accepted), "exact_rechecks": int(st.exact_rechecks)},
    }
    out["settle"] = {"epochs": settle_epochs, "device_ms": settle_ms,
                     "note": "untimed, before the warmup steps: clock transient of a freshly started process"}
    if not args.no_exchange_overhead:
        # the cost of the exchange (Sec. 4.4: it must stay small beside the update itself): kernel time of one epoch
        # with the seeded deterministic schedule, free-running, and with no exchange at all, same data, same run
        per_mode = {args.mode: avg_kernel_ms}
        for mode in ("deterministic", "free", "silent"):
            if mode not in per_mode:
                c = context(mode)
                run(c, max(args.warmup, 20))               # (the first epochs of a fresh context run slower)
                _, cs = timed(c, max(args.steps, 20))
                per_mode[mode] = sum(ms for ms, n in cs) / sum(n for ms, n in cs)
                c.close()
        out["exchange_overhead"] = {
            "kernel_ms": per_mode, "unit": "ms per epoch",
            "deterministic_over_silent": per_mode["deterministic"] / per_mode["silent"] - 1.0,
            "free_over_silent": per_mode["free"] / per_mode["silent"] - 1.0}
    if args.quant_error:
        out["stats"]["quant_error_worker0"] = g.quant_error(0)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, X)
    print(json.dumps(out), flush=True)
    g.close()


if __name__ == "__main__":
    main()
