#!/usr/bin/env python3
"""Benchmark of the ASGD mini-batch K-Means hot path on one MI355X.

A "step" is one pass of the whole path (assignment, gradient, merge, update, send) over the
synthetic streaming workload: one epoch of N = 1e8 fp32 samples, d = 10, k = 10, W = 1024
workers, b = 1000, exchange every 8 mini-batches, deterministic mode.  The samples are
resident in HBM before the timed region starts.  Prints ONE JSON line.
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


def traffic_from_profile():
    """HBM bytes per launch measured with rocprofv3 counters (committed summary), or None."""
    path = os.path.join(ROOT, "profiles", "small_steps_kernel_cfg1_streaming_pmc.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(wl, X_host):
    """The oracle as it stands, timed on the host cores over one full epoch of the same samples."""
    from oracle import asgd_oracle
    asgd_oracle.build()
    cores = min(asgd_oracle.threads(), 16)
    asgd_oracle.set_threads(cores)
    o = asgd_oracle.OracleASGD(X_host, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    t0 = time.perf_counter()
    o.run_epochs(1)
    dt = time.perf_counter() - t0
    return {"value": wl.processed_per_epoch / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": "one full epoch of the same workload (%d samples), fp64, %d OpenMP threads over workers"
                      % (wl.processed_per_epoch, cores)}, o


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = streaming workload of the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", type=int, default=0)
    ap.add_argument("--plain-launch", action="store_true",
                    help="start the single-launch kernel with a plain launch instead of a cooperative one "
                         "(same kernel, same grid); needed under rocprofv3, whose tool library crashes at "
                         "process exit after cooperative launches")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the sample array (known size: N*d*4 bytes read and "
                         "written), so that a counter profile of this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (all workers share one MI355X); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no HIP device visible; there is no CPU fallback for the product path")
    from paper_1505_04956_amd import binding as B
    from paper_1505_04956_amd import workloads

    wl = workloads.CONFIGS[args.config]
    torch.cuda.set_device(0)
    X = workloads.generate_device(wl, device="cuda:0")
    torch.cuda.synchronize()

    if args.calibrate_copy:
        Y = torch.empty_like(X)
        torch.mul(X, 1.0, out=Y)      # an elementwise kernel: reads N*d*4 bytes, writes N*d*4 bytes
        torch.cuda.synchronize()
        del Y
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, tune=args.tune,
               cooperative=not args.plain_launch)
    g.load_shards(X)
    for _ in range(args.warmup):
        g.run_epochs(1)
    torch.cuda.synchronize()
    kernel_ms = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.run_epochs(1)                       # returns after the device has finished
        kernel_ms.append(g.last_run_ms())
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = g.stats()

    samples = wl.processed_per_epoch
    value = args.steps * samples / elapsed
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms)
    algo_bytes = samples * wl.d * 4            # one read of every processed sample
    achieved = algo_bytes / (avg_kernel_ms * 1e-3) / 1e9
    out = {
        "metric": "samples/sec (assign+grad+update+merge) and % of peak HBM GB/s, 1 MI355X",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "d": wl.d, "k": wl.k, "W": wl.W, "b": wl.b, "lr": wl.lr,
                   "exchange_every": wl.E, "epochs_per_step": 1, "mode": "deterministic",
                   "samples_per_step": samples, "kernel": int(st.kernel), "launches_per_step": int(st.launches)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic_from_profile(),
                     "kernel": "small_steps_kernel", "kernel_ms": avg_kernel_ms,
                     "algorithmic_bytes_per_launch": algo_bytes},
        "stats": {"messages_sent": int(st.sent), "messages_received": int(st.received),
                  "messages_accepted": int(st.accepted), "exact_rechecks": int(st.exact_rechecks)},
    }
    if not args.no_cpu_baseline:
        X_host = X.cpu().numpy()
        base, _ = cpu_baseline(wl, X_host)
        out["cpu_baseline"] = base
    print(json.dumps(out), flush=True)
    g.close()


if __name__ == "__main__":
    main()
