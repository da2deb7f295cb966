"""Convergence table of one synthetic workload: Eq. 8 and the error against the generator's centres after every
epoch, for the deterministic, the free-running and the silent (no exchange: SimuParallelSGD with mini-batches)
mode on the same data — the shape of the paper's convergence figures (Sec. 5.4) without its baselines.

    python -m paper_1505_04956_amd.convergence --config 1 --epochs 8

Evaluation helper around the library; needs a HIP device.  Prints one line per epoch and mode:
worker 0's state (what Alg. 5 returns) and the mean over the workers' states (the map-reduce alternative of Sec. 4).
"""
from __future__ import annotations

import argparse
import sys


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--epochs", type=int, default=8)
    ap.add_argument("--buffers", type=int, default=1)
    ap.add_argument("--parts", type=int, default=1)
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        sys.exit("convergence.py: no HIP device visible")
    from . import binding as B
    from . import workloads
    wl = workloads.CONFIGS[args.config]
    X = workloads.generate_device(wl, device="cuda:0")
    torch.cuda.synchronize()
    modes = (("deterministic", dict(E=wl.E)), ("free-running", dict(E=wl.E, mode=B.MODE_FREE_RUNNING)),
             ("silent", dict(E=0)))
    runs = {}
    for name, kw in modes:
        g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, seed=wl.schedule_seed, buffers=(args.buffers if kw["E"] else 1),
                   parts=(args.parts if kw["E"] else 1), **kw)
        g.load_shards(X)
        runs[name] = g
    print("workload %s: N=%d d=%d k=%d W=%d b=%d E=%d, buffers=%d, parts=%d; per sample: E(w)/N" %
          (wl.name, wl.N, wl.d, wl.k, wl.W, wl.b, wl.E, args.buffers, args.parts), flush=True)
    print("%5s %-14s %14s %14s %12s %12s" % ("epoch", "mode", "E(w_0)/N", "E(mean w)/N", "centres w_0", "centres mean"))
    for ep in range(1, args.epochs + 1):
        for name, _ in modes:
            g = runs[name]
            g.run_epochs(1)
            q0, qm = g.quant_error(0) / wl.N, g.quant_error(-1) / wl.N
            c0 = workloads.centre_error(g.get_state(0), wl)
            cm = workloads.centre_error(g.get_mean_state(), wl)
            print("%5d %-14s %14.6f %14.6f %12.5f %12.5f" % (ep, name, q0, qm, c0, cm), flush=True)
    for g in runs.values():
        g.close()


if __name__ == "__main__":
    main()
