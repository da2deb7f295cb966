#!/usr/bin/env python3
"""Writes tests/golden/cfg0_oracle.json: what the CPU oracle computes on the tiny workload
(N = 1e5, d = 10, k = 10, W = 4, b = 500, E = 4, 5 epochs, deterministic mode, seeds 1234 / 1; and three epochs
with N external buffers and / or partial messages).
Calls only the oracle and the seeded input generator.  The paper prints no worked numbers for the
method (Sec. 5.4 reports curves on its own data), so these stored values are a regression pin of
the oracle itself and expected values for the GPU path; run from the repository root:
    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import asgd_oracle          # noqa: E402
from paper_1505_04956_amd import workloads   # noqa: E402


def compute():
    asgd_oracle.build()
    wl = workloads.CONFIGS[0]
    X = workloads.generate_host(wl)
    o = asgd_oracle.OracleASGD(X, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    qe = [o.quant_error(0)]                      # Eq. 8 for worker 0 before and after every epoch
    for _ in range(wl.epochs):
        o.run_epochs(1)
        qe.append(o.quant_error(0))
    variants = {}
    for name, kw in (("buffers2", dict(buffers=2)), ("parts2", dict(parts=2)), ("buffers3_parts5", dict(buffers=3, parts=5))):
        v = asgd_oracle.OracleASGD(X, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed, **kw)
        v.run_epochs(3)
        variants[name] = {
            "options": kw,
            "quant_error_worker0": v.quant_error(0),
            "counters_sent_received_accepted": v.counters.sum(0).tolist(),
            "state_sum_by_worker": v.w.reshape(wl.W, -1).sum(1).tolist(),
        }
    return {
        "workload": wl.name,
        "variants_after_3_epochs": variants,
        "quant_error_worker0_by_epoch": qe,
        "quant_error_mean_state": asgd_oracle.quant_error(X, o.w.mean(0)),
        "counters_sent_received_accepted": o.counters.sum(0).tolist(),
        "state_worker0_row0": o.w[0, 0].tolist(),
        "state_sum_by_worker": o.w.reshape(wl.W, -1).sum(1).tolist(),
        "peers_round0": [asgd_oracle.peer(wl.schedule_seed, 0, i, wl.W) for i in range(wl.W)],
    }


if __name__ == "__main__":
    out = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg0_oracle.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print("wrote", path)
