"""Parity at the workloads' full sizes and in the launch configuration bench.py times
(deterministic mode), against the oracle:
  - streaming workload (N = 1e8, d = 10, k = 10, W = 1024, b = 1000, E = 8): one epoch, every
    assignment and every worker state;
  - wider workload (k = d = 100, W = 512, b = 2000, E = 8): one epoch, all assignments and states;
  - contraction workload (k = 1024, d = 128, W = 256, b = 4096, E = 4): one epoch plus the first
    merge step, all assignments and states;
  - HBM-scale workload (N = 2.5e9, W = 4096, E = 16; 100 GB of samples): the first two
    communication rounds element by element (the oracle runs them on a compacted copy of the rows
    those steps touch), then the whole epoch on properties that hold at any size.
"""
import numpy as np
import pytest

from paper_1505_04956_amd import workloads

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def compare(tag, g, o, ag, ao, gap, state_tol=1e-4):
    """Bar: assignments are identical except at near-ties (oracle relative gap < 1e-6).  A near-tie that is
    resolved the other way moves one sample between two centroids, after which that worker's state differs
    from the oracle's by a few 1e-5 (relative) and later samples of the SAME worker whose gap is below that
    perturbation may follow; those must stay below 1e-3 and are listed."""
    st = g.stats()
    W = o.w.shape[0]
    wg = g.get_state().astype(np.float64).reshape(W, -1)
    wo = o.w.reshape(W, -1)
    err = np.linalg.norm(wg - wo, axis=1) / np.linalg.norm(wo, axis=1)
    diff = ag != ao
    print("\n[%s] %d assignments: mismatches %d, oracle near-ties %d, Parzen near-ties %d; max state err %.3g; "
          "exact rechecks %d; messages sent/received/good %d/%d/%d (oracle %d/%d/%d); kernel %d, launches %d, %.3f ms"
          % (tag, ag.size, diff.sum(), (gap < 1e-6).sum(), o.near[1], err.max(), st.exact_rechecks, st.sent,
             st.received, st.accepted, *o.counters.sum(0), st.kernel, st.launches, st.last_run_ms))
    first_seen = {}
    for t, i, n in zip(*np.nonzero(diff)):
        print("   mismatch step %d worker %d sample %d: gpu %d oracle %d gap %.3g"
              % (t, i, n, ag[t, i, n], ao[t, i, n], gap[t, i, n]))
        if i not in first_seen:
            first_seen[i] = t
        if t == first_seen[i]:
            assert gap[t, i, n] < 1e-6, "first mismatch of worker %d is not a near-tie" % i
        else:
            assert gap[t, i, n] < 1e-3, "mismatch of worker %d after a near-tie flip has a large gap" % i
    assert np.all(np.isfinite(wg))
    assert err.max() <= state_tol
    if o.near[1] == 0:
        assert np.array_equal(g.worker_counters(), o.counters)


def run_config(oracle, wl, steps, expect_kernel, expect_launches=None):
    from paper_1505_04956_amd import binding as B
    X = workloads.generate_device(wl, device="cuda:0")
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
    g.load_shards(X)
    g.enable_assign_dump(steps)
    g.run_steps(steps)
    st = g.stats()
    assert st.kernel == expect_kernel
    if expect_launches is not None:
        assert st.launches == expect_launches
    ag = g.assign_dump(steps)
    oracle.set_threads(16)
    o = oracle.OracleASGD(X.cpu().numpy(), k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    ao, gap = o.run_steps(steps, dump=True)
    compare(wl.name, g, o, ag, ao, gap)
    qg, qo = g.quant_error(0), o.quant_error(0)
    assert abs(qg - qo) <= 1e-4 * qo
    return g, o


def test_streaming_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[1]
    run_config(oracle, wl, wl.S, B.KERNEL_SMALL, expect_launches=1)       # what bench.py times


def test_wider_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[2]
    g, o = run_config(oracle, wl, wl.S, B.KERNEL_MFMA)
    assert o.counters[:, 2].sum() > 0


def test_contraction_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[4]
    g, o = run_config(oracle, wl, wl.S + 1, B.KERNEL_MFMA)                # the step after the epoch is a merge step
    assert o.counters[:, 1].sum() == wl.W


def test_hbm_scale_workload(oracle):
    import torch
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[3]
    free, total = torch.cuda.mem_get_info()
    if free < 115e9:
        pytest.skip("needs 115 GB of free device memory, have %.0f GB" % (free / 1e9))
    X = workloads.generate_device(wl, device="cuda:0")                   # 100 GB
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
    g.load_shards(X)
    # --- the first two rounds, element by element ---
    steps = 2 * wl.E + 1                                                  # ends one step after the second merge point
    g.enable_assign_dump(steps)
    g.run_steps(steps)
    assert g.stats().kernel == B.KERNEL_SMALL and g.stats().launches == 1
    ag = g.assign_dump(steps)
    g.disable_assign_dump()
    rows = steps * wl.b
    Xc = X[:wl.W * wl.H].view(wl.W, wl.H, wl.d)[:, :rows, :].contiguous().cpu().numpy().reshape(wl.W * rows, wl.d)
    oracle.set_threads(16)
    o = oracle.OracleASGD(Xc, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    ao, gap = o.run_steps(steps, dump=True)
    compare(wl.name + " first rounds", g, o, ag, ao, gap)
    assert o.counters[:, 1].sum() == 2 * wl.W                             # every worker has merged twice
    # --- the rest of the epoch: properties ---
    w_before = g.get_state()
    q_before = g.quant_error(0)
    g.run_steps(wl.S - steps)
    st = g.stats()
    w_after = g.get_state()
    q_after = g.quant_error(0)
    rounds = wl.S // wl.E
    print("\n[%s epoch] %.3f ms for %d steps (%.3g samples/s); E(w) of worker 0 %.6g -> %.6g; "
          "messages sent/received/good %d/%d/%d"
          % (wl.name, st.last_run_ms, wl.S - steps, (wl.S - steps) * wl.W * wl.b / st.last_run_ms * 1e3,
             q_before, q_after, st.sent, st.received, st.accepted))
    assert st.steps == wl.S and st.launches == 1
    assert np.all(np.isfinite(w_after))
    assert st.sent == wl.W * rounds                                       # every worker sends once per round
    assert st.received == wl.W * ((wl.S - 1) // wl.E)                     # ... and merges at every multiple of E
    assert 0 < st.accepted <= st.received
    assert q_after <= q_before * 1.001                                    # constant step size: no worse, up to SGD noise
    # the states stay inside the convex hull box of the data they average
    lo, hi = float(X[:1_000_000].min()), float(X[:1_000_000].max())
    assert w_after.min() >= lo - 1.0 and w_after.max() <= hi + 1.0
    assert not np.array_equal(w_before, w_after)


def test_free_running_full_size():
    """Free-running mode (the paper's races, Sec. 4.4) at the streaming workload's full size, against the
    deterministic and the silent run on the same data: no element-wise parity exists for it, so properties:
    finite states, every worker sends once per round, Eq. 8 of worker 0 and of the mean state within 2 % of
    the deterministic run's and not worse than the silent run's by more than 2 %."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[1]
    X = workloads.generate_device(wl, device="cuda:0")
    res = {}
    for name, kw in (("deterministic", dict(E=wl.E)), ("free", dict(E=wl.E, mode=B.MODE_FREE_RUNNING)), ("silent", dict(E=0))):
        g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, seed=wl.schedule_seed, **kw)
        g.load_shards(X)
        g.run_epochs(2)
        st = g.stats()
        w = g.get_state()
        assert np.all(np.isfinite(w)) and st.kernel == B.KERNEL_SMALL and st.launches == 1
        res[name] = (g.quant_error(0), g.quant_error(-1), st.sent, st.received, st.accepted, st.last_run_ms)
        print("[%s] E(w_0) %.6g  E(mean w) %.6g  sent/received/good %d/%d/%d  %.3f ms" % ((name,) + res[name]))
        g.close()
    rounds = (2 * wl.S) // wl.E
    assert res["deterministic"][2] == res["free"][2] == wl.W * rounds and res["silent"][2] == 0
    assert 0 < res["free"][3] <= res["free"][2] and 0 < res["free"][4] <= res["free"][3]
    for q in (0, 1):
        assert abs(res["free"][q] - res["deterministic"][q]) <= 0.02 * res["deterministic"][q]
        assert res["free"][q] <= 1.02 * res["silent"][q]
