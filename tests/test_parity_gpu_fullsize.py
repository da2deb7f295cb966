"""Parity at the workloads' full sizes and in the launch configuration bench.py times
(deterministic mode), against the oracle:
  - streaming workload (N = 1e8, d = 10, k = 10, W = 1024, b = 1000, E = 8): two epochs in one call (one launch), every
    assignment and every worker state;
  - wider workload (k = d = 100, W = 512, b = 2000, E = 8): two epochs in one call (one launch), all assignments and
    states;
  - contraction workload (k = 1024, d = 128, W = 256, b = 4096, E = 4): one epoch plus the first
    merge step (one launch per round), and two epochs plus a merge step in one call (one launch), all assignments
    and states;
  - HBM-scale workload (N = 2.5e9, W = 4096, E = 16; 100 GB of samples): the whole epoch, round by
    round (the oracle is fed the rows of one communication round at a time), every assignment,
    every state at every round boundary, counters, Eq. 8 at the end; then the free-running mode.
"""
import numpy as np
import pytest

from paper_1505_04956_amd import workloads
from tests.parity_rules import NEAR_TIE, check_assignments, check_counters, follow_on_bound, mismatch_shift, rel_fro

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def compare(tag, g, o, ag, ao, gap, q_per_sample, state_tol=1e-4):
    """The rules of tests/parity_rules.py at full size; mismatches are listed and counted by kind."""
    st = g.stats()
    W = o.w.shape[0]
    err = rel_fro(g.get_state(), o.w)
    print("\n[%s] %d assignments, oracle near-ties %d, Parzen near-ties %d; max state err %.3g; "
          "exact rechecks %d; messages sent/received/good %d/%d/%d (oracle %d/%d/%d); kernel %d, launches %d, %.3f ms"
          % (tag, ag.size, (gap < NEAR_TIE).sum(), o.near[1], err.max(), st.exact_rechecks, st.sent,
             st.received, st.accepted, *o.counters.sum(0), st.kernel, st.launches, st.last_run_ms))
    n_tie, n_round, n_follow = check_assignments(ag, ao, gap, follow_on_bound(err, o.w, q_per_sample))
    print("[%s] mismatches: %d at near-ties of the oracle, %d from state rounding, %d follow-on" % (tag, n_tie, n_round, n_follow))
    assert n_round <= 1 + ag.size // 10_000_000
    assert np.all(np.isfinite(g.get_state()))
    assert err.max() <= state_tol
    check_counters(g.worker_counters(), o.counters, o.parzen_near)


def run_config(oracle, wl, steps, expect_kernel, expect_launches=None, kernel=0, **exchange):
    """`exchange`: options both sides take (parts, buffers); `kernel`: the library's kernel choice (0 = its own)."""
    from paper_1505_04956_amd import binding as B
    X = workloads.generate_device(wl, device="cuda:0")
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, kernel=kernel, **exchange)
    g.load_shards(X)
    g.enable_assign_dump(steps)
    g.run_steps(steps)
    st = g.stats()
    assert st.kernel == expect_kernel
    if expect_launches is not None:
        assert st.launches == expect_launches
    ag = g.assign_dump(steps)
    oracle.set_threads(16)
    o = oracle.OracleASGD(X.cpu().numpy(), k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed, **exchange)
    ao, gap = o.run_steps(steps, dump=True)
    qg, qo = g.quant_error(0), o.quant_error(0)
    compare(wl.name + "".join(" %s=%s" % kv for kv in exchange.items()), g, o, ag, ao, gap, qo / wl.N)
    assert abs(qg - qo) <= 1e-4 * qo
    return g, o


def test_streaming_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[1]
    # what bench.py times: several epochs handed over in one call, which this kernel runs as ONE launch
    run_config(oracle, wl, 2 * wl.S, B.KERNEL_SMALL, expect_launches=1)


def test_wider_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[2]
    g, o = run_config(oracle, wl, 2 * wl.S, B.KERNEL_MFMA, expect_launches=1)     # two epochs in one call = one launch
    assert o.counters[:, 2].sum() > 0


def test_wider_workload_is_reproducible_bit_for_bit():
    """Two runs of the k = d = 100 workload in the benchmark's launch configuration (one launch, 512 co-resident
    workgroups, gradient sums added with integer atomics in whatever order the waves arrive) end in identical states
    and counters."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[2]
    X = workloads.generate_device(wl, device="cuda:0")
    out = []
    for rep in range(2):
        g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
        g.load_shards(X)
        g.run_epochs(2)
        assert g.stats().kernel == B.KERNEL_MFMA
        out.append((g.get_state().copy(), g.worker_counters().copy()))
        g.close()
    assert np.array_equal(out[0][0], out[1][0])
    assert np.array_equal(out[0][1], out[1][1])


def test_contraction_workload_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[4]
    g, o = run_config(oracle, wl, wl.S + 1, B.KERNEL_MFMA)                # the step after the epoch is a merge step
    assert o.counters[:, 1].sum() == wl.W


def test_contraction_workload_full_size_one_launch(oracle):
    """The same workload as bench.py times it: a call that covers several rounds is ONE launch of 256 co-resident
    workgroups that wait for each other's messages (two epochs and the merge step after them)."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[4]
    g, o = run_config(oracle, wl, 2 * wl.S + 1, B.KERNEL_MFMA, expect_launches=1)
    assert o.counters[:, 1].sum() == 2 * wl.W


def test_partial_messages_full_size_streaming_kernel(oracle):
    """Sec. 4.4 at full size: messages of one part in five of the rows (two centroid rows each), two buffers, on the
    streaming workload with the kernel the library chooses there; one epoch, every assignment, state and counter."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[1]
    g, o = run_config(oracle, wl, wl.S, B.KERNEL_SMALL, expect_launches=1, parts=5, buffers=2)
    assert o.counters[:, 2].sum() > 0


def test_partial_messages_full_size_wider_workload(oracle):
    """Sec. 4.4 on the k = d = 100 workload at full size (W = 512, 25 rows per message), on the shape-agnostic kernel -
    the matrix-core kernel refuses partial messages for states of this size."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[2]
    g, o = run_config(oracle, wl, wl.S, B.KERNEL_GENERIC, kernel=B.KERNEL_GENERIC, parts=4)
    assert o.counters[:, 2].sum() > 0


def test_partial_messages_full_size_contraction_workload(oracle):
    """Sec. 4.4 where the paper wants it, on the largest state (k = 1024, d = 128: 512 KB per full message, 64 centroid
    rows per partial one with P = 16): one epoch plus the merge step after it, shape-agnostic kernel."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[4]
    g, o = run_config(oracle, wl, wl.S + 1, B.KERNEL_GENERIC, kernel=B.KERNEL_GENERIC, parts=16)
    assert o.counters[:, 1].sum() > 0


@pytest.mark.skip(reason="partial messages (Sec. 4.4) on the matrix-core kernel at full size: the only batch of such runs "
                         "(k = d = 100 and k = 1024, d = 128 workloads, P = 1/4/16, also with 4 buffers) ended with the GPU box "
                         "reporting a fault or a hung queue; its log was lost with the box and no cause was found by reading "
                         "the code, so the case is not run again and the library refuses the combination above the tested sizes")
def test_partial_messages_matrix_core_full_size(oracle):
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[2]
    X = workloads.generate_device(wl, device="cuda:0")
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, parts=4, kernel=B.KERNEL_MFMA)
    g.load_shards(X)
    g.enable_assign_dump(wl.S)
    g.run_steps(wl.S)
    ag = g.assign_dump(wl.S)
    o = oracle.OracleASGD(X.cpu().numpy(), k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed, parts=4)
    ao, gap = o.run_steps(wl.S, dump=True)
    compare(wl.name + " parts=4", g, o, ag, ao, gap, o.quant_error(0) / wl.N)


def test_hbm_scale_workload(oracle):
    """The 100 GB workload, the WHOLE epoch against the oracle: the samples stay on the device, the oracle is fed one
    communication round at a time (the rows those 16 steps touch, copied shard by shard), and after every round all
    assignments of the round, all worker states and the message counters are compared; Eq. 8 of the final state is
    summed by the oracle over chunks of the samples.  Then the same epoch as ONE launch (what the benchmark times) must
    give the same states bit for bit, and the free-running mode (the workload names both) is checked on properties."""
    import time
    import torch
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[3]
    free, total = torch.cuda.mem_get_info()
    if free < 115e9:
        pytest.skip("needs 115 GB of free device memory, have %.0f GB" % (free / 1e9))
    t_begin = time.time()
    X = workloads.generate_device(wl, device="cuda:0")                   # 100 GB
    shards = X[:wl.W * wl.H].view(wl.W, wl.H, wl.d)
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
    g.load_shards(X)
    oracle.set_threads(16)
    o = None
    err_max = q_typ = None
    flipped = set()
    n_round = over = 0
    shift = np.zeros(wl.W)
    n_tie = n_follow = near = 0
    worst = 0.0
    t = 0
    g.enable_assign_dump(wl.E)
    while t < wl.S:
        n = min(wl.E, wl.S - t)                                           # 38 rounds of 16 steps, then 2 steps
        g.run_steps(n)
        assert g.stats().kernel == B.KERNEL_SMALL and g.stats().launches == 1
        ag = g.assign_dump(n)
        Xw = shards[:, t * wl.b:(t + n) * wl.b, :].contiguous().cpu().numpy().reshape(wl.W * n * wl.b, wl.d)
        if o is None:
            o = oracle.OracleASGD(Xw, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
        else:
            o.set_window(Xw, t)
        ao, gap = o.run_steps(n, dump=True)
        err = rel_fro(g.get_state(), o.w)
        err_max = err if err_max is None else np.maximum(err_max, err)
        if q_typ is None:
            q_typ = oracle.quant_error(Xw, o.w[0]) / Xw.shape[0]           # Eq. 8 per sample, from the rows of the first round
        a, r_, f_ = check_assignments(ag, ao, gap, follow_on_bound(err_max, o.w, q_typ), verbose=False, flipped=flipped)
        n_round += r_
        n_tie += a; n_follow += f_; near += int((gap < NEAR_TIE).sum())
        worst = max(worst, float(err.max()))
        # a worker's state may be off by 1e-4 plus what its counted assignment mismatches explain
        shift += mismatch_shift(ag, ao, Xw.reshape(wl.W, n * wl.b, wl.d), o.w, wl.lr, wl.b)
        allowed = 1e-4 + shift / np.linalg.norm(o.w.reshape(wl.W, -1), axis=1)
        if not (np.all(np.isfinite(err)) and np.all(err <= allowed)):
            for i_ in np.nonzero(~(err <= allowed))[0][:10]:
                print("   step %d worker %d: state error %.3g > %.3g" % (t + n, i_, err[i_], allowed[i_]))
        assert np.all(np.isfinite(err)) and np.all(err <= allowed), (t, err.max())
        over = max(over, int((err > 1e-4).sum()))
        check_counters(g.worker_counters(), o.counters, o.parzen_near)
        t += n
    g.disable_assign_dump()
    st = g.stats()
    rounds = wl.S // wl.E
    assert st.steps == wl.S and int(o.t[0]) == wl.S
    assert st.sent == wl.W * rounds and st.received == wl.W * ((wl.S - 1) // wl.E) and 0 < st.accepted <= st.received
    # Eq. 8 of worker 0's final state over all N rows: the oracle sums it chunk by chunk
    qo = 0.0
    chunk = 50_000_000
    for lo in range(0, wl.N, chunk):
        qo += oracle.quant_error(X[lo:lo + chunk].cpu().numpy(), o.w[0])
    qg = g.quant_error(0)
    print("\n[%s whole epoch] %d assignments: %d mismatches at near-ties of the oracle (%d near-ties), %d from state rounding, %d follow-on; worst "
          "state error at a round boundary %.3g; Parzen near-ties %d; messages sent/received/good %d/%d/%d (oracle %d/%d/%d); "
          "workers above 1e-4 at some boundary (explained by their mismatches): %d; E(w_0) gpu %.8g oracle %.8g; %.0f s"
          % (wl.name, wl.S * wl.W * wl.b, n_tie, near, n_round, n_follow, worst, o.near[1], st.sent, st.received, st.accepted,
             *o.counters.sum(0), over, qg, qo, time.time() - t_begin))
    assert abs(qg - qo) <= 1e-4 * qo
    assert n_round <= 1 + (wl.S * wl.W * wl.b) // 10_000_000
    w_rounds = g.get_state()
    g.close()
    # --- the same epoch as one launch, as the benchmark runs it: bit for bit the same ---
    one = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
    one.load_shards(X)
    one.run_epochs(1)
    s1 = one.stats()
    assert s1.launches == 1 and s1.steps == wl.S
    assert np.array_equal(one.get_state(), w_rounds)
    assert [s1.sent, s1.received, s1.accepted] == [st.sent, st.received, st.accepted]
    print("[%s] one launch: %.3f ms (%.3g samples/s)" % (wl.name, s1.last_run_ms, wl.processed_per_epoch / s1.last_run_ms * 1e3))
    one.close()
    # --- free-running mode (no element-wise parity exists for it): properties, and Eq. 8 close to the deterministic run's ---
    fr = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, mode=B.MODE_FREE_RUNNING)
    fr.load_shards(X)
    fr.run_epochs(1)
    sf = fr.stats()
    wf = fr.get_state()
    qf = fr.quant_error(0)
    print("[%s free-running] %.3f ms; E(w_0) %.8g (deterministic %.8g); sent/received/good %d/%d/%d"
          % (wl.name, sf.last_run_ms, qf, qg, sf.sent, sf.received, sf.accepted))
    assert np.all(np.isfinite(wf)) and sf.kernel == B.KERNEL_SMALL and sf.launches == 1
    assert sf.sent == wl.W * rounds and 0 < sf.received <= sf.sent and 0 < sf.accepted <= sf.received
    assert abs(qf - qg) <= 0.02 * qg
    fr.close()


@pytest.mark.parametrize("config", [1, 2, 4])
def test_free_running_full_size(config):
    """Free-running mode (the paper's races, Sec. 4.4) at full size on the streaming, the wider and the contraction
    workload, over three schedule seeds, against the deterministic and the silent run on the same data: no element-wise
    parity exists for it, so properties: finite states, every worker sends once per round, nobody receives more than
    was sent, Eq. 8 of worker 0 within 3 % of the deterministic run's and not worse than the silent run's by more
    than 3 %.  Prints the kernel time per epoch of the three modes (the cost of the exchange)."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[config]
    X = workloads.generate_device(wl, device="cuda:0")
    kernel = B.KERNEL_SMALL if config == 1 else B.KERNEL_MFMA
    silent = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=0)
    silent.load_shards(X)
    silent.run_epochs(2)
    qs, ms_s = silent.quant_error(0), silent.stats().last_run_ms
    assert silent.stats().sent == 0 and silent.stats().kernel == kernel
    silent.close()
    rounds = (2 * wl.S) // wl.E
    for seed in (1, 2, 3):
        res = {}
        for name, mode in (("deterministic", B.MODE_DETERMINISTIC), ("free", B.MODE_FREE_RUNNING)):
            g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=seed, mode=mode)
            g.load_shards(X)
            g.run_epochs(2)
            st = g.stats()
            assert np.all(np.isfinite(g.get_state())) and st.kernel == kernel
            res[name] = (g.quant_error(0), st.sent, st.received, st.accepted, st.last_run_ms)
            g.close()
        qd, qf = res["deterministic"][0], res["free"][0]
        print("[%s seed %d] E(w_0): deterministic %.6g free %.6g silent %.6g; free sent/received/good %d/%d/%d; "
              "ms per 2 epochs: deterministic %.3f free %.3f silent %.3f"
              % (wl.name, seed, qd, qf, qs, *res["free"][1:4], res["deterministic"][4], res["free"][4], ms_s))
        assert res["deterministic"][1] == res["free"][1] == wl.W * rounds
        assert res["deterministic"][2] == wl.W * ((2 * wl.S - 1) // wl.E)
        assert 0 < res["free"][2] <= res["free"][1] and 0 < res["free"][3] <= res["free"][2]
        assert abs(qf - qd) <= 0.03 * qd
        assert qf <= 1.03 * qs


def test_convergence_curves_match_the_oracle(oracle):
    """The convergence table of the tiny workload (Eq. 8 per sample and the error against the generating centres
    after every epoch: the shape of the paper's convergence figures, Sec. 5.4) from the HIP path and from the oracle."""
    from paper_1505_04956_amd import binding as B
    wl = workloads.CONFIGS[0]
    X = workloads.generate_host(wl)
    centres, _ = workloads.mixture_parameters(wl)
    import torch
    g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed)
    g.load_shards(torch.from_numpy(X).to("cuda:0"))
    o = oracle.OracleASGD(X, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    for ep in range(1, wl.epochs + 1):
        g.run_epochs(1)
        o.run_epochs(1)
        qg, qo = g.quant_error(0) / wl.N, o.quant_error(0) / wl.N
        cg, co = workloads.centre_error(g.get_state(0), wl), oracle.centre_error(o.w[0], centres)
        print("epoch %d: E(w_0)/N gpu %.7f oracle %.7f; centre error gpu %.6f oracle %.6f" % (ep, qg, qo, cg, co))
        assert abs(qg - qo) <= 1e-4 * qo and abs(cg - co) <= 1e-4 * co
