"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  The bars (deterministic mode) are stated in tests/parity_rules.py:
assignments identical except at near-ties of the oracle (counted and printed), every worker state
and the quantization error within 1e-4 relative, message counters identical up to flagged
near-ties of Eq. 4.
"""
import numpy as np
import pytest

from paper_1505_04956_amd import workloads
from tests.parity_rules import NEAR_TIE, check_assignments, check_counters, follow_on_bound, rel_fro

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; there is no CPU fallback")
    from paper_1505_04956_amd import binding
    binding.lib()
    return binding


def to_dev(X):
    import torch
    return torch.from_numpy(X).to("cuda:0")


def make_data(N, d, k, seed=3, centres="uniform10", weights="equal", sigma=1.0):
    wl = workloads.Workload("t", N, d, k, 1, 1, 0.1, 0, 1, sigma, centres, weights, data_seed=seed)
    return workloads.generate_host(wl)


def run_both(B, oracle, X, k, W, b, lr, E, steps, seed=1, parzen=True, drop_rate=0.0, lr_mode=0,
             kernel=0, tune=0, dump=True, w0=None, check_qe=True, buffers=1, parts=1):
    """Run `steps` steps on the GPU and in the oracle; assert the bars; return both."""
    N, d = X.shape
    g = B.ASGD(k, d, W, b, lr, E=E, seed=seed, parzen=parzen, drop_rate=drop_rate, lr_mode=lr_mode,
               kernel=kernel, tune=tune, buffers=buffers, parts=parts)
    g.load_shards(to_dev(X))
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=E, seed=seed, parzen=parzen, drop_rate=drop_rate,
                          lr_mode=lr_mode, w0=w0, buffers=buffers, parts=parts)
    if w0 is not None:
        g.set_state(-1, np.asarray(w0, dtype=np.float32))
    if dump:
        g.enable_assign_dump(steps)
    g.run_steps(steps)
    od = o.run_steps(steps, dump=dump)
    wg = g.get_state()
    st = g.stats()
    n_tie = n_round = n_follow = near = 0
    err = rel_fro(wg, o.w)
    if dump:
        ag = g.assign_dump(steps)
        ao, gap = od
        near = int((gap < NEAR_TIE).sum())
        n_tie, n_round, n_follow = check_assignments(ag, ao, gap, follow_on_bound(err, o.w, o.quant_error(0) / N))
    print("\n[parity] k=%d d=%d W=%d b=%d E=%d steps=%d kernel=%d: max state err %.3g, assign mismatches %d at near-ties + %d from state rounding + %d "
          "follow-on (oracle near-ties %d, Parzen near-ties %d), rechecks %d, msgs sent/recv/good gpu %d/%d/%d oracle %d/%d/%d"
          % (k, d, W, b, E, steps, st.kernel, err.max(), n_tie, n_round, n_follow, near, o.near[1], st.exact_rechecks,
             st.sent, st.received, st.accepted, *o.counters.sum(0)))
    assert np.all(np.isfinite(wg))
    assert err.max() <= TOL
    check_counters(g.worker_counters(), o.counters, o.parzen_near)
    if check_qe:
        for wk in sorted({0, W - 1}):
            qg, qo = g.quant_error(wk), o.quant_error(wk)
            assert abs(qg - qo) <= TOL * qo, (qg, qo)
    assert st.steps == steps
    return g, o


# ----------------------------------------------------------------------------------- config 0
@pytest.mark.parametrize("kernel", [0, 1])
def test_config0_full(B, oracle, kernel):
    wl = workloads.CONFIGS[0]
    X = workloads.generate_host(wl)
    g, o = run_both(B, oracle, X, wl.k, wl.W, wl.b, wl.lr, wl.E, wl.epochs * wl.S, seed=wl.schedule_seed,
                    kernel=kernel)
    assert g.stats().kernel == (2 if kernel == 0 else 1)      # small kernel is the default for k=d=10
    assert o.counters[:, 2].sum() > 0                          # merges really happened


@pytest.mark.parametrize("tune", [1, 2, 4, 5, 6, 8, 9, 12])   # ring depths x worker shapes (waves, sharing of accumulator cells)
def test_small_kernel_variants(B, oracle, tune):
    X = make_data(8 * 4000, 10, 10, seed=5)
    run_both(B, oracle, X, 10, 8, 1000, 0.05, 2, 9, kernel=2, tune=tune)


# ------------------------------------------------------------------- shapes, tails, edge cases
@pytest.mark.parametrize("k,d,W,b,E,N", [
    (5, 7, 3, 130, 2, 3 * 1000 + 2),      # odd d, N not divisible by W, b not a multiple of 64
    (1, 4, 2, 64, 1, 2 * 640),            # k = 1, exchange after every step (Alg. 5 as printed)
    (3, 1, 5, 17, 3, 5 * 200 + 4),        # d = 1
    (16, 16, 4, 256, 4, 4 * 2048),
    (10, 10, 1, 500, 4, 5000),            # W = 1: nothing to exchange (Alg. 4)
    (70, 3, 2, 100, 2, 2 * 700),          # k > 64
    (6, 700, 2, 120, 2, 2 * 500),         # long rows: the re-decision threshold follows d (4 (d + 2) 2^-24 > 1e-5)
])
def test_generic_shapes(B, oracle, k, d, W, b, E, N):
    X = make_data(N, d, k, seed=11)
    H = N // W
    run_both(B, oracle, X, k, W, b, 0.1, E, 2 * (H // b) + 3, kernel=1)


def test_small_kernel_ragged(B, oracle):
    # b below one group of 64, b = 64 exactly, and a tail of one sample
    for b in (37, 64, 65, 200, 500, 1000):
        X = make_data(4 * 3000 + 3, 10, 10, seed=b)
        run_both(B, oracle, X, 10, 4, b, 0.05, 3, 11, kernel=2)


@pytest.mark.parametrize("b", [1, 5, 200, 1000])
@pytest.mark.parametrize("kernel,tune", [(2, 0), (2, 4), (2, 8), (1, 0)])
def test_small_kernel_column_ranges(B, oracle, kernel, tune, b):
    # The streaming kernel sums the gradient in fixed point with one power-of-two scale per column, taken from the
    # column's largest magnitude: columns of very different size, a column of zeros, a column far from the origin and
    # a column that is negative throughout each have to come out as exact as an ordinary one, whatever the mini-batch
    # size (which bounds the scale from the other side).  Every column is checked on its own: in the norm of the whole
    # state the small ones would not show.
    X = make_data(4 * 3000, 10, 10, seed=17 + b)
    X = X * np.array([1e-6, 1e-3, 1.0, 1.0, 1.0, 1.0, 1e2, 3e3, 0.0, 1.0], dtype=np.float32)
    X[:, 4] += np.float32(1000.0)
    X[:, 5] = -np.abs(X[:, 5]) - np.float32(2.0)
    X = np.ascontiguousarray(X, dtype=np.float32)
    steps = 11 if b > 5 else 60
    # (initial centroids that no mini-batch of the run contains: a worker's default start, its own first k samples,
    # makes the first mini-batches of b = 1 coincide with their centroids, G = 0 and Eq. 4 an exact tie, which the
    # fixed-point sums decide by rounding - the oracle counts those as Parzen near-ties)
    w0 = X[5000:5010].astype(np.float64)
    g, o = run_both(B, oracle, X, 10, 4, b, 0.05, 3, steps, kernel=kernel, tune=tune, check_qe=False, w0=w0)
    wg = np.asarray(g.get_state(), dtype=np.float64)
    wo = np.asarray(o.w, dtype=np.float64)
    assert np.all(wg[:, :, 8] == 0.0)
    for j in range(10):
        if j == 8:
            continue
        num = np.linalg.norm((wg - wo)[:, :, j].reshape(4, -1), axis=1)
        den = np.linalg.norm(wo[:, :, j].reshape(4, -1), axis=1)
        assert np.all(num <= TOL * den), (j, num / den)


@pytest.mark.parametrize("k,d", [(4, 4), (8, 8), (8, 16), (16, 8), (16, 12)])
@pytest.mark.parametrize("W,b,E,buffers,parts,tune", [
    (6, 200, 2, 1, 1, 0),        # two waves per worker
    (5, 130, 3, 2, 1, 8),        # one wave per worker, two buffers, ragged mini-batch
    (4, 1000, 2, 3, 2, 0),       # the streaming workload's mini-batch, three buffers, partial messages
])
def test_small_kernel_other_shapes(B, oracle, k, d, W, b, E, buffers, parts, tune):
    """The other small shapes the streaming kernel is built for (the automatic choice takes it for them too)."""
    X = make_data(W * b * 4 + 5, d, k, seed=31 + k + d)
    g, o = run_both(B, oracle, X, k, W, b, 0.05, E, 13, kernel=0, tune=tune, buffers=buffers, parts=parts)
    assert g.stats().kernel == B.KERNEL_SMALL and g.stats().launches == 1


def test_small_kernel_other_shapes_many_workers(B, oracle):
    # more workers than workgroups can be resident (one wave per SIMD for the larger of these shapes), message loss
    X = make_data(1500 * 260 + 7, 12, 16, seed=9)
    g, o = run_both(B, oracle, X, 16, 1500, 64, 0.05, 2, 7, kernel=2, drop_rate=0.25)
    assert g.stats().launches == 1


def test_more_workers_than_resident_workgroups(B, oracle):
    # a workgroup of the single-launch path then takes several workers through every round
    X = make_data(2500 * 200 + 7, 10, 10, seed=9)
    g, o = run_both(B, oracle, X, 10, 2500, 64, 0.05, 2, 7, kernel=2, drop_rate=0.25)
    assert g.stats().launches == 1


def test_single_launch_equals_one_launch_per_round(B):
    X = to_dev(make_data(16 * 4000, 10, 10, seed=12))
    res = []
    for tune in (0, 3, 4, 7):   # +3 = end every launch at a multiple of E instead of waiting inside the kernel
        g = B.ASGD(10, 10, 16, 1000, 0.05, E=2, seed=3, kernel=2, tune=tune)
        g.load_shards(X)
        g.run_steps(5)
        g.run_steps(6)
        res.append((g.get_state(), g.worker_counters(), g.stats().launches))
    for a, c in ((0, 1), (2, 3)):
        assert np.array_equal(res[a][0], res[c][0]) and np.array_equal(res[a][1], res[c][1])
        assert res[a][2] == 1 and res[c][2] > 1
    assert np.allclose(res[0][0], res[2][0], rtol=1e-5)      # one or two waves per worker: other summation order


def test_options(B, oracle):
    X = make_data(24_000, 10, 10, seed=2)
    for kernel in (1, 2):
        run_both(B, oracle, X, 10, 6, 200, 0.1, 2, 25, parzen=False, kernel=kernel)
        run_both(B, oracle, X, 10, 6, 200, 0.1, 2, 25, drop_rate=0.5, kernel=kernel)
        run_both(B, oracle, X, 10, 6, 200, 0.1, 0, 25, kernel=kernel)
    run_both(B, oracle, X, 10, 6, 200, 0.1, 0, 25, lr_mode=1, kernel=1)     # 1/count step size
    w0 = np.random.default_rng(0).uniform(0, 10, size=(10, 10))
    run_both(B, oracle, X, 10, 6, 200, 0.1, 2, 25, w0=w0.astype(np.float32).astype(np.float64))


def test_lost_messages_equal_silent_mode_bitwise(B):
    X = to_dev(make_data(24_000, 10, 10, seed=2))
    for kernel in (1, 2):
        a = B.ASGD(10, 10, 6, 200, 0.1, E=2, drop_rate=1.0, kernel=kernel); a.load_shards(X); a.run_steps(25)
        s = B.ASGD(10, 10, 6, 200, 0.1, E=0, kernel=kernel); s.load_shards(X); s.run_steps(25)
        assert np.array_equal(a.get_state(), s.get_state())
        assert a.stats().sent == 6 * 12 and a.stats().received == 0


def test_reproducible_and_resumable(B):
    X = to_dev(make_data(24_000, 10, 10, seed=4))
    for kernel in (1, 2):
        kw = dict(E=3, seed=8, kernel=kernel)
        full = B.ASGD(10, 10, 6, 200, 0.1, **kw); full.load_shards(X); full.run_steps(40)
        again = B.ASGD(10, 10, 6, 200, 0.1, **kw); again.load_shards(X); again.run_steps(40)
        assert np.array_equal(full.get_state(), again.get_state())          # bit for bit
        a = B.ASGD(10, 10, 6, 200, 0.1, **kw); a.load_shards(X); a.run_steps(10); a.run_steps(7)
        c = B.ASGD(10, 10, 6, 200, 0.1, **kw); c.load_shards(X)
        c.set_state(-2, a.get_state()); c.set_step(17)                      # 17 is not a merge point
        c.run_steps(23)
        assert np.array_equal(full.get_state(), c.get_state())


def test_wider_shapes_generic(B, oracle):
    # scaled-down relatives of the k=d=100 and the k=1024, d=128 workloads
    X = make_data(4 * 2000 * 3, 100, 100, seed=6, weights="zipf1.1")
    run_both(B, oracle, X, 100, 4, 2000, 0.02, 2, 7, kernel=1)
    X = make_data(2 * 4096 * 2, 128, 1024, seed=7, centres="sphere10")
    run_both(B, oracle, X, 1024, 2, 4096, 0.01, 2, 4, kernel=1)


@pytest.mark.parametrize("k,d,W,b,E,steps,N,centres,weights", [
    (100, 100, 4, 2000, 2, 7, 4 * 2000 * 3, "uniform10", "zipf1.1"),     # relative of the k = d = 100 workload
    (1024, 128, 2, 4096, 2, 4, 2 * 4096 * 2, "sphere10", "equal"),      # relative of the k = 1024, d = 128 workload
    (70, 8, 3, 100, 2, 9, 3 * 450 + 2, "uniform10", "equal"),           # b below one tile, k not a multiple of 32
    (33, 36, 5, 300, 3, 8, 5 * 1000 + 3, "uniform10", "equal"),         # ragged last tile, odd row length of W'
    (2, 4, 2, 129, 1, 6, 2 * 400, "uniform10", "equal"),                # smallest k and d
    (128, 64, 2, 256, 1, 5, 2 * 1024, "uniform10", "equal"),            # exact multiples of all tile sizes
    (64, 32, 3, 1024, 2, 6, 3 * 1024 * 2 + 5, "uniform10", "zipf1.1"),  # skewed cluster sizes, big and small ones in one gather
    (3, 16, 2, 500, 2, 5, 2 * 1000, "uniform10", "zipf1.1"),            # fewer centroids than half-waves
    (2048, 16, 2, 2304, 1, 3, 2 * 2304 * 2, "uniform10", "equal"),      # many centroids: the sort uses fewer shares than waves
    (104, 40, 2, 512, 1, 5, 2 * 1024, "uniform10", "equal"),            # last 32 rows hold 8 centroids: two groups of 4x4 tiles
    (37, 12, 3, 300, 2, 7, 3 * 900 + 2, "uniform10", "zipf1.1"),        # ... 5 centroids: the second group is partly padding
])
def test_matrix_core_kernel(B, oracle, k, d, W, b, E, steps, N, centres, weights):
    X = make_data(N, d, k, seed=21, centres=centres, weights=weights)
    g, o = run_both(B, oracle, X, k, W, b, 0.02, E, steps, kernel=3)
    assert g.stats().kernel == 3


@pytest.mark.parametrize("k,d,W,b,E,steps,N", [
    (100, 100, 4, 2000, 2, 7, 4 * 2000 * 3),
    (33, 36, 5, 300, 3, 8, 5 * 1000 + 3),
    (70, 8, 3, 100, 2, 9, 3 * 450 + 2),
    (64, 32, 3, 1024, 2, 6, 3 * 1024 * 2 + 5),
    (38, 24, 3, 200, 2, 7, 3 * 200 * 3 + 1),
])
@pytest.mark.parametrize("tune", [2, 66, 130, 258])
def test_matrix_core_kernel_four_waves(B, oracle, k, d, W, b, E, steps, N, tune):
    # the variant with four waves per worker (two workers per CU), which large W selects by itself: the samples of the
    # next tile are fetched a whole tile ahead into a second set of registers and the gradient sums are formed in fixed
    # point in a second pass over the mini-batch; +128: counting sort and gather instead (fp32 sums in sample order);
    # +64: also one set of registers (same arithmetic and order as +128); +256: no 4x4 tiles for a last half-block of
    # at most 8 centroids
    X = make_data(N, d, k, seed=23)
    g, o = run_both(B, oracle, X, k, W, b, 0.02, E, steps, kernel=3, tune=tune)
    assert g.stats().kernel == 3
    if tune == 66:
        plain = B.ASGD(k, d, W, b, 0.02, E=E, kernel=3, tune=130); plain.load_shards(to_dev(X)); plain.run_steps(steps)
        assert np.array_equal(g.get_state(), plain.get_state())


@pytest.mark.parametrize("k,d,W,b,E,steps,N,weights,buffers,parts,drop", [
    (100, 100, 4, 2000, 2, 7, 4 * 2000 * 3, "zipf1.1", 1, 1, 0.0),       # relative of the k = d = 100 workload
    (33, 36, 5, 300, 3, 8, 5 * 1000 + 3, "equal", 1, 1, 0.0),            # ragged last tile, odd row length
    (70, 8, 3, 100, 2, 9, 3 * 450 + 2, "equal", 1, 1, 0.3),              # b below one tile, small clusters
    (2, 4, 2, 129, 1, 6, 2 * 400, "equal", 1, 1, 0.0),                   # smallest k and d: one half-wave holds the row
    (128, 64, 2, 256, 1, 5, 2 * 1024, "equal", 1, 1, 0.0),               # exact multiples of all tile sizes
    (64, 32, 3, 1024, 2, 6, 3 * 1024 * 2 + 5, "zipf1.1", 2, 1, 0.0),     # skewed cluster sizes: many lanes add to one row
    (40, 20, 12, 100, 2, 17, 12 * 1800 + 7, "equal", 2, 4, 0.0),         # with partial messages and two buffers
])
@pytest.mark.parametrize("tune", [32, 2])
def test_matrix_core_kernel_fused_sums(B, oracle, k, d, W, b, E, steps, N, weights, buffers, parts, drop, tune):
    """The variants with gradient sums in fixed point, asked for with their tune bits: 32 forms them tile by tile (no
    second read of the mini-batch), 2 (four waves) in a second pass over the mini-batch in memory order, in the LDS
    the state rows no longer need; against the oracle, and bit for bit against itself (run twice, run in pieces) -
    integer sums do not depend on the order in which the waves get there."""
    X = make_data(N, d, k, seed=29, weights=weights)
    g, o = run_both(B, oracle, X, k, W, b, 0.02, E, steps, kernel=3, tune=tune, buffers=buffers, parts=parts, drop_rate=drop)
    assert g.stats().kernel == 3
    Xg = to_dev(X)
    kw = dict(E=E, kernel=3, tune=tune, buffers=buffers, parts=parts, drop_rate=drop)
    again = B.ASGD(k, d, W, b, 0.02, **kw); again.load_shards(Xg); again.run_steps(2); again.run_steps(steps - 2)
    assert np.array_equal(g.get_state(), again.get_state())
    assert np.array_equal(g.worker_counters(), again.worker_counters())


@pytest.mark.parametrize("b", [7, 100, 600])
@pytest.mark.parametrize("tune", [2, 32, 0])
def test_matrix_core_kernel_column_ranges(B, oracle, tune, b):
    # like test_small_kernel_column_ranges, for the variants of the matrix-core kernel with fixed-point gradient sums
    # (2: second pass, 32: tile by tile) and the one that sums in fp32 (0, eight waves): columns of very different
    # size, a zero column, a column far from the origin, a negative one; every column checked on its own
    k, d, W = 40, 20, 4
    X = make_data(W * 3000, d, k, seed=31 + b)
    scale = np.ones(d, dtype=np.float32)
    scale[[0, 1, 6, 7, 8, 13]] = [1e-6, 1e-3, 1e2, 3e3, 0.0, 1e-2]
    X = X * scale
    X[:, 4] += np.float32(1000.0)
    X[:, 5] = -np.abs(X[:, 5]) - np.float32(2.0)
    X = np.ascontiguousarray(X, dtype=np.float32)
    w0 = X[5000:5000 + k].astype(np.float64)
    g, o = run_both(B, oracle, X, k, W, b, 0.05, 3, 11 if b > 7 else 40, kernel=3, tune=tune, check_qe=False, w0=w0)
    assert g.stats().kernel == 3
    wg = np.asarray(g.get_state(), dtype=np.float64)
    wo = np.asarray(o.w, dtype=np.float64)
    assert np.all(wg[:, :, 8] == 0.0)
    for j in range(d):
        if j == 8:
            continue
        num = np.linalg.norm((wg - wo)[:, :, j].reshape(W, -1), axis=1)
        den = np.linalg.norm(wo[:, :, j].reshape(W, -1), axis=1)
        assert np.all(num <= TOL * den), (j, num / den)


@pytest.mark.parametrize("k,d", [(12, 8), (5, 4), (20, 32)])
def test_automatic_choice_prefers_the_matrix_core_kernel(B, oracle, k, d):
    # shapes the streaming kernel is not built for, with rows the matrix-core kernel can take (d % 4 = 0)
    X = make_data(4 * 900 + 3, d, k, seed=44)
    g, o = run_both(B, oracle, X, k, 4, 150, 0.05, 2, 9)
    assert g.stats().kernel == B.KERNEL_MFMA
    Xo = make_data(4 * 900 + 3, d + 1, k, seed=45)                      # odd row length: the shape-agnostic kernel
    g, o = run_both(B, oracle, Xo, k, 4, 150, 0.05, 2, 9)
    assert g.stats().kernel == B.KERNEL_GENERIC


def test_matrix_core_kernel_options(B, oracle):
    X = make_data(6 * 1200, 20, 40, seed=22)
    run_both(B, oracle, X, 40, 6, 200, 0.05, 2, 11, parzen=False, kernel=3)
    run_both(B, oracle, X, 40, 6, 200, 0.05, 2, 11, drop_rate=0.5, kernel=3)
    run_both(B, oracle, X, 40, 6, 200, 0.05, 0, 11, kernel=3)
    g, o = run_both(B, oracle, X, 40, 6, 200, 0.05, 2, 11)            # chosen automatically for this shape
    assert g.stats().kernel == 3
    # duplicated samples give exact ties between centroids started from them: lowest index wins on both sides
    Xd = X.copy()
    Xd[1] = Xd[0]
    Xd[1200 + 3] = Xd[1200]
    run_both(B, oracle, Xd, 40, 6, 200, 0.05, 2, 6, kernel=3)
    # same run twice: bit for bit; lost messages: same as silent
    Xg = to_dev(X)
    a = B.ASGD(40, 20, 6, 200, 0.05, E=2, kernel=3); a.load_shards(Xg); a.run_steps(11)
    c = B.ASGD(40, 20, 6, 200, 0.05, E=2, kernel=3); c.load_shards(Xg); c.run_steps(4); c.run_steps(7)
    assert np.array_equal(a.get_state(), c.get_state())
    lost = B.ASGD(40, 20, 6, 200, 0.05, E=2, drop_rate=1.0, kernel=3); lost.load_shards(Xg); lost.run_steps(11)
    sil = B.ASGD(40, 20, 6, 200, 0.05, E=0, kernel=3); sil.load_shards(Xg); sil.run_steps(11)
    assert np.array_equal(lost.get_state(), sil.get_state())
    with pytest.raises(B.AsgdError):
        bad = B.ASGD(40, 18, 6, 200, 0.05, kernel=3)                   # d must be a multiple of 4
        bad.load_shards(to_dev(make_data(6 * 1200, 18, 40)))
        bad.run_steps(1)


@pytest.mark.parametrize("tune", [2, 8])
def test_matrix_core_kernel_one_launch(B, oracle, tune):
    """Deterministic mode as ONE launch whose workgroups wait for each other's messages (four waves per worker:
    the default there; eight waves: forced by the tune bit), against the oracle and, bit for bit, against one launch
    per round; with lost messages, and continued in the middle of a round."""
    X = make_data(12 * 900 + 5, 20, 40, seed=27)
    for drop in (0.0, 0.4):
        g, o = run_both(B, oracle, X, 40, 12, 100, 0.05, 2, 17, drop_rate=drop, kernel=3, tune=tune)
        assert g.stats().kernel == 3 and g.stats().launches == 1
        Xg = to_dev(X)
        per_round = B.ASGD(40, 20, 12, 100, 0.05, E=2, drop_rate=drop, kernel=3, tune=(tune & 2) | 4)
        per_round.load_shards(Xg); per_round.run_steps(17)
        assert per_round.stats().launches == 9
        assert np.array_equal(g.get_state(), per_round.get_state())
        assert np.array_equal(g.worker_counters(), per_round.worker_counters())
        parts = B.ASGD(40, 20, 12, 100, 0.05, E=2, drop_rate=drop, kernel=3, tune=tune)
        parts.load_shards(Xg); parts.run_steps(5); parts.run_steps(1); parts.run_steps(11)
        assert np.array_equal(g.get_state(), parts.get_state())


@pytest.mark.parametrize("kernel,tune,k,d,W,b,E,steps,buffers,parzen,drop", [
    (1, 0, 10, 10, 6, 100, 2, 13, 2, True, 0.0),        # generic kernel
    (2, 0, 10, 10, 6, 100, 2, 13, 2, True, 0.0),        # small-state kernel, two waves per worker, one launch
    (2, 0, 10, 10, 9, 500, 1, 12, 4, True, 0.3),
    (2, 0, 10, 10, 7, 130, 3, 14, 3, False, 0.0),
    (2, 8, 10, 10, 6, 100, 2, 13, 2, True, 0.2),        # one wave per worker, shared accumulator cells
    (2, 3, 10, 10, 6, 256, 2, 13, 4, True, 0.0),        # one launch per round
    (1, 0, 7, 5, 5, 64, 1, 9, 4, True, 0.3),
    (1, 0, 12, 9, 6, 50, 3, 14, 3, False, 0.0),
    (3, 2, 40, 20, 12, 100, 2, 17, 2, True, 0.0),       # four waves, one launch
    (3, 2, 40, 20, 12, 100, 2, 17, 4, True, 0.4),
    (3, 6, 40, 20, 12, 100, 2, 17, 3, False, 0.0),      # four waves, one launch per round
    (3, 8, 40, 20, 12, 100, 3, 17, 3, True, 0.2),       # eight waves, one launch
    (3, 0, 70, 36, 5, 300, 2, 9, 4, True, 0.0),         # eight waves, one launch per round
])
def test_n_external_buffers(B, oracle, kernel, tune, k, d, W, b, E, steps, buffers, parzen, drop):
    """Eq. 3 / Eq. 6: N buffers per worker, N recipients per message."""
    X = make_data(W * (steps + 1) * b + 7, d, k, seed=31)
    g, o = run_both(B, oracle, X, k, W, b, 0.05, E, steps, kernel=kernel, tune=tune, buffers=buffers, parzen=parzen,
                    drop_rate=drop)
    assert g.stats().kernel == kernel
    assert o.counters[:, 1].sum() > W                          # several buffers were looked at per merge point
    if parzen and drop == 0.0:
        assert 0 < o.counters[:, 2].sum()


@pytest.mark.parametrize("kernel,tune,k,d,W,b,E,steps,buffers,parts,parzen,drop", [
    (1, 0, 10, 10, 6, 100, 2, 13, 1, 2, True, 0.0),
    (2, 0, 10, 10, 6, 100, 2, 13, 1, 2, True, 0.0),      # small-state kernel, two waves per worker, one launch
    (2, 0, 10, 10, 9, 500, 1, 12, 3, 10, True, 0.3),     # one row per message
    (2, 0, 10, 10, 7, 130, 3, 14, 2, 3, False, 0.0),
    (2, 8, 10, 10, 6, 100, 2, 13, 4, 5, True, 0.2),      # one wave per worker, shared accumulator cells
    (2, 3, 10, 10, 6, 256, 2, 13, 2, 4, True, 0.0),      # one launch per round
    (1, 0, 7, 5, 5, 64, 1, 9, 3, 7, True, 0.3),          # one row per message
    (1, 0, 12, 9, 6, 50, 3, 14, 2, 5, False, 0.0),
    (1, 0, 6, 70, 4, 50, 2, 7, 2, 3, True, 0.0),         # rows longer than a wave
    (3, 2, 40, 20, 12, 100, 2, 17, 1, 4, True, 0.0),     # four waves, one launch
    (3, 2, 40, 20, 12, 100, 1, 12, 3, 3, True, 0.4),
    (3, 6, 40, 20, 12, 100, 2, 17, 2, 8, False, 0.0),    # four waves, one launch per round
    (3, 8, 40, 20, 12, 100, 3, 17, 2, 40, True, 0.0),    # eight waves, one launch
    (3, 0, 70, 36, 5, 300, 2, 9, 4, 6, True, 0.0),       # eight waves, one launch per round
    (3, 0, 100, 100, 4, 2000, 2, 7, 1, 3, True, 0.0),    # two columns of lanes per row
])
def test_partial_messages(B, oracle, kernel, tune, k, d, W, b, E, steps, buffers, parts, parzen, drop):
    """Sec. 4.4: a copy carries the centroid rows of one part; lambda, Eq. 4 and Eq. 6 row by row."""
    X = make_data(W * (steps + 1) * b + 7, d, k, seed=37)
    g, o = run_both(B, oracle, X, k, W, b, 0.05, E, steps, kernel=kernel, tune=tune, buffers=buffers, parts=parts,
                    parzen=parzen, drop_rate=drop)
    assert g.stats().kernel == kernel
    assert o.counters[:, 1].sum() > 0 and o.counters[:, 2].sum() > 0


def test_partial_messages_options(B):
    X = make_data(6 * 1500, 10, 10, seed=33)
    Xg = to_dev(X)
    auto = B.ASGD(10, 10, 6, 100, 0.05, E=2, parts=2); auto.load_shards(Xg); auto.run_steps(5)
    assert auto.stats().kernel == B.KERNEL_SMALL and auto.stats().launches == 1
    with pytest.raises(B.AsgdError):
        auto.set_option(B.OPT_PARTS, 5)                         # not after the first step
    for bad in (0, 11, 2.5):
        with pytest.raises(B.AsgdError):
            B.ASGD(10, 10, 6, 100, 0.05, E=2, parts=bad)
    # free-running mode of the small-state kernel with partial messages: finite, every worker sends, rows arrive
    fs = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=2, parts=5, mode=B.MODE_FREE_RUNNING); fs.load_shards(Xg); fs.run_steps(15)
    assert np.all(np.isfinite(fs.get_state())) and fs.stats().sent == 6 * 7 and 0 < fs.stats().received <= 2 * fs.stats().sent
    # one part set explicitly is the default
    a = B.ASGD(10, 10, 6, 100, 0.05, E=2, parts=1); a.load_shards(Xg); a.run_steps(9)
    c = B.ASGD(10, 10, 6, 100, 0.05, E=2); c.load_shards(Xg); c.run_steps(9)
    assert a.stats().kernel == B.KERNEL_SMALL and np.array_equal(a.get_state(), c.get_state())
    # continued in the middle of a round: bit for bit; free-running mode: finite, messages arrive
    Xm = to_dev(make_data(12 * 1500, 20, 40, seed=34))
    e = B.ASGD(40, 20, 12, 100, 0.05, E=2, buffers=2, parts=4, kernel=3); e.load_shards(Xm); e.run_steps(9)
    f = B.ASGD(40, 20, 12, 100, 0.05, E=2, buffers=2, parts=4, kernel=3); f.load_shards(Xm); f.run_steps(4); f.run_steps(5)
    assert np.array_equal(e.get_state(), f.get_state())
    fr = B.ASGD(40, 20, 12, 100, 0.05, E=2, buffers=2, parts=4, mode=B.MODE_FREE_RUNNING, kernel=3)
    fr.load_shards(Xm); fr.run_steps(15)
    st = fr.stats()
    assert np.all(np.isfinite(fr.get_state())) and st.sent == 12 * 7 and 0 < st.received <= 2 * st.sent


def test_partial_messages_size_limit_of_the_matrix_core_kernel(B, oracle):
    """Above W*k*d = 2^18 the matrix-core kernel refuses partial messages (its full-size runs of that combination are
    not covered by any test: the one batch of them ended in an unexplained device fault); the automatic choice takes the
    shape-agnostic kernel there, with the same results."""
    k, d, W, b = 64, 32, 129, 64                        # 129 * 2048 = 264 192 state elements
    X = make_data(W * b * 4 + 5, d, k, seed=39)
    g, o = run_both(B, oracle, X, k, W, b, 0.05, 2, 5, parts=4, dump=False, check_qe=False)
    assert g.stats().kernel == B.KERNEL_GENERIC
    forced = B.ASGD(k, d, W, b, 0.05, E=2, parts=4, kernel=B.KERNEL_MFMA)
    forced.load_shards(to_dev(X))
    with pytest.raises(B.AsgdError) as e:
        forced.run_steps(1)
    assert e.value.code == B.EINVAL
    whole = B.ASGD(k, d, W, b, 0.05, E=2, kernel=B.KERNEL_MFMA)         # whole messages: no limit
    whole.load_shards(to_dev(X)); whole.run_steps(5)
    assert whole.stats().kernel == B.KERNEL_MFMA


def test_n_external_buffers_options(B, oracle):
    X = make_data(6 * 1500, 10, 10, seed=33)
    Xg = to_dev(X)
    auto = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=2); auto.load_shards(Xg); auto.run_steps(5)
    assert auto.stats().kernel == B.KERNEL_SMALL and auto.stats().launches == 1
    with pytest.raises(B.AsgdError):
        auto.set_option(B.OPT_BUFFERS, 3)                       # not after the first step
    with pytest.raises(B.AsgdError):
        many = B.ASGD(10, 10, 3, 100, 0.05, E=2, buffers=3); many.load_shards(Xg); many.run_steps(1)   # needs N < W
    with pytest.raises(B.AsgdError):
        B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=5)
    # set after load_shards but before the first step: same as set at creation
    late = B.ASGD(10, 10, 6, 100, 0.05, E=2); late.load_shards(Xg)
    late.set_option(B.OPT_BUFFERS, 3); late.set_option(B.OPT_PARTS, 2); late.run_steps(9)
    early = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=3, parts=2); early.load_shards(Xg); early.run_steps(9)
    assert np.array_equal(late.get_state(), early.get_state()) and late.stats().received == early.stats().received > 0
    # one buffer set explicitly is the default; same run twice with three buffers: bit for bit
    a = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=1); a.load_shards(Xg); a.run_steps(9)
    c = B.ASGD(10, 10, 6, 100, 0.05, E=2); c.load_shards(Xg); c.run_steps(9)
    assert a.stats().kernel == B.KERNEL_SMALL and np.array_equal(a.get_state(), c.get_state())
    e = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=3); e.load_shards(Xg); e.run_steps(9)
    f = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=3); f.load_shards(Xg); f.run_steps(4); f.run_steps(5)
    assert np.array_equal(e.get_state(), f.get_state())
    assert e.stats().sent == 6 * 4 and e.stats().received == 6 * 4 * 3 and e.stats().kernel == B.KERNEL_SMALL
    # free-running mode of the small-state kernel with three buffers
    fs = B.ASGD(10, 10, 6, 100, 0.05, E=2, buffers=3, mode=B.MODE_FREE_RUNNING); fs.load_shards(Xg); fs.run_steps(15)
    assert np.all(np.isfinite(fs.get_state())) and fs.stats().sent == 6 * 7 and 0 < fs.stats().received <= 3 * fs.stats().sent
    # free-running mode: no element-wise parity; finite, every worker sends, some messages arrive
    fr = B.ASGD(40, 20, 12, 100, 0.05, E=2, buffers=3, mode=B.MODE_FREE_RUNNING, kernel=3)
    Xm = to_dev(make_data(12 * 1500, 20, 40, seed=34))
    fr.load_shards(Xm); fr.run_steps(15)
    st = fr.stats()
    assert np.all(np.isfinite(fr.get_state())) and st.sent == 12 * 7 and 0 < st.received <= 3 * st.sent


def test_stored_values_of_tiny_workload(B):
    """GPU path against the values the oracle wrote to tests/golden/cfg0_oracle.json."""
    import json
    import os
    stored = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg0_oracle.json")))
    wl = workloads.CONFIGS[0]
    X = workloads.generate_host(wl)
    for kernel in (0, 1):
        g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, kernel=kernel)
        g.load_shards(to_dev(X))
        qe = [g.quant_error(0)]
        for _ in range(wl.epochs):
            g.run_epochs(1)
            qe.append(g.quant_error(0))
        assert np.allclose(qe, stored["quant_error_worker0_by_epoch"], rtol=TOL, atol=0)
        st = g.stats()
        assert [st.sent, st.received, st.accepted] == stored["counters_sent_received_accepted"]
        w = g.get_state()
        assert np.allclose(w[0, 0], stored["state_worker0_row0"], rtol=TOL)
        assert np.allclose(w.reshape(wl.W, -1).sum(1), stored["state_sum_by_worker"], rtol=TOL)
        assert abs(g.quant_error(-1) - stored["quant_error_mean_state"]) <= TOL * stored["quant_error_mean_state"]
        assert [B.asgd_schedule_peer(wl.schedule_seed, 0, i, wl.W) for i in range(wl.W)] == stored["peers_round0"]
    for name, sv in stored["variants_after_3_epochs"].items():       # N external buffers, partial messages
        g = B.ASGD(wl.k, wl.d, wl.W, wl.b, wl.lr, E=wl.E, seed=wl.schedule_seed, **sv["options"])
        g.load_shards(to_dev(X))
        g.run_epochs(3)
        st = g.stats()
        assert [st.sent, st.received, st.accepted] == sv["counters_sent_received_accepted"], name
        assert np.allclose(g.get_state().reshape(wl.W, -1).sum(1), sv["state_sum_by_worker"], rtol=TOL), name
        assert abs(g.quant_error(0) - sv["quant_error_worker0"]) <= TOL * sv["quant_error_worker0"], name


@pytest.mark.parametrize("kernel,k,d,W,b,E", [
    (2, 10, 10, 64, 500, 2),        # small-state kernel
    (1, 10, 10, 64, 500, 2),        # generic kernel
    (3, 64, 32, 16, 512, 2),        # matrix-core kernel
])
def test_free_running_mode(B, kernel, k, d, W, b, E):
    """Free-running mode keeps the paper's races (Sec. 4.4): every sender draws its own recipient, a later
    message overwrites an earlier one, a buffer may be read while it is written.  The result is not
    reproducible, so there is no element-wise parity; what must hold: finite states, every worker sends once
    per round, nobody receives more than was sent, and the quantization error (Eq. 8) ends close to that of
    the deterministic run on the same data."""
    steps = 40
    X = make_data(W * b * 12, d, k, seed=31)
    Xg = to_dev(X)
    res = {}
    for mode in (B.MODE_DETERMINISTIC, B.MODE_FREE_RUNNING):
        g = B.ASGD(k, d, W, b, 0.05, E=E, seed=5, mode=mode, kernel=kernel)
        g.load_shards(Xg)
        q0 = g.quant_error(0)
        g.run_steps(steps)
        st = g.stats()
        w = g.get_state()
        assert st.kernel == kernel and np.all(np.isfinite(w))
        assert st.sent == W * (steps // E)
        assert 0 < st.received <= st.sent and 0 <= st.accepted <= st.received
        res[mode] = (g.quant_error(0), g.quant_error(-1), st)
        assert res[mode][0] < q0
    qd, qf = res[B.MODE_DETERMINISTIC], res[B.MODE_FREE_RUNNING]
    print("\n[free-running] kernel %d: E(w_0) deterministic %.6g, free-running %.6g; received %d vs %d of %d sent"
          % (kernel, qd[0], qf[0], qd[2].received, qf[2].received, qf[2].sent))
    assert abs(qf[0] - qd[0]) <= 0.2 * qd[0]             # about half of the messages are overwritten before use
    assert qd[2].received == W * ((steps - 1) // E)      # the cyclic shift delivers exactly one message per worker and round


def test_error_paths(B):
    import torch
    with pytest.raises(B.AsgdError):
        B.asgd_create(0, 10, 4, 500, 0.05)
    with pytest.raises(B.AsgdError):
        B.asgd_create(10, 10, 4, 500, -1.0)
    g = B.ASGD(10, 10, 4, 500, 0.05)
    with pytest.raises(B.AsgdError) as e:
        g.run_steps(1)                                   # before load_shards
    assert e.value.code == B.ESTATE
    x = torch.zeros((100, 10), device="cuda:0")
    with pytest.raises(B.AsgdError):
        g.load_shards(x)                                 # shard shorter than b
    with pytest.raises(B.AsgdError):
        g.set_option(B.OPT_MODE, 7)
    g2 = B.ASGD(10, 10, 2, 10, 0.05, E=2, lr_mode=1)
    g2.load_shards(torch.rand((100, 10), device="cuda:0"))
    with pytest.raises(B.AsgdError):
        g2.run_steps(1)                                  # 1/count step size needs silent mode


def test_two_contexts_and_a_side_stream(B, oracle):
    # contexts are independent (no global state); the library launches on the stream handed to load_shards
    import torch
    X1 = make_data(24_000, 10, 10, seed=41)
    X2 = make_data(4 * 600 * 4, 20, 40, seed=42)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        a = B.ASGD(10, 10, 6, 200, 0.1, E=2, seed=3)
        a.load_shards(to_dev(X1))
    c = B.ASGD(40, 20, 4, 600, 0.05, E=3, seed=4)
    c.load_shards(to_dev(X2))
    for _ in range(3):                                  # interleave the two
        a.run_steps(5)
        c.run_steps(3)
    assert a.stats().kernel == B.KERNEL_SMALL and c.stats().kernel == B.KERNEL_MFMA
    oa = oracle.OracleASGD(X1, k=10, W=6, b=200, lr=0.1, E=2, seed=3); oa.run_steps(15)
    oc = oracle.OracleASGD(X2, k=40, W=4, b=600, lr=0.05, E=3, seed=4); oc.run_steps(9)
    assert rel_fro(a.get_state(), oa.w).max() <= TOL and rel_fro(c.get_state(), oc.w).max() <= TOL
    assert np.array_equal(a.worker_counters(), oa.counters) and np.array_equal(c.worker_counters(), oc.counters)
    a.run_steps(0)                                      # nothing to do is not an error
    assert a.stats().steps == 15


@pytest.mark.parametrize("fast,k,d,W,b", [(2, 10, 10, 6, 200), (3, 40, 20, 4, 600)])
@pytest.mark.parametrize("buffers,parts", [(1, 1), (2, 1), (1, 5), (3, 2)])
def test_kernel_switch_between_runs(B, oracle, buffers, parts, fast, k, d, W, b):
    # Kernels keep the messages in flight in their own formats; at a change of kernel the library carries them over,
    # also at a merge point, where messages wait (t = 2, 6, 8 below), and with partial messages, where the fill of the
    # never-written rows differs per format.  fast: the specialised kernel of the shape; the other one is shape-agnostic.
    X = make_data(W * b * 4, d, k, seed=2)
    g = B.ASGD(k, d, W, b, 0.1, E=2, kernel=fast, buffers=buffers, parts=parts)
    g.load_shards(to_dev(X))
    g.run_steps(2)                                    # t = 2: the messages of round 0 wait to be merged
    g.set_option(B.OPT_KERNEL, 1)
    g.run_steps(1)                                    # the generic kernel merges what the specialised kernel sent
    g.run_steps(3)                                    # t = 6: sends in its own format
    g.set_option(B.OPT_KERNEL, fast)
    g.run_steps(2)                                    # and back (t = 8)
    g.set_option(B.OPT_KERNEL, 1)
    g.run_steps(1)                                    # t = 9
    assert g.stats().kernel == 1
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=0.1, E=2, buffers=buffers, parts=parts)
    o.run_steps(9)
    assert rel_fro(g.get_state(), o.w).max() <= TOL
    check_counters(g.worker_counters(), o.counters, o.parzen_near)


@pytest.mark.parametrize("kernel,k,d,W,b", [(1, 10, 10, 6, 200), (2, 10, 10, 6, 200), (3, 40, 20, 4, 600), (1, 7, 5, 5, 150)])
@pytest.mark.parametrize("buffers,parts", [(1, 1), (2, 1), (3, 2)])
def test_resume_at_a_merge_point(B, oracle, kernel, k, d, W, b, buffers, parts):
    """A run stopped at a merge point (messages of the finished round in flight), exported (states, step counter,
    messages) and continued in a new context is bit for bit the uninterrupted run; the exported messages are the
    oracle's external buffers at that step (same layout: buffer, worker, row), stamps identical."""
    if kernel == 3 and parts > 1 and W * k * d > (1 << 18):
        pytest.skip("beyond the size limit of partial messages on the matrix-core kernel")
    E, t_stop, t_more = 3, 12, 11
    X = make_data(W * b * 5 + 3, d, k, seed=12)
    Xd = to_dev(X)
    kw = dict(E=E, seed=5, kernel=kernel, buffers=buffers, parts=parts)
    full = B.ASGD(k, d, W, b, 0.1, **kw); full.load_shards(Xd); full.run_steps(t_stop + t_more)
    a = B.ASGD(k, d, W, b, 0.1, **kw); a.load_shards(Xd); a.run_steps(t_stop)
    values, rounds = a.get_exchange()
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=0.1, E=E, seed=5, buffers=buffers, parts=parts)
    o.run_steps(t_stop)
    assert np.array_equal(rounds, np.asarray(o.slot_stamp).reshape(buffers, W))
    assert (rounds == t_stop // E - 1).all()
    oslot = np.asarray(o.slot).reshape(buffers, W, k, d)
    assert np.array_equal(values == 0, oslot == 0)                         # the same rows travel
    assert np.abs(values - oslot).max() <= TOL * np.abs(oslot).max()
    # without the messages the continued run differs; with them it does not
    c = B.ASGD(k, d, W, b, 0.1, **kw); c.load_shards(Xd)
    c.set_state(-2, a.get_state()); c.set_step(t_stop)
    v0, r0 = c.get_exchange()
    assert (r0 == -1).all() and not v0.any()
    c.run_steps(t_more)
    merges = len([t for t in range(t_stop, t_stop + t_more) if t % E == 0])
    assert c.stats().received == (merges - 1) * W * buffers               # the first merge point found nothing
    c.set_state(-2, a.get_state()); c.set_step(t_stop); c.set_exchange(values, rounds)
    v1, r1 = c.get_exchange()                                              # handed over, not yet used: comes back as is
    assert np.array_equal(v1, values) and np.array_equal(r1, rounds)
    c.run_steps(t_more)
    assert c.stats().received == (2 * merges - 1) * W * buffers           # (the counters went on from the first try)
    assert np.array_equal(full.get_state(), c.get_state())
    # inside a round nothing is in flight
    a.run_steps(1)
    v2, r2 = a.get_exchange()
    assert (r2 == -1).all() and not v2.any()
    # a round that cannot wait at this step is refused
    with pytest.raises(B.AsgdError) as e:
        c.set_exchange(values, rounds + 1)
    assert e.value.code == B.EINVAL


@pytest.mark.parametrize("kernel,k,d,W,b", [(2, 10, 10, 6, 200), (3, 40, 20, 4, 600), (1, 7, 5, 5, 150)])
def test_exchange_export_in_free_running_mode(B, kernel, k, d, W, b):
    """Free-running mode makes no promise of reproducibility; the export still has to be a consistent snapshot: rounds
    between -1 and the newest one that has sent, finite rows, zeros where nothing waits; handed to a new context (also
    one that runs another kernel) the run goes on, and the messages are found at the next merge point."""
    E, t_stop = 2, 8
    X = to_dev(make_data(W * b * 5 + 3, d, k, seed=52))
    a = B.ASGD(k, d, W, b, 0.1, E=E, seed=3, kernel=kernel, mode=B.MODE_FREE_RUNNING, buffers=2)
    a.load_shards(X); a.run_steps(t_stop)
    values, rounds = a.get_exchange()
    assert rounds.min() >= -1 and rounds.max() <= t_stop // E - 1 and (rounds >= 0).any()
    assert np.all(np.isfinite(values)) and not values[rounds < 0].any() and values[rounds >= 0].any()
    for other in (kernel, 1):
        c = B.ASGD(k, d, W, b, 0.1, E=E, seed=3, kernel=other, mode=B.MODE_FREE_RUNNING, buffers=2)
        c.load_shards(X)
        c.set_state(-2, a.get_state()); c.set_step(t_stop); c.set_exchange(values, rounds)
        c.run_steps(1)                                        # t_stop is a merge point: the waiting messages are looked at
        assert c.stats().received == int((rounds >= 0).sum()) and np.all(np.isfinite(c.get_state()))
        c.run_steps(5)
        assert np.all(np.isfinite(c.get_state()))


def test_schedule_matches_oracle(B, oracle):
    for W in (2, 5, 1024):
        for r in range(5):
            for i in (0, 1, W - 1):
                assert B.asgd_schedule_peer(9, r, i, W) == oracle.peer(9, r, i, W)


def test_mean_state(B, oracle):
    X = make_data(24_000, 10, 10, seed=2)
    g, o = run_both(B, oracle, X, 10, 6, 200, 0.1, 2, 10)
    assert np.allclose(g.get_mean_state(), o.w.mean(0), rtol=1e-4, atol=1e-5)
    qg = g.quant_error(-1)
    qo = oracle.quant_error(X, o.w.mean(0))
    assert abs(qg - qo) <= TOL * qo


@pytest.mark.parametrize("k,d,kernel_name", [(10, 10, "streaming"), (64, 32, "matrix-core"), (7, 5, "generic"),
                                             (4, 4, "streaming"), (8, 16, "streaming"), (16, 12, "streaming"),
                                             (100, 100, "matrix-core"), (39, 12, "matrix-core"),     # 4x4 tiles at the end
                                             (2048, 16, "matrix-core")])                             # state streamed through LDS
def test_quant_error_of_tight_clusters_far_from_the_origin(B, oracle, k, d, kernel_name):
    """Eq. 8 where |x|^2 is ten orders of magnitude above the distances: centres in [0, 1000]^d, sigma = 0.01.  An
    expanded-form evaluation |x|^2/2 - max score loses everything to cancellation in fp32; the kernels form the winner's
    distance directly."""
    rng = np.random.default_rng(17)
    N = 60_000 + 13
    centres = rng.uniform(0.0, 1000.0, size=(k, d))
    X = (centres[rng.integers(0, k, size=N)] + 0.01 * rng.standard_normal((N, d))).astype(np.float32)
    w = (centres + 0.02 * rng.standard_normal((k, d))).astype(np.float32)
    g = B.ASGD(k, d, 1, 64, 0.05)
    g.load_shards(to_dev(X))
    g.set_state(0, w)
    qg, qo = g.quant_error(0), oracle.quant_error(X, w.astype(np.float64))
    print("\n[Eq. 8, %s kernel] gpu %.8g oracle %.8g (per sample %.3g)" % (kernel_name, qg, qo, qo / N))
    assert abs(qg - qo) <= TOL * qo


@pytest.mark.parametrize("kernel,tune,k,d,W,b", [(2, 0, 10, 10, 8, 64), (3, 2, 40, 20, 12, 32), (3, 8, 40, 20, 12, 32)])
def test_long_call_is_cut_into_launches_of_bounded_length(B, kernel, tune, k, d, W, b):
    """A call that covers more rounds than one launch with in-kernel waits is allowed (1024) becomes several such
    launches; the result is that of the same steps handed over in small pieces, bit for bit."""
    steps = 2500                                      # E = 1: 2500 rounds -> 3 launches
    X = make_data(W * b * 7 + 5, d, k, seed=47)       # (7 steps per epoch: the run wraps around many times)
    Xg = to_dev(X)
    whole = B.ASGD(k, d, W, b, 0.02, E=1, kernel=kernel, tune=tune); whole.load_shards(Xg); whole.run_steps(steps)
    assert whole.stats().launches == 3
    pieces = B.ASGD(k, d, W, b, 0.02, E=1, kernel=kernel, tune=tune); pieces.load_shards(Xg)
    for n in (1000, 1, 1023, 476):
        pieces.run_steps(n)
    assert np.array_equal(whole.get_state(), pieces.get_state())
    assert np.array_equal(whole.worker_counters(), pieces.worker_counters())


@pytest.mark.parametrize("kernel,tune,k,d,W,b", [(2, 0, 10, 10, 8, 200), (3, 2, 40, 20, 12, 100)])
def test_expired_wait_is_reported_and_the_context_recovers(B, kernel, tune, k, d, W, b):
    """The error path of the runs that are one launch: the host makes every message get lost without telling the
    recipients (test hooks) and gives the workgroups four polls for all their waits, so every merge point gives up
    at once and every kernel still ends normally.  The run must return ASGD_ESYNC, leave the step counter alone and
    the context refusing runs; after set_state + set_step the context works again."""
    X = make_data(W * b * 6 + 3, d, k, seed=43)
    Xg = to_dev(X)
    g = B.ASGD(k, d, W, b, 0.05, E=2, drop_rate=1.0, kernel=kernel, tune=tune)
    g.set_option(B.OPT_WAIT_POLLS, 4)
    g.set_option(B.OPT_DROP_UNANNOUNCED, 1)
    g.load_shards(Xg)
    w0 = g.get_state()
    with pytest.raises(B.AsgdError) as e:
        g.run_steps(7)
    assert e.value.code == B.ESYNC
    assert g.stats().steps == 0 and g.stats().launches == 1 and g.stats().kernel == kernel
    with pytest.raises(B.AsgdError) as e:
        g.run_steps(1)
    assert e.value.code == B.ESTATE
    g.set_option(B.OPT_DROP_UNANNOUNCED, 0)                 # lost messages are skipped again: same as silent mode
    g.set_state(-2, w0)
    g.set_step(0)
    g.run_steps(7)
    s = B.ASGD(k, d, W, b, 0.05, E=0, kernel=kernel, tune=tune)
    s.load_shards(Xg)
    s.run_steps(7)
    assert g.stats().steps == 7 and np.array_equal(g.get_state(), s.get_state())
