"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without
reusing the oracle's own code.  Every comparison partner below is written here, in
NumPy/pure Python (or is a library routine), from the definition it cites."""
import numpy as np
import pytest

from paper_1505_04956_amd import workloads

M64 = (1 << 64) - 1


# ---------------------------------------------------------------- helpers (independent)
def brute_assign(X, w):
    """s_i(w) by full enumeration of all k squared distances in fp64 (text after Eq. 8)."""
    D = ((X[:, None, :].astype(np.float64) - w[None, :, :]) ** 2).sum(-1)
    return D.argmin(1), D            # numpy argmin returns the first minimum


def minibatch_kmeans_numpy(X, w0, b, lr, steps):
    """Sequential mini-batch K-Means, Alg. 4 with the K-Means gradient of Eq. 9 (descent sign)."""
    w = w0.astype(np.float64).copy()
    S = X.shape[0] // b
    for t in range(steps):
        M = X[(t % S) * b:(t % S + 1) * b].astype(np.float64)
        a = ((M[:, None] - w[None]) ** 2).sum(-1).argmin(1)
        grad = np.zeros_like(w)
        for i, c in enumerate(a):
            grad[c] += w[c] - M[i]
        w -= lr * grad / b
    return w


def splitmix64_stream(seed, n):
    """First n outputs of the published splitmix64 generator, in Python integers."""
    out, s = [], seed & M64
    for _ in range(n):
        s = (s + 0x9E3779B97F4A7C15) & M64
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        out.append(z ^ (z >> 31))
    return out


def py_peer(seed, r, i, W, n=0):
    return (i + 1 + (splitmix64_stream(seed, r + 1)[r] % (W - 1) + n) % (W - 1)) % W


def asgd_numpy(X, k, W, b, lr, E, seed, steps, parzen=True, buffers=1, parts=1):
    """Whole lockstep ASGD (Alg. 5 + Eq. 4 + Eq. 6/7, partial messages of Sec. 4.4) in NumPy, vectorised differently
    from the oracle.  A buffer entry is (state, boolean row mask of the rows that travelled)."""
    N, d = X.shape
    H = N // W
    S = H // b
    w = np.stack([X[i * H:i * H + k] for i in range(W)]).astype(np.float64)
    buf = [[None] * buffers for _ in range(W)]
    stats = np.zeros((W, 3), dtype=np.int64)
    for t in range(steps):
        s = t % S
        new = np.empty_like(w)
        for i in range(W):
            M = X[i * H + s * b:i * H + (s + 1) * b].astype(np.float64)
            a, _ = brute_assign(M, w[i])
            onehot = np.zeros((b, k))
            onehot[np.arange(b), a] = 1.0
            cnt = onehot.sum(0)
            G = (cnt[:, None] * w[i] - onehot.T @ M) / b
            step = G
            if E > 0 and t > 0 and t % E == 0 and parts == 1:
                good = []
                for ent in buf[i]:
                    if ent is None or np.linalg.norm(ent[0]) == 0:
                        continue
                    we = ent[0]
                    stats[i, 1] += 1
                    ok = np.sum(((w[i] - lr * G) - we) ** 2) < np.sum((w[i] - we) ** 2)
                    if ok or not parzen:
                        good.append(we)
                if good:
                    stats[i, 2] += len(good)
                    step = (w[i] - np.mean(np.stack(good + [w[i]]), axis=0)) + G
            elif E > 0 and t > 0 and t % E == 0:
                total = w[i].copy()                      # per row: local state + accepted external rows
                count = np.ones(k)
                for ent in buf[i]:
                    if ent is None or np.linalg.norm(ent[0][ent[1]]) == 0:
                        continue
                    we, rows = ent
                    stats[i, 1] += 1
                    lhs = np.sum(((w[i] - lr * G) - we) ** 2, axis=1)
                    rhs = np.sum((w[i] - we) ** 2, axis=1)
                    ok = rows & (np.sum(we ** 2, axis=1) > 0) & ((lhs < rhs) if parzen else True)
                    total[ok] += we[ok]
                    count[ok] += 1
                    stats[i, 2] += int(ok.any())
                step = (w[i] - total / count[:, None]) + G
            new[i] = w[i] - lr * step
        if E > 0 and t > 0 and t % E == 0:
            buf = [[None] * buffers for _ in range(W)]
        w = new
        if E > 0 and W > 1 and (t + 1) % E == 0:
            r = t // E
            for i in range(W):
                stats[i, 0] += 1
                for n in range(buffers):
                    p = py_peer(seed, r, i, W, n)
                    buf[p][n] = (w[i].copy(), np.arange(k) % parts == (r + p + n) % parts)
    return w, stats


def small_data(N=4000, d=3, k=4, seed=7):
    wl = workloads.Workload("t", N, d, k, 1, 1, 0.1, 0, 1, 1.0, "uniform10", "equal", data_seed=seed)
    return workloads.generate_host(wl)


# ---------------------------------------------------------------- pin 1: s_i(w)
def test_argmin_matches_brute_force(oracle):
    rng = np.random.default_rng(0)
    for (n, k, d) in [(64, 5, 3), (50, 2, 1), (33, 7, 2)]:
        X = rng.normal(size=(n, d)).astype(np.float32)
        w = rng.normal(size=(k, d))
        idx, gap = oracle.assign(X, w, want_gap=True)
        ref, D = brute_assign(X, w)
        assert np.array_equal(idx, ref)
        Ds = np.sort(D, axis=1)
        assert np.allclose(gap, (Ds[:, 1] - Ds[:, 0]) / Ds[:, 0], rtol=1e-12)


def test_argmin_degenerate_cases(oracle):
    rng = np.random.default_rng(1)
    X = rng.normal(size=(40, 3)).astype(np.float32)
    assert np.all(oracle.assign(X, rng.normal(size=(1, 3))) == 0)            # k = 1
    w = np.tile(rng.normal(size=(1, 3)), (4, 1))
    assert np.all(oracle.assign(X, w) == 0)                                   # duplicates: lowest index
    w = rng.normal(size=(5, 3)); w[3] = w[1]
    idx = oracle.assign(X, w)
    assert not np.any(idx == 3)                                               # never the later twin
    # exact tie by construction: sample midway between two centroids
    w2 = np.array([[0.0, 0.0], [2.0, 0.0], [0.0, 2.0]])
    assert oracle.assign(np.array([[1.0, 0.0]], dtype=np.float32), w2)[0] == 0
    assert oracle.assign(np.array([[1.0, 1.0]], dtype=np.float32), w2[[2, 1, 0]])[0] == 0


# ---------------------------------------------------------------- pin 2: W=1, no exchange
@pytest.mark.parametrize("b,lr", [(50, 0.1), (97, 0.5)])
def test_single_worker_is_sequential_minibatch_kmeans(oracle, b, lr):
    X = small_data()
    k = 4
    o = oracle.OracleASGD(X, k=k, W=1, b=b, lr=lr, E=0)
    steps = 2 * o.S + 3                                   # crosses an epoch boundary
    o.run_steps(steps)
    ref = minibatch_kmeans_numpy(X, X[:k], b, lr, steps)
    assert np.allclose(o.w[0], ref, rtol=1e-12, atol=1e-12)


def test_w1_ignores_exchange_interval(oracle):
    X = small_data()
    a = oracle.OracleASGD(X, k=4, W=1, b=50, lr=0.1, E=0); a.run_steps(30)
    c = oracle.OracleASGD(X, k=4, W=1, b=50, lr=0.1, E=3); c.run_steps(30)
    assert np.array_equal(a.w, c.w) and c.counters.sum() == 0


# ---------------------------------------------------------------- pin 3: 1/count step
def test_inverse_count_rate_is_running_mean(oracle):
    X = small_data(N=3000)
    k, b = 4, 60
    o = oracle.OracleASGD(X, k=k, W=1, b=b, lr=0.1, E=0, lr_mode=oracle.OracleASGD.LR_INV_COUNT)
    steps = 35
    a, _ = o.run_steps(steps, dump=True)
    sums = np.zeros((k, 3)); cnt = np.zeros(k)
    for t in range(steps):
        M = X[t * b:(t + 1) * b].astype(np.float64)
        np.add.at(sums, a[t, 0], M)
        np.add.at(cnt, a[t, 0], 1)
    assert np.array_equal(cnt, o.ncum[0])
    seen = cnt > 0
    assert np.allclose(o.w[0][seen], sums[seen] / cnt[seen, None], rtol=1e-10)
    assert np.array_equal(o.w[0][~seen], X[:k][~seen].astype(np.float64))


def test_inverse_count_full_batch_is_one_lloyd_iteration(oracle):
    from sklearn.cluster import KMeans
    X = small_data(N=2000, d=3, k=4, seed=11)
    k = 4
    o = oracle.OracleASGD(X, k=k, W=1, b=X.shape[0], lr=1.0, E=0, lr_mode=1)
    o.run_steps(1)
    # textbook Lloyd step
    a, _ = brute_assign(X, X[:k].astype(np.float64))
    lloyd = np.stack([X[a == c].astype(np.float64).mean(0) for c in range(k)])
    assert np.allclose(o.w[0], lloyd, rtol=1e-12)
    # library Lloyd, one iteration from the same start
    km = KMeans(n_clusters=k, init=X[:k].astype(np.float64), n_init=1, max_iter=1, algorithm="lloyd", tol=0.0)
    km.fit(X.astype(np.float64))
    assert np.allclose(o.w[0], km.cluster_centers_, rtol=1e-7, atol=1e-7)


def test_inverse_count_needs_silent_mode(oracle):
    X = small_data()
    o = oracle.OracleASGD(X, k=4, W=2, b=50, lr=0.1, E=2, lr_mode=1)
    with pytest.raises(ValueError):
        o.run_steps(1)


# ---------------------------------------------------------------- pin 4: closed form
def test_identical_samples_closed_form(oracle):
    """All samples equal x and one centroid nearest: w_k(t) = x + (1-eps)^t (w_k(0)-x); others fixed.
    Fails for the other sign of Eq. 9, for 1/count instead of 1/b, or a wrong eps."""
    k, d, b, lr = 3, 4, 20, 0.3
    x = np.array([1.0, -2.0, 0.5, 3.0], dtype=np.float32)
    X = np.tile(x, (200, 1)).astype(np.float32)
    w0 = np.array([[1.5, -2.0, 0.5, 3.0], [9, 9, 9, 9], [-7, 0, 0, 1]], dtype=np.float64)
    o = oracle.OracleASGD(X, k=k, W=1, b=b, lr=lr, E=0, w0=w0)
    for t in range(1, 8):
        o.run_steps(1)
        expect = w0.copy()
        expect[0] = x + (1 - lr) ** t * (w0[0] - x)
        assert np.allclose(o.w[0], expect, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- pin 5: merge algebra (Eq. 4, Eq. 7)
def _merge_case(oracle, c, lr=0.2, parzen=True, seed=3):
    """One worker pair at a merge point with the external state placed at w - c*G."""
    X = small_data(N=800, d=3, k=4, seed=seed)
    k, W, b, E = 4, 2, 40, 2
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=E, parzen=parzen)
    o.t[0] = E                                   # next step is a merge point of round 1
    w = o.w.copy()
    G = []
    for i in range(W):
        M = X[i * o.H + (E % o.S) * b:i * o.H + (E % o.S + 1) * b].astype(np.float64)
        a, _ = brute_assign(M, w[i])
        g = np.zeros((k, 3))
        for c_ in range(k):
            g[c_] = ((a == c_).sum() * w[i][c_] - M[a == c_].sum(0)) / b
        G.append(g)
    G = np.stack(G)
    o.slot[:] = w - c * G
    o.slot_stamp[:] = 0                          # message of round 0
    o.run_steps(1)
    return o, w, G


@pytest.mark.parametrize("c", [-1.0, 0.0, 0.05, 0.0999, 0.1001, 0.5, 3.0])
def test_parzen_accepts_iff_peer_is_ahead_by_more_than_half_a_step(oracle, c):
    """With w_ext = w - c*G Eq. 4 reduces to c > eps/2 (here eps/2 = 0.1)."""
    lr = 0.2
    o, w, G = _merge_case(oracle, c, lr=lr)
    accept = c > lr / 2
    assert np.all(o.counters[:, 1] == 1)
    assert np.all(o.counters[:, 2] == int(accept))
    ext = w - c * G
    expect = w - lr * G - (lr / 2) * (w - ext) if accept else w - lr * G
    assert np.allclose(o.w, expect, rtol=1e-12, atol=1e-13)
    assert np.all(o.slot == 0) and np.all(o.slot_stamp == -1)      # used once, then empty


def test_parzen_off_always_merges_and_same_state_is_rejected(oracle):
    o, w, G = _merge_case(oracle, -1.0, parzen=False)
    assert np.all(o.counters[:, 2] == 1)
    ext = w + G
    assert np.allclose(o.w, w - 0.2 * G - 0.1 * (w - ext), rtol=1e-12)
    # w_ext == w: lhs = eps^2 |G|^2 > 0 = rhs -> rejected, plain step
    o2, w2, G2 = _merge_case(oracle, 0.0)
    assert np.all(o2.counters[:, 2] == 0) and np.allclose(o2.w, w2 - 0.2 * G2, rtol=1e-12)


@pytest.mark.parametrize("delta,flagged", [(2.5e-8, True), (-2.5e-8, True), (2.5e-4, False), (-2.5e-4, False)])
def test_parzen_near_tie_flag_is_set_exactly_below_the_margin(oracle, delta, flagged):
    """With w_ext = w - c*G: lhs / rhs = ((c - eps) / c)^2, so c = (eps/2)(1 + delta) gives |lhs - rhs| / rhs = 4|delta|
    to first order: 1e-7 must be counted as a near-tie of Eq. 4, 1e-3 must not; the decision follows the sign."""
    lr = 0.2
    o, w, G = _merge_case(oracle, lr / 2 * (1 + delta), lr=lr)
    assert o.near[1] == (2 if flagged else 0)                       # both workers of the pair
    assert np.array_equal(o.parzen_near, [1, 1] if flagged else [0, 0])
    assert np.all(o.counters[:, 2] == int(delta > 0))
    # one worker near the tie, the other far from it: the per-worker counter tells them apart
    c = np.array([lr / 2 * (1 + 2.5e-8), 3.0]).reshape(2, 1, 1)
    o2, _, _ = _merge_case(oracle, c, lr=lr)
    assert o2.near[1] == 1 and np.array_equal(o2.parzen_near, [1, 0]) and np.array_equal(o2.counters[:, 2], [1, 1])


def test_argmin_near_tie_counter_counts_gaps_below_1e6(oracle):
    """Two centroids at (0,0) and (2,0); a sample at (1 - eta, 0) has (d2 - d1)/d1 = 4 eta / (1 - eta)^2.  eta = 2^-24
    (the fp32 neighbour of 1: gap 2.4e-7) and eta = 0 (exact tie) count as near-ties, eta = 2^-12 (gap 9.8e-4) does not."""
    b = 40
    w0 = np.array([[0.0, 0.0], [2.0, 0.0]])
    for n_near, n_exact in [(0, 0), (3, 0), (5, 2)]:
        X = np.zeros((2 * b, 2), dtype=np.float32)
        X[:, 0] = np.float32(1.0) - np.float32(2.0 ** -12)
        X[:n_near, 0] = np.float32(1.0) - np.float32(2.0 ** -24)
        X[n_near:n_near + n_exact, 0] = 1.0
        assert float(X[0, 0]) < 1.0 or n_near == 0
        o = oracle.OracleASGD(X, k=2, W=1, b=b, lr=0.1, E=0, w0=w0)
        a, gap = o.run_steps(1, dump=True)
        assert o.near[0] == n_near + n_exact
        assert np.all(a == 0)                                        # the nearer one, and the lower index on the tie
        assert int((gap < 1e-6).sum()) == n_near + n_exact
        if n_near:
            assert 2.0e-7 < gap[0, 0, 0] < 2.6e-7
        assert 9.0e-4 < gap[0, 0, -1] < 1.0e-3


def test_zero_gradient_never_accepts(oracle):
    """G = 0 makes both sides of Eq. 4 equal; the strict '<' rejects."""
    x = np.array([2.0, 2.0], dtype=np.float32)
    X = np.tile(x, (400, 1))
    w0 = np.array([[2.0, 2.0], [50.0, 50.0]])
    o = oracle.OracleASGD(X, k=2, W=2, b=10, lr=0.1, E=1, w0=w0)
    o.t[0] = 1
    o.slot[:] = np.array([[3.0, 1.0], [40.0, 60.0]])
    o.slot_stamp[:] = 0
    o.run_steps(1)
    assert np.all(o.counters[:, 1] == 1) and np.all(o.counters[:, 2] == 0)
    assert np.array_equal(o.w, np.broadcast_to(w0, (2, 2, 2)))


def test_one_dimensional_picture_of_the_update(oracle):
    """1-D case in the spirit of Fig. 4: state at 0, samples at 1 (descent goes right)."""
    X = np.ones((200, 1), dtype=np.float32)
    lr, b = 0.5, 10
    for ext, good in [(0.8, True), (0.3, True), (0.2, False), (-0.5, False)]:
        # projected step lands at 0.5: external states right of 0.25 are closer to it than to 0
        o = oracle.OracleASGD(X, k=1, W=2, b=b, lr=lr, E=1, w0=np.zeros((1, 1)))
        o.t[0] = 1
        o.slot[:] = ext
        o.slot_stamp[:] = 0
        o.run_steps(1)
        expect = 0.5 + (lr / 2) * ext if good else 0.5
        assert np.allclose(o.w, expect, atol=1e-15), (ext, o.w)


def test_stale_or_empty_buffers_are_ignored(oracle):
    X = small_data(N=800)
    base = oracle.OracleASGD(X, k=4, W=2, b=40, lr=0.2, E=2); base.t[0] = 2; base.run_steps(1)
    stale = oracle.OracleASGD(X, k=4, W=2, b=40, lr=0.2, E=2); stale.t[0] = 2
    stale.slot[:] = 5.0; stale.slot_stamp[:] = 7            # wrong round
    stale.run_steps(1)
    zero = oracle.OracleASGD(X, k=4, W=2, b=40, lr=0.2, E=2); zero.t[0] = 2
    zero.slot_stamp[:] = 0                                  # right round but all-zero = empty (Eq. 3)
    zero.run_steps(1)
    assert np.array_equal(base.w, stale.w) and np.array_equal(base.w, zero.w)
    assert stale.counters[:, 1].sum() == 0 and zero.counters[:, 1].sum() == 0


# ---------------------------------------------------------------- N external buffers (Eq. 3, Eq. 6)
def _merge_case_n(oracle, cs, lr=0.2, parzen=True, present=None):
    """Worker pair at a merge point with buffer n holding w - cs[n]*G (buffers not in `present` stay empty)."""
    X = small_data(N=1200, d=3, k=4, seed=3)
    k, W, b, E, nb = 4, len(cs) + 1, 40, 2, len(cs)
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=E, parzen=parzen, buffers=nb)
    o.t[0] = E
    w = o.w.copy()
    G = np.zeros_like(w)
    for i in range(W):
        M = X[i * o.H + (E % o.S) * b:i * o.H + (E % o.S + 1) * b].astype(np.float64)
        a, _ = brute_assign(M, w[i])
        for c_ in range(k):
            G[i, c_] = ((a == c_).sum() * w[i][c_] - M[a == c_].sum(0)) / b
    slot = o.slot.reshape(nb, W, k, 3)
    stamp = o.slot_stamp.reshape(nb, W)
    for n, c in enumerate(cs):
        if present is None or n in present:
            slot[n] = w - c * G
            stamp[n] = 0
    o.run_steps(1)
    return o, w, G


@pytest.mark.parametrize("cs", [(0.5,), (0.5, 0.5), (0.5, 0.05), (3.0, 0.11, 0.7), (0.01, -1.0, 0.09), (0.3, 0.3, 0.3, 0.3)])
def test_n_buffers_each_gated_on_its_own(oracle, cs):
    """Buffer n at w - c_n G passes Eq. 4 iff c_n > eps/2, whatever the others hold; Eq. 6 then moves the state by
    eps * (sum of the accepted c_n) / (D + 1) further along -G, D = number accepted."""
    lr = 0.2
    o, w, G = _merge_case_n(oracle, cs, lr=lr)
    acc = [c for c in cs if c > lr / 2]
    assert np.all(o.counters[:, 1] == len(cs)) and np.all(o.counters[:, 2] == len(acc))
    expect = w - lr * G * (1.0 + sum(acc) / (len(acc) + 1.0))
    assert np.allclose(o.w, expect, rtol=1e-12, atol=1e-13)
    assert np.all(o.slot == 0) and np.all(o.slot_stamp == -1)


def test_n_buffers_gate_off_counts_only_the_buffers_that_hold_a_message(oracle):
    """Eq. 3: lambda = 0 for an empty buffer, so the mean runs over the local state and the non-empty ones."""
    cs = (0.4, -2.0, 1.5)
    o, w, G = _merge_case_n(oracle, cs, parzen=False, present=(0, 2))
    assert np.all(o.counters[:, 1] == 2) and np.all(o.counters[:, 2] == 2)
    assert np.allclose(o.w, w - 0.2 * G * (1.0 + (0.4 + 1.5) / 3.0), rtol=1e-12, atol=1e-13)
    o, w, G = _merge_case_n(oracle, cs, parzen=False)
    assert np.allclose(o.w, w - 0.2 * G * (1.0 + (0.4 - 2.0 + 1.5) / 4.0), rtol=1e-12, atol=1e-13)


def test_n_buffers_zero_gradient_unit_step_is_the_plain_average(oracle):
    """eps = 1, gate off, G = 0 (k = 1, every sample equals the centroid): the new state is the arithmetic mean of
    the local state and the N external ones."""
    x = np.array([1.5, -2.0, 0.25], dtype=np.float32)
    X = np.tile(x, (600, 1))
    nb, W = 3, 4
    o = oracle.OracleASGD(X, k=1, W=W, b=10, lr=1.0, E=1, parzen=False, buffers=nb, w0=x[None, :].astype(np.float64))
    o.t[0] = 1
    rng = np.random.default_rng(5)
    ext = rng.normal(size=(nb, W, 1, 3))
    o.slot[:] = ext
    o.slot_stamp[:] = 0
    o.run_steps(1)
    expect = (ext.sum(0) + x.astype(np.float64)) / (nb + 1)
    assert np.allclose(o.w, expect, rtol=1e-14, atol=1e-15)
    # the order of the buffers does not matter
    o2 = oracle.OracleASGD(X, k=1, W=W, b=10, lr=1.0, E=1, parzen=False, buffers=nb, w0=x[None, :].astype(np.float64))
    o2.t[0] = 1
    o2.slot[:] = ext[::-1]
    o2.slot_stamp[:] = 0
    o2.run_steps(1)
    assert np.allclose(o.w, o2.w, rtol=1e-14, atol=1e-15)


def test_n_buffers_schedule(oracle):
    """Copy n of a round's messages is a cyclic shift of its own: every worker gets exactly one message per buffer,
    the N senders of a worker differ, nobody sends to itself; copy 0 is the one-buffer schedule."""
    for W, nb in [(2, 1), (5, 4), (7, 3), (64, 4)]:
        for r in range(40):
            for n in range(nb):
                rec = [oracle.peer(11, r, i, W, n) for i in range(W)]
                assert sorted(rec) == list(range(W)) and all(rec[i] != i for i in range(W))
                assert rec == [py_peer(11, r, i, W, n) for i in range(W)]
            for i in range(W):
                assert len({oracle.peer(11, r, i, W, n) for n in range(nb)}) == nb
            assert [oracle.peer(11, r, i, W) for i in range(W)] == [oracle.peer(11, r, i, W, 0) for i in range(W)]
    X = small_data(N=800)
    with pytest.raises(ValueError):
        oracle.OracleASGD(X, k=4, W=3, b=40, lr=0.2, E=2, buffers=3).run_steps(1)       # needs N < W


def test_n_buffers_loss_hook_is_per_copy(oracle):
    thr = oracle.drop_threshold(0.5)
    lost = np.array([[oracle.dropped(9, r, s, thr, n) for n in range(4)] for r in range(50) for s in range(20)])
    assert np.array_equal(lost[:, 0], np.array([oracle.dropped(9, r, s, thr) for r in range(50) for s in range(20)]))
    frac = lost.mean(0)
    assert np.all(np.abs(frac - 0.5) < 0.06)
    assert np.abs(np.corrcoef(lost[:, 0], lost[:, 1])[0, 1]) < 0.1
    X = small_data(N=2400)
    o = oracle.OracleASGD(X, k=4, W=6, b=20, lr=0.2, E=2, buffers=3, drop_rate=0.5, seed=9)
    o.run_steps(41)
    rounds = 20
    expected = sum(not oracle.dropped(9, r, s, thr, n) for r in range(rounds) for s in range(6) for n in range(3))
    assert o.counters[:, 0].sum() == 6 * rounds and o.counters[:, 1].sum() == expected


# ---------------------------------------------------------------- partial messages (Sec. 4.4)
def test_partial_messages_carry_one_part_and_rotate(oracle):
    """After a send, buffer n of worker p holds the rows c = (r + p + n) mod P (mod P) of its sender's state and
    nothing else; over P rounds a worker sees every part once per buffer."""
    X = small_data(N=4000, d=3, k=6, seed=11)
    k, W, b, E, nb, P = 6, 5, 20, 2, 2, 3
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=0.1, E=E, seed=4, buffers=nb, parts=P)
    seen = {(p, n): set() for p in range(W) for n in range(nb)}
    for r in range(P):
        o.run_steps(E)                               # ends right after the send of round r
        assert int(o.t[0]) == (r + 1) * E
        for n in range(nb):
            for i in range(W):
                p = oracle.peer(4, r, i, W, n)
                part = (r + p + n) % P
                rows = np.arange(k) % P == part
                assert np.array_equal(o.slot[n, p][rows], o.w[i][rows])
                assert np.all(o.slot[n, p][~rows] == 0)
                seen[(p, n)].add(part)
    assert all(v == set(range(P)) for v in seen.values())
    X2 = small_data(N=800)
    for bad in (0, 5):
        with pytest.raises(ValueError):
            oracle.OracleASGD(X2, k=4, W=2, b=40, lr=0.2, E=2, parts=bad).run_steps(1)


@pytest.mark.parametrize("parzen", [True, False])
def test_partial_messages_gate_row_by_row(oracle, parzen):
    """Row c of the external state at w_c - a_c G_c: Eq. 4 over that row alone accepts iff a_c > eps/2 (and
    G_c != 0); only the rows of the part that travelled are looked at; an all-zero row is empty."""
    X = small_data(N=1600, d=3, k=8, seed=3)
    k, W, b, E, P, lr = 8, 2, 60, 2, 2, 0.2
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=E, parzen=parzen, parts=P)
    o.t[0] = E                                   # merge point of round 1: message of round 0, part (0 + i) mod P
    w = o.w.copy()
    G = np.zeros_like(w)
    for i in range(W):
        M = X[i * o.H + (E % o.S) * b:i * o.H + (E % o.S + 1) * b].astype(np.float64)
        a, _ = brute_assign(M, w[i])
        for c_ in range(k):
            G[i, c_] = ((a == c_).sum() * w[i][c_] - M[a == c_].sum(0)) / b
    coef = np.array([0.5, 0.5, 0.05, 0.05, -1.0, 3.0, 0.11, 0.09])
    ext = w - coef[None, :, None] * G
    ext[:, 5] = 0.0                              # row 5 empty, whatever its part
    o.slot[:] = ext
    o.slot_stamp[:] = 0
    o.run_steps(1)
    for i in range(W):
        in_part = np.arange(k) % P == (0 + i) % P
        nonzero_g = np.abs(G[i]).sum(1) > 0
        acc = in_part & (np.arange(k) != 5) & (((coef > lr / 2) & nonzero_g) if parzen else True)
        assert acc.any() and (~acc).any()
        expect = w[i] - lr * G[i]
        expect[acc] -= (lr / 2) * (w[i][acc] - ext[i][acc])
        assert np.allclose(o.w[i], expect, rtol=1e-12, atol=1e-13)
    assert np.all(o.counters[:, 1] == 1) and np.all(o.counters[:, 2] == 1)


def test_partial_messages_with_one_part_are_whole_messages(oracle):
    X = small_data(N=3000, d=3, k=4, seed=5)
    a = oracle.OracleASGD(X, k=4, W=4, b=30, lr=0.3, E=2, seed=9); a.run_steps(40)
    c = oracle.OracleASGD(X, k=4, W=4, b=30, lr=0.3, E=2, seed=9, parts=1); c.run_steps(40)
    assert np.array_equal(a.w, c.w) and np.array_equal(a.counters, c.counters)


# ---------------------------------------------------------------- whole algorithm vs NumPy
@pytest.mark.parametrize("W,E,parzen,buffers,parts", [(4, 3, True, 1, 1), (3, 1, True, 1, 1), (5, 2, False, 1, 1),
                                                      (5, 2, True, 2, 1), (4, 1, True, 3, 1), (6, 3, False, 4, 1),
                                                      (4, 1, True, 1, 2), (5, 2, True, 1, 4), (5, 1, False, 2, 3),
                                                      (6, 2, True, 3, 2)])
def test_full_run_matches_independent_numpy_asgd(oracle, W, E, parzen, buffers, parts):
    X = small_data(N=3000, d=3, k=4, seed=5)
    k, b, lr, seed = 4, 30, 0.3, 42
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=E, seed=seed, parzen=parzen, buffers=buffers, parts=parts)
    steps = 2 * o.S + 5
    o.run_steps(steps)
    ref_w, ref_stats = asgd_numpy(X, k, W, b, lr, E, seed, steps, parzen=parzen, buffers=buffers, parts=parts)
    assert np.allclose(o.w, ref_w, rtol=1e-11, atol=1e-12)
    assert np.array_equal(o.counters, ref_stats)
    assert ref_stats[:, 2].sum() > 0                       # the merge path really ran


# ---------------------------------------------------------------- schedule
def test_round_hash_is_splitmix64():
    # first outputs of splitmix64 for seed 0, as published with the generator
    assert splitmix64_stream(0, 3) == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_peer_schedule(oracle):
    for W in (2, 3, 7, 64):
        for seed in (0, 1, 12345):
            for r in range(6):
                p = [oracle.peer(seed, r, i, W) for i in range(W)]
                assert p == [py_peer(seed, r, i, W) for i in range(W)]
                assert sorted(p) == list(range(W))                 # everyone receives exactly once
                assert all(p[i] != i for i in range(W))            # never to oneself (Alg. 5, send)
    shifts = {oracle.peer(9, r, 0, 64) for r in range(200)}
    assert len(shifts) > 30                                        # rounds use different shifts


# ---------------------------------------------------------------- pin 6: silent mode
def test_silent_mode_equals_independent_single_worker_runs(oracle):
    X = small_data(N=4000)
    W, k, b, lr = 4, 4, 50, 0.2
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=lr, E=0)
    o.run_epochs(2)
    for i in range(W):
        solo = oracle.OracleASGD(X[i * o.H:(i + 1) * o.H], k=k, W=1, b=b, lr=lr, E=0)
        solo.run_epochs(2)
        assert np.array_equal(o.w[i], solo.w[0])


# ---------------------------------------------------------------- pin 7: lost messages
def test_losing_every_message_equals_silent_mode(oracle):
    X = small_data(N=4000)
    a = oracle.OracleASGD(X, k=4, W=4, b=50, lr=0.2, E=2, drop_rate=1.0); a.run_epochs(2)
    s = oracle.OracleASGD(X, k=4, W=4, b=50, lr=0.2, E=0); s.run_epochs(2)
    assert np.array_equal(a.w, s.w)
    assert a.counters[:, 0].min() > 0 and a.counters[:, 1:].sum() == 0


def test_partial_loss_counts(oracle):
    X = small_data(N=4000)
    W, E, seed = 4, 2, 5
    o = oracle.OracleASGD(X, k=4, W=W, b=50, lr=0.2, E=E, seed=seed, drop_rate=0.5)
    steps = 2 * o.S
    o.run_steps(steps)
    thr = oracle.drop_threshold(0.5)
    rounds_sent = steps // E
    rounds_read = (steps - 1) // E                      # the last message is never looked at
    kept = sum(not oracle.dropped(seed, r, i, thr) for r in range(rounds_read) for i in range(W))
    assert o.counters[:, 0].sum() == rounds_sent * W
    assert o.counters[:, 1].sum() == kept
    assert 0 < kept < rounds_read * W
    frac = np.mean([oracle.dropped(1, r, i, thr) for r in range(50) for i in range(40)])
    assert 0.4 < frac < 0.6


# ---------------------------------------------------------------- pin 8: conservation
def test_conservation_and_counters(oracle):
    X = small_data(N=4000)
    W, k, b, E = 4, 4, 50, 3
    o = oracle.OracleASGD(X, k=k, W=W, b=b, lr=0.2, E=E)
    steps = o.S + 7
    a, gap = o.run_steps(steps, dump=True)
    assert a.shape == (steps, W, b) and a.min() >= 0 and a.max() < k
    assert np.all(gap >= 0)
    sent, recv, good = o.counters.T
    assert np.all(sent == steps // E)
    assert np.all(recv == (steps - 1) // E)
    assert np.all(good <= recv)
    assert o.t[0] == steps


# ---------------------------------------------------------------- pin 9: E(w)
def test_quant_error_closed_form_and_invariance(oracle):
    X = small_data(N=3000)
    X64 = X.astype(np.float64)
    w = np.array([[1.0, 2.0, 3.0]])
    xbar = X64.mean(0)
    closed = 0.5 * (len(X) * np.sum((xbar - w[0]) ** 2) + np.sum((X64 - xbar) ** 2))
    assert np.isclose(oracle.quant_error(X, w), closed, rtol=1e-12)
    rng = np.random.default_rng(3)
    w = rng.uniform(0, 10, size=(6, 3))
    _, D = brute_assign(X, w)
    assert np.isclose(oracle.quant_error(X, w), 0.5 * D.min(1).sum(), rtol=1e-12)
    assert np.isclose(oracle.quant_error(X, w), oracle.quant_error(X, w[::-1].copy()), rtol=1e-13)


# ---------------------------------------------------------------- pin 10: resume
def test_resume_from_exported_state(oracle):
    X = small_data(N=4000)
    kw = dict(k=4, W=4, b=50, lr=0.2, E=3, seed=8)
    full = oracle.OracleASGD(X, **kw); full.run_steps(40)
    a = oracle.OracleASGD(X, **kw); a.run_steps(17)
    c = oracle.OracleASGD(X, **kw)
    c.w[:] = a.w; c.slot[:] = a.slot; c.slot_stamp[:] = a.slot_stamp; c.t[:] = a.t
    c.run_steps(23)
    assert np.array_equal(full.w, c.w)


def test_configs_table():
    c = workloads.CONFIGS
    assert [(x.H, x.S) for x in c] == [(25000, 50), (97656, 97), (39062, 19), (610351, 610), (19531, 4)]
    assert c[1].processed_per_epoch == 99_328_000 and c[4].processed_per_epoch == 4_194_304


def test_stored_values_of_tiny_workload(oracle):
    """The stored values under tests/golden were written by tests/golden/make_golden.py (oracle only);
    the oracle must still produce them (guards against silent changes of its arithmetic)."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    stored = json.load(open(os.path.join(here, "golden", "cfg0_oracle.json")))
    assert now["counters_sent_received_accepted"] == stored["counters_sent_received_accepted"]
    assert now["peers_round0"] == stored["peers_round0"]
    for key in ("quant_error_worker0_by_epoch", "state_worker0_row0", "state_sum_by_worker"):
        assert np.allclose(now[key], stored[key], rtol=1e-12, atol=0), key
    assert abs(now["quant_error_mean_state"] - stored["quant_error_mean_state"]) <= 1e-12 * stored["quant_error_mean_state"]
    qe = stored["quant_error_worker0_by_epoch"]
    assert all(b < a for a, b in zip(qe, qe[1:]))          # Eq. 8 falls epoch by epoch on this workload
    assert set(now["variants_after_3_epochs"]) == set(stored["variants_after_3_epochs"])
    for name, sv in stored["variants_after_3_epochs"].items():
        nv = now["variants_after_3_epochs"][name]
        assert nv["counters_sent_received_accepted"] == sv["counters_sent_received_accepted"], name
        assert np.allclose(nv["state_sum_by_worker"], sv["state_sum_by_worker"], rtol=1e-12, atol=0), name
        assert abs(nv["quant_error_worker0"] - sv["quant_error_worker0"]) <= 1e-12 * sv["quant_error_worker0"], name


def test_centre_error_hand_example(oracle):
    """Three generating centres (0,0), (4,0), (0,3) and returned centroids (1,0), (4,1), (10,10): the nearest returned
    centroid is at distance 1, 1 and sqrt(10) (to (1,0); (4,1) is at sqrt(20)), so the error is (2 + sqrt 10) / 3.  A
    squared distance would give 4, a maximum 3.16, a mean over the returned centroids something else again; the
    far centroid (10,10) must not matter, nor the order."""
    centres = np.array([[0.0, 0.0], [4.0, 0.0], [0.0, 3.0]])
    w = np.array([[1.0, 0.0], [4.0, 1.0], [10.0, 10.0]])
    want = (2.0 + np.sqrt(10.0)) / 3.0
    assert abs(oracle.centre_error(w, centres) - want) < 1e-15
    assert abs(oracle.centre_error(w[::-1], centres[[2, 0, 1]]) - want) < 1e-15
    assert oracle.centre_error(centres, centres) == 0.0
    # the evaluation helper of the package (NumPy, vectorised) is the same quantity
    wl = workloads.CONFIGS[0]
    c, _ = workloads.mixture_parameters(wl)
    rng = np.random.default_rng(5)
    wr = rng.uniform(0, 10, size=(wl.k, wl.d))
    assert abs(workloads.centre_error(wr, wl) - oracle.centre_error(wr, c)) < 1e-12


def test_centre_error_convergence_of_tiny_workload(oracle):
    """Shape of the paper's convergence figures on the synthetic generator (Sec. 5.4): the distance between
    the generator's centres and the returned ones falls with the number of samples touched; the helper is
    zero for the centres themselves and invariant to the order of the centroids."""
    wl = workloads.CONFIGS[0]
    c, _ = workloads.mixture_parameters(wl)
    assert workloads.centre_error(c, wl) == 0.0
    assert workloads.centre_error(c[::-1], wl) == 0.0
    X = workloads.generate_host(wl)
    o = oracle.OracleASGD(X, k=wl.k, W=wl.W, b=wl.b, lr=wl.lr, E=wl.E, seed=wl.schedule_seed)
    errs = [workloads.centre_error(o.w[0], wl)]           # the state of the first worker is what Alg. 5 returns
    for _ in range(wl.epochs):
        o.run_epochs(1)
        errs.append(workloads.centre_error(o.w[0], wl))
    print("centre error of worker 0 by epoch:", ["%.3f" % e for e in errs])
    assert errs[-1] < 0.8 * errs[0]
    assert all(b <= a * 1.02 for a, b in zip(errs, errs[1:]))
