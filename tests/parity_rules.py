"""The acceptance rules of the GPU parity tests, in one place (used at the small sizes and at the workloads' full sizes).

Deterministic mode, HIP path against the oracle on the same input:
  assignments  identical, except where the oracle's own relative gap (d2 - d1)/d1 is below 1e-6 (near-ties), and
               except where the gap is below what the measured difference between the two states can turn: the GPU keeps
               fp32 states (the oracle fp64 ones), which drift apart by ~1e-7 relative per step, and a near-tie resolved
               the other way moves one sample between two centroids, after which that worker's states differ by a few
               1e-5.  A state that is off by dw (Frobenius) moves a squared distance d1 by at most 2 sqrt(d1) |dw|, so
               two distances can change order only if (d2 - d1)/d1 <= 4 |dw| / sqrt(d1); with |dw| = err_i |w_i| (err_i:
               relative state error of worker i, measured at the end of the run or at the round boundaries the test
               looks at), the typical squared distance 2 E(w)/N of Eq. 8 for d1, and a factor 2 because the steps
               between a flip and the measurement contract the error (by (1 - eps c_k/b) per step), a mismatch must have
               gap < 8 err_i |w_i| / sqrt(2 E(w)/N).  Mismatches are counted in three kinds: at near-ties; above the
               near-tie band in a worker with no earlier near-tie mismatch (fp32 rounding of the state alone; gaps of a
               few 1e-6, a handful in 1e9 samples); follow-ons of an earlier mismatch of the same worker.
  states       per worker, relative Frobenius error <= 1e-4.  Where a run is long enough for assignment mismatches of one
               worker to add up (the 100 GB workload: 610 steps), the error a worker is allowed grows by what its counted
               mismatches explain: a sample x that goes to centroid a instead of b moves row a by eps (x - w_a)/b and
               row b by -eps (x - w_b)/b, and later steps only contract that (mismatch_shift()).
  counters     messages sent and messages looked at are identical; messages merged may differ per worker by at most the
               number of that worker's merge tests the oracle flags as near-ties of Eq. 4 (|lhs - rhs| / rhs < 1e-6).
"""
import numpy as np

NEAR_TIE = 1e-6
STATE_TOL = 1e-4


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(a.shape[0], -1)
    b = np.asarray(b, dtype=np.float64).reshape(b.shape[0], -1)
    return np.linalg.norm(a - b, axis=1) / np.linalg.norm(b, axis=1)


def follow_on_bound(err, w_oracle, quant_error_per_sample):
    """Per worker: largest relative gap of a follow-on mismatch that a state error err (relative, W values) explains.
    w_oracle: W x k x d states; quant_error_per_sample: E(w)/N of Eq. 8 for a typical state."""
    wn = np.linalg.norm(np.asarray(w_oracle, dtype=np.float64).reshape(len(err), -1), axis=1)
    return np.maximum(NEAR_TIE, 8.0 * np.asarray(err) * wn / np.sqrt(2.0 * quant_error_per_sample))


def check_assignments(ag, ao, gap, bound, verbose=True, flipped=None):
    """ag, ao, gap: steps x W x b (GPU, oracle, oracle's relative gap); bound: W values of follow_on_bound().
    flipped: for runs checked piece by piece, the set of workers with a mismatch in an earlier piece (updated here).
    Returns (mismatches at near-ties, mismatches from state rounding alone, follow-on mismatches)."""
    diff = ag != ao
    n_tie = n_round = n_follow = 0
    seen = set() if flipped is None else flipped
    for t, i, n in zip(*np.nonzero(diff)):                 # ordered by step, then worker, then position
        g = gap[t, i, n]
        if verbose:
            print("   mismatch step %d worker %d sample %d: gpu %d oracle %d gap %.3g" % (t, i, n, ag[t, i, n], ao[t, i, n], g))
        if g < NEAR_TIE:
            n_tie += 1
        else:
            assert g < bound[i], "worker %d: mismatch at step %d with gap %.3g >= %.3g, more than the state error explains" % (i, t, g, bound[i])
            if i in seen:
                n_follow += 1
            else:
                n_round += 1
        seen.add(i)
    return n_tie, n_round, n_follow


def mismatch_shift(ag, ao, Xs, w, eps, b):
    """Per worker, the sum over its assignment mismatches of the Frobenius norm of the state change that moving the
    sample from one centroid to the other causes.  ag, ao: steps x W x b; Xs: W x (steps*b) x d samples of these steps;
    w: W x k x d states (the oracle's, at the end of these steps)."""
    out = np.zeros(ag.shape[1])
    for t, i, n in zip(*np.nonzero(ag != ao)):
        x = Xs[i, t * b + n].astype(np.float64)
        da, db = x - w[i, ag[t, i, n]], x - w[i, ao[t, i, n]]
        out[i] += eps / b * np.sqrt(da @ da + db @ db)
    return out


def check_counters(gpu_counters, oracle_counters, parzen_near):
    """W x 3 (sent, looked at, merged) on both sides; parzen_near: W near-ties of Eq. 4 flagged by the oracle."""
    assert np.array_equal(gpu_counters[:, 0], oracle_counters[:, 0]), "messages sent differ"
    assert np.array_equal(gpu_counters[:, 1], oracle_counters[:, 1]), "messages looked at differ"
    d = np.abs(gpu_counters[:, 2] - oracle_counters[:, 2])
    assert np.all(d <= parzen_near), "merged messages differ beyond the flagged near-ties of Eq. 4: workers %s" % np.nonzero(d > parzen_near)[0][:10]
