/*
 * CPU oracle for the ASGD mini-batch K-Means path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the path computes, written from the
 * paper.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product (the HIP library) shares no code with it and never runs it.
 *
 * Arithmetic: samples are fp32 as stored; every distance, sum, gradient, merge and
 * state update is carried out in fp64 and the worker states stay fp64 throughout.
 * Distances are evaluated in the direct form sum_j (x_j - w_kj)^2 and ties go to the
 * lowest centroid index.  Workers advance in lockstep, one mini-batch step at a
 * time; the `omp parallel for` over workers inside a step reorders nothing, because
 * the workers of one step are independent of each other.
 *
 * What each part follows:
 *   shard split H = floor(N/W), per-worker loop ............ Alg. 5 (ASGD), lines 1-10
 *   nearest prototype s_i(w) ................................ Sec. 5.1, text after Eq. 8
 *   mini-batch gradient with 1/m', m' = b ................... Eq. 9, Alg. 4
 *   Parzen window delta(i,j) ................................ Eq. 4
 *   gated merge of one external state ....................... Eq. 7 (Eq. 5 with mini-batches)
 *   update w <- w - eps * merged step ....................... Alg. 5, update, Fig. 4 stage IV
 *   send of the new state to one other worker ............... Alg. 5, send, Fig. 2 stage I
 *   empty external buffer <=> zero norm ..................... Eq. 3 (lambda)
 *   merge of N external buffers, each gated on its own ...... Eq. 3 (no gate), Eq. 6 (gated)
 *   partial messages, partitioned along the cluster centres . Sec. 4.4 (data races and sparsity)
 *   quantization error E(w) ................................. Eq. 8
 *
 * Readings taken where the paper is silent or inconsistent (each is listed with its
 * reason in the design notes of the repository):
 *   - sign: the step is a descent step on E(w), i.e. the gradient for centroid k is
 *     (1/b) * sum_{assigned i} (w_k - x_i), so that w - eps*gradient moves centroids
 *     towards their samples (Eq. 9 prints the opposite sign of Alg. 5, update);
 *   - the gradient is taken at the state the mini-batch started with (Alg. 4, gradient step);
 *   - mini-batch s of an epoch is rows [s*b, (s+1)*b) of the worker's shard, the
 *     shard tail H mod b is not visited, the order repeats every epoch;
 *   - a state is sent after every E-th mini-batch (E = 1 is Alg. 5 as printed,
 *     E = 0 never sends = SimuParallelSGD with mini-batches); the receiver looks at
 *     its buffer at the start of the following step, uses the message once, and
 *     clears the buffer;
 *   - N external buffers per worker (default 1) and as many recipients per message:
 *     copy n of a message goes to worker (i + 1 + (h(seed, round) + n) mod (W-1)) mod W,
 *     a cyclic shift shared by all senders of a round, into the recipient's buffer n, so
 *     every worker receives exactly N messages per round, from N different senders;
 *   - in Eq. 3 the count |N| runs over the external buffers only (the printed sum starts
 *     at n = 0, which would count the local state twice and would not give Eq. 2 for N = 1);
 *     with the gate switched off every non-empty buffer takes part (Eq. 3), with the gate
 *     on every buffer is tested by Eq. 4 against the same projected local step (Eq. 6);
 *   - Eq. 4 uses whole-state norms and a strict "<";
 *   - partial messages (P parts, P = 1: whole states, the default): Sec. 4.4 partitions "along the
 *     individual cluster centers" and leaves the rest open.  Here part q is the set of centroid
 *     rows c with c mod P = q; copy n of the message of round r to recipient p carries part
 *     (r + p + n) mod P of the sender's state, so the recipient knows the part without knowing the
 *     sender and sees every part once in P rounds.  The parts of Eq. 3/4/6 are then the rows: a
 *     transmitted row is empty iff it is all zero (lambda), is tested by Eq. 4 over that row alone,
 *     and the accepted rows of all buffers enter Eq. 6 row by row; rows that were not transmitted
 *     take the plain step.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- counter-based integer generator (published splitmix64 finaliser) ------------- */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
static uint64_t round_hash(uint64_t seed, int64_t r)
{
    return mix64(seed + 0x9E3779B97F4A7C15ULL * (uint64_t)(r + 1));
}

/* Recipient of copy n of worker i's message of round r (deterministic schedule).
   W >= 2, 0 <= n < W - 1: the shifts of one round are different and never 0. */
int64_t asgd_oracle_peer_n(uint64_t seed, int64_t r, int64_t i, int64_t W, int64_t n)
{
    uint64_t shift = 1 + (round_hash(seed, r) % (uint64_t)(W - 1) + (uint64_t)n) % (uint64_t)(W - 1);
    return (int64_t)(((uint64_t)i + shift) % (uint64_t)W);
}
int64_t asgd_oracle_peer(uint64_t seed, int64_t r, int64_t i, int64_t W)
{
    return asgd_oracle_peer_n(seed, r, i, W, 0);
}

/* Test hook: is copy n of the message that `sender` emits in round r lost on the way?
   drop_threshold is a 24-bit fixed-point probability (0 = never, 2^24 = always). */
int asgd_oracle_dropped_n(uint64_t seed, int64_t r, int64_t sender, int64_t n, uint32_t drop_threshold)
{
    uint64_t u = mix64(round_hash(seed, r) + 0x9E3779B97F4A7C15ULL * (uint64_t)(sender + 1) +
                       0xD1B54A32D192ED03ULL * (uint64_t)n) >> 40;
    return u < (uint64_t)drop_threshold;
}
int asgd_oracle_dropped(uint64_t seed, int64_t r, int64_t sender, uint32_t drop_threshold)
{
    return asgd_oracle_dropped_n(seed, r, sender, 0, drop_threshold);
}

int asgd_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void asgd_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- s_i(w): index of the closest prototype (text after Eq. 8) --------------------
   Returns the argmin; *best and *second receive the smallest and second smallest
   squared distance (second = +inf when k == 1). */
static int nearest(const float *x, const double *w, int k, int d, double *best, double *second)
{
    int arg = 0;
    double d1 = INFINITY, d2 = INFINITY;
    for (int c = 0; c < k; ++c) {
        double s = 0.0;
        for (int j = 0; j < d; ++j) {
            double diff = (double)x[j] - w[(size_t)c * d + j];
            s += diff * diff;
        }
        if (s < d1) { d2 = d1; d1 = s; arg = c; }   /* strict: first minimum wins */
        else if (s < d2) { d2 = s; }
    }
    *best = d1;
    *second = d2;
    return arg;
}

/* Assignment of n samples under one state; gap_out (optional) = (d2 - d1) / d1. */
void asgd_oracle_assign(const float *X, int64_t n, int d, int k, const double *w,
                        int32_t *idx_out, double *gap_out)
{
    for (int64_t i = 0; i < n; ++i) {
        double d1, d2;
        idx_out[i] = nearest(X + i * d, w, k, d, &d1, &d2);
        if (gap_out) gap_out[i] = (d2 - d1) / d1;
    }
}

/* ---- Eq. 8: E(w) = sum_i 1/2 * min_k ||x_i - w_k||^2 over n samples ---------------- */
double asgd_oracle_quant_error(const float *X, int64_t n, int d, int k, const double *w)
{
    double total = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int64_t i = 0; i < n; ++i) {
        double d1, d2;
        (void)nearest(X + i * d, w, k, d, &d1, &d2);
        total += 0.5 * d1;
    }
    return total;
}

/* ---- one worker, one mini-batch step ------------------------------------------------
   w:       k*d state at the start of the step (read only)
   wnew:    k*d state after the step
   ext:     the next non-empty external buffers of this merge point (next = 0: nothing to merge)
   parts:   P; extpart[n] = which part buffer n carries (P = 1: the whole state, gated as a whole)
   returns the number of buffers accepted by Eq. 4 (or merged without the gate; P > 1: with at
           least one accepted row) in bits 0-7,
           bit 8 = a Parzen near-tie (|lhs-rhs|/rhs < 1e-6) in one of them                  */
static int worker_step(const float *M, int b, int k, int d, double eps, int lr_mode, int parzen,
                       const double *w, double *wnew, const double *const *ext, int next, int parts,
                       const int *extpart, int64_t *ncum,
                       int32_t *assign_out, double *gap_out, int64_t *argmin_near)
{
    const size_t kd = (size_t)k * d;
    int64_t *cnt = (int64_t *)calloc((size_t)k, sizeof(int64_t));
    double *Ssum = (double *)calloc(kd, sizeof(double));
    double *G = (double *)malloc(kd * sizeof(double));
    int flags = 0;
    int64_t near = 0;

    /* Alg. 4 lines 3-5 with Eq. 9: every sample is assigned under the SAME state w. */
    for (int i = 0; i < b; ++i) {
        const float *x = M + (size_t)i * d;
        double d1, d2;
        int a = nearest(x, w, k, d, &d1, &d2);
        cnt[a] += 1;
        for (int j = 0; j < d; ++j) Ssum[(size_t)a * d + j] += (double)x[j];
        double gap = (d2 - d1) / d1;
        if (gap < 1e-6) near += 1;
        if (assign_out) assign_out[i] = a;
        if (gap_out) gap_out[i] = gap;
    }
    *argmin_near += near;

    if (lr_mode == 1) {
        /* Per-centroid 1/count step (Sculley-style): running mean of everything ever
           assigned to the centroid.  Exchange is not defined in this mode. */
        for (int c = 0; c < k; ++c) {
            ncum[c] += cnt[c];
            for (int j = 0; j < d; ++j) {
                size_t e = (size_t)c * d + j;
                wnew[e] = w[e];
                if (cnt[c] > 0) wnew[e] = w[e] + (Ssum[e] - (double)cnt[c] * w[e]) / (double)ncum[c];
            }
        }
    } else {
        /* Eq. 9 as a descent gradient: G_k = (1/b) * sum_{assigned} (w_k - x_i). */
        for (int c = 0; c < k; ++c)
            for (int j = 0; j < d; ++j) {
                size_t e = (size_t)c * d + j;
                G[e] = ((double)cnt[c] * w[e] - Ssum[e]) / (double)b;
            }
        int delta[256];
        int ndelta = 0;
        if (parts > 1) {
            /* Sec. 4.4: the units of Eq. 3/4/6 are the transmitted centroid rows. */
            for (int n = 0; n < next; ++n) delta[n] = 0;
            for (int c = 0; c < k; ++c) {
                int nacc = 0;
                int accn[256];
                for (int n = 0; n < next; ++n) {
                    if (c % parts != extpart[n]) continue;
                    const double *er = ext[n] + (size_t)c * d;
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
                    for (int j = 0; j < d; ++j) {
                        size_t e = (size_t)c * d + j;
                        double a = (w[e] - eps * G[e]) - er[j];
                        double c2 = w[e] - er[j];
                        lhs += a * a; rhs += c2 * c2; nrm += er[j] * er[j];
                    }
                    if (!(nrm > 0.0)) continue;                 /* lambda: an all-zero row is empty */
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) flags |= 256;
                    if (parzen ? (lhs < rhs) : 1) { accn[nacc++] = n; delta[n] = 1; }
                }
                for (int j = 0; j < d; ++j) {
                    size_t e = (size_t)c * d + j;
                    double Gbar = G[e];
                    if (nacc > 0) {
                        double s2 = w[e];
                        for (int q = 0; q < nacc; ++q) s2 += ext[accn[q]][e];
                        Gbar += w[e] - s2 / (double)(nacc + 1);
                    }
                    wnew[e] = w[e] - eps * Gbar;
                }
            }
            for (int n = 0; n < next; ++n) ndelta += delta[n];
            flags |= ndelta;
            free(cnt);
            free(Ssum);
            free(G);
            return flags;
        }
        for (int n = 0; n < next; ++n) {
            /* Eq. 4: compare the projected local step with the current state, both
               measured from the external state. */
            double lhs = 0.0, rhs = 0.0;
            for (size_t e = 0; e < kd; ++e) {
                double a = (w[e] - eps * G[e]) - ext[n][e];
                double c2 = w[e] - ext[n][e];
                lhs += a * a;
                rhs += c2 * c2;
            }
            delta[n] = parzen ? (lhs < rhs) : 1;
            if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) flags |= 256;
            ndelta += delta[n];
        }
        flags |= ndelta;
        /* Eq. 6 (one buffer: Eq. 7; gate off: Eq. 3) with the mini-batch gradient, then Alg. 5, update. */
        for (size_t e = 0; e < kd; ++e) {
            double Gbar = G[e];
            if (ndelta > 0) {
                double sum = w[e];
                for (int n = 0; n < next; ++n)
                    if (delta[n]) sum += ext[n][e];
                Gbar += w[e] - sum / (double)(ndelta + 1);
            }
            wnew[e] = w[e] - eps * Gbar;
        }
    }
    free(cnt);
    free(Ssum);
    free(G);
    return flags;
}

/*
 * Advance all W workers by nsteps mini-batch steps in lockstep.
 *
 * X           N x d fp32 row-major; shard i = rows [i*H, (i+1)*H), H = floor(N/W)
 * w           W*k*d fp64 states, in/out
 * nb          external buffers per worker = recipients per message (1 <= nb <= 255, nb < W or W == 1)
 * parts       P of the partial messages (1 = whole states; 1 <= P <= k)
 * slot        nb*W*k*d fp64 external buffers, buffer n of worker i at (n*W + i)*k*d, in/out
 *             (all-zero = empty, Eq. 3)
 * slot_stamp  nb*W round numbers of the buffered messages (-1 = none), in/out
 * ncum        W*k cumulative assignment counts (lr_mode 1 only), in/out
 * t_io        global step counter shared by all workers, in/out
 * counters    W*3: sending rounds, messages looked at, messages merged ("good" messages), in/out
 * near        2 counters: argmin near-ties, Parzen near-ties, in/out
 * parzen_near_w  optional W counters: Parzen near-ties per worker (steps of that worker with a flagged test), in/out
 * assign_out  optional nsteps*W*b assignments, step-major then worker then sample
 * gap_out     optional, same shape: (d2-d1)/d1 of each assignment
 * lr_mode     0 = constant eps, 1 = per-centroid 1/count (requires E == 0)
 * returns 0, or -1 on invalid arguments
 */
int asgd_oracle_steps(const float *X, int64_t N, int k, int d, int W, int b, double eps, int E, int nb, int parts,
                      uint64_t seed, int parzen, int lr_mode, uint32_t drop_threshold,
                      int64_t nsteps, double *w, double *slot, int64_t *slot_stamp, int64_t *ncum,
                      int64_t *t_io, int64_t *counters, int64_t *near, int64_t *parzen_near_w, int32_t *assign_out,
                      double *gap_out)
{
    if (k < 1 || d < 1 || W < 1 || b < 1 || !(eps > 0.0) || E < 0) return -1;
    const int64_t H = N / W;           /* Alg. 5, partition of the data */
    const int64_t S = H / b;           /* full mini-batches per epoch */
    if (H < k || S < 1) return -1;
    if (lr_mode == 1 && E != 0) return -1;
    if (nb < 1 || nb > 255 || (W > 1 && nb > W - 1)) return -1;
    if (parts < 1 || parts > k) return -1;
    const size_t kd = (size_t)k * d;
    double *wnew = (double *)malloc((size_t)W * kd * sizeof(double));
    int *flags = (int *)malloc((size_t)W * sizeof(int));
    int *looked = (int *)malloc((size_t)W * sizeof(int));
    int64_t *near_w = (int64_t *)calloc((size_t)W, sizeof(int64_t));
    int64_t t = *t_io;

    for (int64_t n = 0; n < nsteps; ++n, ++t) {
        const int64_t s = t % S;       /* position inside the epoch */
        const int merge_point = (E > 0 && t > 0 && t % E == 0);
#pragma omp parallel for schedule(static)
        for (int i = 0; i < W; ++i) {
            const float *M = X + ((size_t)i * H + (size_t)s * b) * d;
            const double *ext[256];
            int extpart[256];
            int next = 0;
            for (int n = 0; merge_point && n < nb; ++n) {
                const double *buf = slot + ((size_t)n * W + i) * kd;
                if (slot_stamp[(size_t)n * W + i] != t / E - 1) continue;
                const int part = (int)((t / E - 1 + i + n) % parts);    /* which rows the copy carries */
                double nrm = 0.0;
                for (int c = 0; c < k; ++c) {
                    if (c % parts != part) continue;
                    for (int j = 0; j < d; ++j) nrm += buf[(size_t)c * d + j] * buf[(size_t)c * d + j];
                }
                if (nrm > 0.0) { extpart[next] = part; ext[next++] = buf; }       /* lambda of Eq. 3 */
            }
            looked[i] = next;
            int32_t *ao = assign_out ? assign_out + ((size_t)n * W + i) * b : NULL;
            double *go = gap_out ? gap_out + ((size_t)n * W + i) * b : NULL;
            flags[i] = worker_step(M, b, k, d, eps, lr_mode, parzen, w + i * kd, wnew + i * kd, ext, next, parts,
                                   extpart, ncum + (size_t)i * k, ao, go, &near_w[i]);
        }
        for (int i = 0; i < W; ++i) {
            counters[i * 3 + 1] += looked[i];
            counters[i * 3 + 2] += flags[i] & 255;
            if (flags[i] & 256) {
                near[1] += 1;
                if (parzen_near_w) parzen_near_w[i] += 1;
            }
        }
        if (merge_point) {               /* a buffer is looked at once, then emptied */
            memset(slot, 0, (size_t)nb * W * kd * sizeof(double));
            for (size_t q = 0; q < (size_t)nb * W; ++q) slot_stamp[q] = -1;
        }
        memcpy(w, wnew, (size_t)W * kd * sizeof(double));
        if (E > 0 && W > 1 && (t + 1) % E == 0) {       /* Alg. 5, send */
            const int64_t r = t / E;
            for (int i = 0; i < W; ++i) {
                counters[i * 3 + 0] += 1;
                for (int n = 0; n < nb; ++n) {
                    if (asgd_oracle_dropped_n(seed, r, i, n, drop_threshold)) continue;
                    int64_t p = asgd_oracle_peer_n(seed, r, i, W, n);
                    const int part = (int)((r + p + n) % parts);
                    for (int c = 0; c < k; ++c)            /* only the rows of the part travel */
                        if (c % parts == part)
                            memcpy(slot + ((size_t)n * W + p) * kd + (size_t)c * d, w + i * kd + (size_t)c * d,
                                   (size_t)d * sizeof(double));
                    slot_stamp[(size_t)n * W + p] = r;
                }
            }
        }
    }
    for (int i = 0; i < W; ++i) near[0] += near_w[i];
    *t_io = t;
    free(wnew);
    free(flags);
    free(looked);
    free(near_w);
    return 0;
}
