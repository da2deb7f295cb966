/*
 * asgd.h — C ABI of the MI355X (gfx950) ASGD mini-batch K-Means library.
 *
 * The library runs W independent SGD workers on one GPU.  Every worker streams its
 * own shard of fp32 samples through mini-batch K-Means steps (nearest prototype,
 * per-centroid gradient, update) and every E steps sends its state to one other
 * worker, whose next step merges it under the paper's Parzen-window rule.
 *
 * Conventions
 *   - every function returns ASGD_OK (0) or a negative ASGD_E* code; nothing throws
 *     or aborts across this boundary; asgd_strerror() names a code;
 *   - "device pointer" = HIP device memory of the current device, "host pointer" =
 *     ordinary host memory; the library never frees caller memory;
 *   - a context belongs to the device that was current in asgd_create(); calls on
 *     one context must not overlap in time (one context per host thread);
 *   - there is no CPU fallback: without a usable HIP device the calls fail.
 *
 * Notation: k centroids, d dimensions, W workers, b mini-batch size, eps step size,
 * E exchange interval, H = floor(N / W) shard length, S = floor(H / b) steps per
 * epoch, t = step counter (the same for all workers, it continues across epochs and
 * across calls), round r = floor(t / E).
 */
#ifndef ASGD_H
#define ASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asgd_ctx asgd_ctx; /* opaque: worker states, exchange buffers, counters */

enum {
    ASGD_OK = 0,
    ASGD_EINVAL = -1,   /* bad argument (null pointer, size out of range, unknown option) */
    ASGD_ENOMEM = -2,   /* device or host allocation failed */
    ASGD_ESTATE = -3,   /* call out of order (e.g. run before load_shards) */
    ASGD_EHIP = -4,     /* a HIP runtime call failed; asgd_last_hip_error() has its code */
    ASGD_ESYNC = -5     /* a bounded wait inside a kernel expired (runs that are one launch of workgroups
                           which wait for each other's messages; all the waits of a workgroup draw on one
                           budget of polls that grows with the rounds of the launch, and a launch covers
                           at most 1024 rounds, so such a launch ends within a second plus a few
                           milliseconds per round of waiting).  The run is lost: the step counter is not advanced and later runs
                           fail with ASGD_ESTATE until asgd_load_shards(), or asgd_set_state() followed by
                           asgd_set_step(), have put the context back on a known footing. */
};

/* Keys of asgd_set_option().  Values are passed as double and rounded to integers
   where an integer is meant. */
enum {
    ASGD_OPT_EXCHANGE_EVERY = 1, /* E >= 0; 0 = never send: silent mode = SimuParallelSGD with
                                    mini-batches (Sec. 4, first paragraph; Sec. 5.4 "silent");
                                    E = 1 is Alg. 5 as printed.  Default 0. */
    ASGD_OPT_SEED = 2,           /* seed of the peer schedule (integer < 2^53).  Default 1. */
    ASGD_OPT_MODE = 3,           /* ASGD_MODE_*.  Default deterministic. */
    ASGD_OPT_PARZEN = 4,         /* 1 = gate merges with Eq. 4 (default), 0 = delta = 1 (Eq. 2) */
    ASGD_OPT_LR_MODE = 5,        /* ASGD_LR_*.  Default constant. */
    ASGD_OPT_DROP_RATE = 6,      /* test hook: probability in [0,1] that a message is lost on
                                    the way (Sec. 4.4: a lost message is harmless).  Default 0. */
    ASGD_OPT_KERNEL = 7,         /* ASGD_KERNEL_*: which implementation runs the steps.
                                    Default auto.  All give the same results to rounding.  The kernels keep
                                    messages in flight in different formats; when the kernel changes between
                                    two runs the library carries them over (see asgd_get_exchange). */
    ASGD_OPT_TUNE = 8,           /* launch-shape variant of the chosen kernel (0 = default); for
                                    performance experiments: the variants compute the same thing and may
                                    differ in the rounding of their sums */
    ASGD_OPT_COOPERATIVE = 9,    /* 1 (default): a run that needs all its workgroups resident at the
                                    same time is started with a cooperative launch, which refuses
                                    grids that cannot be; 0: plain launch of the same grid (for tools
                                    that cannot follow cooperative launches).  The in-kernel waits are
                                    bounded either way. */
    ASGD_OPT_BUFFERS = 10,       /* N of Eq. 3 / Eq. 6: external buffers per worker, 1 (default) .. 4.  A
                                    worker then sends every message to N different workers (copy n goes
                                    into the recipient's buffer n; deterministic schedule: a cyclic shift
                                    per round and copy, so every worker receives N messages per round from
                                    N different senders) and merges, of the buffers that hold a message,
                                    those that pass Eq. 4 on their own: w - (sum of them + w)/(their
                                    number + 1) is added to the step.  With ASGD_OPT_PARZEN = 0 every
                                    non-empty buffer takes part (Eq. 3).  Needs N < W at run time
                                    (ASGD_EINVAL otherwise); may only be set before the first step
                                    (ASGD_ESTATE after); reallocates the exchange buffers (2 * N * W states).
                                    Available in all three kernels. */
    ASGD_OPT_PARTS = 11          /* partial messages (Sec. 4.4, partitioned along the cluster centres):
                                    P in 1 .. k, default 1 = whole states.  With P > 1 part q is the set of
                                    centroid rows c with c mod P = q, and copy n of the message of round r
                                    to worker p carries part (r + p + n) mod P only (1/P of the bytes); the
                                    recipient treats every transmitted row as a unit of its own: empty iff
                                    all zero, tested by Eq. 4 over that row, merged by Eq. 6 with the other
                                    buffers' accepted copies of the same row; rows that did not travel take
                                    the plain step.  "received" then counts buffers with a non-empty row,
                                    "accepted" buffers with an accepted row.  May only be set before the
                                    first step (ASGD_ESTATE after).  Available in all three kernels; in the
                                    matrix-core kernel only while W*k*d <= ASGD_MFMA_PARTS_MAX_STATE (the sizes
                                    its tests cover: the only batch of larger runs of that combination ended in
                                    a device fault that was never explained).  Above that the automatic choice
                                    takes the shape-agnostic kernel and an explicit ASGD_KERNEL_MFMA fails with
                                    ASGD_EINVAL. */
};
enum { ASGD_MFMA_PARTS_MAX_STATE = 1 << 18 };
enum {
    ASGD_OPT_WAIT_POLLS = 12,       /* test hook: polls a workgroup may spend, in total, on the waits of one launch
                                       (0 = the library's default of some 10^5, i.e. a fraction of a second) */
    ASGD_OPT_DROP_UNANNOUNCED = 13  /* test hook: 1 = the recipient does not know which messages ASGD_OPT_DROP_RATE
                                       loses, so a run that is one launch waits for them until its poll budget is
                                       gone and then returns ASGD_ESYNC (every kernel still ends normally); 0 (default):
                                       a lost message is skipped at once */
};
enum { ASGD_MODE_DETERMINISTIC = 0, ASGD_MODE_FREE_RUNNING = 1 };
enum { ASGD_LR_CONST = 0, ASGD_LR_INV_COUNT = 1 };
enum { ASGD_KERNEL_AUTO = 0, ASGD_KERNEL_GENERIC = 1, ASGD_KERNEL_SMALL = 2, ASGD_KERNEL_MFMA = 3 };

typedef struct asgd_stats {
    int64_t steps;            /* value of the step counter t */
    int64_t samples;          /* samples processed so far = t * W * b */
    int64_t sent;             /* messages written, summed over workers (Alg. 5, send) */
    int64_t received;         /* messages found in a buffer and tested with Eq. 4 */
    int64_t accepted;         /* of those, messages with delta = 1 ("good" messages, Sec. 5.4) */
    int64_t parzen_near_ties; /* tested messages with |lhs - rhs| / rhs < 1e-6 in Eq. 4 */
    int64_t exact_rechecks;   /* samples whose two best fp32 scores were too close to call and
                                 whose assignment was therefore recomputed in fp64 */
    double last_run_ms;       /* device time of the last asgd_run_* call (HIP events) */
    int32_t kernel;           /* ASGD_KERNEL_* that the last run used */
    int32_t launches;         /* kernel launches of the last run */
} asgd_stats;

/*
 * Create a context for the problem of Sec. 5.1 (k prototypes for points in R^d) run by
 * Alg. 5 with W workers ("nodes"), mini-batch size b and step size eps = lr.
 * Requires k, d, W, b >= 1 and lr > 0 (Alg. 5 "Require"; W = 1 is allowed and equals
 * Alg. 4).  Allocates W*k*d floats of state and the exchange buffers on the current
 * device.  *out is set only on success and must be released with asgd_destroy().
 */
int asgd_create(asgd_ctx **out, int k, int d, int W, int b, float lr);

/* Set one option (see the key list).  Allowed at any time between runs. */
int asgd_set_option(asgd_ctx *ctx, int key, double value);

/*
 * Hand the samples to the workers (Sec. 4 "Initialization": the data is split into
 * packages, one per worker; Alg. 5 lines 1-2).
 *   x_dev       device pointer, N x d fp32 row-major, at least 8-byte aligned.  BORROWED:
 *               the caller keeps it alive and unchanged until asgd_destroy() or the
 *               next asgd_load_shards().
 *   N           number of rows; worker i owns rows [i*H, (i+1)*H), the last N mod W rows
 *               are not used by the optimisation.  Requires H >= max(k, b).
 *   hip_stream  a hipStream_t (0 = default stream) on which this and all later calls of
 *               the context enqueue their work.
 * Effects: every worker's state is set to the first k rows of its own shard, exchange
 * buffers, counters and the step counter are cleared.  Synchronises the stream.
 */
int asgd_load_shards(asgd_ctx *ctx, const float *x_dev, int64_t N, void *hip_stream);

/*
 * Overwrite worker states from host memory: w_host holds k*d floats (worker >= 0 sets
 * that worker, worker = -1 gives the same w0 to all workers, Sec. 4 "Initialization") or
 * W*k*d floats (worker = -2 sets each worker from its own block).  Needed to continue an
 * earlier run (Sec. 4: w0 may be the result of a run that was stopped early).
 */
int asgd_set_state(asgd_ctx *ctx, int worker, const float *w_host);

/* Set the step counter t (>= 0) when continuing an earlier run.  Exchange buffers are
   emptied: at a multiple of E the messages of the round just finished are in flight
   (Alg. 5: sent at the end of one step, looked at in the merge of the next), so a run resumed
   there equals the uninterrupted one only if asgd_set_exchange() hands them over too. */
int asgd_set_step(asgd_ctx *ctx, int64_t t);

/*
 * The messages in flight (Alg. 5 lines 5 and 9, Eq. 3 / Eq. 6: N external buffers per
 * worker; Sec. 4 "Initialization": a run may start from the result of an earlier one), in
 * a layout that does not depend on the kernel that ran:
 *   values_host  float [buffers][W][k][d], host memory: the rows waiting in buffer n of
 *                worker i; rows that a partial message (Sec. 4.4) does not carry, and
 *                empty buffers, are zeros.
 *   rounds_host  int32 [buffers][W], host memory: the round the message was sent in,
 *                -1 = nothing waiting.
 * Deterministic mode: messages wait exactly when t is a positive multiple of E, and all
 * carry round t/E - 1; anywhere else every entry is -1.  Free-running mode: whatever the
 * buffers hold at this moment (the newest message of a buffer; its rows only).
 * asgd_get_exchange() copies them out (sizes in bytes are checked: ASGD_EINVAL if too
 * small).  asgd_set_exchange() is called after asgd_set_state() and asgd_set_step(t) of a
 * continued run; the library keeps a host copy until the next run, which writes it into
 * the buffers in its kernel's format.  A deterministic run continued this way at a merge
 * point is bit-identical to the uninterrupted run.  ASGD_EINVAL: a round that cannot wait
 * at step t (deterministic mode: anything but -1 and t/E - 1 at a merge point).
 * The same conversion happens by itself when ASGD_OPT_KERNEL changes between two runs.
 */
int asgd_get_exchange(asgd_ctx *ctx, float *values_host, size_t values_bytes, int32_t *rounds_host, size_t rounds_bytes);
int asgd_set_exchange(asgd_ctx *ctx, const float *values_host, const int32_t *rounds_host);

/*
 * Run `epochs` passes over every shard: epochs * S steps of Alg. 5 lines 6-10 per
 * worker, mini-batch s of an epoch being rows [s*b, (s+1)*b) of the shard (the tail
 * H mod b is skipped).  A step = assignment s_i(w) (Sec. 5.1), gradient (Eq. 9 with
 * m' = b), merge of a buffered external state when t > 0 and t mod E == 0 (Eq. 4,
 * Eq. 7), update w <- w - eps * step (Alg. 5, update) and, when (t+1) mod E == 0, the
 * send of the new state to one other worker (Alg. 5, send).  Returns after the work
 * has finished on the device.  The result does not depend on how a run is cut into
 * calls (deterministic mode: bit for bit), the time does: where all workers fit the
 * device at once, a call is ONE kernel launch for every 1024 communication rounds it
 * covers, and the start and the tail of a launch are then paid once per launch, not once
 * per epoch (asgd_stats.launches).
 */
int asgd_run_epochs(asgd_ctx *ctx, int epochs);

/* Same, for an arbitrary number of steps (continues inside an epoch). */
int asgd_run_steps(asgd_ctx *ctx, int64_t steps);

/*
 * Test aid: record the assignment s_i of every sample processed by later runs.
 *   assign_dev  device pointer to capacity int32 values, BORROWED, or NULL to stop.
 * A run of n steps writes n*W*b values, step-major, then worker, then position in the
 * mini-batch, and fails with ASGD_EINVAL if that exceeds `capacity`.
 */
int asgd_set_assign_dump(asgd_ctx *ctx, int32_t *assign_dev, size_t capacity);

/*
 * Copy states to host memory.  worker >= 0: that worker's k*d floats (worker 0 is the
 * result Alg. 5, return returns); worker = -1: all W states, W*k*d floats.
 * out_bytes must be at least the size copied.
 */
int asgd_get_state(asgd_ctx *ctx, int worker, float *out_host, size_t out_bytes);

/*
 * The mean of the W worker states (the alternative final aggregation of Sec. 4.3),
 * k*d floats, computed on the device in worker order.
 */
int asgd_get_mean_state(asgd_ctx *ctx, float *out_host, size_t out_bytes);

/*
 * Quantization error of Eq. 8, E(w) = sum_i 1/2 * min_k |x_i - w_k|^2, over all N loaded
 * rows for the state of `worker` (>= 0) or the mean state (worker = -1).  fp32: the nearest
 * centroid of a sample is found from expanded-form scores x.w_c - |w_c|^2/2 (any shape but the
 * smallest ones: on the matrix cores), the distance to it is then formed directly as
 * sum_j (x_j - w_cj)^2, so clusters far from the origin lose nothing to cancellation; the sum
 * over the samples is fp64 in a fixed order.  *out is host memory.
 */
int asgd_quant_error(asgd_ctx *ctx, int worker, double *out);

/*
 * Eq. 8 without a context and without any allocation, for callers that cannot call hipMalloc: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same kernels and the same result as
 * asgd_quant_error(); the partial sums of the reduction live in a static device array of the library (16 KB on every
 * GPU the library runs on, held until the process ends) instead of a context's scratch.
 *   x_dev    device pointer, N x d fp32 row-major, at least 8-byte aligned (BORROWED for the duration of the work)
 *   w_dev    device pointer, k x d fp32 state
 *   out_dev  device pointer to ONE double, 8-byte aligned: receives E(w) when the work enqueued on `hip_stream`
 *            (a hipStream_t, 0 = default stream) has finished; the call itself does not wait
 * Limits: N <= 2^40, d <= 65536, k*d <= 2^24; anything larger, a null pointer or a misaligned one gives ASGD_EINVAL
 * and nothing is enqueued.  Calls neither hipMalloc/hipFree nor any routine that allocates (the first call on a
 * device looks up the address of the static array, nothing more).  All calls on one GPU share that array: calls that
 * overlap in time on one GPU (different streams or threads) race on it; calls on one stream are ordered and safe.
 * The array keeps the last call's partial sums; every call overwrites all it reads, so nothing is cleared.
 */
int asgd_quant_error_noalloc(const float *x_dev, int64_t N, int k, int d, const float *w_dev, double *out_dev,
                             void *hip_stream);

/* Device time in milliseconds of the last asgd_run_* call, measured with HIP events recorded on
   the context's stream around its kernel launches.  No device access. */
int asgd_last_run_ms(asgd_ctx *ctx, double *out);

/* Totals since asgd_load_shards(). */
int asgd_get_stats(asgd_ctx *ctx, asgd_stats *out);

/* Per-worker message counters (Sec. 5.4, "messages sent or received by a single CPU"):
   each array receives W values; any pointer may be NULL. */
int asgd_get_worker_counters(asgd_ctx *ctx, int64_t *sent, int64_t *received, int64_t *accepted);

/* Recipient of worker i's message of round r under the deterministic schedule
   (host-side copy of what the kernels compute; W >= 2); _n: of copy n of it, 0 <= n < W - 1
   (ASGD_OPT_BUFFERS; copy 0 is the one-buffer schedule).  -1 on invalid arguments. */
int64_t asgd_schedule_peer(uint64_t seed, int64_t r, int64_t i, int64_t W);
int64_t asgd_schedule_peer_n(uint64_t seed, int64_t r, int64_t i, int64_t W, int64_t n);

/* hipError_t of the last failed HIP call of this context (0 if none). */
int asgd_last_hip_error(asgd_ctx *ctx);

/* Release the context and everything it allocated (not the samples, not the dump). */
void asgd_destroy(asgd_ctx *ctx);

/* Static description of a return code. */
const char *asgd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ASGD_H */
