// Internal declarations shared by the translation units of the HIP library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "asgd.h"
#include "exchange_index.h"

namespace asgd {

enum { MAX_BUFFERS = 4 };   // external buffers per worker (Eq. 3)

// Per-worker counters kept in device memory.
enum { CNT_SENT = 0, CNT_RECEIVED = 1, CNT_ACCEPTED = 2, CNT_PARZEN_NEAR = 3, CNT_RECHECK = 4, CNT_STRIDE = 8 };

// Everything a step kernel needs; passed by value.
struct StepParams {
    const float *x;        // N x d samples
    float *w;              // W x k x d states
    float *slot;           // 2 x nb x W exchange buffers (parity, buffer, worker): k x d floats, or the small-state kernel's pairs
    int *stamp;            // 2 x nb x W round number of the buffered message, -1 = empty
    int *consumed;         // W: last round whose merge point the worker has passed
    long long *ncum;       // W x k cumulative counts (1/count step size only)
    long long *counters;   // W x CNT_STRIDE
    float *acc;            // W x k x d gradient-sum scratch (generic/large kernels)
    int *cnt;              // W x k count scratch
    int *assign_tmp;       // W x b assignment scratch
    int32_t *dump;         // optional assignment dump (step-major), or nullptr
    const float *xabsmax;  // d per-dimension max |x| over the loaded samples
    int *error_flag;       // pinned host memory, set to 1 by a kernel whose bounded wait expired
    const int *shift_tab;  // deterministic schedule: cyclic shift of round r at [r - shift_r0] (small-state kernel)
    long long shift_r0;
    long long H, S;        // shard length, steps per epoch
    long long t_dump0;     // step counter value at which the dump buffer starts
    uint64_t seed;
    int k, d, W, b, E;
    int nb;                // external buffers per worker = recipients per message (Eq. 3), 1 .. MAX_BUFFERS
    int parts;             // partial messages: a copy carries the centroid rows of one of `parts` parts (1: whole state)
    float eps;
    int parzen, lr_mode, mode;
    uint32_t drop_thr;
    int tune;              // variant selector for experiments (0 = default)
    int cooperative;       // use the cooperative launch API for single-launch runs
    int wait_polls;        // polls a workgroup may spend on all the waits of a launch (test hook; 0 = the kernel's default)
    int drop_unannounced;  // test hook: the recipient does not know which messages the loss hook drops and waits for them
};

// Launchers (each returns the hipError_t of its launch).
hipError_t launch_init_first_k(const StepParams &p, hipStream_t s);
hipError_t launch_absmax(const float *x, long long rows, int d, float *out, hipStream_t s);
hipError_t launch_generic_steps(const StepParams &p, long long t0, long long t1, hipStream_t s);
bool small_kernel_supports(int k, int d, int b);
// bytes of one exchange buffer in the small-state kernel's own message format (0: kernel not applicable)
size_t small_kernel_message_bytes(int k, int d);
// host side of that format: rows = k x d floats, row_round[c] = round stamped on row c (-1: row empty or torn)
void small_kernel_unpack_message(int k, int d, const void *msg, float *rows, int *row_round);
void small_kernel_pack_message(int k, int d, const float *rows, const int *row_round, void *msg);
// persistent = true: the whole range in one cooperative launch with in-kernel waits between rounds
hipError_t launch_small_steps(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent);
// Matrix-core kernel: needs d % 4 == 0, d <= 128, 16-byte aligned samples and its LDS budget.
bool mfma_kernel_supports(int k, int d, int b, const void *x);
hipError_t launch_rownorm2max(const float *x, long long rows, int d, float *out, hipStream_t s);   // max_n |x_n|^2
// persistent = true: as for the small-state kernel (deterministic mode; hipErrorCooperativeLaunchTooLarge when the
// workers do not all fit the device at once)
hipError_t launch_mfma_steps(const StepParams &p, long long t0, long long t1, const float *xnorm2max, hipStream_t s,
                             bool persistent);
// shift_tab[q] = 1 + round_hash(seed, r0 + q) % (W - 1) for q in [0, n)
hipError_t launch_schedule_table(uint64_t seed, long long r0, int n, int W, int *shift_tab, hipStream_t s);
hipError_t launch_mean_state(const float *w, int W, int kd, float *out, hipStream_t s);
// Eq. 8 over rows [0, N): partials is scratch of quant_partials_count() doubles.
int quant_partials_count();
// specialisations of Eq. 8 (each fills `nblocks` <= quant_partials_count() partial sums; the generic launcher
// below picks one and adds the partials in a fixed order)
hipError_t launch_quant_error_small(const float *x, long long N, int d, int k, const float *w, double *partials, int nblocks,
                                    hipStream_t s);   // shapes of small_kernel_supports()
bool mfma_quant_error_supports(int k, int d, const void *x);
hipError_t launch_quant_error_mfma(const float *x, long long N, int d, int k, const float *w, double *partials,
                                   int nblocks, hipStream_t s);
hipError_t launch_quant_error(const float *x, long long N, int d, int k, const float *w, double *partials,
                              double *out, hipStream_t s);

}  // namespace asgd
