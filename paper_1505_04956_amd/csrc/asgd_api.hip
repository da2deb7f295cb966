// Host side of the C ABI declared in asgd.h: argument checks, device memory of a context,
// splitting of a run into launches, timing, copies to and from the host.
#include <math.h>
#include <new>
#include <string.h>
#include <vector>

#include "asgd_internal.h"

using namespace asgd;

struct asgd_ctx {
    int k = 0, d = 0, W = 0, b = 0;
    float lr = 0.f;
    int E = 0;
    uint64_t seed = 1;
    int mode = ASGD_MODE_DETERMINISTIC;
    int parzen = 1;
    int lr_mode = ASGD_LR_CONST;
    double drop_rate = 0.0;
    int kernel_opt = ASGD_KERNEL_AUTO;
    int tune = 0;
    int nb = 1;                 // external buffers per worker
    int parts = 1;              // partial messages: parts of a state (1 = whole states)
    size_t slot_bytes_one = 0;  // bytes of both parities of ONE buffer per worker
    int cooperative = 1;
    int wait_polls = 0;
    int drop_unannounced = 0;

    int device = 0;
    hipStream_t stream = nullptr;
    bool loaded = false;
    const float *x = nullptr;
    long long N = 0, H = 0, S = 0;
    long long t = 0;

    float *w = nullptr, *slot = nullptr, *acc = nullptr, *xabsmax = nullptr, *mean = nullptr;
    float *xnorm2max = nullptr;    // matrix-core kernel only, allocated on first use
    size_t slot_bytes = 0;         // size of the exchange buffers (both parities, all workers)
    int *shift_tab = nullptr;      // schedule table of the small-state kernel, grown on demand
    long long shift_cap = 0;
    long long tab_r0 = 0, tab_n = 0;   // rounds [tab_r0, tab_r0 + tab_n) the table holds, for tab_seed and tab_W
    uint64_t tab_seed = 0;
    int tab_W = 0;
    bool xnorm2max_valid = false;
    int *stamp = nullptr, *consumed = nullptr, *cnt = nullptr, *assign_tmp = nullptr;
    // Error flag of the kernels (an expired bounded wait), in pinned host memory that the device writes directly: the
    // host clears and reads it around a run without a memset or a copy on the stream (each is a separate operation
    // of several microseconds, which counts when a run is one launch of less than a millisecond).
    int *flag_host = nullptr;
    long long *ncum = nullptr, *counters = nullptr;
    double *qpart = nullptr, *qout = nullptr;
    int32_t *dump = nullptr;
    size_t dump_cap = 0;

    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    double last_ms = 0.0;
    int last_kernel = 0, last_launches = 0;
    long long passed_t = -1;    // step up to which `consumed` holds what a one-launch run needs (-1: unknown)
    int fill_kernel = 0;        // kernel whose message format the exchange buffers were last emptied for
    bool desynced = false;      // a bounded wait expired in the last run: states and buffers are not those of any step
    // messages handed over by asgd_set_exchange(), kept until the next run knows which kernel's format they take
    std::vector<float> pending_values;
    std::vector<int32_t> pending_rounds;
    bool pending = false;
    int hip_err = 0;
};

namespace {

// rounds one launch with in-kernel waits covers at most (a longer call becomes several such launches)
constexpr long long ONE_LAUNCH_MAX_ROUNDS = 1024;

#define HIP_TRY(ctx, call)                              \
    do {                                                \
        hipError_t e__ = (call);                        \
        if (e__ != hipSuccess) {                        \
            (ctx)->hip_err = (int)e__;                  \
            return e__ == hipErrorOutOfMemory ? ASGD_ENOMEM : ASGD_EHIP; \
        }                                               \
    } while (0)

size_t kd_of(const asgd_ctx *c) { return (size_t)c->k * c->d; }

void free_all(asgd_ctx *c)
{
    void *ptrs[] = {c->w, c->slot, c->acc, c->xabsmax, c->mean, c->stamp, c->consumed, c->cnt, c->assign_tmp,
                    c->ncum, c->counters, c->qpart, c->qout, c->xnorm2max, c->shift_tab};
    for (void *q : ptrs)
        if (q) (void)hipFree(q);
    if (c->flag_host) (void)hipHostFree(c->flag_host);
    if (c->ev0) (void)hipEventDestroy(c->ev0);
    if (c->ev1) (void)hipEventDestroy(c->ev1);
}

StepParams make_params(const asgd_ctx *c)
{
    StepParams p;
    memset(&p, 0, sizeof(p));
    p.x = c->x; p.w = c->w; p.slot = c->slot; p.stamp = c->stamp; p.consumed = c->consumed; p.ncum = c->ncum;
    p.counters = c->counters; p.acc = c->acc; p.cnt = c->cnt; p.assign_tmp = c->assign_tmp;
    p.dump = c->dump; p.xabsmax = c->xabsmax; p.error_flag = c->flag_host;
    p.H = c->H; p.S = c->S; p.t_dump0 = c->t; p.seed = c->seed;
    p.k = c->k; p.d = c->d; p.W = c->W; p.b = c->b; p.E = c->E; p.eps = c->lr; p.nb = c->nb; p.parts = c->parts;
    p.parzen = c->parzen; p.lr_mode = c->lr_mode; p.mode = c->mode;
    p.drop_thr = (uint32_t)llround(c->drop_rate * (double)(1u << 24));
    p.tune = c->tune;
    p.cooperative = c->cooperative;
    p.wait_polls = c->wait_polls;
    p.drop_unannounced = c->drop_unannounced;
    return p;
}

// Empties the exchange buffers for the kernel that is going to use them.  Small-state kernel: all bits set = stamp -1
// inside its (value, stamp) pairs.  The other kernels look at `stamp` before they read a buffer; with partial messages
// rows of a buffer stay unwritten, which a free-running recipient may look at: those start as zeros = empty rows.
int clear_exchange(asgd_ctx *c, int kernel)
{
    const int fill = (c->parts > 1 && kernel != ASGD_KERNEL_SMALL) ? 0 : 0xFF;
    HIP_TRY(c, hipMemsetAsync(c->slot, fill, c->slot_bytes, c->stream));
    HIP_TRY(c, hipMemsetAsync(c->stamp, 0xFF, exchange_buffers_total(c->nb, c->W) * sizeof(int), c->stream));   // -1
    c->fill_kernel = kernel;
    return ASGD_OK;
}

// ---- messages in flight, in a format of their own -------------------------------------------------------------
// Logical content of the exchange buffers: values[n][i] = the k x d rows waiting in buffer n of worker i (rows that a
// partial message does not carry: zeros), rounds[n][i] = the round it was sent in, -1 = nothing waiting.  The
// kernels hold this in two device formats: plain rows + a stamp per buffer (shape-agnostic and matrix-core kernels),
// or (value, stamp) pairs in padded rows (small-state kernel).  Conversion runs on the host, in chunks of workers.

// parity of the buffers that hold what the next merge point reads, and the round those messages carry (-1: none can)
void inflight(const asgd_ctx *c, int *parity, long long *round)
{
    const bool det = c->mode == ASGD_MODE_DETERMINISTIC;
    *parity = 0;
    *round = -1;
    if (c->E <= 0 || c->W < 2 || c->t <= 0) return;
    if (!det) { *round = c->t / c->E - 1; return; }       // newest round that has sent; older stamps count too
    if (c->t % c->E != 0) return;                           // inside a round nothing is in flight
    *round = c->t / c->E - 1;
    *parity = (int)(*round & 1);
}

bool row_in_part(const asgd_ctx *c, int row, long long round, int worker, int n)
{
    return row_travels(row, round, worker, n, c->parts);
}

enum { EXCHANGE_CHUNK_BYTES = 32 << 20 };

int export_exchange(asgd_ctx *c, int kernel, float *values, int32_t *rounds)
{
    const size_t kd = kd_of(c), W = (size_t)c->W;
    const bool det = c->mode == ASGD_MODE_DETERMINISTIC;
    int par;
    long long r_want;
    inflight(c, &par, &r_want);
    for (size_t q = 0; q < (size_t)c->nb * W; ++q) rounds[q] = -1;
    memset(values, 0, (size_t)c->nb * W * kd * sizeof(float));
    if (r_want < 0 || kernel == 0) return ASGD_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const bool small = kernel == ASGD_KERNEL_SMALL;
    const size_t msg_bytes = small ? small_kernel_message_bytes(c->k, c->d) : kd * sizeof(float);
    const size_t per_chunk = EXCHANGE_CHUNK_BYTES / msg_bytes > 0 ? EXCHANGE_CHUNK_BYTES / msg_bytes : 1;
    std::vector<unsigned char> stage;
    std::vector<int> stamps, row_round;
    try {
        stage.resize((per_chunk < W ? per_chunk : W) * msg_bytes);
        stamps.resize(W);
        row_round.resize((size_t)c->k);
    } catch (...) {
        return ASGD_ENOMEM;
    }
    for (int n = 0; n < c->nb; ++n) {
        const size_t buf0 = exchange_buffer(par, c->nb, n, c->W, 0);
        if (!small)
            HIP_TRY(c, hipMemcpy(stamps.data(), c->stamp + buf0, W * sizeof(int), hipMemcpyDeviceToHost));
        for (size_t i0 = 0; i0 < W; i0 += per_chunk) {
            const size_t cnt = W - i0 < per_chunk ? W - i0 : per_chunk;
            HIP_TRY(c, hipMemcpy(stage.data(), (const unsigned char *)c->slot + (buf0 + i0) * msg_bytes, cnt * msg_bytes,
                                 hipMemcpyDeviceToHost));
            for (size_t q = 0; q < cnt; ++q) {
                const size_t i = i0 + q;
                float *out = values + ((size_t)n * W + i) * kd;
                long long st = -1;
                if (small) {
                    small_kernel_unpack_message(c->k, c->d, stage.data() + q * msg_bytes, out, row_round.data());
                    for (int row = 0; row < c->k; ++row)
                        if (row_round[row] > st) st = row_round[row];
                } else {
                    st = stamps[i];
                    if (st >= 0) memcpy(out, stage.data() + q * msg_bytes, kd * sizeof(float));
                }
                const bool there = det ? st == r_want : st >= 0;
                for (int row = 0; row < c->k; ++row) {
                    const bool keep = there && row_in_part(c, row, st, (int)i, n) && (!small || row_round[row] == st);
                    if (!keep) memset(out + (size_t)row * c->d, 0, (size_t)c->d * sizeof(float));
                }
                rounds[(size_t)n * W + i] = there ? (int32_t)st : -1;
            }
        }
    }
    return ASGD_OK;
}

// Writes the messages into the (freshly emptied) buffers in the format of `kernel`.
int import_exchange(asgd_ctx *c, int kernel, const float *values, const int32_t *rounds)
{
    const size_t kd = kd_of(c), W = (size_t)c->W;
    int par;
    long long r_want;
    inflight(c, &par, &r_want);
    if (r_want < 0) return ASGD_OK;
    const bool small = kernel == ASGD_KERNEL_SMALL;
    const size_t msg_bytes = small ? small_kernel_message_bytes(c->k, c->d) : kd * sizeof(float);
    const size_t per_chunk = EXCHANGE_CHUNK_BYTES / msg_bytes > 0 ? EXCHANGE_CHUNK_BYTES / msg_bytes : 1;
    std::vector<unsigned char> stage;
    std::vector<int> stamps, row_round;
    try {
        stage.resize((per_chunk < W ? per_chunk : W) * msg_bytes);
        stamps.resize(W);
        row_round.resize((size_t)c->k);
    } catch (...) {
        return ASGD_ENOMEM;
    }
    const int fill = (c->parts > 1 && !small) ? 0 : 0xFF;              // what clear_exchange() left in an empty buffer
    for (int n = 0; n < c->nb; ++n) {
        const size_t buf0 = exchange_buffer(par, c->nb, n, c->W, 0);
        for (size_t i0 = 0; i0 < W; i0 += per_chunk) {
            const size_t cnt = W - i0 < per_chunk ? W - i0 : per_chunk;
            for (size_t q = 0; q < cnt; ++q) {
                const size_t i = i0 + q;
                const long long st = rounds[(size_t)n * W + i];
                const float *in = values + ((size_t)n * W + i) * kd;
                unsigned char *dst = stage.data() + q * msg_bytes;
                stamps[i] = (int)st;
                if (small) {
                    for (int row = 0; row < c->k; ++row)
                        row_round[row] = (st >= 0 && row_in_part(c, row, st, (int)i, n)) ? (int)st : -1;
                    small_kernel_pack_message(c->k, c->d, in, row_round.data(), dst);
                } else if (st >= 0) {
                    memcpy(dst, in, kd * sizeof(float));
                } else {
                    memset(dst, fill, msg_bytes);
                }
            }
            HIP_TRY(c, hipMemcpy((unsigned char *)c->slot + (buf0 + i0) * msg_bytes, stage.data(), cnt * msg_bytes,
                                 hipMemcpyHostToDevice));
        }
        if (!small)
            HIP_TRY(c, hipMemcpy(c->stamp + buf0, stamps.data(), W * sizeof(int), hipMemcpyHostToDevice));
    }
    return ASGD_OK;
}

}  // namespace

extern "C" {

const char *asgd_strerror(int code)
{
    switch (code) {
        case ASGD_OK: return "success";
        case ASGD_EINVAL: return "invalid argument";
        case ASGD_ENOMEM: return "out of memory";
        case ASGD_ESTATE: return "call out of order";
        case ASGD_EHIP: return "HIP runtime error";
        case ASGD_ESYNC: return "bounded wait inside a kernel expired";
        default: return "unknown error code";
    }
}

int64_t asgd_schedule_peer_n(uint64_t seed, int64_t r, int64_t i, int64_t W, int64_t n)
{
    if (W < 2 || W > 0x7fffffff || i < 0 || i >= W || r < 0 || n < 0 || n >= W - 1) return -1;
    return peer_deterministic(seed, r, (int)i, (int)W, (int)n);
}

int64_t asgd_schedule_peer(uint64_t seed, int64_t r, int64_t i, int64_t W)
{
    if (W < 2 || i < 0 || i >= W || r < 0) return -1;
    return peer_deterministic(seed, r, (int)i, (int)W);
}

int asgd_create(asgd_ctx **out, int k, int d, int W, int b, float lr)
{
    if (!out || k < 1 || d < 1 || W < 1 || b < 1 || !(lr > 0.0f) || !isfinite(lr)) return ASGD_EINVAL;
    if ((double)k * d > (double)(1 << 28) || (double)W * k * d > 4e10) return ASGD_EINVAL;
    asgd_ctx *c = new (std::nothrow) asgd_ctx();
    if (!c) return ASGD_ENOMEM;
    c->k = k; c->d = d; c->W = W; c->b = b; c->lr = lr;
    int rc = ASGD_OK;
    auto fail = [&](hipError_t e) {
        c->hip_err = (int)e;
        rc = (e == hipErrorOutOfMemory) ? ASGD_ENOMEM : ASGD_EHIP;
    };
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { delete c; return ASGD_EHIP; }
    const size_t kd = kd_of(c), Wz = (size_t)W;
    {
        const size_t plain = kd * sizeof(float), own = small_kernel_message_bytes(k, d);
        c->slot_bytes_one = exchange_buffers_total(1, W) * (plain > own ? plain : own);
        c->slot_bytes = c->slot_bytes_one;
    }
    struct { void **p; size_t bytes; } allocs[] = {
        {(void **)&c->w, Wz * kd * sizeof(float)},
        {(void **)&c->slot, c->slot_bytes},
        {(void **)&c->acc, Wz * kd * sizeof(float)},
        {(void **)&c->xabsmax, (size_t)d * sizeof(float)},
        {(void **)&c->mean, kd * sizeof(float)},
        {(void **)&c->stamp, exchange_buffers_total(1, W) * sizeof(int)},
        {(void **)&c->consumed, Wz * sizeof(int)},
        {(void **)&c->cnt, Wz * k * sizeof(int)},
        {(void **)&c->assign_tmp, Wz * (size_t)b * sizeof(int)},
        {(void **)&c->ncum, Wz * k * sizeof(long long)},
        {(void **)&c->counters, Wz * CNT_STRIDE * sizeof(long long)},
        {(void **)&c->qpart, (size_t)quant_partials_count() * sizeof(double)},
        {(void **)&c->qout, sizeof(double)},
    };
    for (auto &a : allocs) {
        e = hipMalloc(a.p, a.bytes);
        if (e != hipSuccess) { fail(e); break; }
    }
    if (rc == ASGD_OK && (e = hipHostMalloc((void **)&c->flag_host, sizeof(int), hipHostMallocDefault)) != hipSuccess) fail(e);
    if (rc == ASGD_OK && (e = hipEventCreate(&c->ev0)) != hipSuccess) fail(e);
    if (rc == ASGD_OK && (e = hipEventCreate(&c->ev1)) != hipSuccess) fail(e);
    if (rc != ASGD_OK) {
        free_all(c);
        delete c;
        return rc;
    }
    *out = c;
    return ASGD_OK;
}

void asgd_destroy(asgd_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->stream || ctx->loaded) (void)hipStreamSynchronize(ctx->stream);
    free_all(ctx);
    delete ctx;
}

int asgd_last_hip_error(asgd_ctx *ctx) { return ctx ? ctx->hip_err : 0; }

int asgd_set_option(asgd_ctx *ctx, int key, double value)
{
    if (!ctx || !isfinite(value)) return ASGD_EINVAL;
    ctx->passed_t = -1;
    switch (key) {
        case ASGD_OPT_EXCHANGE_EVERY:
            if (value < 0 || value > 2e9 || value != floor(value)) return ASGD_EINVAL;
            ctx->E = (int)value;
            return ASGD_OK;
        case ASGD_OPT_SEED:
            if (value < 0 || value > 9007199254740992.0 || value != floor(value)) return ASGD_EINVAL;
            ctx->seed = (uint64_t)value;
            return ASGD_OK;
        case ASGD_OPT_MODE:
            if (value != ASGD_MODE_DETERMINISTIC && value != ASGD_MODE_FREE_RUNNING) return ASGD_EINVAL;
            ctx->mode = (int)value;
            return ASGD_OK;
        case ASGD_OPT_PARZEN:
            if (value != 0 && value != 1) return ASGD_EINVAL;
            ctx->parzen = (int)value;
            return ASGD_OK;
        case ASGD_OPT_LR_MODE:
            if (value != ASGD_LR_CONST && value != ASGD_LR_INV_COUNT) return ASGD_EINVAL;
            ctx->lr_mode = (int)value;
            return ASGD_OK;
        case ASGD_OPT_DROP_RATE:
            if (value < 0.0 || value > 1.0) return ASGD_EINVAL;
            ctx->drop_rate = value;
            return ASGD_OK;
        case ASGD_OPT_KERNEL:
            if (value != ASGD_KERNEL_AUTO && value != ASGD_KERNEL_GENERIC && value != ASGD_KERNEL_SMALL &&
                value != ASGD_KERNEL_MFMA)
                return ASGD_EINVAL;
            ctx->kernel_opt = (int)value;
            return ASGD_OK;
        case ASGD_OPT_COOPERATIVE:
            if (value != 0 && value != 1) return ASGD_EINVAL;
            ctx->cooperative = (int)value;
            return ASGD_OK;
        case ASGD_OPT_BUFFERS: {
            if (value < 1 || value > MAX_BUFFERS || value != floor(value)) return ASGD_EINVAL;
            if (ctx->t != 0) return ASGD_ESTATE;
            const int nb = (int)value;
            if (nb == ctx->nb) return ASGD_OK;
            HIP_TRY(ctx, hipSetDevice(ctx->device));
            HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
            float *slot = nullptr;
            int *stamp = nullptr;
            hipError_t e = hipMalloc((void **)&slot, (size_t)nb * ctx->slot_bytes_one);
            if (e == hipSuccess) e = hipMalloc((void **)&stamp, exchange_buffers_total(nb, ctx->W) * sizeof(int));
            if (e != hipSuccess) {
                if (slot) (void)hipFree(slot);
                HIP_TRY(ctx, e);
            }
            (void)hipFree(ctx->slot);
            (void)hipFree(ctx->stamp);
            ctx->slot = slot;
            ctx->stamp = stamp;
            ctx->slot_bytes = (size_t)nb * ctx->slot_bytes_one;
            ctx->nb = nb;
            return clear_exchange(ctx, ASGD_KERNEL_SMALL);
        }
        case ASGD_OPT_PARTS:
            if (value < 1 || value > ctx->k || value != floor(value)) return ASGD_EINVAL;
            if (ctx->t != 0) return ASGD_ESTATE;
            ctx->parts = (int)value;
            ctx->fill_kernel = 0;          // the first run empties the buffers for its kernel
            return ASGD_OK;
        case ASGD_OPT_WAIT_POLLS:
            if (value < 0 || value > (double)(1 << 24) || value != floor(value)) return ASGD_EINVAL;
            ctx->wait_polls = (int)value;
            return ASGD_OK;
        case ASGD_OPT_DROP_UNANNOUNCED:
            if (value != 0 && value != 1) return ASGD_EINVAL;
            ctx->drop_unannounced = (int)value;
            return ASGD_OK;
        case ASGD_OPT_TUNE:
            if (value < 0 || value > 1000 || value != floor(value)) return ASGD_EINVAL;
            ctx->tune = (int)value;
            return ASGD_OK;
        default:
            return ASGD_EINVAL;
    }
}

int asgd_load_shards(asgd_ctx *ctx, const float *x_dev, int64_t N, void *hip_stream)
{
    if (!ctx || !x_dev || N < 1) return ASGD_EINVAL;
    if (((uintptr_t)x_dev & 7u) != 0 || ctx->d > 65536) return ASGD_EINVAL;
    const long long H = N / ctx->W;
    if (H < ctx->k || H < ctx->b) return ASGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    ctx->x = x_dev; ctx->N = N; ctx->H = H; ctx->S = H / ctx->b;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->t = 0;
    ctx->passed_t = -1;
    ctx->desynced = false;
    ctx->pending = false;
    ctx->loaded = false;
    ctx->xnorm2max_valid = false;
    StepParams p = make_params(ctx);
    HIP_TRY(ctx, launch_init_first_k(p, ctx->stream));
    int rc = clear_exchange(ctx, ASGD_KERNEL_SMALL);
    if (rc != ASGD_OK) return rc;
    ctx->fill_kernel = 0;
    HIP_TRY(ctx, hipMemsetAsync(ctx->ncum, 0, (size_t)ctx->W * ctx->k * sizeof(long long), ctx->stream));
    HIP_TRY(ctx, hipMemsetAsync(ctx->counters, 0, (size_t)ctx->W * CNT_STRIDE * sizeof(long long), ctx->stream));
    // per-dimension max |x| over the rows the workers own: input of the rounding-error bound
    // that decides when an assignment is recomputed exactly
    HIP_TRY(ctx, launch_absmax(x_dev, H * ctx->W, ctx->d, ctx->xabsmax, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->loaded = true;
    return ASGD_OK;
}

int asgd_set_state(asgd_ctx *ctx, int worker, const float *w_host)
{
    if (!ctx || !w_host || worker < -2 || worker >= ctx->W) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const size_t kdb = kd_of(ctx) * sizeof(float);
    if (worker >= 0) {
        HIP_TRY(ctx, hipMemcpy(ctx->w + (size_t)worker * kd_of(ctx), w_host, kdb, hipMemcpyHostToDevice));
    } else if (worker == -1) {
        for (int i = 0; i < ctx->W; ++i)
            HIP_TRY(ctx, hipMemcpy(ctx->w + (size_t)i * kd_of(ctx), w_host, kdb, hipMemcpyHostToDevice));
    } else {
        HIP_TRY(ctx, hipMemcpy(ctx->w, w_host, kdb * ctx->W, hipMemcpyHostToDevice));
    }
    return ASGD_OK;
}

int asgd_set_step(asgd_ctx *ctx, int64_t t)
{
    if (!ctx || t < 0) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    ctx->t = t;
    ctx->passed_t = -1;
    ctx->desynced = false;
    ctx->pending = false;
    ctx->last_kernel = 0;       // the buffers are empty: no format to carry over
    int rc = clear_exchange(ctx, ASGD_KERNEL_SMALL);
    if (rc != ASGD_OK) return rc;
    ctx->fill_kernel = 0;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return ASGD_OK;
}

int asgd_get_exchange(asgd_ctx *ctx, float *values_host, size_t values_bytes, int32_t *rounds_host, size_t rounds_bytes)
{
    if (!ctx || !values_host || !rounds_host) return ASGD_EINVAL;
    if (!ctx->loaded || ctx->desynced) return ASGD_ESTATE;
    const size_t nmsg = (size_t)ctx->nb * ctx->W;
    if (values_bytes < nmsg * kd_of(ctx) * sizeof(float) || rounds_bytes < nmsg * sizeof(int32_t)) return ASGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    if (ctx->pending) {          // handed over and not yet used by a run: give the same messages back
        memcpy(values_host, ctx->pending_values.data(), nmsg * kd_of(ctx) * sizeof(float));
        memcpy(rounds_host, ctx->pending_rounds.data(), nmsg * sizeof(int32_t));
        return ASGD_OK;
    }
    return export_exchange(ctx, ctx->last_kernel, values_host, rounds_host);
}

int asgd_set_exchange(asgd_ctx *ctx, const float *values_host, const int32_t *rounds_host)
{
    if (!ctx || !values_host || !rounds_host) return ASGD_EINVAL;
    if (!ctx->loaded || ctx->desynced) return ASGD_ESTATE;
    const size_t nmsg = (size_t)ctx->nb * ctx->W;
    int par;
    long long r_want;
    inflight(ctx, &par, &r_want);
    const bool det = ctx->mode == ASGD_MODE_DETERMINISTIC;
    for (size_t q = 0; q < nmsg; ++q) {
        const long long st = rounds_host[q];
        if (st < -1 || st > r_want || (det && st >= 0 && st != r_want)) return ASGD_EINVAL;   // no such message can wait here
    }
    try {
        ctx->pending_values.assign(values_host, values_host + nmsg * kd_of(ctx));
        ctx->pending_rounds.assign(rounds_host, rounds_host + nmsg);
    } catch (...) {
        return ASGD_ENOMEM;
    }
    ctx->pending = true;
    ctx->passed_t = -1;
    return ASGD_OK;
}

int asgd_set_assign_dump(asgd_ctx *ctx, int32_t *assign_dev, size_t capacity)
{
    if (!ctx) return ASGD_EINVAL;
    ctx->dump = assign_dev;
    ctx->dump_cap = assign_dev ? capacity : 0;
    return ASGD_OK;
}

int asgd_run_steps(asgd_ctx *ctx, int64_t steps)
{
    if (!ctx || steps < 0) return ASGD_EINVAL;
    if (!ctx->loaded || ctx->desynced) return ASGD_ESTATE;
    if (ctx->lr_mode == ASGD_LR_INV_COUNT && ctx->E != 0) return ASGD_EINVAL;
    if (ctx->dump && (double)steps * ctx->W * ctx->b > (double)ctx->dump_cap) return ASGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));

    int kernel = ctx->kernel_opt;
    if (ctx->W > 1 && ctx->E > 0 && ctx->nb > ctx->W - 1) return ASGD_EINVAL;       // a message has nb different recipients
    const bool small_ok = small_kernel_supports(ctx->k, ctx->d, ctx->b) && ctx->lr_mode == ASGD_LR_CONST &&
                          ((ctx->nb == 1 && ctx->parts == 1) || ((ctx->tune >> 2) & 3) != 1);   // several buffers, partial messages: not in the private-rows shape
    // Partial messages in the matrix-core kernel are limited to the sizes its parity tests cover: the one batch of
    // full-size runs of that combination ended with a device fault whose cause was never found, so larger runs of
    // it are refused (an explicit choice of the kernel) or go to the shape-agnostic kernel (automatic choice).
    const bool mfma_parts_ok = ctx->parts == 1 || (double)ctx->W * ctx->k * ctx->d <= (double)ASGD_MFMA_PARTS_MAX_STATE;
    const bool mfma_ok = mfma_kernel_supports(ctx->k, ctx->d, ctx->b, ctx->x) && ctx->lr_mode == ASGD_LR_CONST && mfma_parts_ok;
    if (kernel == ASGD_KERNEL_AUTO) {
        // the streaming kernel for the small shapes it is built for; else the matrix-core kernel wherever its
        // layout rules allow (measured faster than the shape-agnostic kernel down to k = d = 4); else the latter
        kernel = small_ok ? ASGD_KERNEL_SMALL : (mfma_ok ? ASGD_KERNEL_MFMA : ASGD_KERNEL_GENERIC);
    }
    if (kernel == ASGD_KERNEL_SMALL && !small_ok) return ASGD_EINVAL;
    if (kernel == ASGD_KERNEL_MFMA) {
        if (!mfma_ok) return ASGD_EINVAL;
        if (!ctx->xnorm2max) HIP_TRY(ctx, hipMalloc((void **)&ctx->xnorm2max, sizeof(float)));
        if (!ctx->xnorm2max_valid) {
            HIP_TRY(ctx, launch_rownorm2max(ctx->x, ctx->H * ctx->W, ctx->d, ctx->xnorm2max, ctx->stream));
            ctx->xnorm2max_valid = true;
        }
    }

    // The kernels keep a message in flight in different formats.  Messages handed over by asgd_set_exchange(), and
    // those a run of another kernel left behind, are written into the buffers in the format of this run's kernel.
    const bool switched = ctx->last_kernel != 0 && kernel != ctx->last_kernel && ctx->E > 0 && ctx->W > 1 && ctx->t > 0;
    if (ctx->pending || switched) {
        if (!ctx->pending) {
            try {
                ctx->pending_values.resize((size_t)ctx->nb * ctx->W * kd_of(ctx));
                ctx->pending_rounds.resize((size_t)ctx->nb * ctx->W);
            } catch (...) {
                return ASGD_ENOMEM;
            }
            const int rc = export_exchange(ctx, ctx->last_kernel, ctx->pending_values.data(), ctx->pending_rounds.data());
            if (rc != ASGD_OK) return rc;
        }
        int rc = clear_exchange(ctx, kernel);
        if (rc != ASGD_OK) return rc;
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        rc = import_exchange(ctx, kernel, ctx->pending_values.data(), ctx->pending_rounds.data());
        if (rc != ASGD_OK) return rc;
        ctx->pending = false;
        std::vector<float>().swap(ctx->pending_values);
        std::vector<int32_t>().swap(ctx->pending_rounds);
        ctx->passed_t = -1;
    } else if (ctx->parts > 1 && ctx->fill_kernel != kernel) {
        // Partial messages: the fill of the never-written rows of the exchange buffers depends on the kernel's
        // message format.  (No message is in flight here: first run after load / set_step.)
        const int rc = clear_exchange(ctx, kernel);
        if (rc != ASGD_OK) return rc;
    }

    StepParams p = make_params(ctx);
    const long long t_end = ctx->t + steps;
    if (kernel == ASGD_KERNEL_SMALL && ctx->mode == ASGD_MODE_DETERMINISTIC && ctx->E > 0 && ctx->W > 1 && steps > 0) {
        // cyclic shifts of the rounds this call touches: the round before the first step up to the last step's
        const long long r_lo = ctx->t / ctx->E > 0 ? ctx->t / ctx->E - 1 : 0;
        const long long r_hi = (t_end - 1) / ctx->E;
        if (r_hi - r_lo + 1 > (long long)1 << 30) return ASGD_EINVAL;
        const bool held = ctx->tab_n > 0 && ctx->tab_seed == ctx->seed && ctx->tab_W == ctx->W && r_lo >= ctx->tab_r0 &&
                          r_hi < ctx->tab_r0 + ctx->tab_n;
        if (!held) {
            // some rounds ahead as well, so that a run of many short calls computes the table once in a while
            long long n = r_hi - r_lo + 1;
            if (n < 4096) n = 4096;
            if (n > ctx->shift_cap) {
                if (ctx->shift_tab) (void)hipFree(ctx->shift_tab);
                ctx->shift_tab = nullptr;
                ctx->shift_cap = 0;
                ctx->tab_n = 0;
                HIP_TRY(ctx, hipMalloc((void **)&ctx->shift_tab, (size_t)n * sizeof(int)));
                ctx->shift_cap = n;
            }
            HIP_TRY(ctx, launch_schedule_table(ctx->seed, r_lo, (int)n, ctx->W, ctx->shift_tab, ctx->stream));
            ctx->tab_r0 = r_lo; ctx->tab_n = n; ctx->tab_seed = ctx->seed; ctx->tab_W = ctx->W;
        }
        p.shift_tab = ctx->shift_tab;
        p.shift_r0 = ctx->tab_r0;
    }
    // Deterministic mode: a worker may only read the message of round r-1 once its sender has
    // finished that round.  Either the whole run is one launch of co-resident workgroups that wait
    // for each other's stamps (small-state and matrix-core kernels, when the workers all fit the
    // device), or a launch never crosses a multiple of E, so that the message was written by an
    // earlier launch on the same stream.
    const bool rounds = (ctx->mode == ASGD_MODE_DETERMINISTIC && ctx->E > 0 && ctx->W > 1);
    int launches = 0;
    *ctx->flag_host = 0;         // (no kernel of this context is in flight: every run ends with a wait for the stream)
    HIP_TRY(ctx, hipEventRecord(ctx->ev0, ctx->stream));
    long long t_done = ctx->t;           // steps [ctx->t, t_done) have been launched
    const bool one_launch = (kernel == ASGD_KERNEL_SMALL && (ctx->tune & 3) != 3) || (kernel == ASGD_KERNEL_MFMA && !(ctx->tune & 4));
    if (rounds && one_launch && steps > 0) {
        // every worker has passed the merge points before the first step of this run
        const long long r0 = ctx->t / ctx->E;
        const int passed = (int)((ctx->t % ctx->E) != 0 ? r0 : (r0 > 0 ? r0 - 1 : 0));
        // (a one-launch run leaves exactly these values behind: no need to write them again for the run that follows it)
        if (ctx->passed_t != ctx->t)
            HIP_TRY(ctx, hipMemsetD32Async((hipDeviceptr_t)ctx->consumed, passed, (size_t)ctx->W, ctx->stream));
        // A launch covers at most ONE_LAUNCH_MAX_ROUNDS rounds and ends on a round boundary: the waits of a workgroup
        // draw on one budget of polls per launch, which the short waits of a healthy run must not use up however long
        // the call is.
        while (t_done < t_end) {
            long long tb = (t_done / ctx->E + ONE_LAUNCH_MAX_ROUNDS) * (long long)ctx->E;
            if (tb > t_end) tb = t_end;
            hipError_t e = (kernel == ASGD_KERNEL_SMALL) ? launch_small_steps(p, t_done, tb, ctx->stream, true)
                                                         : launch_mfma_steps(p, t_done, tb, ctx->xnorm2max, ctx->stream, true);
            if (e == hipSuccess) {
                ++launches;
                t_done = tb;
                ctx->passed_t = tb;
            } else if (e == hipErrorCooperativeLaunchTooLarge || e == hipErrorNotSupported) {
                (void)hipGetLastError();     // the rest (or all of it): one launch per round
                break;
            } else {
                HIP_TRY(ctx, e);
            }
        }
    }
    for (long long ta = t_done; ta < t_end;) {
        long long tb = t_end;
        if (rounds) {
            const long long next = (ta / ctx->E + 1) * (long long)ctx->E;
            if (next < tb) tb = next;
        }
        hipError_t e = (kernel == ASGD_KERNEL_SMALL) ? launch_small_steps(p, ta, tb, ctx->stream, false)
                       : (kernel == ASGD_KERNEL_MFMA)
                           ? launch_mfma_steps(p, ta, tb, ctx->xnorm2max, ctx->stream, false)
                           : launch_generic_steps(p, ta, tb, ctx->stream);
        HIP_TRY(ctx, e);
        ++launches;
        ta = tb;
        ctx->passed_t = -1;
    }
    HIP_TRY(ctx, hipEventRecord(ctx->ev1, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev0, ctx->ev1));
    ctx->last_ms = ms;
    ctx->last_kernel = kernel;
    ctx->last_launches = launches;
    if (*ctx->flag_host) {
        // A bounded wait inside a kernel expired: some worker went on without a message it was owed, so the states are
        // not those of any step of the deterministic run.  The step counter stays where it was and the context refuses
        // further runs until asgd_load_shards() or asgd_set_state() + asgd_set_step() put it back on a known footing.
        ctx->passed_t = -1;
        ctx->desynced = true;
        return ASGD_ESYNC;
    }
    ctx->t = t_end;
    return ASGD_OK;
}

int asgd_run_epochs(asgd_ctx *ctx, int epochs)
{
    if (!ctx || epochs < 0) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    return asgd_run_steps(ctx, (int64_t)epochs * ctx->S);
}

int asgd_get_state(asgd_ctx *ctx, int worker, float *out_host, size_t out_bytes)
{
    if (!ctx || !out_host || worker < -1 || worker >= ctx->W) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    const size_t kdb = kd_of(ctx) * sizeof(float);
    const size_t need = worker >= 0 ? kdb : kdb * ctx->W;
    if (out_bytes < need) return ASGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const float *src = worker >= 0 ? ctx->w + (size_t)worker * kd_of(ctx) : ctx->w;
    HIP_TRY(ctx, hipMemcpy(out_host, src, need, hipMemcpyDeviceToHost));
    return ASGD_OK;
}

int asgd_get_mean_state(asgd_ctx *ctx, float *out_host, size_t out_bytes)
{
    if (!ctx || !out_host) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    const size_t kdb = kd_of(ctx) * sizeof(float);
    if (out_bytes < kdb) return ASGD_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, launch_mean_state(ctx->w, ctx->W, (int)kd_of(ctx), ctx->mean, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, hipMemcpy(out_host, ctx->mean, kdb, hipMemcpyDeviceToHost));
    return ASGD_OK;
}

int asgd_quant_error(asgd_ctx *ctx, int worker, double *out)
{
    if (!ctx || !out || worker < -1 || worker >= ctx->W) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const float *w = ctx->w + (size_t)(worker >= 0 ? worker : 0) * kd_of(ctx);
    if (worker == -1) {
        HIP_TRY(ctx, launch_mean_state(ctx->w, ctx->W, (int)kd_of(ctx), ctx->mean, ctx->stream));
        w = ctx->mean;
    }
    HIP_TRY(ctx, launch_quant_error(ctx->x, ctx->N, ctx->d, ctx->k, w, ctx->qpart, ctx->qout, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, hipMemcpy(out, ctx->qout, sizeof(double), hipMemcpyDeviceToHost));
    return ASGD_OK;
}

int asgd_get_worker_counters(asgd_ctx *ctx, int64_t *sent, int64_t *received, int64_t *accepted)
{
    if (!ctx) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<long long> h;
    try {
        h.resize((size_t)ctx->W * CNT_STRIDE);
    } catch (...) {
        return ASGD_ENOMEM;
    }
    HIP_TRY(ctx, hipMemcpy(h.data(), ctx->counters, h.size() * sizeof(long long), hipMemcpyDeviceToHost));
    for (int i = 0; i < ctx->W; ++i) {
        if (sent) sent[i] = h[(size_t)i * CNT_STRIDE + CNT_SENT];
        if (received) received[i] = h[(size_t)i * CNT_STRIDE + CNT_RECEIVED];
        if (accepted) accepted[i] = h[(size_t)i * CNT_STRIDE + CNT_ACCEPTED];
    }
    return ASGD_OK;
}

int asgd_last_run_ms(asgd_ctx *ctx, double *out)
{
    if (!ctx || !out) return ASGD_EINVAL;
    *out = ctx->last_ms;
    return ASGD_OK;
}

int asgd_get_stats(asgd_ctx *ctx, asgd_stats *out)
{
    if (!ctx || !out) return ASGD_EINVAL;
    if (!ctx->loaded) return ASGD_ESTATE;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<long long> h;
    try {
        h.resize((size_t)ctx->W * CNT_STRIDE);
    } catch (...) {
        return ASGD_ENOMEM;
    }
    HIP_TRY(ctx, hipMemcpy(h.data(), ctx->counters, h.size() * sizeof(long long), hipMemcpyDeviceToHost));
    memset(out, 0, sizeof(*out));
    for (int i = 0; i < ctx->W; ++i) {
        out->sent += h[(size_t)i * CNT_STRIDE + CNT_SENT];
        out->received += h[(size_t)i * CNT_STRIDE + CNT_RECEIVED];
        out->accepted += h[(size_t)i * CNT_STRIDE + CNT_ACCEPTED];
        out->parzen_near_ties += h[(size_t)i * CNT_STRIDE + CNT_PARZEN_NEAR];
        out->exact_rechecks += h[(size_t)i * CNT_STRIDE + CNT_RECHECK];
    }
    out->steps = ctx->t;
    out->samples = ctx->t * (long long)ctx->W * ctx->b;
    out->last_run_ms = ctx->last_ms;
    out->kernel = ctx->last_kernel;
    out->launches = ctx->last_launches;
    return ASGD_OK;
}

}  // extern "C"
