// Step kernel for small states (k*d of the order of 100): the streaming workloads.
//
// One wavefront per worker.  A lane takes one sample at a time:
//   - the sample's d floats come straight from HBM into registers through a ring of PF
//     register buffers, so that PF-1 groups of 64 samples are in flight per wave; the ring
//     runs across mini-batch boundaries (the addresses of the next mini-batch do not depend on
//     the state), so the update between two mini-batches overlaps with loads;
//   - the k scores x.w_k - |w_k|^2/2 (largest score = nearest centroid, the |x|^2 term is
//     common to all k) are fused multiply-add chains against a wave-uniform copy of the state
//     held in registers;
//   - the two best scores are tracked; when they are closer than a rigorous bound on the fp32
//     rounding error of the scores, the lane recomputes its assignment exactly (fp64, direct
//     form), so the assignment is the exact-arithmetic nearest centroid of the fp32 state;
//   - the gradient sums of Eq. 9 are kept per lane in LDS: row (centroid, lane) holds the d
//     sums and the count; a lane reads its row, adds its sample and writes the row back (plain
//     128-bit LDS accesses; the 48-byte lane stride keeps them free of bank conflicts).  The
//     read is issued one group ahead of the add.  Lanes past the end of a mini-batch use a
//     scratch row.  A fixed-order reduction over the 64 lanes follows once per step.
// Every sum is formed in one fixed order, so a run is reproducible bit for bit.
#include "asgd_internal.h"

namespace asgd {

namespace {

template <int D>
__device__ __forceinline__ void load_row(float (&x)[D], const float *__restrict__ row)
{
    if constexpr (D % 2 == 0) {
        const float2 *r2 = reinterpret_cast<const float2 *>(row);   // rows are 8-byte aligned when d is even
#pragma unroll
        for (int j = 0; j < D / 2; ++j) {
            float2 v = r2[j];
            x[2 * j] = v.x;
            x[2 * j + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int j = 0; j < D; ++j) x[j] = row[j];
    }
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Exchange buffers are written and read with relaxed device-scope atomic accesses: these go through
// to the memory level all workgroups share, so that no cache-wide write-back or invalidation is
// needed.  Order (payload before stamp on the sender, stamp before payload on the receiver) is kept
// by waiting for the outstanding accesses of the wave (a workgroup-scope fence) in between.
__device__ __forceinline__ void store_shared(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_shared(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded wait until *flag (device memory written by another workgroup) satisfies `flag >= want`
// (at_least) or `flag == want`.  Returns false when the bound expires; the caller then goes on
// without the message (and waits for nothing else) and the host reports the failure, so the
// kernel always terminates: a wait lasts at most a fraction of a second.
__device__ __forceinline__ bool wait_flag(const int *flag, int want, bool at_least)
{
    for (int spin = 0; spin < (1 << 18); ++spin) {
        const int v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (at_least ? (v >= want) : (v == want)) return true;
        __builtin_amdgcn_s_sleep(4);
    }
    return false;
}

// Steps [t0, t1) of the workers blockIdx.x, blockIdx.x + gridDim.x, ...
//   sync = 0: the launch contains nothing a worker has to wait for (silent or free-running mode,
//             or the host ends every launch at a multiple of E); one workgroup per worker.
//   sync = 1: the whole run is one launch of co-resident workgroups.  A workgroup takes its workers
//             through one round (E steps) after the other; at the first step of a round a worker
//             waits for the stamp of the message addressed to it (written by the sender at the end
//             of the previous round), and a sender waits until the recipient has consumed the older
//             message that sits in the same buffer.  Every wait is on an earlier round, so the
//             waits cannot form a cycle.
template <int K, int D, int PF>
__global__ __launch_bounds__(64) void small_steps_kernel(StepParams p, long long t0, long long t1, int sync)
{
    constexpr int KD = K * D;
    constexpr int ROWF = (D + 1 + 3) / 4 * 4;       // floats per accumulator row: d sums, count, padding
    constexpr int NQ = ROWF / 4;                    // float4 per row
    constexpr int NT = K * NQ;                      // reduction tasks: one float4 column each
    constexpr int NPART = 64 / NT;                  // lanes sharing a task split the 64 rows
    constexpr int NSLOT = (KD + 63) / 64;           // state elements a lane owns (element e = slot*64 + lane)
    static_assert(PF >= 2, "the ring needs the previous group's buffer");
    static_assert(NT <= 64 && NPART >= 1 && 64 % NPART == 0, "state too large for this kernel");
    static_assert(ROWF % 4 == 0 && ((ROWF / 4) % 2) == 1, "row stride must be an odd number of 16-byte units");

    __shared__ __attribute__((aligned(16))) float acc[(K + 1) * 64 * ROWF];   // row K: scratch for masked lanes
    __shared__ __attribute__((aligned(16))) float wbc[KD];                    // state, wave-uniform reads
    __shared__ __attribute__((aligned(16))) float sq[KD];
    __shared__ __attribute__((aligned(16))) float part[NPART][NT][4];

    const int lane = threadIdx.x;
    const int b = p.b;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);
    const bool rounds = (p.E > 0 && p.W > 1 && det);   // work is cut at multiples of E
    const float inv_b = 1.0f / (float)b;
    // groups of 64 samples per mini-batch, rounded up to a multiple of the ring depth (the extra
    // groups are fully masked)
    const int ngroups = ((b + 63) / 64 + PF - 1) / PF * PF;

    float sum_xmax = 0.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) sum_xmax += p.xabsmax[j];
    {
        float4 *a4 = reinterpret_cast<float4 *>(acc);
        for (int q = lane; q < (K + 1) * 64 * NQ; q += 64) a4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    long long rechecks = 0;
    int wait_failed = 0;

    // first work item: worker i, steps [ta, tb)
    int i = blockIdx.x;
    long long ta = t0;
    long long tb = rounds ? min(t1, (ta / p.E + 1) * (long long)p.E) : t1;
    long long s_seg = ta % p.S;                     // position of step ta inside the epoch

    // ring of sample buffers: buffer u holds group g with g % PF == u
    float xr[PF][D];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
#pragma unroll
        for (int j = 0; j < D; ++j) xr[u][j] = 0.0f;
    }
    {
        const float *x0 = p.x + ((size_t)i * p.H + (size_t)s_seg * b) * D;
#pragma unroll
        for (int u = 0; u + 1 < PF; ++u) {
            const int n = u * 64 + lane;
            load_row<D>(xr[u], x0 + (size_t)(n < b ? n : b - 1) * D);
        }
    }

    for (;;) {
        // ---- what this workgroup does after the current item ----
        bool has_next = true;
        int next_i = i;
        long long next_ta = ta, next_s = s_seg;
        if ((long long)i + gridDim.x < p.W) {
            next_i = i + gridDim.x;
        } else if (tb < t1) {
            next_i = blockIdx.x;
            next_ta = tb;
            next_s = (s_seg + (tb - ta)) % p.S;
        } else {
            has_next = false;
        }
        const float *xs = p.x + (size_t)i * p.H * D;            // this worker's shard
        const float *x_after = has_next ? p.x + ((size_t)next_i * p.H + (size_t)next_s * b) * D : xs + (size_t)s_seg * b * D;

        float wl[NSLOT];                                        // element e = slot*64 + lane of the state
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int e = q * 64 + lane;
            wl[q] = e < KD ? p.w[(size_t)i * KD + e] : 0.0f;
        }
        long long s_epoch = s_seg;
        long long round = p.E > 0 ? ta / p.E : 0;
        int te = p.E > 0 ? (int)(ta % p.E) : 0;

        for (long long t = ta; t < tb; ++t) {
            // ---- wave-uniform copy of the state, -|w_k|^2/2, and the rounding-error bound ----
            float wabs = 0.0f;
#pragma unroll
            for (int q = 0; q < NSLOT; ++q) {
                const int e = q * 64 + lane;
                if (e < KD) {
                    wbc[e] = wl[q];
                    sq[e] = wl[q] * wl[q];
                }
                wabs = fmaxf(wabs, fabsf(wl[q]));
            }
            __syncthreads();
            float wv[KD];
#pragma unroll
            for (int e = 0; e < KD; ++e) wv[e] = wbc[e];
            float hl = 0.0f;
            if (lane < K) {
#pragma unroll
                for (int j = 0; j < D; ++j) hl += sq[lane * D + j];
            }
            hl *= -0.5f;
            float hn[K];
            float hmax = 0.0f;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                hn[c] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hl), c));
                hmax = fmaxf(hmax, -hn[c]);
            }
            const float wmax = wave_max(wabs);
            // Each score is a chain of D fused multiply-adds started from hn (itself a sum of D squares),
            // so its rounding error is below (2D+1) * 2^-24 * (max|w| * sum_j max|x_j| + max_k |hn_k|).
            // Two scores that differ by more than twice that (here with a factor 1.5 to spare) are
            // ordered correctly by the fp32 comparison.
            const float thr = 3.0f * (float)(2 * D + 1) * 5.9604645e-8f * (wmax * sum_xmax + hmax);

            const long long s_next = (s_epoch + 1 == p.S) ? 0 : s_epoch + 1;
            const float *xb = xs + (size_t)s_epoch * b * D;                       // this mini-batch
            const float *xbn = (t + 1 < tb) ? xs + (size_t)s_next * b * D : x_after;   // the one after it

            // pending read-modify-write: row pointer and row content of the group before the current one
            float4 *prow = reinterpret_cast<float4 *>(&acc[(K * 64 + lane) * ROWF]);
            float4 pr[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) pr[q] = prow[q];

            for (int g0 = 0; g0 < ngroups; g0 += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int up = (u + PF - 1) % PF;           // buffer of the previous group
                    const int g = g0 + u;
                    const int n = g * 64 + lane;
                    const float(&xc)[D] = xr[u];

                    float best = -INFINITY, second = -INFINITY;
                    int arg = 0;
#pragma unroll
                    for (int c = 0; c < K; ++c) {
                        float sc = hn[c];
#pragma unroll
                        for (int j = 0; j < D; ++j) sc = fmaf(xc[j], wv[c * D + j], sc);
                        second = __builtin_amdgcn_fmed3f(best, second, sc);   // second largest so far
                        arg = sc > best ? c : arg;
                        best = fmaxf(best, sc);
                    }
                    const bool valid = n < b;
                    if (valid && !(best - second > thr)) {
                        // too close to call in fp32: exact assignment, fp64 direct form, lowest index on ties
                        float xe[D];
#pragma unroll
                        for (int j = 0; j < D; ++j) {
                            xe[j] = xc[j];
                            asm volatile("" : "+v"(xe[j]));     // keep the conversions below inside this branch
                        }
                        double dbest = INFINITY;
                        int darg = 0;
                        for (int c = 0; c < K; ++c) {
                            double sd = 0.0;
#pragma unroll
                            for (int j = 0; j < D; ++j) {
                                double diff = (double)xe[j] - (double)wbc[c * D + j];
                                sd += diff * diff;
                            }
                            if (sd < dbest) { dbest = sd; darg = c; }
                        }
                        arg = darg;
                        rechecks += 1;
                    }
                    if (p.dump && valid) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;

                    // finish the previous group's row: add its sample (still in buffer `up`), write back
                    {
                        float *rf = reinterpret_cast<float *>(pr);
#pragma unroll
                        for (int j = 0; j < D; ++j) rf[j] += xr[up][j];
                        rf[D] += 1.0f;
#pragma unroll
                        for (int q = 0; q < NQ; ++q) prow[q] = pr[q];
                    }
                    // buffer `up` is free now: refill it with the group PF-1 turns ahead
                    {
                        const int gg = g + PF - 1;
                        const bool same = gg < ngroups;
                        const float *src = same ? xb : xbn;
                        const int nn = (same ? gg : gg - ngroups) * 64 + lane;
                        load_row<D>(xr[up], src + (size_t)(nn < b ? nn : b - 1) * D);
                    }
                    // start this group's row
                    prow = reinterpret_cast<float4 *>(&acc[((valid ? arg : K) * 64 + lane) * ROWF]);
#pragma unroll
                    for (int q = 0; q < NQ; ++q) pr[q] = prow[q];
                }
            }
            // finish the last group of the mini-batch (buffer PF-1)
            {
                float *rf = reinterpret_cast<float *>(pr);
#pragma unroll
                for (int j = 0; j < D; ++j) rf[j] += xr[PF - 1][j];
                rf[D] += 1.0f;
#pragma unroll
                for (int q = 0; q < NQ; ++q) prow[q] = pr[q];
            }
            __syncthreads();

            // ---- sum the 64 rows of every centroid in a fixed order, clear them ----
            // lane = (part, task): task = one float4 column (centroid c, quarter q4); part = its share of the rows
            {
                const int task = lane % NT, prt = lane / NT;
                if (prt < NPART) {
                    constexpr int ROWS = 64 / NPART;
                    const int c = task / NQ, q4 = task % NQ;
                    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
#pragma unroll
                    for (int r = 0; r < ROWS; r += 2) {
                        float4 *a0 = reinterpret_cast<float4 *>(&acc[((c * 64) + prt * ROWS + r) * ROWF]) + q4;
                        float4 *a1 = reinterpret_cast<float4 *>(&acc[((c * 64) + prt * ROWS + r + 1) * ROWF]) + q4;
                        const float4 v0 = *a0, v1 = *a1;
                        *a0 = make_float4(0.f, 0.f, 0.f, 0.f);
                        *a1 = make_float4(0.f, 0.f, 0.f, 0.f);
                        s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
                        s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
                    }
                    part[prt][task][0] = s0.x + s1.x;
                    part[prt][task][1] = s0.y + s1.y;
                    part[prt][task][2] = s0.z + s1.z;
                    part[prt][task][3] = s0.w + s1.w;
                }
            }
            __syncthreads();
            float S[NSLOT], cntv[NSLOT];
#pragma unroll
            for (int q = 0; q < NSLOT; ++q) {
                const int e = q * 64 + lane;
                float sv = 0.0f, cv = 0.0f;
                if (e < KD) {
                    const int c = e / D, j = e % D;
#pragma unroll
                    for (int v = 0; v < NPART; ++v) {
                        sv += part[v][c * NQ + j / 4][j % 4];
                        cv += part[v][c * NQ + D / 4][D % 4];
                    }
                }
                S[q] = sv;
                cntv[q] = cv;
            }

            // ---- merge point? (a buffer is looked at once, at the first step of a round) ----
            const bool merge_point = (p.E > 0 && p.W > 1 && t > 0 && te == 0);
            const int rpar = det ? (int)((round - 1) & 1) : 0;
            bool has_ext = false;
            if (merge_point) {
                const int *stp = p.stamp + (size_t)rpar * p.W + i;
                if (sync && det) {
                    // the sender of the message of round-1 under the cyclic-shift schedule
                    const uint64_t shift = 1 + round_hash(p.seed, round - 1) % (uint64_t)(p.W - 1);
                    const int sender = (int)(((uint64_t)i + (uint64_t)p.W - shift) % (uint64_t)p.W);
                    if (!wait_failed && !message_dropped(p.seed, round - 1, sender, p.drop_thr)) {
                        if (!wait_flag(stp, (int)(round - 1), false)) wait_failed = 1;
                    }
                }
                const int st = __hip_atomic_load(stp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                has_ext = det ? (st == (int)(round - 1)) : (st >= 0);
            }
            const float *ext = p.slot + ((size_t)rpar * p.W + i) * KD;
            float G[NSLOT], we[NSLOT];
            double lhs = 0.0, rhs = 0.0, nrm = 0.0;
#pragma unroll
            for (int q = 0; q < NSLOT; ++q) {
                const int e = q * 64 + lane;
                G[q] = (cntv[q] * wl[q] - S[q]) * inv_b;      // descent gradient of Eq. 9
                we[q] = 0.0f;
                if (has_ext && e < KD) {
                    we[q] = load_shared(ext + e);
                    const double wed = (double)we[q];
                    const double a = ((double)wl[q] - (double)p.eps * (double)G[q]) - wed;
                    const double c2 = (double)wl[q] - wed;
                    lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                }
            }
            int delta = 0;
            if (has_ext) {           // uniform over the wave
                lhs = wave_sum(lhs); rhs = wave_sum(rhs); nrm = wave_sum(nrm);
                if (nrm > 0.0) {     // lambda of Eq. 3: an all-zero buffer is empty
                    delta = p.parzen ? (lhs < rhs) : 1;       // Eq. 4
                    if (lane == 0) {
                        long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                        cn[CNT_RECEIVED] += 1;
                        cn[CNT_ACCEPTED] += delta;
                        if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                    }
                }
            }
            // Eq. 7 and Alg. 5 line 8
#pragma unroll
            for (int q = 0; q < NSLOT; ++q) {
                float step = G[q];
                if (delta) step += wl[q] - 0.5f * (wl[q] + we[q]);
                wl[q] = wl[q] - p.eps * step;
            }
            if (merge_point) {
                // the buffer has been read: empty it and tell senders of later rounds so
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                if (lane == 0) {
                    __hip_atomic_store(p.stamp + (size_t)rpar * p.W + i, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(p.consumed + i, (int)round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }

            // ---- send (Alg. 5 line 9) ----
            if (p.E > 0 && p.W > 1 && te + 1 == p.E) {
                if (!message_dropped(p.seed, round, i, p.drop_thr)) {
                    const int peer = det ? peer_deterministic(p.seed, round, i, p.W) : peer_free(p.seed, round, i, p.W);
                    const int spar = det ? (int)(round & 1) : 0;
                    if (sync && det && round >= 2 && !wait_failed) {
                        // the buffer still holds the message of round-2 until the recipient has passed
                        // the merge point of round-1
                        if (!wait_flag(p.consumed + peer, (int)(round - 1), true)) wait_failed = 1;
                    }
                    float *dst = p.slot + ((size_t)spar * p.W + peer) * KD;
#pragma unroll
                    for (int q = 0; q < NSLOT; ++q) {
                        const int e = q * 64 + lane;
                        if (e < KD) store_shared(dst + e, wl[q]);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    if (lane == 0)
                        __hip_atomic_store(p.stamp + (size_t)spar * p.W + peer, (int)round, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
                if (lane == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
            }

            // advance the clock
            s_epoch = s_next;
            if (p.E > 0 && ++te == p.E) { te = 0; ++round; }
        }

#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int e = q * 64 + lane;
            if (e < KD) p.w[(size_t)i * KD + e] = wl[q];
        }
        if (!has_next) break;
        i = next_i;
        if (next_ta != ta) {
            ta = next_ta;
            tb = rounds ? min(t1, (ta / p.E + 1) * (long long)p.E) : t1;
        }
        s_seg = next_s;
    }

    for (int off = 32; off > 0; off >>= 1) rechecks += __shfl_xor(rechecks, off, 64);
    if (lane == 0 && rechecks)
        atomicAdd((unsigned long long *)&p.counters[(size_t)blockIdx.x * CNT_STRIDE + CNT_RECHECK],
                  (unsigned long long)rechecks);
    if (lane == 0 && wait_failed) atomicOr(p.error_flag, 1);
}

template <int K, int D, int PF>
hipError_t launch_variant(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    auto kern = small_steps_kernel<K, D, PF>;
    if (!persistent) {
        hipLaunchKernelGGL(kern, dim3(p.W), dim3(64), 0, s, p, t0, t1, 0);
        return hipGetLastError();
    }
    // one launch for the whole run: every workgroup must be resident at the same time
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 64, 0);
    if (e != hipSuccess) return e;
    const long long capacity = (long long)per_cu * prop.multiProcessorCount;
    if (capacity < 1) return hipErrorCooperativeLaunchTooLarge;
    const int grid = (int)(p.W < capacity ? p.W : capacity);
    StepParams pp = p;
    long long a0 = t0, a1 = t1;
    int sync = 1;
    void *args[] = {&pp, &a0, &a1, &sync};
    return hipLaunchCooperativeKernel((const void *)kern, dim3(grid), dim3(64), args, 0, s);
}

}  // namespace

bool small_kernel_supports(int k, int d, int b)
{
    (void)b;
    return k == 10 && d == 10;
}

hipError_t launch_small_steps(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    if (!(p.k == 10 && p.d == 10)) return hipErrorInvalidValue;
    const int ngroups = (p.b + 63) / 64;
    // ring depth: the largest of 8, 4 that divides the number of groups per mini-batch, else 2
    // (the kernel then pads an odd group count with one masked group)
    int pf = (ngroups % 8 == 0) ? 8 : (ngroups % 4 == 0) ? 4 : 2;
    if (p.tune == 1 && pf > 4) pf = 4;
    if (p.tune == 2 && pf > 2) pf = 2;
    switch (pf) {
        case 8: return launch_variant<10, 10, 8>(p, t0, t1, s, persistent);
        case 4: return launch_variant<10, 10, 4>(p, t0, t1, s, persistent);
        default: return launch_variant<10, 10, 2>(p, t0, t1, s, persistent);
    }
}

}  // namespace asgd
