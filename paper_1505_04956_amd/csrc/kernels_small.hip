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
//   NW   wavefronts per worker: wave v takes the groups v, v+NW, ... of every mini-batch.
//        NW = 1: a lane owns one accumulator row per centroid and its read-modify-write is
//                software-pipelined (the row is read one group before it is added to);
//        NW = 2: lanes l and l+32 share a row and update it one after the other, which halves
//                the LDS per wave so that two waves per SIMD are resident and hide each other's
//                latencies.
//   sync = 0: the launch contains nothing a worker has to wait for (silent or free-running mode,
//             or the host ends every launch at a multiple of E); one workgroup per worker.
//   sync = 1: the whole run is one launch of co-resident workgroups.  A workgroup takes its workers
//             through one round (E steps) after the other; at the first step of a round a worker
//             waits for the stamp of the message addressed to it (written by the sender at the end
//             of the previous round), and a sender waits until the recipient has consumed the older
//             message that sits in the same buffer.  Every wait is on an earlier round, so the
//             waits cannot form a cycle.
template <int K, int D, int PF, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW, NW))) void small_steps_kernel(StepParams p, long long t0, long long t1, int sync)
{
    constexpr int KD = K * D;
    constexpr int NQ = (D + 1 + 3) / 4;             // float4 per accumulator row: d sums, count, padding
    constexpr int NT = K * NQ;                      // reduction tasks: one float4 column each
    constexpr int NPART = 64 / NT;                  // lanes sharing a task split the rows
    constexpr int NSLOT = (KD + 63) / 64;           // state elements a lane owns (element e = slot*64 + lane)
    constexpr int RL = 64 / NW;                     // accumulator rows per centroid and wave
    constexpr int RPP = RL / NPART;                 // rows one lane sums in the reduction
    static_assert(NW == 1 || NW == 2, "one or two waves per worker");
    static_assert(PF >= 2, "the ring needs the previous group's buffer");
    static_assert(NT <= 64 && NPART >= 1 && RL % NPART == 0 && RPP % 2 == 0, "state too large for this kernel");

    // acc[wave][row][q][r]: float4 number q of the row that lane r (NW = 2: lanes r and r+32) keeps for
    // centroid `row`; row K is scratch for masked lanes.  Consecutive lanes are 16 bytes apart.
    __shared__ float4 acc[NW][K + 1][NQ][RL];
    __shared__ __attribute__((aligned(16))) float wbc[NW][KD];   // state, wave-uniform reads, one copy per wave
    __shared__ __attribute__((aligned(16))) float sq[NW][KD];
    __shared__ float4 part[2][NW][NPART][NT];                    // per-wave totals, double-buffered by step parity

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = p.b;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);
    const bool rounds = (p.E > 0 && p.W > 1 && det);   // work is cut at multiples of E
    const float inv_b = 1.0f / (float)b;
    // groups of 64 samples per mini-batch and wave, rounded up to a multiple of the ring depth (the
    // extra groups are fully masked); group m of wave v covers samples [(v + m*NW)*64, +64)
    const int ngw = (((b + 63) / 64 + NW - 1) / NW + PF - 1) / PF * PF;

    float sum_xmax = 0.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) sum_xmax += p.xabsmax[j];
    for (int q = lane; q < (K + 1) * NQ * RL; q += 64) (&acc[wave][0][0][0])[q] = make_float4(0.f, 0.f, 0.f, 0.f);

    long long rechecks = 0;
    int wait_failed = 0;
    int parity = 0;

    // first work item: worker i, steps [ta, tb)
    int i = blockIdx.x;
    long long ta = t0;
    long long tb = rounds ? min(t1, (ta / p.E + 1) * (long long)p.E) : t1;
    long long s_seg = ta % p.S;                     // position of step ta inside the epoch

    // ring of sample buffers: buffer u holds this wave's group m with m % PF == u
    float xr[PF][D];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
#pragma unroll
        for (int j = 0; j < D; ++j) xr[u][j] = 0.0f;
    }
    {
        const float *x0 = p.x + ((size_t)i * p.H + (size_t)s_seg * b) * D;
#pragma unroll
        for (int u = 0; u < (NW == 1 ? PF - 1 : PF); ++u) {
            const int n = (wave + u * NW) * 64 + lane;
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
                    wbc[wave][e] = wl[q];
                    sq[wave][e] = wl[q] * wl[q];
                }
                wabs = fmaxf(wabs, fabsf(wl[q]));
            }
            __syncthreads();
            float wv[KD];
#pragma unroll
            for (int e = 0; e < KD; ++e) wv[e] = wbc[wave][e];
            float hl = 0.0f;
            if (lane < K) {
#pragma unroll
                for (int j = 0; j < D; ++j) hl += sq[wave][lane * D + j];
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

            // NW = 1: pending read-modify-write (row pointer and content) of the group before the current one
            float4 *prow = &acc[wave][K][0][lane % RL];
            float4 pr[NQ];
            if constexpr (NW == 1) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) pr[q] = prow[q * RL];
            }

            for (int m0 = 0; m0 < ngw; m0 += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int up = (u + PF - 1) % PF;           // buffer of the previous group
                    const int m = m0 + u;
                    const int n = (wave + m * NW) * 64 + lane;
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
                                double diff = (double)xe[j] - (double)wbc[wave][c * D + j];
                                sd += diff * diff;
                            }
                            if (sd < dbest) { dbest = sd; darg = c; }
                        }
                        arg = darg;
                        rechecks += 1;
                    }
                    if (p.dump && valid) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;

                    if constexpr (NW == 1) {
                        // finish the previous group's row: add its sample (still in buffer `up`), write back
                        {
                            float *rf = reinterpret_cast<float *>(pr);
#pragma unroll
                            for (int j = 0; j < D; ++j) rf[j] += xr[up][j];
                            rf[D] += 1.0f;
#pragma unroll
                            for (int q = 0; q < NQ; ++q) prow[q * RL] = pr[q];
                        }
                        // start this group's row
                        prow = &acc[wave][valid ? arg : K][0][lane];
#pragma unroll
                        for (int q = 0; q < NQ; ++q) pr[q] = prow[q * RL];
                    } else {
                        // lanes l and l+32 share a row: lower half first, then upper half
                        float4 *row = &acc[wave][valid ? arg : K][0][lane % RL];
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            if ((lane >> 5) == h) {
                                float4 rr[NQ];
#pragma unroll
                                for (int q = 0; q < NQ; ++q) rr[q] = row[q * RL];
                                float *rf = reinterpret_cast<float *>(rr);
#pragma unroll
                                for (int j = 0; j < D; ++j) rf[j] += xc[j];
                                rf[D] += 1.0f;
#pragma unroll
                                for (int q = 0; q < NQ; ++q) row[q * RL] = rr[q];
                            }
                        }
                    }
                    // refill a free buffer with the group PF-1 (NW = 1) or PF (NW = 2) turns ahead
                    {
                        constexpr int ahead = (NW == 1) ? PF - 1 : PF;
                        const int mm = m + ahead;
                        const bool same = mm < ngw;
                        const float *src = same ? xb : xbn;
                        const int nn = (wave + (same ? mm : mm - ngw) * NW) * 64 + lane;
                        load_row<D>(xr[NW == 1 ? up : u], src + (size_t)(nn < b ? nn : b - 1) * D);
                    }
                }
            }
            if constexpr (NW == 1) {
                // finish the last group of the mini-batch (buffer PF-1)
                float *rf = reinterpret_cast<float *>(pr);
#pragma unroll
                for (int j = 0; j < D; ++j) rf[j] += xr[PF - 1][j];
                rf[D] += 1.0f;
#pragma unroll
                for (int q = 0; q < NQ; ++q) prow[q * RL] = pr[q];
            }
            __syncthreads();

            // ---- sum the rows of every centroid in a fixed order, clear them ----
            // lane = (part, task): task = one float4 column (centroid c, quarter q4); part = its share of the rows
            {
                const int task = lane % NT, prt = lane / NT;
                if (prt < NPART) {
                    const int c = task / NQ, q4 = task % NQ;
                    float4 *col = &acc[wave][c][q4][prt * RPP];
                    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
#pragma unroll
                    for (int r = 0; r < RPP; r += 2) {
                        // start at a task-dependent row so that the lanes of one access hit different banks
                        const int r0 = (r + task) % RPP, r1 = (r + 1 + task) % RPP;
                        const float4 v0 = col[r0], v1 = col[r1];
                        col[r0] = make_float4(0.f, 0.f, 0.f, 0.f);
                        col[r1] = make_float4(0.f, 0.f, 0.f, 0.f);
                        s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
                        s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
                    }
                    part[parity][wave][prt][task] = make_float4(s0.x + s1.x, s0.y + s1.y, s0.z + s1.z, s0.w + s1.w);
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
                    const float *pf = reinterpret_cast<const float *>(&part[parity][0][0][0]);
#pragma unroll
                    for (int v = 0; v < NW * NPART; ++v) {      // waves, then parts: one fixed order
                        sv += pf[(v * NT + c * NQ + j / 4) * 4 + j % 4];
                        cv += pf[(v * NT + c * NQ + D / 4) * 4 + D % 4];
                    }
                }
                S[q] = sv;
                cntv[q] = cv;
            }
            parity ^= 1;

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
            if (has_ext) {           // uniform over the workgroup
                lhs = wave_sum(lhs); rhs = wave_sum(rhs); nrm = wave_sum(nrm);
                if (nrm > 0.0) {     // lambda of Eq. 3: an all-zero buffer is empty
                    delta = p.parzen ? (lhs < rhs) : 1;       // Eq. 4
                    if (threadIdx.x == 0) {
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
                // every wave has read the buffer: empty it and tell senders of later rounds so
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                if constexpr (NW > 1) __syncthreads();
                if (threadIdx.x == 0) {
                    __hip_atomic_store(p.stamp + (size_t)rpar * p.W + i, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(p.consumed + i, (int)round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }

            // ---- send (Alg. 5 line 9): the first wave writes ----
            if (p.E > 0 && p.W > 1 && te + 1 == p.E && wave == 0) {
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

        if (wave == 0) {
#pragma unroll
            for (int q = 0; q < NSLOT; ++q) {
                const int e = q * 64 + lane;
                if (e < KD) p.w[(size_t)i * KD + e] = wl[q];
            }
        }
        if (!has_next) break;
        if constexpr (NW > 1) __syncthreads();      // the other wave reloads the state written above
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

template <int K, int D, int PF, int NW>
hipError_t launch_variant(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    auto kern = small_steps_kernel<K, D, PF, NW>;
    if (!persistent) {
        hipLaunchKernelGGL(kern, dim3(p.W), dim3(64 * NW), 0, s, p, t0, t1, 0);
        return hipGetLastError();
    }
    // one launch for the whole run: every workgroup must be resident at the same time
    // resident workgroups of this kernel on the current device (queried once per device and variant)
    static long long cached_capacity[64] = {0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    long long capacity = (dev >= 0 && dev < 64) ? cached_capacity[dev] : 0;
    if (capacity == 0) {
        int per_cu = 0, cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 64 * NW, 0);
        if (e != hipSuccess) return e;
        capacity = (long long)per_cu * cus;
        if (dev >= 0 && dev < 64) cached_capacity[dev] = capacity;
    }
    if (capacity < 1) return hipErrorCooperativeLaunchTooLarge;
    const int grid = (int)(p.W < capacity ? p.W : capacity);
    StepParams pp = p;
    long long a0 = t0, a1 = t1;
    int sync = 1;
    void *args[] = {&pp, &a0, &a1, &sync};
    if (p.cooperative) return hipLaunchCooperativeKernel((const void *)kern, dim3(grid), dim3(64 * NW), args, 0, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), 0, s, pp, a0, a1, sync);
    return hipGetLastError();
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
    // tune: bit 2 (value 4) = one wave per worker; bits 0-1 limit the ring depth (1: 4, 2: 2); 3 is
    // handled by the caller (one launch per round)
    const int nw = (p.tune & 4) ? 1 : 2;
    const int ngw = ((p.b + 63) / 64 + nw - 1) / nw;
    // ring depth: the largest of 8, 4 that divides the number of groups per mini-batch and wave, else 2
    // (the kernel then pads the group count with masked groups)
    int pf = (ngw % 8 == 0) ? 8 : (ngw % 4 == 0) ? 4 : 2;
    if (nw == 2 && pf > 4) pf = 4;                 // two waves per SIMD: 256 registers each
    if ((p.tune & 3) == 1 && pf > 4) pf = 4;
    if ((p.tune & 3) == 2 && pf > 2) pf = 2;
    if (nw == 1) {
        switch (pf) {
            case 8: return launch_variant<10, 10, 8, 1>(p, t0, t1, s, persistent);
            case 4: return launch_variant<10, 10, 4, 1>(p, t0, t1, s, persistent);
            default: return launch_variant<10, 10, 2, 1>(p, t0, t1, s, persistent);
        }
    }
    switch (pf) {
        case 4: return launch_variant<10, 10, 4, 2>(p, t0, t1, s, persistent);
        default: return launch_variant<10, 10, 2, 2>(p, t0, t1, s, persistent);
    }
}

}  // namespace asgd
