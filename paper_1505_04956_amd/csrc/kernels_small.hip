// Step kernel for small states (k <= 16, k*d of the order of 100): the streaming workloads.
//
// One workgroup of NW wavefronts per worker; a lane takes one sample at a time:
//   - the sample's d floats come straight from HBM into registers through a ring of PF register
//     buffers, so that PF-1 groups of 64 samples are in flight per wave; the ring runs across
//     mini-batch, round and worker boundaries (the addresses of later mini-batches do not depend on
//     the state), so the update between two mini-batches overlaps with loads;
//   - scores relative to centroid 0, t_k = x.(w_k - w_0) + (h_k - h_0) + 1 with h_k = -|w_k|^2/2
//     (largest t_k = nearest centroid; the |x|^2 term is common to all k), are chains of fused
//     multiply-adds against a wave-uniform copy of w_k - w_0 held in registers;
//   - the centroid index rides in the low 4 mantissa bits of t_k, and the two largest t_k come out
//     of a network of three-input max/median instructions; when they are closer than a rigorous
//     bound on the fp32 rounding error (packing included), the lane decides exactly in fp64, so the
//     assignment is the exact-arithmetic nearest centroid of the fp32 state;
//   - the gradient sums of Eq. 9 are kept per lane in LDS: a row holds the d sums and the count of
//     one centroid, as NQ float4, for one lane (RS = 1) or for the lane pair l, l+32 (RS = 2).  A
//     sample is added to its row in NQ phases of one 128-bit read, four adds and one 128-bit write;
//     in phase p the lower lanes work on float4 number p and the upper lanes on number p+1 (mod NQ),
//     so a shared row is never touched twice in one phase and every LDS instruction serves all 64
//     lanes.  The phases of a group are interleaved with the score computation of the next group,
//     which hides their LDS latency.  Lanes past the end of a mini-batch use a scratch row.  A
//     fixed-order reduction follows once per step.
// The LDS pipeline is the scarce resource of this kernel (it was measured ~85 % busy with twice as
// many, half-filled accesses), hence the care for few, full LDS instructions and for DPP instead of
// LDS-backed shuffles in the per-step part.
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

// max over the wave of a non-negative value, without LDS: butterfly inside rows of 16 lanes with DPP
// (lane ^ 1, lane ^ 2, mirror inside 8, mirror inside 16), then the four rows through scalar reads.
__device__ __forceinline__ float wave_max_nonneg(float v)
{
    int x = __float_as_int(v);      // non-negative floats order like their bit patterns
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xF, 0xF, true));   // row_half_mirror
    x = max(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xF, 0xF, true));   // row_mirror
    const int a = __builtin_amdgcn_readlane(x, 0), b = __builtin_amdgcn_readlane(x, 16);
    const int c = __builtin_amdgcn_readlane(x, 32), d = __builtin_amdgcn_readlane(x, 48);
    return __int_as_float(max(max(a, b), max(c, d)));
}

// min and max of floats through the integer instructions on their bit patterns.  For non-negative
// values the integer order is the float order and every negative value is below every non-negative
// one; negative values compare in reverse among themselves.  That is enough for top2() below, whose
// callers guarantee that the largest value is at least 1 and only look at the second largest when
// it is within a small distance of the largest.  (Integer instructions need no NaN quieting.)
__device__ __forceinline__ float fmin2(float a, float b) { return __int_as_float(min(__float_as_int(a), __float_as_int(b))); }
__device__ __forceinline__ float fmax2(float a, float b) { return __int_as_float(max(__float_as_int(a), __float_as_int(b))); }
__device__ __forceinline__ float fmax3(float a, float b, float c)
{
    return __int_as_float(max(max(__float_as_int(a), __float_as_int(b)), __float_as_int(c)));
}

// Largest and second largest of t[0..N) with three-input max/median instructions: triples are reduced
// to (max, median) and merged pairwise.  Exact when the second largest is non-negative (see above).
template <int N>
__device__ __forceinline__ void top2(const float (&t)[N], float &best, float &second)
{
    static_assert(N >= 2, "need two values");
    float H, M;
    int i;
    if constexpr (N >= 3) {
        H = fmax3(t[0], t[1], t[2]);
        M = __builtin_amdgcn_fmed3f(t[0], t[1], t[2]);
        i = 3;
    } else {
        H = fmax2(t[0], t[1]);
        M = fmin2(t[0], t[1]);
        i = 2;
    }
#pragma unroll
    for (; i + 2 < N; i += 3) {
        const float h = fmax3(t[i], t[i + 1], t[i + 2]);
        const float m = __builtin_amdgcn_fmed3f(t[i], t[i + 1], t[i + 2]);
        const float lo = fmin2(H, h);
        H = fmax2(H, h);
        M = fmax3(lo, M, m);
    }
#pragma unroll
    for (; i < N; ++i) {
        M = __builtin_amdgcn_fmed3f(H, M, t[i]);
        H = fmax2(H, t[i]);
    }
    best = H;
    second = M;
}

// Lanes l and l+32 hand parts of an accumulator row to each other through LDS.  The hardware executes
// the LDS accesses of a wave in program order; this keeps the compiler from moving the read of one
// phase above the write of the previous one (to a single lane the two look unrelated).
__device__ __forceinline__ void phase_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// A message of this kernel is self-validating: every element travels as a 64-bit pair (value, round
// stamp), written and read with relaxed device-scope 64-bit atomic accesses (single-copy atomic; they go
// through to the memory level all workgroups share, so no cache-wide write-back or invalidation is
// needed).  The receiver accepts a message when every pair carries the expected stamp.  Hence the sender
// needs no ordering between payload and a separate flag - it never waits for its stores, which on this
// chip would also drain the sample loads in flight - and the receiver can fetch the pairs long before it
// needs them and only has to look again if they had not arrived yet.  A message of lane l < NT is the four
// pairs [4l, 4l+4) of its buffer (task layout, elements that do not exist included).
__device__ __forceinline__ unsigned long long pack_pair(float v, int stamp)
{
    return ((unsigned long long)(unsigned)stamp << 32) | (unsigned long long)__float_as_uint(v);
}
__device__ __forceinline__ void store_pair(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_pair(const unsigned long long *p)
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
//   RS   lanes sharing an accumulator row: 1 = every lane has its own rows (64 per centroid and
//        wave); 2 = lanes l and l+32 share a row, which halves the LDS per wave so that twice as many
//        waves are resident.
//   sync = 0: the launch contains nothing a worker has to wait for (silent or free-running mode,
//             or the host ends every launch at a multiple of E); one workgroup per worker.
//   sync = 1: the whole run is one launch of co-resident workgroups.  A workgroup takes its workers
//             through one round (E steps) after the other; at the first step of a round a worker
//             waits for the stamp of the message addressed to it (written by the sender at the end
//             of the previous round), and a sender waits until the recipient has consumed the older
//             message that sits in the same buffer.  Every wait is on an earlier round, so the
//             waits cannot form a cycle.
//
// State layout in registers ("task layout"): lane l < NT = K*NQ holds the four elements
// (c, 4q .. 4q+3) of the state with c = l / NQ, q = l % NQ (elements past d do not exist and stay 0);
// the same lane sums float4 column (c, q) of the accumulator rows once per step.
//   NB   external buffers per worker = recipients per message (Eq. 3 / Eq. 6); NB = p.nb
template <int K, int D, int PF, int NW, int RS, int NB>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(RS, RS)))
void small_steps_kernel(StepParams p, long long t0, long long t1, int sync)
{
    constexpr int KD = K * D;
    constexpr int NQ = (D + 1 + 3) / 4;             // float4 per accumulator row: d sums, count, padding
    constexpr int NT = K * NQ;                      // tasks: one float4 column each
    constexpr int NPART = 64 / NT;                  // lanes sharing a task split the rows in the reduction
    constexpr int RL = 64 / RS;                     // accumulator rows per centroid and wave
    constexpr int RPP = RL / NPART;                 // rows one lane sums in the reduction
    constexpr int CPC = (K - 1 + NQ - 1) / NQ;      // score chains between two row phases
    constexpr int CQ = D / 4, CI = D % 4;           // float4 and component that hold the count
    static_assert(NW == 1 || NW == 2, "one or two waves per worker");
    static_assert(RS == 1 || (RS == 2 && NQ >= 2), "two lanes share a row only if it has two float4 or more");
    static_assert(K >= 2 && K <= 16, "index packing uses 4 bits");
    static_assert(PF >= 2, "the ring needs the previous group's buffer");
    static_assert(NT <= 64 && NPART >= 1 && RL % NPART == 0 && RPP % 2 == 0, "state too large for this kernel");

    // acc[wave][row][q][r]: float4 number q of the row that lane r (RS = 2: lanes r and r+32) keeps for
    // centroid `row`; row K is scratch for masked lanes.  Consecutive lanes are 16 bytes apart.
    __shared__ float4 acc[NW][K + 1][NQ][RL];
    __shared__ __attribute__((aligned(16))) float wbc[NW][KD];         // state, one copy per wave
    __shared__ __attribute__((aligned(16))) float wdc[NW][KD - D + 4]; // w_k - w_0 for k >= 1
    __shared__ float hq[NW][64];                                       // per-task sums of squares
    __shared__ float hnc[NW][16];                                      // (h_k - h_0) + 1
    __shared__ float4 part[2][NW][NPART][NT];                          // per-wave totals, double-buffered by step parity

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool lower = RS == 1 || lane < 32;        // the half of the wave that starts with float4 number 0
    const int b = p.b;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);
    const bool rounds = (p.E > 0 && p.W > 1 && det);   // work is cut at multiples of E
    const float inv_b = 1.0f / (float)b;
    // groups of 64 samples per mini-batch and wave, rounded up to a multiple of the ring depth (the
    // extra groups are fully masked); group m of wave v covers samples [(v + m*NW)*64, +64)
    const int ngw = (((b + 63) / 64 + NW - 1) / NW + PF - 1) / PF * PF;

    // this lane's task
    const bool has_task = lane < NT;
    const int tc = has_task ? lane / NQ : 0, tq = has_task ? lane % NQ : 0;
    bool tv[4];                                     // which of the four elements exist
    int te_[4];                                     // their index in the state
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
        tv[c4] = has_task && (4 * tq + c4 < D);
        te_[c4] = tc * D + 4 * tq + c4;
    }
    // float4 number this lane works on in phase ph of a row update, as an offset in float4 units
    int qoff[NQ];
#pragma unroll
    for (int ph = 0; ph < NQ; ++ph) qoff[ph] = (lower ? ph : (ph + 1) % NQ) * RL;

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
        for (int u = 0; u + 1 < PF; ++u) {
            const int n = (wave + u * NW) * 64 + lane;
            load_row<D>(xr[u], x0 + (size_t)(n < b ? n : b - 1) * D);
        }
    }

    // part of sample x that goes to float4 number q of a row, component c4: the d values, then the count
    auto row_part = [](const float(&x)[D], int q, int c4) -> float {
        const int j = 4 * q + c4;
        return j < D ? x[j] : (j == D ? 1.0f : 0.0f);
    };

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

        float w4[4];                                            // this lane's four elements of the state
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) w4[c4] = tv[c4] ? p.w[(size_t)i * KD + te_[c4]] : 0.0f;
        long long s_epoch = s_seg;
        long long round = p.E > 0 ? ta / p.E : 0;
        int te = p.E > 0 ? (int)(ta % p.E) : 0;

        for (long long t = ta; t < tb; ++t) {
            // ---- wave-uniform copies: state (for exact re-evaluation), differences to centroid 0, offsets ----
            // centroid 0 lives in the lanes 0 .. NQ-1
            float w0[4 * NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4)
                    w0[4 * q + c4] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w4[c4]), q));
            }
            float dabs = 0.0f, hsq = 0.0f;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                float w0q = w0[c4];
#pragma unroll
                for (int q = 1; q < NQ; ++q) w0q = (tq == q) ? w0[4 * q + c4] : w0q;
                const float wd = tv[c4] ? w4[c4] - w0q : 0.0f;
                if (tv[c4]) {
                    wbc[wave][te_[c4]] = w4[c4];
                    if (tc >= 1) wdc[wave][te_[c4] - D] = wd;
                }
                dabs = fmaxf(dabs, fabsf(wd));
                hsq = fmaf(w4[c4], w4[c4], hsq);
            }
            hq[wave][lane] = hsq;
            phase_fence();      // the copies are per wave: the lanes of this wave only have to see each other's writes
            float wv[KD - D];                                    // w_k - w_0 for k >= 1
#pragma unroll
            for (int e = 0; e < KD - D; ++e) wv[e] = wdc[wave][e];
            float hl = 0.0f;
            if (lane < K) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) hl += hq[wave][lane * NQ + q];
            }
            hl *= -0.5f;
            const float h0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hl), 0));
            const float hdl = hl - h0;
            const float hol = hdl + 1.0f;
            if (lane < K) hnc[wave][lane] = hol;
            float hn[K];                                         // hn[k] = (h_k - h_0) + 1
#pragma unroll
            for (int c = 0; c < K; ++c) hn[c] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hol), c));
            // max_k |h_k| bounds max_k |h_k - h_0| up to a factor 2; one wave-wide max serves both
            const float hmax = wave_max_nonneg(lane < K ? fabsf(hl) : 0.0f);
            const float hdmax = 2.0f * hmax;
            // Rounding-error bound of one t_k, with u = 2^-24, A = max|w_k - w_0| * sum_j max|x_j| (a bound of
            // sum_j |x_j||w_kj - w_0j|) and Hd = max_k |h_k - h_0|:
            //   differences w_k - w_0 ................. u A
            //   D fused multiply-adds ................. D u (A + Hd + 1)
            //   h_k (D squares and adds, one product) . (D+1) u max|h| each, two of them in h_k - h_0
            //   the subtraction and the +1 ............ 2 u (Hd + 1)
            //   index in the low 4 mantissa bits ...... 32 u (A + Hd + 1)
            // Two values that differ by more than twice the sum (times 1.5 to spare) are ordered correctly.
            const float Abound = wave_max_nonneg(dabs) * sum_xmax;
            const float thr = 3.0f * 5.9604645e-8f *
                              ((float)(D + 33) * Abound + (float)(D + 34) * (hdmax + 1.0f) + (float)(2 * D + 2) * hmax);

            // The instruction arbiter of a SIMD prefers the older of its two waves, which makes the workgroups that
            // were dispatched later run ~40 % slower - and with rounds coupled through the exchange everybody ends
            // up waiting for them.  Alternating the wave priority step by step, in opposite phase for the two
            // halves of the grid (dispatch order), evens the shares out.
            if (((int)(t & 1) ^ (blockIdx.x * 2 >= gridDim.x ? 1 : 0)) != 0)
                __builtin_amdgcn_s_setprio(1);
            else
                __builtin_amdgcn_s_setprio(0);

            // ---- exchange, early part: fetch what the end of this step will need, so that the latency of these
            // accesses (they bypass the caches) runs behind the mini-batch ----
            const bool merge_point = (p.E > 0 && p.W > 1 && t > 0 && te == 0);
            const bool send_point = (p.E > 0 && p.W > 1 && te + 1 == p.E);
            const int rpar = det ? (int)((round - 1) & 1) : 0;
            // buffer n of this worker (parity rpar): NT lanes x 4 pairs each; copy n of a message goes to buffer n
            const unsigned long long *mslot[NB];
            unsigned long long mp[NB][4];
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                mslot[n] = reinterpret_cast<const unsigned long long *>(p.slot) +
                           (((size_t)(rpar * NB + n) * p.W + i) * NT + (has_task ? lane : 0)) * 4;
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) mp[n][c4] = merge_point ? load_pair(mslot[n] + c4) : 0ull;
            }
            // cyclic shift of copy n in round r: 1 + (shift of copy 0 - 1 + n) mod (W - 1)
            auto shift_of = [&](long long r, int n) -> int {
                int sh = p.shift_tab[r - p.shift_r0] + n;
                if (sh > p.W - 1) sh -= p.W - 1;
                return sh;
            };
            int peer[NB], ackv[NB];
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                peer[n] = 0; ackv[n] = 0;
                if (send_point && wave == 0) {
                    if (det) {
                        // (the shifts of the rounds of this launch come from a table: no 64-bit division in here)
                        peer[n] = i + shift_of(round, n);
                        if (peer[n] >= p.W) peer[n] -= p.W;
                        if (sync && round >= 2)
                            ackv[n] = __hip_atomic_load(p.consumed + peer[n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        peer[n] = peer_free(p.seed, round, i, p.W, n);
                    }
                }
            }

            const long long s_next = (s_epoch + 1 == p.S) ? 0 : s_epoch + 1;
            const float *xb = xs + (size_t)s_epoch * b * D;                       // this mini-batch
            const float *xbn = (t + 1 < tb) ? xs + (size_t)s_next * b * D : x_after;   // the one after it

            // pending row update of the group before the current one: row pointer (float4 number 0 of the
            // row) and the float4 read for the coming phase.  At the start of a step: the scratch row.
            float4 *prow = &acc[wave][K][0][lane % RL];
            float4 pr = prow[qoff[0]];

            for (int m0 = 0; m0 < ngw; m0 += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int up = (u + PF - 1) % PF;           // buffer of the previous group
                    const int m = m0 + u;
                    const int n = (wave + m * NW) * 64 + lane;
                    const float(&xc)[D] = xr[u];
                    const float(&xp)[D] = xr[up];

                    // t_k with the centroid index in the low 4 mantissa bits (15 - k, so that the lower index
                    // wins exact ties of positive values); between the chains, the row phases of the
                    // previous group: add, write, (fence,) read for the next phase
                    float tk[K];
                    const float tk0 = __uint_as_float(0x3F800000u | 15u);
                    tk[0] = tk0;
#pragma unroll
                    for (int ph = 0; ph < NQ; ++ph) {
#pragma unroll
                        for (int c = 1 + ph * CPC; c < 1 + (ph + 1) * CPC && c < K; ++c) {
                            float sc = hn[c];
#pragma unroll
                            for (int j = 0; j < D; ++j) sc = fmaf(xc[j], wv[(c - 1) * D + j], sc);
                            tk[c] = __uint_as_float((__float_as_uint(sc) & 0xFFFFFFF0u) | (unsigned)(15 - c));
                        }
                        // keep the order chains / row phase / chains ...: the LDS read issued at the end of a phase
                        // then returns under the next chains instead of being waited for at once
                        __builtin_amdgcn_sched_barrier(0);
                        float add[4];
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4) {
                            const float lo = row_part(xp, ph, c4);
                            if constexpr (RS == 1) {
                                add[c4] = lo;
                            } else {
                                const float hi = row_part(xp, (ph + 1) % NQ, c4);
                                add[c4] = lower ? lo : hi;
                            }
                        }
                        pr.x += add[0]; pr.y += add[1]; pr.z += add[2]; pr.w += add[3];
                        prow[qoff[ph]] = pr;
                        if (ph + 1 < NQ) {
                            if constexpr (RS == 2) phase_fence();
                            pr = prow[qoff[ph + 1]];
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // buffer `up` is free now: refill it with the group PF-1 turns ahead
                    {
                        const int mm = m + PF - 1;
                        const bool same = mm < ngw;
                        const float *src = same ? xb : xbn;
                        const int nn = (wave + (same ? mm : mm - ngw) * NW) * 64 + lane;
                        load_row<D>(xr[up], src + (size_t)(nn < b ? nn : b - 1) * D);
                    }

                    float best, second;
                    top2<K>(tk, best, second);
                    int arg = 15 - (int)(__float_as_uint(best) & 15u);
                    const bool valid = n < b;
                    if (valid && !(best - second > thr)) {
                        // Too close to call in fp32.  Candidates are the centroids within thr of the best; with
                        // two of them their distances are compared exactly (fp64), with more all k distances
                        // are recomputed in fp64, direct form; the lowest index wins exact ties.
                        float xe[D];
#pragma unroll
                        for (int j = 0; j < D; ++j) {
                            xe[j] = xc[j];
                            asm volatile("" : "+v"(xe[j]));     // keep the conversions below inside this branch
                        }
                        // count the candidates by forming every t_k again (same operations, same values)
                        int ncand = (tk0 >= best - thr) ? 1 : 0;
#pragma unroll 1
                        for (int c = 1; c < K; ++c) {
                            float sc = hnc[wave][c];
#pragma unroll
                            for (int j = 0; j < D; ++j) sc = fmaf(xe[j], wdc[wave][(c - 1) * D + j], sc);
                            const float tc2 = __uint_as_float((__float_as_uint(sc) & 0xFFFFFFF0u) | (unsigned)(15 - c));
                            ncand += (tc2 >= best - thr) ? 1 : 0;
                        }
                        if (ncand <= 2) {
                            const int ca = arg, cb = 15 - (int)(__float_as_uint(second) & 15u);
                            // |x - w_a|^2 - |x - w_b|^2 = sum_j (w_aj - w_bj) (w_aj + w_bj - 2 x_j)
                            double dd = 0.0;
#pragma unroll
                            for (int j = 0; j < D; ++j) {
                                const double wa = (double)wbc[wave][ca * D + j], wb = (double)wbc[wave][cb * D + j];
                                dd += (wa - wb) * ((wa + wb) - 2.0 * (double)xe[j]);
                            }
                            arg = (dd < 0.0 || (dd == 0.0 && ca < cb)) ? ca : cb;
                        } else {
                            double dbest = INFINITY;
                            int darg = 0;
#pragma unroll 1
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
                        }
                        rechecks += 1;
                    }
                    if (p.dump && valid) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;

                    // start this group's row update: read for phase 0
                    if constexpr (RS == 2) phase_fence();
                    prow = &acc[wave][valid ? arg : K][0][lane % RL];
                    pr = prow[qoff[0]];
                }
            }
            // finish the last group of the mini-batch (buffer PF-1)
            {
                const float(&xp)[D] = xr[PF - 1];
#pragma unroll
                for (int ph = 0; ph < NQ; ++ph) {
                    float add[4];
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        const float lo = row_part(xp, ph, c4);
                        if constexpr (RS == 1) {
                            add[c4] = lo;
                        } else {
                            const float hi = row_part(xp, (ph + 1) % NQ, c4);
                            add[c4] = lower ? lo : hi;
                        }
                    }
                    pr.x += add[0]; pr.y += add[1]; pr.z += add[2]; pr.w += add[3];
                    prow[qoff[ph]] = pr;
                    if (ph + 1 < NQ) {
                        if constexpr (RS == 2) phase_fence();
                        pr = prow[qoff[ph + 1]];
                    }
                }
            }
            phase_fence();      // a wave sums its own rows

            // ---- sum the rows of every centroid in a fixed order, clear them ----
            // lane = (part, task): task = one float4 column (centroid, float4 number); part = its share of the rows
            {
                const int task = lane % NT, prt = lane / NT;
                if (prt < NPART) {
                    float4 *col = &acc[wave][task / NQ][task % NQ][prt * RPP];
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
            // totals of this lane's float4 column and the count of its centroid: waves, then parts, one fixed order
            float S4[4] = {0.f, 0.f, 0.f, 0.f};
            float cnt = 0.0f;
            if (has_task) {
#pragma unroll
                for (int v = 0; v < NW * NPART; ++v) {
                    const float4 sv = (&part[parity][0][0][0])[v * NT + lane];
                    const float4 cv = (&part[parity][0][0][0])[v * NT + tc * NQ + CQ];
                    S4[0] += sv.x; S4[1] += sv.y; S4[2] += sv.z; S4[3] += sv.w;
                    cnt += CI == 0 ? cv.x : (CI == 1 ? cv.y : (CI == 2 ? cv.z : cv.w));
                }
            }
            parity ^= 1;

            // ---- merge point? (a buffer is looked at once, at the first step of a round) ----
            bool has_ext[NB], in_part[NB];
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                has_ext[n] = false;
                in_part[n] = has_task;
                if (merge_point) {
                    // complete = every pair of every task lane carries the stamp of round-1 (free-running: any stamp).
                    // Partial messages: only the lanes whose centroid row belongs to the part that this copy carries
                    // (free-running mode: the part follows from the round in the lane's own first stamp).
                    auto complete = [&]() -> bool {
                        bool ok = true;
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4) {
                            const int st = (int)(mp[n][c4] >> 32);
                            ok = ok && (det ? st == (int)(round - 1) : st >= 0);
                        }
                        if (p.parts > 1) {
                            const int mr = det ? (int)(round - 1) : (int)(mp[n][0] >> 32);
                            in_part[n] = has_task && mr >= 0 && tc % p.parts == (mr + i + n) % p.parts;
                            if (!det) return __ballot(in_part[n] && ok) != 0ull;      // some row is there
                            return __ballot(in_part[n] && !ok) == 0ull;
                        }
                        return __ballot(has_task && !ok) == 0ull;
                    };
                    has_ext[n] = complete();
                    if (!has_ext[n] && sync && det && !wait_failed) {
                        // not there yet: wait for the sender of round-1 under the cyclic-shift schedule, unless its
                        // message is one of those the loss hook drops
                        int sender = i - shift_of(round - 1, n);
                        if (sender < 0) sender += p.W;
                        if (!(p.drop_thr != 0 && message_dropped(p.seed, round - 1, sender, p.drop_thr, n))) {
                            for (int spin = 0; spin < (1 << 18) && !has_ext[n]; ++spin) {
                                __builtin_amdgcn_s_sleep(4);
#pragma unroll
                                for (int c4 = 0; c4 < 4; ++c4) mp[n][c4] = load_pair(mslot[n] + c4);
                                has_ext[n] = complete();
                            }
                            if (!has_ext[n]) wait_failed = 1;
                        }
                    }
                }
            }
            float G[4], wesum[4];
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                G[c4] = tv[c4] ? (cnt * w4[c4] - S4[c4]) * inv_b : 0.0f;      // descent gradient of Eq. 9
                wesum[c4] = 0.0f;
            }
            int ndelta = 0;
            if (p.parts > 1) {
                // Partial messages (Sec. 4.4): lambda, Eq. 4 and Eq. 6 per centroid row.  A row is spread over the NQ
                // task lanes NQ*c .. NQ*c + NQ - 1; their partial sums are added with lane reads.  ndelta counts,
                // per lane, the accepted copies of ITS row.
                int nz = 0, accb = 0, near = 0;
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if (!has_ext[n]) continue;          // uniform
                    float we[4];
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
                    bool okl = in_part[n];
                    if (!det) {
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4) okl = okl && (int)(mp[n][c4] >> 32) >= 0;
                    }
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        we[c4] = 0.0f;
                        if (okl && tv[c4]) {
                            we[c4] = __uint_as_float((unsigned)(mp[n][c4] & 0xFFFFFFFFull));
                            const double wed = (double)we[c4];
                            const double a = ((double)w4[c4] - (double)p.eps * (double)G[c4]) - wed;
                            const double c2 = (double)w4[c4] - wed;
                            lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                        }
                    }
                    double l3 = 0.0, r3 = 0.0, n3 = 0.0;
                    int all3 = 1;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const int src = tc * NQ + q;
                        l3 += __shfl(lhs, src, 64); r3 += __shfl(rhs, src, 64); n3 += __shfl(nrm, src, 64);
                        all3 &= __shfl((int)okl, src, 64);
                    }
                    const bool rowok = has_task && all3 && n3 > 0.0;       // every lane of the row is there; lambda
                    const bool acc = rowok && (p.parzen ? (l3 < r3) : true);
                    if (acc) {
                        ndelta += 1;
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4) wesum[c4] += we[c4];
                    }
                    if (__ballot(rowok) != 0ull) nz |= 1 << n;
                    if (__ballot(acc) != 0ull) accb |= 1 << n;
                    if (__ballot(rowok && r3 > 0.0 && fabs(l3 - r3) / r3 < 1e-6) != 0ull) near = 1;
                }
                if (threadIdx.x == 0 && nz) {
                    long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                    cn[CNT_RECEIVED] += __builtin_popcount(nz);
                    cn[CNT_ACCEPTED] += __builtin_popcount(accb);
                    cn[CNT_PARZEN_NEAR] += near;
                }
            }
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                if (has_ext[n] && p.parts == 1) {           // uniform over the workgroup
                    float we[4];
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        we[c4] = 0.0f;
                        if (tv[c4]) {
                            we[c4] = __uint_as_float((unsigned)(mp[n][c4] & 0xFFFFFFFFull));
                            const double wed = (double)we[c4];
                            const double a = ((double)w4[c4] - (double)p.eps * (double)G[c4]) - wed;
                            const double c2 = (double)w4[c4] - wed;
                            lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                        }
                    }
                    lhs = wave_sum(lhs); rhs = wave_sum(rhs); nrm = wave_sum(nrm);
                    if (nrm > 0.0) {     // lambda of Eq. 3: an all-zero buffer is empty
                        const int delta = p.parzen ? (lhs < rhs) : 1;       // Eq. 4, every buffer on its own (Eq. 6)
                        if (delta) {
                            ndelta += 1;
#pragma unroll
                            for (int c4 = 0; c4 < 4; ++c4) wesum[c4] += we[c4];
                        }
                        if (threadIdx.x == 0) {
                            long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                            cn[CNT_RECEIVED] += 1;
                            cn[CNT_ACCEPTED] += delta;
                            if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                        }
                    }
                }
            }
            // Eq. 6 (one buffer: Eq. 7) and Alg. 5 line 8
            const float inv_n = (NB == 1 && p.parts == 1) ? 0.5f : 1.0f / (float)(ndelta + 1);
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                float step = G[c4];
                if (ndelta) step += w4[c4] - inv_n * (w4[c4] + wesum[c4]);
                w4[c4] = w4[c4] - p.eps * step;
            }
            if (merge_point) {
                // every wave has read the buffers (the values were used above): tell senders of later rounds so.
                // Deterministic mode: the stamps in a buffer never match again, which empties it.  Free-running
                // mode: a message is used once, so it is marked empty.
                if constexpr (NW > 1) __syncthreads();
                if (threadIdx.x == 0)
                    __hip_atomic_store(p.consumed + i, (int)round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if (!det && has_ext[n] && wave == 0 && has_task && in_part[n]) {
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4)
                            store_pair(const_cast<unsigned long long *>(mslot[n]) + c4, ~0ull);
                    }
                }
            }

            // ---- send (Alg. 5 line 9): the first wave writes ----
            if (send_point && wave == 0) {
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if (p.drop_thr != 0 && message_dropped(p.seed, round, i, p.drop_thr, n)) continue;
                    const int spar = det ? (int)(round & 1) : 0;
                    if (sync && det && round >= 2 && !wait_failed && ackv[n] < (int)(round - 1)) {
                        // the buffer still holds the message of round-2 until the recipient has passed
                        // the merge point of round-1 (it had not when this step began: look again)
                        if (!wait_flag(p.consumed + peer[n], (int)(round - 1), true)) wait_failed = 1;
                    }
                    unsigned long long *dst = reinterpret_cast<unsigned long long *>(p.slot) +
                                              (((size_t)(spar * NB + n) * p.W + peer[n]) * NT + (has_task ? lane : 0)) * 4;
                    if (has_task && (p.parts == 1 || tc % p.parts == (int)((round + peer[n] + n) % p.parts))) {
#pragma unroll
                        for (int c4 = 0; c4 < 4; ++c4) store_pair(dst + c4, pack_pair(w4[c4], (int)round));
                    }
                }
                if (lane == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
            }

            // advance the clock
            s_epoch = s_next;
            if (p.E > 0 && ++te == p.E) { te = 0; ++round; }
        }

        if (wave == 0) {
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                if (tv[c4]) p.w[(size_t)i * KD + te_[c4]] = w4[c4];
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

template <int K, int D, int PF, int NW, int RS, int NB>
hipError_t launch_variant_nb(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    auto kern = small_steps_kernel<K, D, PF, NW, RS, NB>;
    if (!persistent) {
        hipLaunchKernelGGL(kern, dim3(p.W), dim3(64 * NW), 0, s, p, t0, t1, 0);
        return hipGetLastError();
    }
    // one launch for the whole run: every workgroup must be resident at the same time
    // (resident workgroups of this kernel on the current device: queried once per device and variant)
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

// Several buffers: the message pairs of all buffers sit in registers during a step, so the ring depth is at most 4, and
// 2 for four buffers (measured on the streaming workload: 1.22 ms against 1.38 ms with depth 4 and register spills;
// three buffers: 1.10 ms with depth 4 and a few spills against 1.15 ms with depth 2); the caller limits it.  Only the
// shapes with shared rows are built.
template <int K, int D, int PF, int NW, int RS>
hipError_t launch_variant(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    if (p.nb == 1) return launch_variant_nb<K, D, PF, NW, RS, 1>(p, t0, t1, s, persistent);
    if constexpr (PF <= 4 && RS == 2) {
        if (p.nb == 2) return launch_variant_nb<K, D, PF, NW, RS, 2>(p, t0, t1, s, persistent);
        if (p.nb == 3) return launch_variant_nb<K, D, PF, NW, RS, 3>(p, t0, t1, s, persistent);
    }
    if constexpr (PF == 2 && RS == 2) {
        if (p.nb == 4) return launch_variant_nb<K, D, PF, NW, RS, 4>(p, t0, t1, s, persistent);
    }
    return hipErrorInvalidValue;
}

template <int NW, int RS>
hipError_t launch_shape(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent, int pf)
{
    // RS = 2 leaves 256 registers per wave: ring depth at most 4
    if constexpr (RS == 1) {
        if (pf >= 8) return launch_variant<10, 10, 8, NW, RS>(p, t0, t1, s, persistent);
    }
    if (pf >= 4) return launch_variant<10, 10, 4, NW, RS>(p, t0, t1, s, persistent);
    return launch_variant<10, 10, 2, NW, RS>(p, t0, t1, s, persistent);
}

}  // namespace

namespace {

// Eq. 8 for k = d = 10: a lane takes a sample (40 B straight into registers, four samples in flight), forms
// the expanded-form scores x.w_c - |w_c|^2/2 against register copies of the state and adds
// |x|^2/2 - max_c score = min_c |x - w_c|^2 / 2 in fp64.  The assignment of samples to threads is fixed,
// so is every order of summation: the result does not depend on scheduling.
template <int K, int D>
__global__ __launch_bounds__(256) void quant_error_small_kernel(const float *__restrict__ x, long long N,
                                                                const float *__restrict__ w, double *partials)
{
    __shared__ float sw[K * D];
    __shared__ float sh[K];
    __shared__ double red[256];
    for (int e = threadIdx.x; e < K * D; e += 256) sw[e] = w[e];
    __syncthreads();
    if (threadIdx.x < K) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) s = fmaf(sw[threadIdx.x * D + j], sw[threadIdx.x * D + j], s);
        sh[threadIdx.x] = -0.5f * s;
    }
    __syncthreads();
    float wv[K * D], hv[K];
#pragma unroll
    for (int e = 0; e < K * D; ++e) wv[e] = sw[e];
#pragma unroll
    for (int c = 0; c < K; ++c) hv[c] = sh[c];

    constexpr int U = 4;
    const long long stride = (long long)gridDim.x * 256;
    double sum = 0.0;
    for (long long n0 = (long long)blockIdx.x * 256 + threadIdx.x; n0 < N; n0 += U * stride) {
        float xr[U][D];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long n = n0 + u * stride;
            load_row<D>(xr[u], x + (size_t)(n < N ? n : N - 1) * D);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float x2 = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) x2 = fmaf(xr[u][j], xr[u][j], x2);
            float best = -INFINITY;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                float sc = hv[c];
#pragma unroll
                for (int j = 0; j < D; ++j) sc = fmaf(xr[u][j], wv[c * D + j], sc);
                best = fmaxf(best, sc);
            }
            if (n0 + u * stride < N) sum += (double)fmaxf(0.5f * x2 - best, 0.0f);
        }
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0];
}

}  // namespace

hipError_t launch_quant_error_small(const float *x, long long N, const float *w, double *partials, int nblocks, hipStream_t s)
{
    hipLaunchKernelGGL((quant_error_small_kernel<10, 10>), dim3(nblocks), dim3(256), 0, s, x, N, w, partials);
    return hipGetLastError();
}

size_t small_kernel_message_bytes(int k, int d)
{
    if (!(k == 10 && d == 10)) return 0;
    return (size_t)k * ((d + 1 + 3) / 4) * 4 * sizeof(unsigned long long);      // NT lanes x 4 (value, stamp) pairs
}

bool small_kernel_supports(int k, int d, int b)
{
    (void)b;
    return k == 10 && d == 10;
}

hipError_t launch_small_steps(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    if (!(p.k == 10 && p.d == 10)) return hipErrorInvalidValue;
    // Shape of a worker: two waves sharing accumulator rows pairwise (default: 8 waves per CU with one
    // worker per 4 SIMD slots), one wave with shared rows (many workers: twice as many resident), or
    // one wave with private rows.  tune: bits 2-3 pick the shape, bits 0-1 limit the ring depth
    // (1: 4, 2: 2); the value 3 in bits 0-1 is handled by the caller (one launch per round).
    int shape = (p.tune >> 2) & 3;          // 0 = by number of workers, 1 = 1 wave private rows, 2 = 1 wave shared rows, 3 = 2 waves
    if (shape == 0) shape = p.W > 1024 ? 2 : 3;
    const int nw = shape == 3 ? 2 : 1;
    const int ngw = ((p.b + 63) / 64 + nw - 1) / nw;
    // ring depth: the largest of 8, 4 that divides the number of groups per mini-batch and wave, else 2
    // (the kernel then pads the group count with masked groups)
    int pf = (ngw % 8 == 0) ? 8 : (ngw % 4 == 0) ? 4 : 2;
    if ((p.tune & 3) == 1 && pf > 4) pf = 4;
    if ((p.tune & 3) == 2 && pf > 2) pf = 2;
    if (p.nb >= 4 && pf > 2) pf = 2;        // registers: see launch_variant
    switch (shape) {
        case 1: return launch_shape<1, 1>(p, t0, t1, s, persistent, pf);
        case 2: return launch_shape<1, 2>(p, t0, t1, s, persistent, pf);
        default: return launch_shape<2, 2>(p, t0, t1, s, persistent, pf);
    }
}

}  // namespace asgd
