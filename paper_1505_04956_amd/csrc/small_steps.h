// Step kernel for small states (k <= 16, a state of a few hundred floats): the streaming workloads.
//
// One workgroup of NW wavefronts per worker; a lane takes one sample at a time:
//   - the sample's d floats come straight from HBM into registers through a ring of PF register
//     buffers, so that PF-1 groups of 64 samples are in flight per wave; the ring runs across
//     mini-batch, round and worker boundaries (the addresses of later mini-batches do not depend on
//     the state), so the update between two mini-batches overlaps with loads; an address is a
//     wave-uniform base plus a 32-bit lane offset, two vector instructions per group;
//   - scores relative to centroid 0, t_k = x.(w_k - w_0) + (h_k - h_0) + 1 with h_k = -|w_k|^2/2
//     (largest t_k = nearest centroid; the |x|^2 term is common to all k), are chains of fused
//     multiply-adds against a wave-uniform copy of w_k - w_0 held in vector registers;
//   - the centroid index rides in the low 4 mantissa bits of t_k, and the two largest t_k come out
//     of a network of three-input max/median instructions; when they are closer than a rigorous
//     bound on the fp32 rounding error (packing included), the lane decides exactly in fp64, so the
//     assignment is the exact-arithmetic nearest centroid of the fp32 state;
//   - the gradient sums of Eq. 9 are kept in LDS as 32-bit fixed-point cells, one copy per lane (RS = 1) or sixteen
//     copies per wave, one for the lanes l, l+16, l+32, l+48 (RS = 2): a sample adds its d values, each scaled by its column's power of two and rounded
//     to an integer, and a one for the count to the cells of its centroid with d + 1 LDS atomics that return
//     nothing.  Lanes past the end of a mini-batch use a scratch centroid.  Once per step the copies of every cell
//     are summed; the cells are never cleared, a step's sums are the totals now minus the totals a step ago,
//     modulo 2^32.
// The part of a step that does not stream (row sums, totals, update, the new wave-uniform copies) is
// on every worker's critical path, once per mini-batch; it is written for few instructions: all step
// bookkeeping is 32-bit and scalar, the state lives in registers in the layout the row sums come out
// in, and the wave-uniform copies are made with one LDS write and broadcast reads.
// The sums are integers, so they do not depend on the order of the additions; everything after them is formed in one
// fixed order: a run is reproducible bit for bit.
#pragma once

#include <string.h>

#include "asgd_internal.h"
#include "fixed_point_sums.h"

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
// Three sums over the wave at once, level by level: the lane reads of a level are issued together and waited for
// once, instead of three butterflies of six dependent round trips each one after the other.  Same additions in the
// same order as wave_sum for each of the three, so every lane ends with the same bits.
__device__ __forceinline__ void wave_sum3(double &a, double &b, double &c)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double pa = __shfl_xor(a, off, 64), pb = __shfl_xor(b, off, 64), pc = __shfl_xor(c, off, 64);
        __builtin_amdgcn_sched_barrier(0);
        a += pa; b += pb; c += pc;
        __builtin_amdgcn_sched_barrier(0);
    }
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

// value of `v` in lane `src_lane_x4 / 4` (any lane may read any lane; one LDS-pipe instruction, no LDS memory)
__device__ __forceinline__ float lane_read(int src_lane_x4, float v)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane_x4, __float_as_int(v)));
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

// The lanes of a wave hand values to each other through LDS (the copies of the state, the accumulator cells).  The
// hardware executes the LDS accesses of a wave in program order; this keeps the compiler from moving a read above
// the write or atomic of another lane that it has to see (to a single lane the two look unrelated).
__device__ __forceinline__ void phase_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One 32-bit value from a wave-uniform address, through the scalar unit: a vector load would have to be waited for with
// the vector-memory counter, and loads return in order, so that wait would cover every sample load issued before it.
// (Read only: the table it is used for was written by an earlier kernel.)
__device__ __forceinline__ int uniform_load(const int *ptr)
{
    int v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(ptr) : "memory");
    return v;
}

// Adds to a counter in global memory without reading it back: an atomic without return value is not waited for,
// whereas "counter += v" is a load the wave would have to wait for, and on this chip that wait also covers every
// sample load issued before it.
__device__ __forceinline__ void bump(long long *counter, int v)
{
    if (v) (void)__hip_atomic_fetch_add(reinterpret_cast<unsigned long long *>(counter), (unsigned long long)v, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT);
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

// Polls a workgroup may spend, in total, on all the waits of a launch: every wait of this kernel draws on one
// budget, so a launch whose workgroups do not find each other ends after a fraction of a second plus under a
// millisecond per round it covers (a poll takes ~0.3 us of sleep plus one uncached load).  When the budget is gone the caller
// goes on without the message (and waits for nothing else) and the host reports the failure.
constexpr int WAIT_BUDGET = 1 << 19;
constexpr int WAIT_PER_ROUND = 512;      // ... plus this many per round of the launch (the host keeps launches to 1024 rounds)

__device__ __forceinline__ bool wait_at_least(const int *flag, int want, int &budget)
{
    while (budget > 0) {
        if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= want) return true;
        __builtin_amdgcn_s_sleep(4);
        --budget;
    }
    return false;
}

// Geometry of a small state: per centroid d sums and a count, padded to NQ groups of four elements.
template <int K, int D>
struct SmallGeo {
    static constexpr int KD = K * D;
    static constexpr int NQ = (D + 1 + 3) / 4;      // groups of four elements per centroid: d sums, count, padding
    static constexpr int RW = 4 * NQ;               // floats per padded row
    static constexpr int NT = K * NQ;               // tasks: four elements of one centroid each
    static constexpr int NPART = 64 / NT;           // lanes of a wave that share a task split the copies in the reduction
    static constexpr int CQ = D / 4, CI = D % 4;    // float4 and component that hold the count
    static_assert(K >= 2 && K <= 16, "index packing uses 4 bits");
    static_assert(NT <= 64 && NPART >= 1, "state too large for this kernel");
};

// Nearest centroid of a lane's sample from its tagged scores tk and the two largest of them (largest = nearest;
// tag = 15 - index in the low 4 mantissa bits): exact where the fp32 scores are closer than thr.  wsf: the copy of the
// state in LDS, rows padded to RW floats.
template <int K, int D>
__device__ __forceinline__ int decide(const float (&tk)[K], float best, float second, const float (&xc)[D], bool valid,
                                      float thr, const float *wsf, int &rechecks)
{
    constexpr int RW = SmallGeo<K, D>::RW;
    int arg = 15 - (int)(__float_as_uint(best) & 15u);
    if (valid && !(best - second > thr)) {
        // Too close to call in fp32.  Candidates are the centroids within thr of the best; with two of them their
        // distances are compared exactly (fp64), with more all k distances are recomputed in fp64, direct form; the
        // lowest index wins exact ties.
        float xe[D];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            xe[j] = xc[j];
            asm volatile("" : "+v"(xe[j]));     // keep the conversions below inside this branch
        }
        // count the candidates
        int ncand = 0;
#pragma unroll
        for (int c = 0; c < K; ++c) ncand += (tk[c] >= best - thr) ? 1 : 0;
        if (ncand <= 2) {
            const int ca = arg, cb = 15 - (int)(__float_as_uint(second) & 15u);
            // |x - w_a|^2 - |x - w_b|^2 = sum_j (w_aj - w_bj) (w_aj + w_bj - 2 x_j)
            double dd = 0.0;
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const double wa = (double)wsf[ca * RW + j], wb = (double)wsf[cb * RW + j];
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
                    double diff = (double)xe[j] - (double)wsf[c * RW + j];
                    sd += diff * diff;
                }
                if (sd < dbest) { dbest = sd; darg = c; }
            }
            arg = darg;
        }
        rechecks += 1;
    }
    return arg;
}

// Row updates: the accumulator of a wave holds 32-bit fixed-point sums (fixed_point_sums.h), element-major - cell
// (centroid c, element j, copy r) lies at ((c * CE + j) * RL + r) * 4 bytes, element D being the count and CE = D + 1 or
// D + 2, whichever is odd -, and a sample
// adds its D terms and a one for the count with D + 1 LDS atomics that return nothing.  The lanes of one such instruction
// (same j, consecutive r) fall into consecutive banks; there is no read-modify-write chain through LDS and no exchange
// of operands between lanes that share a copy, and because integer addition does not depend on the order, the sums
// - and with them the whole run - are the same whatever order the lanes get their turn in.
typedef __attribute__((address_space(3))) unsigned *lds_u32_ptr;
typedef int lds_ivec4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) lds_ivec4 *lds_ivec4_ptr;
__device__ __forceinline__ void lds_add_u32(unsigned addr, unsigned v)
{
    (void)__hip_atomic_fetch_add((lds_u32_ptr)(size_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Sums the cells of elements 4q .. 4q+3 of one centroid over ROWS copies (they are not cleared, see the caller): `cells` is the LDS byte address of
// copy 0 of element 4q (a multiple of ROWS * 4), elem_bytes the distance between elements.  Four copies are read at a
// time; block rb of the visit is block rb ^ (task mod ROWS/4), so that the lanes of one access do not all hit the same
// banks, and its address is ONE exclusive-or away from the first (no add, mask and shift per block).
template <int ROWS>
__device__ __forceinline__ void sum_cells(unsigned cells, unsigned elem_bytes, int task, int (&s)[4])
{
    static_assert(ROWS % 4 == 0 && ((ROWS / 4) & (ROWS / 4 - 1)) == 0, "blocks of four copies, rotated by exclusive-or");
    unsigned first = cells + ((unsigned)(task & (ROWS / 4 - 1)) << 4);
    // (the addresses are formed here, at every call, from a value the compiler cannot see through: hoisted out of
    // the step loop they would be registers held across the streaming part)
    asm volatile("" : "+v"(first));
    const lds_ivec4 zero = {0, 0, 0, 0};
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
        lds_ivec4 t = zero;
#pragma unroll
        for (int rb = 0; rb < ROWS / 4; ++rb) {
            lds_ivec4_ptr q = (lds_ivec4_ptr)(size_t)((first ^ (unsigned)(rb << 4)) + (unsigned)c4 * elem_bytes);
            const lds_ivec4 v = *q;
            t = rb == 0 ? v : t + v;
        }
        s[c4] = (t.x + t.y) + (t.z + t.w);
    }
}

// The walk of a workgroup through its work, the same in every wave: segments of steps (in deterministic mode a
// segment ends at a multiple of E), inside a segment the workers blockIdx.x, blockIdx.x + gridDim.x, ... in turn.
// All 32-bit and scalar; the only 64-bit divisions are in the constructor.
struct SmallWalk {
    int nsteps, E, S, W, b;
    bool xchg, rounds;
    int done, seg, s_seg, s_next_seg, te_seg, round_seg;
    bool last_seg;
    long long dump0;
    __device__ __forceinline__ SmallWalk(const StepParams &p, long long t0, long long t1)
    {
        E = p.E; S = (int)p.S; W = p.W; b = p.b;        // (the host keeps S and t1 - t0 below 2^31)
        xchg = (E > 0 && W > 1);
        rounds = xchg && p.mode == ASGD_MODE_DETERMINISTIC;      // work is cut at multiples of E
        nsteps = (int)(t1 - t0);
        round_seg = xchg ? (int)(t0 / E) : 0;
        te_seg = xchg ? (int)(t0 % E) : 0;
        s_seg = (int)(t0 % p.S);
        dump0 = t0 - p.t_dump0;                         // step of the dump buffer that step t0 goes to
        done = 0;
        begin_segment();
    }
    __device__ __forceinline__ void begin_segment()
    {
        seg = rounds ? min(nsteps - done, E - te_seg) : nsteps - done;
        last_seg = done + seg >= nsteps;
        s_next_seg = (int)(((unsigned)s_seg + (unsigned)seg) % (unsigned)S);
    }
    __device__ __forceinline__ void end_segment()
    {
        done += seg;
        s_seg = s_next_seg;
        if (rounds) {                       // (otherwise there is only one segment)
            te_seg += seg;
            if (te_seg == E) { te_seg = 0; ++round_seg; }
        }
        if (done < nsteps) begin_segment();
    }
    // First mini-batch of this segment in a shard, and of whatever the workgroup does after this segment of worker i
    // (only loaded from; at the very end any valid address will do).  shard: first row of worker i's shard; first:
    // of the workgroup's first worker; stride: elements between the shards of two successive workers of the
    // workgroup.  (Pointers are carried along instead of being formed from the worker number: 64-bit products are
    // many scalar instructions, and this runs on every worker's critical path at every round boundary.)
    __device__ __forceinline__ const float *first_batch(const float *shard, int d) const
    {
        return shard + (size_t)((unsigned)s_seg * (unsigned)b) * (unsigned)d;
    }
    __device__ __forceinline__ const float *batch_after(const float *shard, const float *first, size_t stride, int i, int d) const
    {
        if (i + (int)gridDim.x < W) return shard + stride + (size_t)((unsigned)s_seg * (unsigned)b) * (unsigned)d;
        if (!last_seg) return first + (size_t)((unsigned)s_next_seg * (unsigned)b) * (unsigned)d;
        return first_batch(shard, d);
    }
};

// What a wave that holds a worker's state does in a step besides streaming: the wave-uniform copies of the state, the
// early fetch of the messages, gradient, merge (Eq. 4, Eq. 6 / Eq. 7), update (Alg. 5, update), send (Alg. 5, send).
//
// State layout in registers ("task layout"): lane l < NT = K*NQ holds the four elements (c, 4q .. 4q+3) of the state
// with c = l / NQ, q = l % NQ (elements past d do not exist and stay 0); the same lane receives the totals of the
// accumulator cells of these four elements once per step.  Written to LDS as one float4 per lane this is the state with
// its rows padded to 4*NQ floats.
//   NB     external buffers per worker = recipients per message (Eq. 3 / Eq. 6); NB = p.nb
//   PARTS  partial messages (Sec. 4.4) compiled in; p.parts > 1 needs it
template <int K, int D, int NB, bool PARTS>
struct SmallKeeper {
    using G = SmallGeo<K, D>;
    static constexpr int NQ = G::NQ, NT = G::NT, CQ = G::CQ, CI = G::CI, KD = G::KD;

    int lane, tc, tq, elem0, bp_row, bp_w0;
    bool has_task, tv[4];
    float w4[4];                                    // this lane's four elements of the state
    float sum_xmax, inv_b, eps;
    const unsigned long long *mslot[NB];
    unsigned long long mp[NB][4];
    int peer[NB], ackv[NB];
    int wait_failed, budget;

    __device__ __forceinline__ void init(const StepParams &p, int lane_)
    {
        lane = lane_;
        has_task = lane < NT;
        tc = has_task ? lane / NQ : 0;
        tq = has_task ? lane % NQ : 0;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            tv[c4] = has_task && (4 * tq + c4 < D);         // which of the four elements exist
            w4[c4] = 0.0f;
        }
        elem0 = tc * D + 4 * tq;                    // index of the first of them in the k x d state
        bp_row = (lane - tq) * 4;                   // lane_read address of the first lane of this lane's centroid
        bp_w0 = tq * 4;                             // ... of the lane that holds the same float4 of centroid 0
        sum_xmax = 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) sum_xmax += p.xabsmax[j];
        inv_b = 1.0f / (float)p.b;
        eps = p.eps;
        wait_failed = 0;
        budget = p.wait_polls > 0 ? p.wait_polls : WAIT_BUDGET;
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            mslot[n] = nullptr; peer[n] = 0; ackv[n] = 0;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) mp[n][c4] = 0ull;
        }
    }
    __device__ __forceinline__ void load_state(const StepParams &p, int i)
    {
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) w4[c4] = tv[c4] ? p.w[(size_t)i * KD + elem0 + c4] : 0.0f;
        // wait for the state here, once, not at the head of the step loop, where the wait would also cover the
        // samples fetched ahead
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) asm volatile("" : "+v"(w4[c4]));
    }
    __device__ __forceinline__ void store_state(const StepParams &p, int i) const
    {
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            if (tv[c4]) p.w[(size_t)i * KD + elem0 + c4] = w4[c4];
        }
    }

    // Writes the copies of the state that the score chains and the exact re-evaluation read (one float4 per task lane
    // each: wst = the state, wdt = row k: w_k - w_0 in elements < D and (h_k - h_0) + 1 in element D, h_k = -|w_k|^2/2)
    // and returns the rounding-error bound below which two scores count as too close to call.  The caller fences.
    __device__ __forceinline__ float publish(float4 *wst, float4 *wdt) const
    {
        float hs = 0.0f;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) hs = fmaf(w4[c4], w4[c4], hs);
        float hsum = lane_read(bp_row, hs);
#pragma unroll
        for (int q = 1; q < NQ; ++q) hsum += lane_read(bp_row + 4 * q, hs);      // same order in all lanes of a row
        const float hl = -0.5f * hsum;                                           // h_k, in every lane of centroid k
        const float h0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hl), 0));
        const float hol = (hl - h0) + 1.0f;
        float wdv[4];
        float dabs = 0.0f;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            const float w0q = lane_read(bp_w0, w4[c4]);
            wdv[c4] = tv[c4] ? w4[c4] - w0q : 0.0f;
            dabs = fmaxf(dabs, fabsf(wdv[c4]));
        }
        if (tq == CQ) wdv[CI] = hol;
        if (has_task) {
            wst[lane] = make_float4(w4[0], w4[1], w4[2], w4[3]);
            wdt[lane] = make_float4(wdv[0], wdv[1], wdv[2], wdv[3]);
        }
        // max_k |h_k| bounds max_k |h_k - h_0| up to a factor 2; one wave-wide max serves both
        const float hmax = wave_max_nonneg(has_task ? fabsf(hl) : 0.0f);
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
        return 3.0f * 5.9604645e-8f *
               ((float)(D + 33) * Abound + (float)(D + 34) * (hdmax + 1.0f) + (float)(2 * D + 2) * hmax);
    }

    // cyclic shift of copy n in round r: 1 + (shift of copy 0 - 1 + n) mod (W - 1)
    // (the shifts of the rounds of a launch come from a table: no 64-bit division in the kernel)
    __device__ __forceinline__ int shift_of(const StepParams &p, int r, int n) const
    {
        int sh = uniform_load(p.shift_tab + ((long long)r - p.shift_r0)) + n;
        if (sh > p.W - 1) sh -= p.W - 1;
        return sh;
    }

    // Called once the ring has gone round after fetch(): every load that fetch() issued has returned by then (loads
    // return in order, and samples requested after them have been used).  Telling the compiler so here, where it can
    // count the loads issued since, keeps it from waiting for ALL outstanding loads - the samples of the next
    // mini-batch among them - where the values are first used, at the end of the step.
    __device__ __forceinline__ void settle_fetched()
    {
#pragma unroll
        for (int n = 0; n < NB; ++n) {
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) asm volatile("" : "+v"(mp[n][c4]));
            asm volatile("" : "+v"(ackv[n]));
        }
    }

    // Exchange, early part: fetch at the start of a step what its end will need, so that the latency of these
    // accesses (they bypass the caches) runs behind the mini-batch.  sender: this wave writes the worker's messages.
    __device__ __forceinline__ void fetch(const StepParams &p, int i, int round, bool merge_point, bool send_point, bool det,
                                          int sync, bool sender)
    {
        const int W = p.W;
        if (merge_point) {
            const int rpar = det ? ((round - 1) & 1) : 0;
            // buffer n of this worker (parity rpar): NT lanes x 4 pairs each; copy n of a message goes to buffer n
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                mslot[n] = reinterpret_cast<const unsigned long long *>(p.slot) +
                           (((size_t)(rpar * NB + n) * W + i) * NT + (has_task ? lane : 0)) * 4;
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) mp[n][c4] = load_pair(mslot[n] + c4);
            }
        }
        if (send_point && sender) {
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                ackv[n] = 0;
                if (det) {
                    peer[n] = i + shift_of(p, round, n);
                    if (peer[n] >= W) peer[n] -= W;
                    if (sync && round >= 2)
                        ackv[n] = __hip_atomic_load(p.consumed + peer[n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    peer[n] = peer_free(p.seed, round, i, W, n);
                }
            }
        }
    }

    // End of a step: S4 = totals of this lane's four elements of the gradient sums, cnt = the number of samples of the
    // lane's centroid.  BAR: several waves hold the state and read the buffers, a workgroup barrier
    // separates their reads from the release of the buffers.  sender: this wave writes messages, state and counters.
    template <bool BAR>
    __device__ __forceinline__ void finish(const StepParams &p, int i, int round, const float (&S4)[4], float cnt, bool merge_point,
                                           bool send_point, bool det, int sync, bool sender)
    {
        const int W = p.W;
        float Gr[4], wesum[4];
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            Gr[c4] = tv[c4] ? (cnt * w4[c4] - S4[c4]) * inv_b : 0.0f;      // descent gradient of Eq. 9
            wesum[c4] = 0.0f;
        }
        int ndelta = 0;
        const bool first = sender && lane == 0;

        if (merge_point) {
            // ---- a buffer is looked at once, at the first step of a round ----
            bool has_ext[NB], in_part[NB];
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                // complete = every pair of every task lane carries the stamp of round-1 (free-running: any stamp).
                // Partial messages: only the lanes whose centroid row belongs to the part that this copy carries
                // (free-running mode: the part follows from the round in the lane's own first stamp).
                in_part[n] = has_task;
                auto complete = [&]() -> bool {
                    bool ok = true;
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        const int st = (int)(mp[n][c4] >> 32);
                        ok = ok && (det ? st == round - 1 : st >= 0);
                    }
                    if constexpr (PARTS) {
                        if (p.parts > 1) {
                            const int mr = det ? round - 1 : (int)(mp[n][0] >> 32);
                            in_part[n] = has_task && mr >= 0 && tc % p.parts == (mr + i + n) % p.parts;
                            if (!det) return __ballot(in_part[n] && ok) != 0ull;      // some row is there
                            return __ballot(in_part[n] && !ok) == 0ull;
                        }
                    }
                    return __ballot(has_task && !ok) == 0ull;
                };
                has_ext[n] = complete();
                if (!has_ext[n] && sync && det && !wait_failed) {
                    // not there yet: wait for the sender of round-1 under the cyclic-shift schedule, unless its
                    // message is one of those the loss hook drops
                    int from = i - shift_of(p, round - 1, n);
                    if (from < 0) from += W;
                    if (p.drop_unannounced || !(p.drop_thr != 0 && message_dropped(p.seed, round - 1, from, p.drop_thr, n))) {
                        while (budget > 0 && !has_ext[n]) {
                            __builtin_amdgcn_s_sleep(4);
                            --budget;
#pragma unroll
                            for (int c4 = 0; c4 < 4; ++c4) mp[n][c4] = load_pair(mslot[n] + c4);
                            // (all four have returned before any is looked at: the test below stops at the first
                            // pair that does not match, and a load left pending here would make the compiler wait
                            // for ALL outstanding loads where the values are used, on every path)
#pragma unroll
                            for (int c4 = 0; c4 < 4; ++c4) asm volatile("" : "+v"(mp[n][c4]));
                            has_ext[n] = complete();
                        }
                        if (!has_ext[n]) wait_failed = 1;
                    }
                }
            }
            bool whole = true;
            if constexpr (PARTS) {
                if (p.parts > 1) {
                    whole = false;
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
                                const double a = ((double)w4[c4] - (double)eps * (double)Gr[c4]) - wed;
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
                        const bool accr = rowok && (p.parzen ? (l3 < r3) : true);
                        if (accr) {
                            ndelta += 1;
#pragma unroll
                            for (int c4 = 0; c4 < 4; ++c4) wesum[c4] += we[c4];
                        }
                        if (__ballot(rowok) != 0ull) nz |= 1 << n;
                        if (__ballot(accr) != 0ull) accb |= 1 << n;
                        if (__ballot(rowok && r3 > 0.0 && fabs(l3 - r3) / r3 < 1e-6) != 0ull) near = 1;
                    }
                    if (first && nz) {
                        long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                        bump(cn + CNT_RECEIVED, __builtin_popcount(nz));
                        bump(cn + CNT_ACCEPTED, __builtin_popcount(accb));
                        bump(cn + CNT_PARZEN_NEAR, near);
                    }
                }
            }
            if (whole) {
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    if (!has_ext[n]) continue;              // uniform over the workgroup
                    float we[4];
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        we[c4] = 0.0f;
                        if (tv[c4]) {
                            we[c4] = __uint_as_float((unsigned)(mp[n][c4] & 0xFFFFFFFFull));
                            const double wed = (double)we[c4];
                            const double a = ((double)w4[c4] - (double)eps * (double)Gr[c4]) - wed;
                            const double c2 = (double)w4[c4] - wed;
                            lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                        }
                    }
                    wave_sum3(lhs, rhs, nrm);
                    if (nrm > 0.0) {     // lambda of Eq. 3: an all-zero buffer is empty
                        const int delta = p.parzen ? (lhs < rhs) : 1;       // Eq. 4, every buffer on its own (Eq. 6)
                        if (delta) {
                            ndelta += 1;
#pragma unroll
                            for (int c4 = 0; c4 < 4; ++c4) wesum[c4] += we[c4];
                        }
                        if (first) {
                            long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                            bump(cn + CNT_RECEIVED, 1);
                            bump(cn + CNT_ACCEPTED, delta);
                            bump(cn + CNT_PARZEN_NEAR, (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) ? 1 : 0);
                        }
                    }
                }
            }
            // every wave has read the buffers (the values were used above): tell senders of later rounds so.
            // Deterministic mode: the stamps in a buffer never match again, which empties it.  Free-running
            // mode: a message is used once, so it is marked empty.
            if constexpr (BAR) __syncthreads();
            if (first) __hip_atomic_store(p.consumed + i, round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                if (!det && has_ext[n] && sender && has_task && in_part[n]) {
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) store_pair(const_cast<unsigned long long *>(mslot[n]) + c4, ~0ull);
                }
            }
        }

        // Eq. 6 (one buffer: Eq. 7) and Alg. 5, update
        {
            const bool half = (NB == 1) && !(PARTS && p.parts > 1);
            const float inv_n = half ? 0.5f : 1.0f / (float)(ndelta + 1);
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                float step = Gr[c4];
                if (ndelta) step += w4[c4] - inv_n * (w4[c4] + wesum[c4]);
                w4[c4] = w4[c4] - eps * step;
            }
        }

        // ---- send (Alg. 5, send) ----
        if (send_point && sender) {
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                if (p.drop_thr != 0 && message_dropped(p.seed, round, i, p.drop_thr, n)) continue;
                const int spar = det ? (round & 1) : 0;
                if (sync && det && round >= 2 && !wait_failed && ackv[n] < round - 1) {
                    // the buffer still holds the message of round-2 until the recipient has passed
                    // the merge point of round-1 (it had not when this step began: look again)
                    if (!wait_at_least(p.consumed + peer[n], round - 1, budget)) wait_failed = 1;
                }
                unsigned long long *dst = reinterpret_cast<unsigned long long *>(p.slot) +
                                          (((size_t)(spar * NB + n) * W + peer[n]) * NT + (has_task ? lane : 0)) * 4;
                bool mine = has_task;
                if constexpr (PARTS) {
                    if (p.parts > 1) mine = has_task && tc % p.parts == (round + peer[n] + n) % p.parts;
                }
                if (mine) {
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) store_pair(dst + c4, pack_pair(w4[c4], round));
                }
            }
            if (lane == 0) bump(p.counters + (size_t)i * CNT_STRIDE + CNT_SENT, 1);
        }
    }
};

// Steps [t0, t1) of the workers blockIdx.x, blockIdx.x + gridDim.x, ..., with NW like waves per worker: wave v takes
// the groups v, v+NW, ... of every mini-batch from the loads to the accumulator cells, and every wave holds the state.
//   RS   lanes sharing a copy of the accumulator cells: 1 = every lane has its own (64 copies per wave); 2 = sixteen
//        copies per wave (32 for the shapes whose once-per-step sums need them), a quarter of the LDS and a quarter of the
//        once-per-step sums; lanes that share a copy and hold samples of one centroid take turns in the LDS unit.
//   sync = 0: the launch contains nothing a worker has to wait for (silent or free-running mode,
//             or the host ends every launch at a multiple of E); one workgroup per worker.
//   sync = 1: the whole run is one launch of co-resident workgroups.  A workgroup takes its workers
//             through one round (E steps) after the other; at the first step of a round a worker
//             waits for the stamp of the message addressed to it (written by the sender at the end
//             of the previous round), and a sender waits until the recipient has consumed the older
//             message that sits in the same buffer.  Every wait is on an earlier round, so the
//             waits cannot form a cycle.
// Score chains of the centroids C0 .. C0 + NC - 1 against the wave-uniform copy wv (row c - 1: w_c - w_0, element D:
// (h_c - h_0) + 1), advancing together element by element; the result goes to tk[c] with 15 - c in the low 4 mantissa
// bits.
template <int K, int D, int C0, int NC>
__device__ __forceinline__ void score_chains(const float (&xc)[D], const float (&wv)[K - 1][SmallGeo<K, D>::RW], float (&tk)[K])
{
    if constexpr (NC > 0) {
        float sc[NC];
#pragma unroll
        for (int e = 0; e < NC; ++e) sc[e] = fmaf(xc[0], wv[C0 + e - 1][0], wv[C0 + e - 1][D]);
#pragma unroll
        for (int j = 1; j < D; ++j) {
#pragma unroll
            for (int e = 0; e < NC; ++e) sc[e] = fmaf(xc[j], wv[C0 + e - 1][j], sc[e]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // (the chains end here, not further down where their results are used: without this the compiler sinks the
        // tails of the chains of one set into the next and serialises them)
#pragma unroll
        for (int e = 0; e < NC; ++e) asm volatile("" : "+v"(sc[e]));
#pragma unroll
        for (int e = 0; e < NC; ++e)
            tk[C0 + e] = __uint_as_float((__float_as_uint(sc[e]) & 0xFFFFFFF0u) | (unsigned)(15 - (C0 + e)));
    }
}

// Waves per SIMD the kernel is compiled for: RS (shared rows halve the LDS per wave so that two fit), unless the
// registers of the shape (the wave-uniform copy of w_k - w_0, the ring, about a hundred more) go past the 256 that two
// waves per SIMD leave each.
template <int K, int D, int PF, int RS>
constexpr int small_waves_per_simd()
{
    return (K - 1) * SmallGeo<K, D>::RW + PF * D + 96 <= 256 ? RS : 1;
}

template <int K, int D, int PF, int NW, int RS, int NB, bool PARTS>
__global__ __launch_bounds__(64 * NW)
__attribute__((amdgpu_waves_per_eu(small_waves_per_simd<K, D, PF, RS>(), small_waves_per_simd<K, D, PF, RS>())))
void small_steps_kernel(StepParams p, long long t0, long long t1, int sync)
{
    using G = SmallGeo<K, D>;
    constexpr int NQ = G::NQ, RW = G::RW, NT = G::NT, NPART = G::NPART;
    // copies of an accumulator cell per wave: one per lane, or sixteen (lanes r, r + 16, r + 32, r + 48 share one; 32 where
    // the once-per-step sums need that many to give every lane of a task four)
    constexpr int RL = RS == 1 ? 64 : (16 >= 4 * NPART ? 16 : 32);
    // Elements per centroid in the accumulator: d sums and the count, one more if that makes the number odd - then the
    // cells of neighbouring centroids start in different banks (with 16 copies: 48 banks on), and lanes that share a
    // copy but hold samples of different centroids seldom collide.  The once-per-step sums read 4 NQ elements from a
    // centroid's first, i.e. into the next centroid's cells, which is harmless: nothing is written there.
    constexpr int CE = (D + 1) % 2 ? D + 1 : D + 2;
    constexpr int RPP = RL / NPART;                 // copies one lane sums in the reduction
    static_assert(NW == 1 || NW == 2, "one or two waves per worker");
    static_assert(RS == 1 || RS == 2, "one copy of the cells per lane, or shared copies");
    static_assert(PF >= 2, "the ring needs the previous group's buffer");
    static_assert(RL % NPART == 0 && RPP % 4 == 0, "state too large for this kernel");

    // acc[wave][c * CE + j][r]: copy r (lanes r, r + RL, ...) of the fixed-point sum of element j of the samples of
    // centroid c, j = D: their count; centroid K is scratch for masked lanes; four elements of slack behind it for the
    // reads of the once-per-step sums
    __shared__ __align__(1024) unsigned acc[NW][(K + 1) * CE + 4][RL];      // (alignment: see sum_cells)
    __shared__ int4 before[NW][NT];                 // totals of a task lane's four elements after the previous step
    __shared__ float4 wst[NW][NT];                  // state, rows padded to RW floats; one copy per wave
    __shared__ float4 wdt[NW][NT];                  // row k: w_k - w_0 in elements < D, (h_k - h_0) + 1 in element D
    __shared__ int4 part[2][NW][NPART][NT];         // per-wave totals, double-buffered by step parity

    const int wave = NW == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int b = p.b, W = p.W, E = p.E;
    const bool det = (p.mode == ASGD_MODE_DETERMINISTIC);
    // groups of 64 samples per mini-batch and wave, rounded up to a multiple of the ring depth (the
    // extra groups are fully masked); group m of wave v covers samples [(v + m*NW)*64, +64)
    const int ngw = (((b + 63) / 64 + NW - 1) / NW + PF - 1) / PF * PF;
    // byte offset of a lane's sample inside a mini-batch: group*64*D*4 + lane*D*4, clamped to the last sample
    const unsigned lane_off = (unsigned)lane * (D * 4);
    const unsigned max_off = (unsigned)(b - 1) * (D * 4);
    constexpr unsigned GROUP_BYTES = 64u * D * 4u;
    auto sample_ptr = [&](const float *batch, int g) -> const float * {
        const unsigned goff = (unsigned)g * GROUP_BYTES;                      // scalar
        const unsigned off = min(lane_off + goff, max_off);
        return reinterpret_cast<const float *>(reinterpret_cast<const char *>(batch) + off);
    };

    SmallKeeper<K, D, NB, PARTS> kp;
    kp.init(p, lane);
    // the budget of polls grows with the rounds the launch covers: a healthy run of the streaming workload spends up
    // to ~30 polls per round on the workgroup that waits most
    if (p.wait_polls <= 0 && p.E > 0) kp.budget += WAIT_PER_ROUND * (int)min((t1 - t0) / p.E + 1, (long long)(1 << 20));
    for (int q = lane; q < ((K + 1) * CE + 4) * RL; q += 64) (&acc[wave][0][0])[q] = 0u;
    if (lane < NT) before[wave][lane] = make_int4(0, 0, 0, 0);

    // Fixed-point sums: the scale of every column (2^e with b * max|x_j| * 2^e < 2^30 and max|x_j| * 2^e < 2^22; 0 for a
    // column of zeros), the inverse scales of this lane's four elements in the task layout (the count needs none),
    // and the LDS byte address of this lane's copy of element 0 of centroid 0
    constexpr unsigned ELEM_BYTES = RL * 4u, CENT_BYTES = (unsigned)CE * ELEM_BYTES;
    float scl[D], inv4[4];
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) inv4[c4] = 0.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        int e = 0;
        const bool okj = fx_scale_exponent(b, p.xabsmax[j], true, &e);
        scl[j] = okj ? ldexpf(1.0f, e) : 0.0f;
        const float iv = okj ? ldexpf(1.0f, -e) : 0.0f;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4)
            if (kp.has_task && 4 * kp.tq + c4 == j) inv4[c4] = iv;
    }
    const unsigned wave_cells = (unsigned)(size_t)(lds_u32_ptr)&acc[wave][0][0];
    const unsigned lane_cell = wave_cells + (unsigned)(lane % RL) * 4u;
    unsigned scratch_cell = lane_cell + (unsigned)K * CENT_BYTES;
    // (opaque to the compiler, which would otherwise select between the two products and add lane_cell afterwards:
    // three instructions per group instead of a multiply-add and a select)
    asm volatile("" : "+v"(scratch_cell));
    const int lane_room = b - wave * 64 - lane;     // group m of this wave holds a sample for this lane iff m NW 64 < lane_room

    int rechecks = 0;
    int parity = 0;
    // LDS byte address of the totals of this lane's four elements over all copies after the previous step
    const unsigned before_cell = (unsigned)(size_t)(lds_u32_ptr)(unsigned *)&before[wave][kp.has_task ? lane : 0];
    SmallWalk wk(p, t0, t1);

    // ring of sample buffers: buffer u holds this wave's group m with m % PF == u
    float xr[PF][D];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
#pragma unroll
        for (int j = 0; j < D; ++j) xr[u][j] = 0.0f;
    }
    {
        const float *x0 = wk.first_batch(p.x + (size_t)blockIdx.x * (size_t)p.H * D, D);
#pragma unroll
        for (int u = 0; u + 1 < PF; ++u) load_row<D>(xr[u], sample_ptr(x0, wave + u * NW));
        // Wait for them here, once per launch.  The compiler may issue these loads in any order, and a loop entered
        // with buffer 0 as the youngest load outstanding would make it wait, at the head of EVERY turn of the ring,
        // until no load at all is outstanding (the count it waits for has to hold on every path into the loop).
#pragma unroll
        for (int u = 0; u + 1 < PF; ++u) {
#pragma unroll
            for (int j = 0; j < D; ++j) asm volatile("" : "+v"(xr[u][j]));
        }
    }

    // A workgroup with one worker keeps its state in registers from segment to segment (every wave holds the same
    // values); one that takes several workers in turn stores and reloads it.
    const bool one_worker = (long long)blockIdx.x + gridDim.x >= W;

    const float *xs_first = p.x + (size_t)blockIdx.x * (size_t)p.H * D;      // shard of the workgroup's first worker
    const size_t xs_stride = (size_t)gridDim.x * (size_t)p.H * D;
    while (wk.done < wk.nsteps) {
        const float *xs = xs_first;                                 // shard of the worker in turn
        for (int i = blockIdx.x; i < W; i += gridDim.x, xs += xs_stride) {
            const float *xb = wk.first_batch(xs, D);                // the current mini-batch
            const float *x_after = wk.batch_after(xs, xs_first, xs_stride, i, D);
            if (!one_worker || wk.done == 0) kp.load_state(p, i);
            int s_epoch = wk.s_seg, te = wk.te_seg, round = wk.round_seg;

            for (int ls = 0; ls < wk.seg; ++ls) {
                // ---- wave-uniform copies of the state: every lane gets w_k - w_0 and (h_k - h_0) + 1 ----
                const float thr = kp.publish(wst[wave], wdt[wave]);
                phase_fence();      // the copies are per wave: the lanes of this wave only have to see each other's writes
                float wv[K - 1][RW];                                 // row k-1: w_k - w_0, (h_k - h_0) + 1 at element D
#pragma unroll
                for (int c = 1; c < K; ++c) {
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const float4 v = wdt[wave][c * NQ + q];
                        wv[c - 1][4 * q] = v.x; wv[c - 1][4 * q + 1] = v.y; wv[c - 1][4 * q + 2] = v.z; wv[c - 1][4 * q + 3] = v.w;
                    }
                }
                const float *wsf = reinterpret_cast<const float *>(&wst[wave][0]);

                // The instruction arbiter of a SIMD prefers the older of its two waves, which makes the workgroups that
                // were dispatched later run slower - and with rounds coupled through the exchange everybody ends
                // up waiting for them.  Alternating the wave priority step by step, in opposite phase for the two
                // halves of the grid (dispatch order), evens the shares out.
                if ((((wk.done + ls) & 1) ^ (blockIdx.x * 2 >= gridDim.x ? 1 : 0)) != 0)
                    __builtin_amdgcn_s_setprio(1);
                else
                    __builtin_amdgcn_s_setprio(0);

                const bool merge_point = wk.xchg && te == 0 && round > 0;      // t > 0 and t mod E == 0
                const bool send_point = wk.xchg && te + 1 == E;
                // what the first step of a launch finds in the buffers was sent before the launch: nothing to wait for
                const int sync_now = (wk.done + ls) > 0 ? sync : 0;
                kp.fetch(p, i, round, merge_point, send_point, det, sync_now, wave == 0);

                const bool last_step = ls + 1 == wk.seg;
                const int s_next = (s_epoch + 1 == wk.S) ? 0 : s_epoch + 1;
                // the mini-batch after this one
                const float *xbn = last_step ? x_after : (s_next == 0 ? xs : xb + (size_t)b * D);
                int32_t *dump = p.dump ? p.dump + ((size_t)(wk.dump0 + wk.done + ls) * W + i) * b : nullptr;
                const float tk0 = __uint_as_float(0x3F800000u | 15u);     // t_0 = 1 with the index of centroid 0

                int m0 = 0;
                do {        // (ngw >= PF: at least one turn, which the compiler has to know for settle_fetched)
                    // Refills of this turn: slot 0 takes group m0 + PF - 1 of this mini-batch, slot u >= 1 group
                    // m0 + PF + u - 1, which lies in the next mini-batch for all of them at once in the last turn
                    // (ngw is a multiple of PF).  One scalar decision per turn, constants per slot.
                    const bool tail = m0 + PF >= ngw;
                    const float *pbase = tail ? xbn : xb;
                    const unsigned turn_off = lane_off + (unsigned)(wave + NW * (tail ? 0 : m0 + PF)) * GROUP_BYTES;
                    const unsigned own_off = lane_off + (unsigned)(wave + NW * (m0 + PF - 1)) * GROUP_BYTES;
#pragma unroll
                    for (int u = 0; u < PF; ++u) {
                        const int up = (u + PF - 1) % PF;           // buffer of the previous group
                        const int m = m0 + u;
                        const float(&xc)[D] = xr[u];

                        // t_k with the centroid index in the low 4 mantissa bits (15 - k, so that the lower index
                        // wins exact ties of positive values)
                        float tk[K];
                        tk[0] = tk0;
                        // The chains advance together, in two sets (a wave issues an instruction that depends on the
                        // one before it at two thirds of the rate of independent ones, and four or more independent
                        // chains issue at the full rate; the scheduling barriers in score_chains keep the compiler from
                        // putting the chains one after the other).
                        constexpr int CA = K / 2, CB = K - 1 - CA;
                        score_chains<K, D, 1, CA>(xc, wv, tk);
                        __builtin_amdgcn_sched_barrier(0);
                        score_chains<K, D, 1 + CA, CB>(xc, wv, tk);
                        __builtin_amdgcn_sched_barrier(0);
                        float best, second;
                        top2<K>(tk, best, second);
                        __builtin_amdgcn_sched_barrier(0);
                        // buffer `up` is free now: refill it with the group PF-1 turns ahead
                        {
                            const unsigned off = u == 0 ? own_off : turn_off + (unsigned)(NW * (u - 1)) * GROUP_BYTES;
                            load_row<D>(xr[up], reinterpret_cast<const float *>(
                                                    reinterpret_cast<const char *>(u == 0 ? xb : pbase) + min(off, max_off)));
                        }

                        // sample (wave + m NW) 64 + lane of the mini-batch exists: a scalar against a per-lane constant
                        const bool valid = (m * NW) * 64 < lane_room;
                        const int arg = decide<K, D>(tk, best, second, xc, valid, thr, wsf, rechecks);
                        if (dump && valid) dump[(wave + m * NW) * 64 + lane] = arg;

                        // this group's row update: D fixed-point terms and a one for the count, added to the lane's
                        // cells of the centroid (masked lanes: the scratch row)
                        const unsigned cell = valid ? (__umul24((unsigned)arg, CENT_BYTES) + lane_cell) : scratch_cell;
#pragma unroll
                        for (int j = 0; j < D; ++j) lds_add_u32(cell + (unsigned)j * ELEM_BYTES, fx_term_bits(xc[j], scl[j]));
                        lds_add_u32(cell + (unsigned)D * ELEM_BYTES, 1u);
                    }
                    kp.settle_fetched();
                    m0 += PF;
                } while (m0 < ngw);
                // the part of the step that does not stream is on the worker's critical path: it goes first on its SIMD
                // until the next step sets the streaming priority again
                __builtin_amdgcn_s_setprio(3);
                phase_fence();      // a wave sums its own cells: its atomics have to be done

                // ---- sum the copies of every cell ----
                // lane = (part, task): task = four elements of a centroid (centroid, float4 number); part = its share of
                // the copies
                {
                    const int task = lane % NT, prt = lane / NT;
                    if (prt < NPART) {
                        int si[4];
                        sum_cells<RPP>(wave_cells + (unsigned)(task / NQ) * CENT_BYTES +
                                                     (unsigned)(4 * (task % NQ)) * ELEM_BYTES + (unsigned)(prt * RPP) * 4u,
                                                 ELEM_BYTES, task, si);
                        part[parity][wave][prt][task] = make_int4(si[0], si[1], si[2], si[3]);
                    }
                }
                if constexpr (NW > 1) __syncthreads(); else phase_fence();
                // Totals of this lane's four elements over waves and parts, as integers.  The count of the centroid
                // (element D) times the rounding constant comes off the sums (modulo 2^32, like the additions), then
                // the column's inverse scale.
                int Si[4] = {0, 0, 0, 0};
                if (kp.has_task) {
#pragma unroll
                    for (int v = 0; v < NW * NPART; ++v) {
                        const int4 sv = (&part[parity][0][0][0])[v * NT + lane];
                        Si[0] += sv.x; Si[1] += sv.y; Si[2] += sv.z; Si[3] += sv.w;
                    }
                }
                // the cells are never cleared: they run on, modulo 2^32, and a step's sums are the totals now minus the
                // totals a step ago (exact, since a step's sums are below 2^30 in magnitude)
                // (every wave keeps its own copy of the totals a step ago, the values are the same)
                if (kp.has_task) {
                    const lds_ivec4_ptr bq = (lds_ivec4_ptr)(size_t)before_cell;
                    const lds_ivec4 bv = *bq;
                    const lds_ivec4 nv = {Si[0], Si[1], Si[2], Si[3]};
                    *bq = nv;
                    Si[0] = (int)((unsigned)Si[0] - (unsigned)bv.x); Si[1] = (int)((unsigned)Si[1] - (unsigned)bv.y);
                    Si[2] = (int)((unsigned)Si[2] - (unsigned)bv.z); Si[3] = (int)((unsigned)Si[3] - (unsigned)bv.w);
                }
                const int cnt_i = __float_as_int(lane_read(kp.bp_row + 4 * G::CQ, __int_as_float(Si[G::CI])));
                // (inv4 is zero where the lane has no column: no select for those)
                float S4[4];
                const unsigned bias_off = (unsigned)cnt_i * FX_BIAS;
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) S4[c4] = (float)(int)((unsigned)Si[c4] - bias_off) * inv4[c4];
                if (kp.tq == G::CQ) S4[G::CI] = (float)cnt_i;
                parity ^= 1;
                kp.template finish<(NW > 1)>(p, i, round, S4, (float)cnt_i, merge_point, send_point, det, sync_now, wave == 0);

                // advance the clock
                xb = xbn;
                s_epoch = s_next;
                if (wk.xchg && ++te == E) { te = 0; ++round; }
            }

            // (several workers per workgroup: a wave reloads the state of a worker that comes round again only after
            // a whole pass over the other workers, whose steps each contain a workgroup barrier)
            if (wave == 0 && (!one_worker || wk.last_seg)) kp.store_state(p, i);
        }
        wk.end_segment();
    }

    for (int off = 32; off > 0; off >>= 1) rechecks += __shfl_xor(rechecks, off, 64);
    if (lane == 0 && rechecks)
        atomicAdd((unsigned long long *)&p.counters[(size_t)blockIdx.x * CNT_STRIDE + CNT_RECHECK],
                  (unsigned long long)rechecks);
    if (lane == 0 && kp.wait_failed) __hip_atomic_store(p.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // host memory
}

// resident workgroups of a kernel on the current device (queried once per device and kernel)
template <typename Kern>
hipError_t resident_capacity(Kern kern, int threads, long long *out)
{
    static long long cached_capacity[64] = {0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    long long capacity = (dev >= 0 && dev < 64) ? cached_capacity[dev] : 0;
    if (capacity == 0) {
        int per_cu = 0, cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, threads, 0);
        if (e != hipSuccess) return e;
        capacity = (long long)per_cu * cus;
        if (dev >= 0 && dev < 64) cached_capacity[dev] = capacity;
    }
    *out = capacity;
    return hipSuccess;
}

template <typename Kern>
hipError_t launch_kernel(Kern kern, int threads, const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    if (!persistent) {
        hipLaunchKernelGGL(kern, dim3(p.W), dim3(threads), 0, s, p, t0, t1, 0);
        return hipGetLastError();
    }
    // one launch for the whole run: every workgroup must be resident at the same time
    long long capacity = 0;
    hipError_t e = resident_capacity(kern, threads, &capacity);
    if (e != hipSuccess) return e;
    if (capacity < 1) return hipErrorCooperativeLaunchTooLarge;
    const int grid = (int)(p.W < capacity ? p.W : capacity);
    StepParams pp = p;
    long long a0 = t0, a1 = t1;
    int sync = 1;
    void *args[] = {&pp, &a0, &a1, &sync};
    if (p.cooperative) return hipLaunchCooperativeKernel((const void *)kern, dim3(grid), dim3(threads), args, 0, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), 0, s, pp, a0, a1, sync);
    return hipGetLastError();
}

// Like waves.  Several buffers: the message pairs of all buffers sit in registers during a step, so the ring depth is
// at most 4, and 2 for four buffers; the caller limits it.  Several buffers and partial messages are only built for
// the shapes with shared rows.
template <int K, int D, int PF, int NW, int RS>
hipError_t launch_variant(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    if (p.nb == 1 && p.parts == 1)
        return launch_kernel(small_steps_kernel<K, D, PF, NW, RS, 1, false>, 64 * NW, p, t0, t1, s, persistent);
    if constexpr (PF <= 4 && RS == 2) {
        if (p.nb == 1) return launch_kernel(small_steps_kernel<K, D, PF, NW, RS, 1, true>, 64 * NW, p, t0, t1, s, persistent);
        if (p.nb == 2) return launch_kernel(small_steps_kernel<K, D, PF, NW, RS, 2, true>, 64 * NW, p, t0, t1, s, persistent);
        if (p.nb == 3) return launch_kernel(small_steps_kernel<K, D, PF, NW, RS, 3, true>, 64 * NW, p, t0, t1, s, persistent);
    }
    if constexpr (PF == 2 && RS == 2) {
        if (p.nb == 4) return launch_kernel(small_steps_kernel<K, D, PF, NW, RS, 4, true>, 64 * NW, p, t0, t1, s, persistent);
    }
    return hipErrorInvalidValue;
}

// ring depth the registers of a shape leave room for: the wave-uniform copy of w_k - w_0 takes (K - 1) * RW registers,
// a ring buffer D
template <int K, int D>
constexpr int max_ring_depth()
{
    return (K - 1) * SmallGeo<K, D>::RW + 4 * D <= 160 ? 4 : 2;
}

template <int K, int D, int NW, int RS>
hipError_t launch_shape(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent, int pf)
{
    // RS = 2 leaves 256 registers per wave: ring depth at most 4
    if constexpr (RS == 1) {
        if (pf >= 8) return launch_variant<K, D, 8, NW, RS>(p, t0, t1, s, persistent);
    }
    if constexpr (max_ring_depth<K, D>() >= 4) {
        if (pf >= 4) return launch_variant<K, D, 4, NW, RS>(p, t0, t1, s, persistent);
    }
    return launch_variant<K, D, 2, NW, RS>(p, t0, t1, s, persistent);
}

// Steps [t0, t1) of a K x D state.  Shape of a worker: two waves with shared copies of the accumulator cells (default: 8
// waves per CU with one worker per 4 SIMD slots), one wave with shared cells (many workers: twice as many resident), or
// one wave with private cells (ALL: built for the streaming workload's own shape only, the others take shared cells).
// tune: bits 2-3 pick the shape, bits 0-1 limit the ring depth (1: 4, 2: 2); the value 3 in bits 0-1 is handled by
// the caller (one launch per round).
template <int K, int D, bool ALL>
hipError_t launch_small_kd(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    int shape = (p.tune >> 2) & 3;          // 0 = by number of workers, 1 = 1 wave private cells, 2 = 1 wave shared cells, 3 = 2 waves
    if (shape == 0) shape = p.W > 1024 ? 2 : 3;
    if (!ALL && shape == 1) shape = 2;
    const int nw = shape == 3 ? 2 : 1;
    const int ngw = ((p.b + 63) / 64 + nw - 1) / nw;
    // ring depth: the largest of 8, 4 that divides the number of groups per mini-batch and wave, else 2
    // (the kernel then pads the group count with masked groups)
    int pf = (ngw % 8 == 0) ? 8 : (ngw % 4 == 0) ? 4 : 2;
    if ((p.tune & 3) == 1 && pf > 4) pf = 4;
    if ((p.tune & 3) == 2 && pf > 2) pf = 2;
    if (p.nb >= 4 && pf > 2) pf = 2;        // registers: see launch_variant
    if constexpr (ALL) {
        if (shape == 1) return launch_shape<K, D, 1, 1>(p, t0, t1, s, persistent, pf);
    }
    if (shape == 2) return launch_shape<K, D, 1, 2>(p, t0, t1, s, persistent, pf);
    return launch_shape<K, D, 2, 2>(p, t0, t1, s, persistent, pf);
}

}  // namespace

namespace {

// Eq. 8 for a small state: a lane takes a sample (d floats straight into registers, four samples in flight), finds the
// nearest centroid with the expanded-form scores x.w_c - |w_c|^2/2 against register copies of the state, and adds
// half the squared distance to THAT centroid, formed directly as sum_j (x_j - w_cj)^2 (no cancellation, whatever
// the distance of the data from the origin; a near-tie picks a centroid whose distance differs by less than the
// rounding error of the scores, which is far below the 1e-4 the sum is asked for), in fp64.  The assignment of
// samples to threads is fixed, so is every order of summation: the result does not depend on scheduling.
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
            float best = -INFINITY;
            int arg = 0;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                float sc = hv[c];
#pragma unroll
                for (int j = 0; j < D; ++j) sc = fmaf(xr[u][j], wv[c * D + j], sc);
                if (sc > best) { best = sc; arg = c; }
            }
            float d2 = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const float diff = xr[u][j] - sw[arg * D + j];
                d2 = fmaf(diff, diff, d2);
            }
            if (n0 + u * stride < N) sum += (double)(0.5f * d2);
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

template <int K, int D>
hipError_t launch_quant_error_small_kd(const float *x, long long N, const float *w, double *partials, int nblocks, hipStream_t s)
{
    hipLaunchKernelGGL((quant_error_small_kernel<K, D>), dim3(nblocks), dim3(256), 0, s, x, N, w, partials);
    return hipGetLastError();
}

}  // namespace

// One translation unit per shape defines these two (the shapes compile side by side).
#define ASGD_SMALL_SHAPE_DEFINE(K, D, ALL)                                                                            \
    hipError_t launch_small_steps_##K##x##D(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent) \
    {                                                                                                                 \
        return launch_small_kd<K, D, ALL>(p, t0, t1, s, persistent);                                                  \
    }                                                                                                                 \
    hipError_t launch_quant_error_small_##K##x##D(const float *x, long long N, const float *w, double *partials, int nblocks, hipStream_t s) \
    {                                                                                                                 \
        return launch_quant_error_small_kd<K, D>(x, N, w, partials, nblocks, s);                                      \
    }

}  // namespace asgd
