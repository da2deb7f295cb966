// Step kernel for large states (k*d too large for registers): the contraction-bound workloads
// (k = 100, d = 100 and k = 1024, d = 128).
//
// One workgroup of 8 wavefronts (two per SIMD, so that one wave's vector work overlaps the other's
// matrix work) per worker.  A step has two phases.
//
// Phase 1, assignment.  The scores x.w_c - |w_c|^2/2 of a tile of 256 samples against all centroids
// are a dense contraction over d and run on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32).
//   - Matrix rows are centroids, columns are samples.  Wave v owns 32 samples of the tile and keeps
//     their operand fragments in registers for the whole pass over the centroids (a lane holds, for
//     its sample, 4 consecutive dimensions of every 8-dimension chunk: half-wave 0 dimensions 0-3,
//     half-wave 1 dimensions 4-7); the fragments of the next tile are fetched into the same registers
//     during the last centroid block of this one.  Samples never pass through LDS.
//   - Blocks of 64 centroid rows stream from the state (L2 resident) through a double-buffered LDS
//     stage, zero-padded to a multiple of 8 columns and of 64 rows; rows are padded to a stride that
//     is an odd multiple of 4 floats, which keeps the 128-bit operand reads free of bank conflicts.
//   - The accumulators start at h_c = -|w_c|^2/2 (kept in LDS), so the offset costs nothing.
//     Matrix instruction q of a group of four contracts dimensions q and q+4 of a chunk: the order of
//     the contraction is a fixed permutation of 0..d-1 and no transposition is needed.
//   - In the 32x32 result a lane holds 16 centroid scores of ONE sample per tile, so the running
//     arg-max is lane-local; the two half-waves (same sample, other rows) are merged once per tile.
//   - The three largest scores and the indices of the two largest are tracked.  If the first two are
//     closer than a bound on the fp32 rounding error, the sample is decided exactly in fp64 (pair
//     comparison, or all k distances when the third is close too), lowest index on ties.
// Phase 2, gradient and update.  The samples are sorted by centroid with a stable counting sort in
// LDS (centroids ordered by owner wave c mod 8); each wave then streams the rows of its samples from
// memory, 16 loads in flight, and adds them in sample order into per-centroid sums, which makes every
// sum reproducible without atomics.  Gradient, Parzen sums (fp64), merge and update are row passes.
#include <type_traits>

#include "asgd_internal.h"
#include "fixed_point_sums.h"
#include "mfma_geom.h"

namespace asgd {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Waves per workgroup is a template parameter NWV (8 or 4): a tile has 32 samples per wave.
constexpr int WB = MFMA_WB;      // centroid rows per block (2 matrix tiles of 32)
constexpr int RB = 8;            // rows per wave and iteration in the row passes (loads in flight)
constexpr int GS = 16;           // sample rows in flight per wave in the gather (small clusters)
constexpr int GU = 16;           // sample rows in flight per half-wave in the gather (large clusters)
constexpr float PAD_SCORE = -1.0e30f;   // offset of the padding rows: never the nearest

// Bounded wait for a flag that another workgroup writes.  All the waits of a workgroup draw on ONE budget of polls
// (*budget, in LDS, used by the one thread that waits; a poll is ~0.5 us of sleep plus an uncached load, the waits of
// a healthy run last microseconds to a few milliseconds): false when it is used up.  A workgroup whose wait has failed
// waits for nothing any more (s_wait_failed), so a launch outlasts its normal duration by about a quarter of a second
// at most, however many rounds it covers.
constexpr int MF_WAIT_BUDGET = 1 << 18;
constexpr int MF_WAIT_PER_ROUND = 4096;
__device__ __forceinline__ bool mf_wait_flag(const int *flag, int want, bool at_least, int *budget)
{
    int left = *budget;
    bool ok = false;
    while (left > 0) {
        const int v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (at_least ? (v >= want) : (v == want)) { ok = true; break; }
        __builtin_amdgcn_s_sleep(8);
        --left;
    }
    *budget = left;
    return ok;
}

struct Top3 {
    float v1, v2, v3;
    int i1, i2;
};
__device__ __forceinline__ void top3_insert(Top3 &t, float s, int c)
{
    const bool g1 = s > t.v1, g2 = s > t.v2, g3 = s > t.v3;
    t.v3 = g2 ? t.v2 : (g3 ? s : t.v3);
    t.i2 = g1 ? t.i1 : (g2 ? c : t.i2);
    t.v2 = g1 ? t.v1 : (g2 ? s : t.v2);
    t.i1 = g1 ? c : t.i1;
    t.v1 = g1 ? s : t.v1;
}

// Value-only insert into a sorted triple (v1 >= v2 >= v3): three instructions.  Used on scores whose low five
// mantissa bits were replaced by the number of the accumulator register they came from.
// `big` is +infinity in a register the compiler cannot see through: med3(v1, s, +inf) = max(v1, s) stays ONE
// instruction (folded to a maximum it would be preceded by an instruction that quiets a signalling NaN, which a
// tagged score can look like).  Every vector instruction between two matrix instructions costs matrix-pipe time.
__device__ __forceinline__ void top3_insert_value(Top3 &t, float s, float big)
{
    t.v3 = __builtin_amdgcn_fmed3f(t.v2, t.v3, s);
    t.v2 = __builtin_amdgcn_fmed3f(t.v1, t.v2, s);
    t.v1 = __builtin_amdgcn_fmed3f(t.v1, s, big);
}
__device__ __forceinline__ float opaque_infinity()
{
    float big = INFINITY;
    asm volatile("" : "+s"(big));
    return big;
}
__device__ __forceinline__ float tag_low5(float v, int r)
{
    return __int_as_float((__float_as_int(v) & ~31) | r);
}

__device__ __forceinline__ double wave_sum_d(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
// Sum over the wave without LDS traffic: butterfly inside rows of 16 lanes with DPP (lane ^ 1, lane ^ 2, mirror inside 8,
// mirror inside 16), then the four rows through scalar reads.  The order of the additions is fixed.
__device__ __forceinline__ float wave_sum_f(float v)
{
    v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x141, 0xF, 0xF, true));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x140, 0xF, 0xF, true));   // row_mirror
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}


// max over rows of |x|^2 (one value), used by the rounding-error bound.  A half-wave takes a row (32 lanes x float4
// cover d <= 128 floats, d a multiple of 4, rows 16-byte aligned: what the matrix-core kernel requires anyway), so
// the reads are contiguous; the squares of a row are added in a fixed order (lane-local, then a butterfly).
__global__ void rownorm2_partial_kernel(const float *__restrict__ x, long long rows, int d, float *partial)
{
    __shared__ float red[256];
    const int lane = threadIdx.x & 63, q4 = lane & 31;
    const long long hw = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 5;      // half-wave number
    const long long nhw = ((long long)gridDim.x * blockDim.x) >> 5;
    const bool colok = 4 * q4 < d;
    float m = 0.0f;
    for (long long r0 = 0; r0 < rows; r0 += nhw) {          // uniform trip count: the shuffles below need every lane
        const long long r = r0 + hw;
        float s = 0.0f;
        if (r < rows && colok) {
            const float4 v = *reinterpret_cast<const float4 *>(x + (size_t)r * d + 4 * q4);
            s = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, v.w * v.w)));
        }
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);         // stays inside the half-wave
        m = fmaxf(m, s);
    }
    red[threadIdx.x] = m;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + off]);
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}
__global__ void rownorm2_final_kernel(const float *partial, int n, float *out)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        float m = 0.0f;
        for (int q = 0; q < n; ++q) m = fmaxf(m, partial[q]);
        *out = m;
    }
}

// NCH = number of 8-dimension chunks of the contraction (d <= 8 * NCH).
// RES: the whole padded state fits in LDS.  It is then staged once per step and phase 1 needs no barriers.
// Otherwise blocks of WB rows are streamed through a two-deep stage with one barrier per block.
// NWV: waves per workgroup.  8 by default (two per SIMD).  4 when the state is resident, two workgroups fit a CU
// and there are more workers than CUs: two workers then share a CU and one's memory-bound phase 2 runs under the
// other's matrix work.
// sync = 0: the launch holds nothing a worker has to wait for (silent or free-running mode, or the host ends every
//           launch at a multiple of E).
// sync = 1: deterministic mode, the whole run is one launch of co-resident workgroups.  At a merge point a worker
//           waits for the stamp of the message addressed to it (its sender writes it at the end of the round
//           before), and a sender waits until the recipient has passed the merge point that read the older message
//           in the same buffer.  Every wait is on an earlier round, so the waits cannot form a cycle, and every
//           wait is bounded: when the bound expires the worker goes on without the message and the host reports it.
// FS (fused sums, resident state only): the per-centroid sums of Eq. 9 are formed tile by tile from the sample
//     fragments a wave still holds in registers when the assignments of the tile are final, so the mini-batch is read
//     from memory ONCE.  The sums are 32-bit fixed-point numbers in LDS, added with integer atomics: integer addition
//     is associative, so the result does not depend on the order in which waves and lanes get there (reproducible
//     bit for bit), and with the scale of column j chosen as the largest power of two with b * max|x_j| * scale < 2^30
//     a sum cannot overflow and is more accurate than an fp32 sum of the same terms (every term is off by at most
//     half a unit = 2^-31 of the largest possible sum).  No counting sort, no gather.
// FSM: 0 = sort and gather, 1 = FS, 2 = sort and gather with the sample fragments of the NEXT tile fetched into a second
//     set of registers during the first half-block of a tile (instead of into the same set during the last one), so
//     that a fetch has a whole tile of matrix work to arrive (resident state only), 3 = as 2, but no sort and no gather:
//     once the assignments of the mini-batch are final, the state rows in LDS make room for fixed-point sums as in FS
//     and the mini-batch is read a second time in memory order (see the pass itself).
template <int NCH, bool RES, int NWV, int FSM>
__global__ __launch_bounds__(64 * NWV) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_steps_kernel(StepParams p, long long t0, long long t1,
                                                                 const float *xnorm2max_ptr, int sync)
{
    constexpr int DP8 = NCH * 8;                 // padded row length
    constexpr int DP = DP8 + 4;                  // LDS row stride
    constexpr int NJ = DP8 > 64 ? 2 : 1;         // dimensions per lane in the row passes (lane l owns l, l + 64)
    constexpr int ROW4 = NCH * 2;                // float4 per padded row
    constexpr int NVEC = WB * ROW4;              // float4 per staged block
    constexpr int MF_THREADS = 64 * NWV, MF_WAVES = NWV, TM = 32 * NWV;
    constexpr int NST = (NVEC + MF_THREADS - 1) / MF_THREADS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ double red_d[3][MF_WAVES];
    __shared__ float red_f[MF_WAVES];
    __shared__ int s_has_ext;
    __shared__ int s_wait_failed;
    __shared__ int s_wait_budget;
    __shared__ int s_ext_round[MAX_BUFFERS];   // round of the message in buffer n (free-running mode: any earlier one)
    __shared__ int s_rowflags[3];     // partial messages: buffers with a non-empty row, with an accepted row, near-ties
    __shared__ int s_next_rows;
    __shared__ int s_next_item;       // gather: next ticket (slot, first or second round)
    __shared__ int s_tot[MF_WAVES];   // samples in the slots of a wave (counting sort)

    const int i = blockIdx.x;                       // worker
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int k = p.k, d = p.d, b = p.b;
    constexpr bool FS = FSM == 1, TWO = FSM != 0, PRE = FSM >= 2, SS = FSM == 3;
    static_assert(!TWO || RES, "fused sums and the second set of fragments need the resident state");
    const MfmaGeom g = mfma_geom(k, b, NCH, RES, NWV, FS ? 1 : (SS ? 2 : 0));
    const size_t kd = (size_t)k * d;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);

    float *Ws = reinterpret_cast<float *>(smem_raw);                                  // (RES ? kpad : 2 x WB) x DP
    float *hs = reinterpret_cast<float *>(smem_raw + g.off_h);                        // kpad offsets h_c
    int *cstart = reinterpret_cast<int *>(smem_raw + g.off_cstart);                   // ns + 1 list starts
    int *cursor = reinterpret_cast<int *>(smem_raw + g.off_cursor);                   // ns x nr counts (slot-major: one per slot and share), then cursors
    unsigned short *idx = reinterpret_cast<unsigned short *>(smem_raw + g.off_idx);   // b assignments
    unsigned short *perm = reinterpret_cast<unsigned short *>(smem_raw + g.off_perm); // b samples sorted by centroid
    unsigned short *flist = reinterpret_cast<unsigned short *>(smem_raw + g.off_flist);
    int *fxsum = reinterpret_cast<int *>(smem_raw + g.off_sums);                       // FS: k x DP8 fixed-point sums
    float *colscale = reinterpret_cast<float *>(smem_raw + g.off_scale);              // FS: DP8 scales, then DP8 inverse scales

    // the last half-block of 32 rows holds at most eight centroids and is the second one of its block: 4x4 tiles there
    constexpr bool TAILOK = RES && NCH <= 13 && FSM != 1;       // (the other variants have no registers to spare)
    const int tail_groups = (TAILOK && !(p.tune & 256) && (k & 31) >= 1 && (k & 31) <= 8 && ((k >> 5) & 1)) ? ((k & 31) + 3) / 4 : 0;
    const int tail_row0 = k & ~31;
    float *wst = p.w + (size_t)i * kd;                  // state of this worker
    float *gsc = p.acc + (size_t)i * kd;                // per-centroid sums of assigned samples
    const float xn2 = *xnorm2max_ptr;

    if (threadIdx.x == 0) {              // read after the barriers below
        s_wait_failed = 0;
        // the budget grows with the rounds of the launch: a healthy run of the k = d = 100 workload spends up to ~700
        // polls per round on the workgroup that waits most (the host keeps launches to 1024 rounds)
        const long long rounds_here = p.E > 0 ? (t1 - t0) / p.E + 1 : 0;
        s_wait_budget = p.wait_polls > 0 ? p.wait_polls : MF_WAIT_BUDGET + MF_WAIT_PER_ROUND * (int)min(rounds_here, (long long)(1 << 16));
    }
    // ---- h_c = -|w_c|^2/2 and max_c |w_c|^2 ----
    float wn2max = 0.0f;
    for (int c0 = wave * RB; c0 < g.kpad; c0 += MF_WAVES * RB) {
        float s[RB];
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            const int c = c0 + q;
            s[q] = 0.0f;
#pragma unroll
            for (int jq = 0; jq < NJ; ++jq) {
                const int j = lane + 64 * jq;
                const float v = wst[(size_t)(c < k ? c : 0) * d + (j < d ? j : 0)];
                if (c < k && j < d) s[q] = fmaf(v, v, s[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            const float sq = wave_sum_f(s[q]);
            if (lane == 0) hs[c0 + q] = c0 + q < k ? -0.5f * sq : PAD_SCORE;      // kpad is a multiple of RB
            wn2max = fmaxf(wn2max, sq);
        }
    }
    if (lane == 0) red_f[wave] = wn2max;
    __syncthreads();
    wn2max = 0.0f;
#pragma unroll
    for (int v = 0; v < MF_WAVES; ++v) wn2max = fmaxf(wn2max, red_f[v]);
    if constexpr (FS || SS) {
        // scale of column j: 2^e with b * max|x_j| * 2^e in [2^29, 2^30) (max|x_j| over the loaded samples)
        for (int j = tid; j < DP8; j += MF_THREADS) {
            float sc = 0.0f, inv = 0.0f;
            int e = 0;
            // (streamed sums: a single term must also stay below 2^22, it is rounded inside a float)
            if (j < d && fx_scale_exponent(b, p.xabsmax[j], SS, &e)) {
                sc = ldexpf(1.0f, e);
                inv = ldexpf(1.0f, -e);
            }
            colscale[j] = sc;
            colscale[DP8 + j] = inv;
        }
    }
    __syncthreads();

    long long rechecks = 0;

    for (long long t = t0; t < t1; ++t) {
        // Two workgroups share a CU and the older one would win every arbitration for the matrix pipe, finish the
        // launch early and leave the CU half empty: they take turns at the higher priority instead.  The phases
        // after the matrix work issue few instructions and wait on memory: highest priority.
        if (((int)(t & 1) != 0) != (blockIdx.x * 2 >= gridDim.x)) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(1);
        // Fresh, opaque copies of the lane id per phase: everything derived from them (addresses, masks) is then
        // recomputed per phase instead of being kept in registers across the whole step loop.
        int lane_p1 = threadIdx.x & 63;
        asm volatile("" : "+v"(lane_p1));
        const int lane = lane_p1, tid = wave * 64 + lane, half = lane >> 5, l32 = lane & 31;
        const long long s_ep = t % p.S;
        const float *xb = p.x + ((size_t)i * p.H + (size_t)s_ep * b) * d;
        // Bound on the rounding error of a score difference: DP8 products and sums on the matrix core plus the
        // roundings inside h_c, each relative to |x||w_c| + |h_c| <= sqrt(max|x|^2 max|w|^2) + max|w|^2/2,
        // doubled in case the matrix core truncates where a vector instruction would round to nearest.
        const float Bb = sqrtf(xn2) * sqrtf(wn2max) + 0.5f * wn2max;
        // ... plus 2^-18 relative for each of the two scores compared: the register tag in their low mantissa bits.
        const float thr = (2.0f * (float)(2 * DP8 + 18) * 5.9604645e-8f + 7.62939453125e-6f) * Bb;

        // ================= phase 1: assignment =================
        // Fragment ch of the sample in row `rowoff` (an offset in floats).  Columns past d are read from a clamped,
        // valid address instead of being zeroed: they meet the zero padding of the state rows.  Likewise lanes past
        // the mini-batch read row 0 and their scores are never used.
        // half-wave 0 reads columns 8*ch + 0..3, half-wave 1 columns 8*ch + 4..7: the last start that is inside a row
        const int col0 = (half && d >= 8) ? 4 : 0;
        const int collim = half ? (d >= 8 ? (d - 8) / 8 * 8 + 4 : 0) : (d - 4) / 8 * 8;
        auto frag = [&](unsigned rowoff, int ch) -> float4 {
            const int col = ch * 8 + col0 < collim ? ch * 8 + col0 : collim;
            return *reinterpret_cast<const float4 *>(xb + (rowoff + (unsigned)col));
        };
        auto rowoff_of = [&](int nbase) -> unsigned {      // nbase: first of the wave's 32 rows
            const int n = nbase + l32;
            return (unsigned)(n < b ? n : 0) * (unsigned)d;
        };
        auto fetch_block = [&](float4(&st)[NST], int cb) {       // block cb of the state -> registers
#pragma unroll
            for (int q = 0; q < NST; ++q) {
                const int e = tid + q * MF_THREADS;
                const int r = (e < NVEC ? e : 0) / ROW4, c4 = (e < NVEC ? e : 0) - r * ROW4;
                const int c = cb * WB + r, col = 4 * c4;
                const bool ok = c < k && col < d;
                float4 v = *reinterpret_cast<const float4 *>(wst + (size_t)(ok ? c : 0) * d + (ok ? col : 0));
                if (!ok) v = make_float4(0.f, 0.f, 0.f, 0.f);
                st[q] = v;
            }
        };
        auto store_block = [&](const float4(&st)[NST], float *dst) {
#pragma unroll
            for (int q = 0; q < NST; ++q) {
                const int e = tid + q * MF_THREADS;
                if (e < NVEC) {
                    const int r = e / ROW4, c4 = e - r * ROW4;
                    *reinterpret_cast<float4 *>(&dst[r * DP + 4 * c4]) = st[q];
                }
            }
        };
        // FS: adds the sample whose fragments the lane pair (l32, half) holds to the fixed-point sums of centroid c.
        // A fragment past the last column start of its half-wave is a clamped duplicate (see frag) and is left out.
        auto add_sample = [&](const float4(&xv)[NCH], int c) {
            int *row = fxsum + c * DP8 + col0;
            const float *sc = colscale + col0;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                if (ch * 8 + col0 <= collim && (half == 0 || d >= 8)) {
                    const float4 s4 = *reinterpret_cast<const float4 *>(sc + ch * 8);
                    atomicAdd(row + ch * 8 + 0, __float2int_rn(xv[ch].x * s4.x));
                    atomicAdd(row + ch * 8 + 1, __float2int_rn(xv[ch].y * s4.y));
                    atomicAdd(row + ch * 8 + 2, __float2int_rn(xv[ch].z * s4.z));
                    atomicAdd(row + ch * 8 + 3, __float2int_rn(xv[ch].w * s4.w));
                }
            }
            if (half == 0) atomicAdd(&cursor[(c % NWV) * g.kq + c / NWV], 1);      // samples of the centroid's slot
        };
        // the wave's rows nbase .. nbase + 31 (fragments xf); its next rows start at nbase_next (past the mini-batch:
        // none) and their fragments go to xn (FS: another set of registers, xf is still needed when the tile is done;
        // otherwise the same set)
        auto do_tile = [&](float4(&xf)[NCH], float4(&xn)[NCH], int nbase, int nbase_next, bool refill) {
            float4 st[NST];
            if constexpr (!RES) {
                __syncthreads();             // nobody still reads the stage
                fetch_block(st, 0);
                store_block(st, Ws);
            }
            if constexpr (PRE) {
                // The loads into xf were issued a whole tile ago; touching the registers here makes the compiler wait
                // for them now, BEFORE this tile issues the loads into xn.  Otherwise it cannot tell the two sets'
                // loads apart (loads return in order, it counts them) and waits for the new ones at every use of xf.
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch)
                    asm volatile("" : "+v"(xf[ch].x), "+v"(xf[ch].y), "+v"(xf[ch].z), "+v"(xf[ch].w));
            }
            Top3 top;
            const float big = opaque_infinity();
            top.v1 = top.v2 = top.v3 = -INFINITY;
            top.i1 = top.i2 = 0;
            // The 64 rows of a block are done as two half-blocks of 32 rows (one 32x32 accumulator each), and the running
            // top three of a half-block's scores is updated while the matrix cores work on the NEXT half-block: the
            // wave issues one matrix instruction per 64 cycles, the vector instructions of the inserts fit in between.
            // acc1 therefore lives across iterations.
            floatx16 acc0, acc1;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
            // Inserts the 16 scores of `prev` (tag = 2*block + which accumulator; -1: nothing real) spread over the
            // chunks of the half-block that is being computed into `acc`.  The register number (0..15) rides in the
            // low mantissa bits of a score (2^-18 relative, covered by thr), so an insert is three value-only
            // instructions; which half-block the two largest came from is found by comparing bit patterns before and
            // after (i1, i2 hold tags until the loop ends).  Two different elements with the same bit pattern end up
            // as v1 == v2 or v2 == v3, which the decisions below treat as "more than two candidates".
            // TAIL (resident state): the half-block holds at most eight centroids (k mod 32 <= 8), whose scores come from
            // v_mfma_f32_4x4x1 instead - in each block of four lanes a column of four state rows (lane 4q + r supplies
            // row r) times a row of four samples (lane 4q + j supplies its own), D[r][j] in register r of lane 4q + j:
            // 8 cycles of the matrix pipe per instruction instead of 64 for 28 rows of padding.  A lane's sum covers
            // the columns of its own half-wave; the two halves are added afterwards and the scores are put where
            // a 32x32 tile would have left them (row 4 * half + r in register r), so that everything downstream is
            // unchanged.  wrow: row (lane mod 4) of the half-block, this half-wave's columns.
            auto half_block = [&](auto mode, auto ins, auto tail, floatx16 &acc, const float *wrow, const floatx16 &prev,
                                  int prev_tag, int cb) {
                constexpr int MODE = decltype(mode)::value;
                constexpr bool INS = decltype(ins)::value;      // false: first half-block of a tile, nothing to insert
                constexpr bool TAIL = decltype(tail)::value;
                // TAIL: one chain of 4x4 tiles per component of the operand fragments, so that consecutive matrix
                // instructions do not depend on each other; rows 0..3 in this loop, rows 4..7 (if any) in one of their own
                floatx4 tq[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) tq[q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
                unsigned nextoff = 0;
                if constexpr (MODE == 2) {
                    nextoff = rowoff_of(nbase_next);
                    asm volatile("" : "+v"(nextoff));          // keep the address arithmetic inside this block
                }
                const int o1 = __float_as_int(top.v1), o2 = __float_as_int(top.v2);
                float4 a = *reinterpret_cast<const float4 *>(wrow);
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    // operands of the next chunk are read under the matrix work of this one; the scheduling
                    // barrier keeps the compiler from hoisting the reads of ALL chunks to the top (registers)
                    float4 nx = a;
                    if (ch + 1 < NCH) nx = *reinterpret_cast<const float4 *>(wrow + (ch + 1) * 8);
                    const float4 xv = xf[ch];
                    if constexpr (TAIL) {
                        tq[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.x, xv.x, tq[0], 0, 0, 0);
                        tq[1] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.y, xv.y, tq[1], 0, 0, 0);
                        tq[2] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.z, xv.z, tq[2], 0, 0, 0);
                        tq[3] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.w, xv.w, tq[3], 0, 0, 0);
                    } else {
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, xv.x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, xv.y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, xv.z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, xv.w, acc, 0, 0, 0);
                    }
                    if constexpr (INS) {
#pragma unroll
                        for (int r = ch * 16 / NCH; r < (ch + 1) * 16 / NCH; ++r)
                            top3_insert_value(top, tag_low5(prev[r], r), big);
                    }
                    if constexpr (MODE == 1) {
                        if (ch == 0) fetch_block(st, cb + 1);   // not before the first chunk: it waits for all loads
                    }
                    // the last half-block has used this fragment for the last time: fetch the next tile's into its
                    // place, so that the fetch runs behind the matrix work and the epilogue of this tile
                    if constexpr (MODE == 2) {
                        // (one set of registers and a second group of 4x4 tiles to come: that loop refills)
                        if (!TAIL || tail_groups <= 1) xn[ch] = frag(nextoff, ch);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    a = nx;
                }
                if constexpr (TAIL) {
                    const floatx4 lo = (tq[0] + tq[1]) + (tq[2] + tq[3]);
                    floatx4 hi = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (tail_groups > 1) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) tq[q] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
                        const float *wrow2 = wrow + 4 * DP;
#pragma unroll
                        for (int ch = 0; ch < NCH; ++ch) {
                            const float4 a2 = *reinterpret_cast<const float4 *>(wrow2 + ch * 8);
                            const float4 xv = xf[ch];
                            tq[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.x, xv.x, tq[0], 0, 0, 0);
                            tq[1] = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.y, xv.y, tq[1], 0, 0, 0);
                            tq[2] = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.z, xv.z, tq[2], 0, 0, 0);
                            tq[3] = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.w, xv.w, tq[3], 0, 0, 0);
                            if constexpr (MODE == 2) xn[ch] = frag(nextoff, ch);
                        }
                        hi = (tq[0] + tq[1]) + (tq[2] + tq[3]);
                    }
                    // rows 0..3 belong to the registers of half-wave 0, rows 4..7 to those of half-wave 1
                    const float4 hv = *reinterpret_cast<const float4 *>(hs + tail_row0 + 4 * half);
                    const float hq[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // v_permlane32_swap exchanges the upper half of its first operand with the lower half of its
                        // second: afterwards the lower half-wave holds both halves' sums of rows 0..3, the upper
                        // half-wave those of rows 4..7
                        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo[r]), __float_as_uint(hi[r]), false, false);
                        acc[r] = (__uint_as_float(sw[0]) + __uint_as_float(sw[1])) + hq[r];
                    }
                    // (registers 4..15 are not looked at after a half-block of this kind)
                }
                if constexpr (INS) {
                    const int n1 = __float_as_int(top.v1), n2 = __float_as_int(top.v2);
                    const int nb2 = (n2 == o2) ? top.i2 : ((n2 == o1) ? top.i1 : prev_tag);
                    top.i1 = (n1 != o1) ? prev_tag : top.i1;
                    top.i2 = nb2;
                }
            };
            using M0 = std::integral_constant<int, 0>;
            using M1 = std::integral_constant<int, 1>;
            using M2 = std::integral_constant<int, 2>;
            for (int cb = 0; cb < g.nblocks; ++cb) {
                if constexpr (!RES) __syncthreads();      // Ws[cb & 1] complete; Ws[(cb + 1) & 1] free
                const float *Wc = Ws + (RES ? cb : (cb & 1)) * WB * DP;
                const bool more = !RES && cb + 1 < g.nblocks;
                const bool lastb = !PRE && refill && cb + 1 == g.nblocks;
                const float4 *hp = reinterpret_cast<const float4 *>(hs + cb * WB + 4 * half);
                const float *w0row = Wc + l32 * DP + 4 * half;
                const float *w1row = Wc + (32 + l32) * DP + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 h0 = hp[2 * q];
                    acc0[4 * q + 0] = h0.x; acc0[4 * q + 1] = h0.y; acc0[4 * q + 2] = h0.z; acc0[4 * q + 3] = h0.w;
                }
                // rows 0..31 of this block; meanwhile the scores of rows 32..63 of the previous block are inserted
                if (cb == 0) {
                    if (PRE && refill) half_block(M2(), std::false_type(), std::false_type(), acc0, w0row, acc1, -1, cb);
                    else if (more) half_block(M1(), std::false_type(), std::false_type(), acc0, w0row, acc1, -1, cb);
                    else half_block(M0(), std::false_type(), std::false_type(), acc0, w0row, acc1, -1, cb);
                } else {
                    if (more) half_block(M1(), std::true_type(), std::false_type(), acc0, w0row, acc1, 2 * cb - 1, cb);
                    else half_block(M0(), std::true_type(), std::false_type(), acc0, w0row, acc1, 2 * cb - 1, cb);
                }
                bool tail_done = false;
                if constexpr (TAILOK) {
                    if (tail_groups > 0 && cb + 1 == g.nblocks) {
                        const float *wtail = Wc + (32 + (lane & 3)) * DP + 4 * half;
                        if (lastb) half_block(M2(), std::true_type(), std::true_type(), acc1, wtail, acc0, 2 * cb, cb);
                        else half_block(M0(), std::true_type(), std::true_type(), acc1, wtail, acc0, 2 * cb, cb);
                        tail_done = true;
                    }
                }
                if (!tail_done) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 h1 = hp[8 + 2 * q];
                    acc1[4 * q + 0] = h1.x; acc1[4 * q + 1] = h1.y; acc1[4 * q + 2] = h1.z; acc1[4 * q + 3] = h1.w;
                }
                // rows 32..63; meanwhile the scores of rows 0..31 are inserted
                if (lastb) half_block(M2(), std::true_type(), std::false_type(), acc1, w1row, acc0, 2 * cb, cb);
                else half_block(M0(), std::true_type(), std::false_type(), acc1, w1row, acc0, 2 * cb, cb);
                }
                if (more) store_block(st, Ws + ((cb + 1) & 1) * WB * DP);
            }
            {
                // the last half-block's scores
                const int o1 = __float_as_int(top.v1), o2 = __float_as_int(top.v2);
#pragma unroll
                for (int r = 0; r < 4; ++r) top3_insert_value(top, tag_low5(acc1[r], r), big);
                if (tail_groups == 0) {          // (4x4 tiles: the other registers hold padding)
#pragma unroll
                    for (int r = 4; r < 16; ++r) top3_insert_value(top, tag_low5(acc1[r], r), big);
                }
                const int n1 = __float_as_int(top.v1), n2 = __float_as_int(top.v2), tg = 2 * g.nblocks - 1;
                const int nb2 = (n2 == o2) ? top.i2 : ((n2 == o1) ? top.i1 : tg);
                top.i1 = (n1 != o1) ? tg : top.i1;
                top.i2 = nb2;
            }
            {
                // half-block tag + register number -> centroid: register r of a 32x32 tile is row 8*(r/4) + 4*half + r%4
                const int r1 = __float_as_int(top.v1) & 15, r2 = __float_as_int(top.v2) & 15;
                top.i1 = top.i1 * 32 + 8 * (r1 >> 2) + 4 * half + (r1 & 3);
                top.i2 = top.i2 * 32 + 8 * (r2 >> 2) + 4 * half + (r2 & 3);
            }
            // merge the two half-waves (same sample, other centroid rows)
            {
                // only the lower half-wave's result is used below: it gets the upper one's values (second result of
                // v_permlane32_swap of a register with itself), the upper half-wave sees its own again
                auto upper = [](unsigned v) -> unsigned { return __builtin_amdgcn_permlane32_swap(v, v, false, false)[1]; };
                const float pv1 = __uint_as_float(upper(__float_as_uint(top.v1))), pv2 = __uint_as_float(upper(__float_as_uint(top.v2))),
                            pv3 = __uint_as_float(upper(__float_as_uint(top.v3)));
                const int pi1 = (int)upper((unsigned)top.i1), pi2 = (int)upper((unsigned)top.i2);
                top3_insert(top, pv1, pi1);
                top3_insert(top, pv2, pi2);
                top.v3 = fmaxf(top.v3, pv3);
            }
            const int n = nbase + l32;                    // this lane pair's sample
            const bool mine = half == 0 && n < b;
            int arg = top.i1;
            const bool close2 = mine && !(top.v1 - top.v2 > thr);
            const bool close3 = close2 && (!(top.v1 - top.v3 > thr) || __float_as_int(top.v1) == __float_as_int(top.v2));
            // exact decision between two candidates, four flagged samples at a time:
            // |x - w_a|^2 - |x - w_b|^2 = sum_j (w_aj - w_bj)(w_aj + w_bj - 2 x_j), in fp64
            unsigned long long pm = RES ? 0ull : __ballot(close2 && !close3);
            while (pm) {
                int L[4], ca[4], cb2[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    L[q] = -1; ca[q] = 0; cb2[q] = 0;
                    if (pm) {
                        L[q] = __builtin_ctzll(pm);
                        pm &= pm - 1;
                        ca[q] = __builtin_amdgcn_readlane(top.i1, L[q]);
                        cb2[q] = __builtin_amdgcn_readlane(top.i2, L[q]);
                        rechecks += (lane == 0);
                    }
                }
                double dd[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    dd[q] = 0.0;
                    const float *xl = xb + (size_t)(nbase + (L[q] < 0 ? 0 : L[q])) * d;      // in bounds: that lane was valid
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq, jc = j < d ? j : 0;
                        const double wa = (double)wst[(size_t)ca[q] * d + jc], wb = (double)wst[(size_t)cb2[q] * d + jc];
                        const double xx = (double)xl[jc];
                        if (j < d) dd[q] += (wa - wb) * ((wa + wb) - 2.0 * xx);
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const double s = wave_sum_d(dd[q]);
                    const int lo = ca[q] < cb2[q] ? ca[q] : cb2[q];
                    const int res = s < 0.0 ? ca[q] : (s > 0.0 ? cb2[q] : lo);
                    if (lane == L[q]) arg = res;
                }
            }
            // all k distances in fp64, direct form; lane l takes centroids l, l + 64, ...
            unsigned long long fm = __ballot(close3);
            while (fm) {
                const int L = __builtin_ctzll(fm);
                fm &= fm - 1;
                const float *xl = xb + (size_t)(nbase + L) * d;
                double best = INFINITY;
                int barg = 0x7fffffff;
                for (int c = lane; c < k; c += 64) {
                    double sd = 0.0;
                    for (int j = 0; j < d; ++j) {
                        const double diff = (double)xl[j] - (double)wst[(size_t)c * d + j];
                        sd += diff * diff;
                    }
                    if (sd < best) { best = sd; barg = c; }
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const double ob = __shfl_xor(best, off, 64);
                    const int oa = __shfl_xor(barg, off, 64);
                    if (ob < best || (ob == best && oa < barg)) { best = ob; barg = oa; }
                }
                if (lane == L) arg = barg;
                rechecks += (lane == 0);
            }
            if (mine) {
                idx[n] = (unsigned short)arg;
                if constexpr (RES) {
                    // two close candidates: decided after the last tile, all such samples of the wave at once;
                    // until then perm[] (unused during this phase) keeps the second candidate
                    const bool pairf = close2 && !close3;
                    perm[n] = pairf ? (unsigned short)top.i2 : (unsigned short)0xFFFF;
                    if (p.dump && !pairf) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;
                } else {
                    if (p.dump) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;
                }
            }
            if constexpr (FS) {
                // the assignment is final unless the sample waits for the exact decision between two candidates
                // (those are added when they are decided); both lanes of the pair need it
                const int settled = (mine && !(close2 && !close3)) ? arg : -1;
                const int c = __shfl(settled, l32, 64);
                if (c >= 0) add_sample(xf, c);
            }
        };
        if constexpr (RES) {
            {
                float4 st[NST];
                for (int cb = 0; cb < g.nblocks; ++cb) {     // the whole state -> LDS (readers of the old one are done)
                    fetch_block(st, cb);
                    store_block(st, Ws + cb * WB * DP);
                }
            }
            if (tid == 0) s_next_rows = TM;                   // the first 32 rows of every wave are fixed
            if constexpr (FS) {
                for (int e = tid; e < k * DP8; e += MF_THREADS) fxsum[e] = 0;
                for (int e = tid; e < g.ns; e += MF_THREADS) cursor[e] = 0;
            }
            __syncthreads();
        }
        {
            float4 xa[NCH];
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) xa[ch] = frag(rowoff_of(wave * 32), ch);
            if constexpr (RES) {
                // No barrier inside this phase: the waves take their groups of 32 rows from a counter, so that a
                // wave that is held up (it shares its SIMD with a wave of another workgroup) does fewer of them.
                auto next_rows = [&]() -> int {
                    int v = 0;
                    if (lane == 0) v = atomicAdd(&s_next_rows, 32);
                    return __builtin_amdgcn_readfirstlane(v);
                };
                int cur = wave * 32;
                if constexpr (TWO) {
                    // two sets of fragment registers take turns
                    float4 xb2[NCH];
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) xb2[ch] = xa[ch];
                    while (cur < b) {
                        int nxt = next_rows();
                        do_tile(xa, xb2, cur, nxt, nxt < b);
                        cur = nxt;
                        if (cur >= b) break;
                        nxt = next_rows();
                        do_tile(xb2, xa, cur, nxt, nxt < b);
                        cur = nxt;
                    }
                } else {
                    while (cur < b) {
                        const int nxt = next_rows();
                        do_tile(xa, xa, cur, nxt, nxt < b);
                        cur = nxt;
                    }
                }
            } else {
                for (int tile0 = 0; tile0 < b; tile0 += TM)
                    do_tile(xa, xa, tile0 + wave * 32, tile0 + TM + wave * 32, tile0 + TM < b);
            }
        }
        __builtin_amdgcn_s_setprio(3);
        if constexpr (RES) {
            // ---- deferred exact decisions between two candidates ----
            // The state rows are still in LDS.  A lane pair (l32, half 0/1) takes one flagged sample: its half of the
            // dimensions of sum_j (w_aj - w_bj)(w_aj + w_bj - 2 x_j) in fp64, x fetched again (it is cache-hot), then
            // the halves are added.  32 samples per pass, so the memory latency is paid once per pass, not per sample.
            __syncthreads();       // the flags of a wave's rows below may come from any wave
            unsigned short *mylist = flist + wave * 32 * ((b + TM - 1) / TM);
            int nfl = 0;
            for (int tile0 = 0; tile0 < b; tile0 += TM) {
                const int n = tile0 + wave * 32 + l32;
                const bool fl = half == 0 && n < b && perm[n] != (unsigned short)0xFFFF;
                const unsigned long long m = __ballot(fl);
                if (fl) mylist[nfl + __popcll(m & ((1ull << lane) - 1ull))] = (unsigned short)n;
                nfl += __popcll(m);
            }
            for (int e0 = 0; e0 < nfl; e0 += 32) {
                const bool act = e0 + l32 < nfl;
                const int n = act ? (int)mylist[e0 + l32] : 0;
                const int ca = idx[n], cb2 = act ? (int)perm[n] : ca;
                const float *ra = Ws + ca * DP + 4 * half, *rb = Ws + cb2 * DP + 4 * half;
                const unsigned rowoff = (unsigned)n * (unsigned)d;
                float4 xv[NCH];
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) xv[ch] = frag(rowoff, ch);
                double dd = 0.0;
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const float4 wa = *reinterpret_cast<const float4 *>(ra + ch * 8);
                    const float4 wb = *reinterpret_cast<const float4 *>(rb + ch * 8);
                    // columns past d: the state rows are zero there, so the term vanishes whatever x holds
                    dd += ((double)wa.x - (double)wb.x) * (((double)wa.x + (double)wb.x) - 2.0 * (double)xv[ch].x);
                    dd += ((double)wa.y - (double)wb.y) * (((double)wa.y + (double)wb.y) - 2.0 * (double)xv[ch].y);
                    dd += ((double)wa.z - (double)wb.z) * (((double)wa.z + (double)wb.z) - 2.0 * (double)xv[ch].z);
                    dd += ((double)wa.w - (double)wb.w) * (((double)wa.w + (double)wb.w) - 2.0 * (double)xv[ch].w);
                }
                dd += __shfl_xor(dd, 32, 64);
                const int lo = ca < cb2 ? ca : cb2;
                const int res = dd < 0.0 ? ca : (dd > 0.0 ? cb2 : lo);
                if (act && half == 0) {
                    idx[n] = (unsigned short)res;
                    if (p.dump) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = res;
                }
                if constexpr (FS) {
                    if (act) add_sample(xv, res);
                }
            }
            rechecks += (lane == 0) ? nfl : 0;
        }

        // ================= phase 2: gradient, merge, update =================
        {
        int lane_p2 = threadIdx.x & 63;
        asm volatile("" : "+v"(lane_p2));
        const int lane = lane_p2, tid = wave * 64 + lane;
        // ---- stable counting sort of the samples by centroid slot ----
        // The mini-batch is cut into nr shares of whole groups of 64 samples (nr = number of waves unless the
        // counters would not fit).  Wave w < nr counts the samples of share w per slot and later places them, behind
        // those of the shares before it.  Entry slot * nr + w of `cursor` first holds that count, then the position of
        // the share's next sample of the slot.  (Every vector instruction of this part competes with the matrix work
        // of the other workgroup on the CU, so each wave looks at its share of the samples only.)
        const int NR = g.nr;
        const int spw = ((b + 63) / 64 + NR - 1) / NR * 64;
        const int n_lo = min(b, wave * spw), n_hi = wave < NR ? min(b, n_lo + spw) : n_lo;
        if constexpr (SS) {
            // Second pass over the mini-batch, in memory order (whole cache lines, many loads in flight, no sort): the
            // state rows in LDS are not needed any more, the fixed-point sums take their place.  The workgroup sweeps
            // R = threads / (d / 4) whole rows at a time, a thread keeps its group of four columns for the whole pass
            // (its scales stay in registers; threads past R rows idle), and the four sums of a group lie DP8/4 apart,
            // so that neighbouring lanes add to neighbouring addresses.  A term x * scale is rounded to an integer by
            // adding 1.5 * 2^23 in the same fused multiply-add; the BIT PATTERN of that float is what is added: it is
            // 0x4B400000 plus the integer, and the count of the centroid times that constant is taken off when the
            // sums are read (all modulo 2^32).
            constexpr int SU = 8, Q4 = DP8 / 4;
            const int c4n = d >> 2;                              // float4 per row
            const int R = MF_THREADS / c4n;
            const int myr = tid / c4n, myc = tid - myr * c4n;
            const bool act = myr < R;
            const float4 *xq = reinterpret_cast<const float4 *>(xb) + tid;      // sweep s: + s * R * c4n
            const unsigned sweep4 = (unsigned)(R * c4n);
            const float4 s4 = *reinterpret_cast<const float4 *>(colscale + (act ? 4 * myc : 0));
            int *cell0 = fxsum + myc;
            const int nfull = b / R;                             // sweeps with R valid rows
            const int nsweep = (b + R - 1) / R;
            // (the full sweeps are taken from the end of the mini-batch to its start: the rows that the assignment
            // read last are the ones most likely to be in a cache still; integer sums do not depend on the order)
            auto place = [&](int sw) { return sw < nfull ? nfull - 1 - sw : sw; };
            auto fetch = [&](float4(&v)[SU], int s0) {
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int sw = place(s0 + u);
                    v[u] = xq[(sw * R + myr < b ? (unsigned)sw : 0u) * sweep4];
                }
            };
            auto add = [&](auto guard, const float4(&v)[SU], int s0) {
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int n = place(s0 + u) * R + myr;
                    if (!decltype(guard)::value || n < b) {
                        int *cell = cell0 + (int)idx[n] * DP8;
                        atomicAdd(cell, (int)fx_term_bits(v[u].x, s4.x));
                        atomicAdd(cell + Q4, (int)fx_term_bits(v[u].y, s4.y));
                        atomicAdd(cell + 2 * Q4, (int)fx_term_bits(v[u].z, s4.z));
                        atomicAdd(cell + 3 * Q4, (int)fx_term_bits(v[u].w, s4.w));
                    }
                }
            };
            // two sets of SU loads take turns: one is in flight while the other is added
            float4 va[SU], vb[SU];
            if (act) fetch(va, 0);
            __syncthreads();                                   // every wave is through with the state rows; idx complete
            for (int e = tid; e < k * (DP8 / 4); e += MF_THREADS) reinterpret_cast<int4 *>(fxsum)[e] = make_int4(0, 0, 0, 0);
            for (int e = tid; e < g.ns; e += MF_THREADS) cursor[e] = 0;
            __syncthreads();
            for (int n = tid; n < b; n += MF_THREADS) {          // samples per centroid slot
                const int c = idx[n];
                atomicAdd(&cursor[(c % NWV) * g.kq + c / NWV], 1);
            }
            if (act) {
                int s0 = 0;
                for (; s0 + 2 * SU <= nfull; s0 += 2 * SU) {
                    fetch(vb, s0 + SU);
                    __builtin_amdgcn_sched_barrier(0);
                    add(std::false_type(), va, s0);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(va, s0 + 2 * SU);
                    __builtin_amdgcn_sched_barrier(0);
                    add(std::false_type(), vb, s0 + SU);
                    __builtin_amdgcn_sched_barrier(0);
                }
                for (; s0 < nsweep; s0 += SU) {
                    add(std::true_type(), va, s0);
                    if (s0 + SU < nsweep) fetch(va, s0 + SU);
                }
            }
        }
        if constexpr (FS) {
            // The sums and the counts per slot are complete once every wave is here.  The row passes below take the
            // count of a centroid from the list starts: an exclusive prefix over the slots (one wave), and the
            // fixed-point sums go to the scratch rows in fp32 (exact integers times a power of two).
            __syncthreads();
            if (wave == 0) {
                int running = 0;
                for (int base = 0; base < g.ns; base += 64) {
                    const int e = base + lane;
                    const int v = e < g.ns ? cursor[e] : 0;
                    int incl = v;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const int o = __shfl_up(incl, off, 64);
                        if (lane >= off) incl += o;
                    }
                    if (e < g.ns) cstart[e] = incl - v + running;
                    running += __shfl(incl, 63, 64);
                }
                if (lane == 0) cstart[g.ns] = running;
            }
            for (int e = tid; e < k * (DP8 / 4); e += MF_THREADS) {
                const int c = e / (DP8 / 4), j = 4 * (e - c * (DP8 / 4));
                if (j < d) {
                    const int4 v = *reinterpret_cast<const int4 *>(fxsum + c * DP8 + j);
                    const float4 inv = *reinterpret_cast<const float4 *>(colscale + DP8 + j);
                    *reinterpret_cast<float4 *>(gsc + (size_t)c * d + j) =
                        make_float4((float)v.x * inv.x, (float)v.y * inv.y, (float)v.z * inv.z, (float)v.w * inv.w);
                }
            }
        } else if constexpr (!SS) {
        for (int s = tid; s < g.ns * NR; s += MF_THREADS) cursor[s] = 0;
        if (tid == 0) s_next_item = 0;
        __syncthreads();                                   // also: idx complete
        for (int n = n_lo + lane; n < n_hi; n += 64) {
            const int c = idx[n];
            atomicAdd(&cursor[((c % NWV) * g.kq + c / NWV) * NR + wave], 1);
        }
        __syncthreads();
        {
            // exclusive prefix over the ns * nr entries: wave w scans those of its own slots (they are contiguous),
            // the totals of the waves give the offsets
            const int ne = g.kq * NR;
            int *mine = cursor + wave * ne;
            int running = 0;
            for (int base = 0; base < ne; base += 64) {
                const int e = base + lane;
                const int v = e < ne ? mine[e] : 0;
                int incl = v;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int o = __shfl_up(incl, off, 64);
                    if (lane >= off) incl += o;
                }
                if (e < ne) mine[e] = incl - v + running;
                running += __shfl(incl, 63, 64);
            }
            if (lane == 0) s_tot[wave] = running;
            __syncthreads();
            int woff = 0;
#pragma unroll
            for (int v = 0; v < MF_WAVES; ++v) woff += v < wave ? s_tot[v] : 0;
            for (int e = lane; e < ne; e += 64) {
                const int pos = mine[e] + woff;
                mine[e] = pos;
                if (e % NR == 0) cstart[wave * g.kq + e / NR] = pos;
            }
            if (wave == MF_WAVES - 1 && lane == 0) cstart[g.ns] = woff + running;
        }
        }
        const bool merge_point = (p.E > 0 && p.W > 1 && t > 0 && (t % p.E) == 0);
        const long long r_now = p.E > 0 ? t / p.E : 0;
        const int rpar = det ? (int)((r_now - 1) & 1) : 0;
        if (tid == MF_THREADS - 1) {
            int has = 0;                       // bit n: buffer n holds a message for this merge point
            for (int n = 0; merge_point && n < p.nb; ++n) {
                int *stp = p.stamp + exchange_buffer(rpar, p.nb, n, p.W, i);
                if (det) {
                    // stamps of one buffer only grow, so the test for the round needs no clearing
                    if (sync && t > t0) {      // (at the first step of a launch the message, if any, was sent before it)
                        const long long rs = r_now - 1;
                        const int sender = (i - shift_deterministic(p.seed, rs, p.W, n) + p.W) % p.W;
                        if ((p.drop_unannounced || !message_dropped(p.seed, rs, sender, p.drop_thr, n)) && !s_wait_failed &&
                            !mf_wait_flag(stp, (int)rs, false, &s_wait_budget)) {
                            s_wait_failed = 1;
                            __hip_atomic_store(p.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // host memory
                        }
                    }
                    if (__hip_atomic_load(stp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)(r_now - 1)) has |= 1 << n;
                    s_ext_round[n] = (int)(r_now - 1);
                } else {
                    const int st = *stp;
                    if (st >= 0) has |= 1 << n;
                    s_ext_round[n] = st;
                    *stp = -1;
                }
            }
            s_has_ext = has;
        }
        __syncthreads();
        // the message was written by another workgroup, maybe on another XCD, during this launch
        if (sync && merge_point) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if constexpr (!FS && !SS) {
        // placement: a wave walks its samples in order
        int nbits = 1;
        while ((1 << nbits) < k) ++nbits;
        for (int n0 = n_lo; n0 < n_hi; n0 += 64) {
            const int n = n0 + lane;
            const bool valid = n < n_hi;
            const int c = valid ? (int)idx[n] : -1;
            // lanes of this group with the same centroid as this lane: intersect, bit by bit of the index, the
            // ballot of the lanes that agree with this lane in that bit (no loop over distinct values)
            unsigned long long same = __ballot(valid);
            for (int bit = 0; bit < nbits; ++bit) {
                const unsigned long long set = __ballot(((c >> bit) & 1) != 0);
                same &= ((c >> bit) & 1) ? set : ~set;
            }
            const int rank = __popcll(same & ((1ull << lane) - 1ull));
            const bool last = (same >> lane) == 1ull;
            if (valid) {
                const int e = ((c % NWV) * g.kq + c / NWV) * NR + wave;
                const int base = cursor[e];
                perm[base + rank] = (unsigned short)n;
                if (last) cursor[e] = base + rank + 1;
            }
        }
        __syncthreads();        // the lists of a wave's centroids were written by all waves
        // gather, large clusters: the wave's 64 lanes are two half-waves of 32 float4 columns; a half-wave sums the
        // sample rows of one centroid at a time, in sample order, GU rows in flight, and takes its next centroid from a
        // counter when it is through: first the centroids with many samples, then the others, so that skewed cluster
        // sizes (the workload with Zipf weights) still spread evenly over the half-waves.  Which half-wave sums a
        // centroid does not change its sum.
        if (b >= 8 * k) {
            const int hw = lane >> 5, q4 = lane & 31;
            const bool colok = 4 * q4 < d;
            const int col = colok ? 4 * q4 : 0;
            const int big = max(b / (8 * NWV), GU);       // a quarter of a half-wave's share of the mini-batch
            int a = 0, nrow = 0, it = 0, c_cur = 0;
            bool done = false;
            float4 S = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            for (;;) {
                bool need = !done && it >= nrow;
                while (__ballot(need) != 0ull) {
                    // ticket v: slot v in the first round (taken if it is a big one), slot v - ns in the second
                    int v = 0;
                    if (need && q4 == 0) v = atomicAdd(&s_next_item, 1);
                    v = __shfl(v, hw * 32, 64);
                    if (need) {
                        if (v < 2 * g.ns) {
                            const int sl = v < g.ns ? v : v - g.ns;
                            const int a2 = cstart[sl], n2 = cstart[sl + 1] - a2;
                            if (v < g.ns ? (n2 >= big) : (n2 > 0 && n2 < big)) {
                                a = a2; nrow = n2; it = 0;
                                c_cur = (sl % g.kq) * NWV + sl / g.kq;
                                S = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                                need = false;
                            }
                        } else {
                            done = true;
                            need = false;
                        }
                    }
                }
                if (__ballot(!done) == 0ull) break;
                // past the end of its list a half-wave re-reads a valid row and adds 0 instead, so the loop
                // has no divergent branch
                float4 v[GU];
                int id[GU];
#pragma unroll
                for (int u = 0; u < GU; ++u) id[u] = perm[(!done && it + u < nrow) ? a + it + u : 0];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < GU; ++u) v[u] = *reinterpret_cast<const float4 *>(xb + (id[u] * d + col));
#pragma unroll
                for (int u = 0; u < GU; ++u) {
                    const bool ok = !done && it + u < nrow;
                    S.x += ok ? v[u].x : 0.0f; S.y += ok ? v[u].y : 0.0f;
                    S.z += ok ? v[u].z : 0.0f; S.w += ok ? v[u].w : 0.0f;
                }
                it += GU;
                if (!done && it >= nrow && colok) *reinterpret_cast<float4 *>(gsc + (size_t)c_cur * d + 4 * q4) = S;
            }
        }
        // gather, small clusters: this wave's samples in (centroid, sample) order, GS rows in flight whatever the
        // cluster boundaries; one lane per column
        else {
            const int pos0 = __builtin_amdgcn_readfirstlane(cstart[wave * g.kq]);
            const int pos1 = __builtin_amdgcn_readfirstlane(cstart[(wave + 1) * g.kq]);
            int cur = -1;
            float S[NJ];
#pragma unroll
            for (int jq = 0; jq < NJ; ++jq) S[jq] = 0.0f;
            for (int g0 = pos0; g0 < pos1; g0 += GS) {
                const int myid = (lane < GS && g0 + lane < pos1) ? (int)perm[g0 + lane] : -1;
                const int myc = myid >= 0 ? (int)idx[myid] : -1;
                float v[GS][NJ];
#pragma unroll
                for (int q = 0; q < GS; ++q) {
                    const int id = __builtin_amdgcn_readlane(myid, q);
                    const float *row = xb + (size_t)(id < 0 ? 0 : id) * d;
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        v[q][jq] = row[j < d ? j : 0];
                    }
                }
#pragma unroll
                for (int q = 0; q < GS; ++q) {
                    const int cq = __builtin_amdgcn_readlane(myc, q);
                    if (cq >= 0) {
                        if (cq != cur) {
                            if (cur >= 0) {
#pragma unroll
                                for (int jq = 0; jq < NJ; ++jq) {
                                    const int j = lane + 64 * jq;
                                    if (j < d) gsc[(size_t)cur * d + j] = S[jq];
                                }
                            }
                            cur = cq;
#pragma unroll
                            for (int jq = 0; jq < NJ; ++jq) S[jq] = 0.0f;
                        }
#pragma unroll
                        for (int jq = 0; jq < NJ; ++jq) S[jq] += v[q][jq];
                    }
                }
            }
            if (cur >= 0) {
#pragma unroll
                for (int jq = 0; jq < NJ; ++jq) {
                    const int j = lane + 64 * jq;
                    if (j < d) gsc[(size_t)cur * d + j] = S[jq];
                }
            }
        }
        }
        __threadfence_block();
        __syncthreads();

        // Samples and sum of the samples of a centroid, for the row passes below (lane l owns columns l and l + 64).
        // Streamed sums: straight from the fixed-point cells in LDS - the count times the rounding constant comes off
        // (modulo 2^32, like the additions), then the column's inverse scale; no list starts are formed.
        float invs[NJ];
        int cellofs[NJ];
#pragma unroll
        for (int jq = 0; jq < NJ; ++jq) {
            const int j = lane + 64 * jq, jc = j < d ? j : 0;
            invs[jq] = SS ? colscale[DP8 + jc] : 0.0f;
            cellofs[jq] = (jc & 3) * (DP8 / 4) + (jc >> 2);
        }
        auto count_of = [&](int c) -> int {
            const int sl = (c % NWV) * g.kq + c / NWV;
            if constexpr (SS) return cursor[sl];
            else return cstart[sl + 1] - cstart[sl];
        };
        auto sum_of = [&](int c, int cn, int jq, unsigned e) -> float {
            if constexpr (SS) return (float)fx_unbias((unsigned)fxsum[c * DP8 + cellofs[jq]], (unsigned)cn) * invs[jq];
            else return gsc[e];
        };
        const int has_mask = s_has_ext;      // uniform over the workgroup
        const float inv_b = 1.0f / (float)b;
        const float *ext0 = p.slot + exchange_buffer(rpar, p.nb, 0, p.W, i) * kd;          // buffer n: + n * W * kd
        const size_t ext_stride = (size_t)p.W * kd;
        if (p.parts > 1) {
            // ---- partial messages (Sec. 4.4): copy n for this worker carries the centroid rows c with
            // c mod P = (round + worker + n) mod P; lambda, Eq. 4 and Eq. 6 row by row, gate and update of a row in
            // one pass of the wave that takes it ----
            if (tid < 3) s_rowflags[tid] = 0;
            __syncthreads();
            int nz = 0, acc = 0, near = 0;
            wn2max = 0.0f;
            for (int c = wave; c < k; c += MF_WAVES) {
                const int cn = count_of(c);
                float w[NJ], gq[NJ], wesum[NJ];
#pragma unroll
                for (int jq = 0; jq < NJ; ++jq) {
                    const int j = lane + 64 * jq;
                    const unsigned e = (unsigned)c * (unsigned)d + (unsigned)(j < d ? j : 0);
                    w[jq] = wst[e];
                    const float sums = cn > 0 ? sum_of(c, cn, jq, e) : 0.0f;
                    gq[jq] = ((float)cn * w[jq] - sums) * inv_b;            // descent gradient of Eq. 9
                    wesum[jq] = 0.0f;
                }
                int rowmask = 0;
                for (int n = 0; n < p.nb; ++n) {
                    if (!(has_mask >> n & 1) || !row_travels(c, s_ext_round[n], i, n, p.parts)) continue;
                    float we[NJ];
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        we[jq] = ext0[n * ext_stride + (size_t)c * d + (j < d ? j : 0)];
                        if (j < d) {
                            const double wed = (double)we[jq];
                            const double a = ((double)w[jq] - (double)p.eps * (double)gq[jq]) - wed;
                            const double c2 = (double)w[jq] - wed;
                            lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                        }
                    }
                    lhs = wave_sum_d(lhs); rhs = wave_sum_d(rhs); nrm = wave_sum_d(nrm);
                    if (!(nrm > 0.0)) continue;
                    nz |= 1 << n;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) near = 1;
                    if (p.parzen ? (lhs < rhs) : 1) {
                        rowmask |= 1 << n;
#pragma unroll
                        for (int jq = 0; jq < NJ; ++jq) wesum[jq] += we[jq];
                    }
                }
                acc |= rowmask;
                const float inv = 1.0f / (float)(__builtin_popcount(rowmask) + 1);
                float s2 = 0.0f;
#pragma unroll
                for (int jq = 0; jq < NJ; ++jq) {
                    const int j = lane + 64 * jq;
                    if (j < d) {
                        float step = gq[jq];
                        if (rowmask) step += w[jq] - inv * (w[jq] + wesum[jq]);
                        const float wn = w[jq] - p.eps * step;
                        wst[(size_t)c * d + j] = wn;
                        s2 = fmaf(wn, wn, s2);
                    }
                }
                const float sq = wave_sum_f(s2);
                if (lane == 0) hs[c] = -0.5f * sq;
                wn2max = fmaxf(wn2max, sq);
            }
            if (lane == 0) {
                red_f[wave] = wn2max;
                if (nz) atomicOr(&s_rowflags[0], nz);
                if (acc) atomicOr(&s_rowflags[1], acc);
                if (near) atomicOr(&s_rowflags[2], near);
            }
            __threadfence_block();
            __syncthreads();
            wn2max = 0.0f;
#pragma unroll
            for (int v = 0; v < MF_WAVES; ++v) wn2max = fmaxf(wn2max, red_f[v]);
            if (tid == 0) {
                long long *cnp = p.counters + (size_t)i * CNT_STRIDE;
                cnp[CNT_RECEIVED] += __builtin_popcount(s_rowflags[0]);
                cnp[CNT_ACCEPTED] += __builtin_popcount(s_rowflags[1]);
                cnp[CNT_PARZEN_NEAR] += s_rowflags[2];
            }
        } else {
        // ---- Parzen sums (Eq. 4) over the whole state, fp64, every buffer on its own (Eq. 6) ----
        int delta_mask = 0;
        for (int n = 0; n < p.nb; ++n) {
            if (!(has_mask >> n & 1)) continue;
            const float *ext = ext0 + n * ext_stride;
            double lhs = 0.0, rhs = 0.0, nrm = 0.0;
            for (int c0 = wave * RB; c0 < k; c0 += MF_WAVES * RB) {
                float w[RB][NJ], sm[RB][NJ], we[RB][NJ];
                int cn[RB];
#pragma unroll
                for (int q = 0; q < RB; ++q) {
                    const int c = c0 + q < k ? c0 + q : k - 1;
                    cn[q] = count_of(c);
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        const unsigned e = (unsigned)c * (unsigned)d + (unsigned)(j < d ? j : 0);
                        w[q][jq] = wst[e]; sm[q][jq] = sum_of(c, cn[q], jq, e); we[q][jq] = ext[e];
                    }
                }
#pragma unroll
                for (int q = 0; q < RB; ++q) {
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        if (c0 + q < k && j < d) {
                            const float sums = cn[q] > 0 ? sm[q][jq] : 0.0f;
                            const float gq = ((float)cn[q] * w[q][jq] - sums) * inv_b;     // descent gradient of Eq. 9
                            const double wed = (double)we[q][jq];
                            const double a = ((double)w[q][jq] - (double)p.eps * (double)gq) - wed;
                            const double c2 = (double)w[q][jq] - wed;
                            lhs += a * a; rhs += c2 * c2; nrm += wed * wed;
                        }
                    }
                }
            }
            lhs = wave_sum_d(lhs); rhs = wave_sum_d(rhs); nrm = wave_sum_d(nrm);
            if (lane == 0) { red_d[0][wave] = lhs; red_d[1][wave] = rhs; red_d[2][wave] = nrm; }
            __syncthreads();
            lhs = rhs = nrm = 0.0;
#pragma unroll
            for (int v = 0; v < MF_WAVES; ++v) { lhs += red_d[0][v]; rhs += red_d[1][v]; nrm += red_d[2][v]; }
            if (nrm > 0.0) {                          // lambda of Eq. 3
                const int delta = p.parzen ? (lhs < rhs) : 1;   // Eq. 4
                delta_mask |= delta << n;
                if (tid == 0) {
                    long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                    cn[CNT_RECEIVED] += 1;
                    cn[CNT_ACCEPTED] += delta;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                }
            }
            __syncthreads();                          // red_d is written again for the next buffer
        }
        // ---- update: Eq. 6 (one buffer: Eq. 7), Alg. 5, update; new offsets h_c and max |w_c|^2 ----
        {
            const int delta = delta_mask != 0;
            const int first = delta ? __builtin_ctz(delta_mask) : 0;
            const int more_mask = delta_mask & (delta_mask - 1);             // accepted buffers after the first
            const float inv = 1.0f / (float)(__builtin_popcount(delta_mask) + 1);
            const float *extp = ext0 + first * ext_stride;                  // read only when a message was accepted
            wn2max = 0.0f;
            // four waves: twice the rows per wave in flight (the pass is a chain of load latencies, its registers are free here)
            constexpr int UB = NWV == 4 ? 2 * RB : RB;
            for (int c0 = wave * UB; c0 < k; c0 += MF_WAVES * UB) {
                float w[UB][NJ], sm[UB][NJ], we[UB][NJ], s2[UB];
                int cn[UB];
#pragma unroll
                for (int q = 0; q < UB; ++q) {
                    const int c = c0 + q < k ? c0 + q : k - 1;
                    cn[q] = count_of(c);
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        const unsigned e = (unsigned)c * (unsigned)d + (unsigned)(j < d ? j : 0);
                        w[q][jq] = wst[e]; sm[q][jq] = sum_of(c, cn[q], jq, e);
                        we[q][jq] = delta ? extp[e] : 0.0f;
                        for (int m = more_mask; m; m &= m - 1) we[q][jq] += ext0[__builtin_ctz(m) * ext_stride + e];
                    }
                }
#pragma unroll
                for (int q = 0; q < UB; ++q) {
                    s2[q] = 0.0f;
#pragma unroll
                    for (int jq = 0; jq < NJ; ++jq) {
                        const int j = lane + 64 * jq;
                        if (c0 + q < k && j < d) {
                            const float sums = cn[q] > 0 ? sm[q][jq] : 0.0f;
                            float step = ((float)cn[q] * w[q][jq] - sums) * inv_b;
                            if (delta) step += w[q][jq] - inv * (w[q][jq] + we[q][jq]);
                            const float wn = w[q][jq] - p.eps * step;
                            wst[(size_t)(c0 + q) * d + j] = wn;
                            s2[q] = fmaf(wn, wn, s2[q]);
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < UB; ++q) {
                    const float sq = wave_sum_f(s2[q]);
                    if (lane == 0 && c0 + q < k) hs[c0 + q] = -0.5f * sq;
                    wn2max = fmaxf(wn2max, sq);
                }
            }
            if (lane == 0) red_f[wave] = wn2max;
            __threadfence_block();
            __syncthreads();
            wn2max = 0.0f;
#pragma unroll
            for (int v = 0; v < MF_WAVES; ++v) wn2max = fmaxf(wn2max, red_f[v]);
        }

        }
        // every wave has read the external state for the last time (barrier above): its buffer may be written again
        if (sync && merge_point && tid == 0)
            __hip_atomic_store(p.consumed + i, (int)r_now, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // ---- send (Alg. 5, send) ----
        if (p.E > 0 && p.W > 1 && ((t + 1) % p.E) == 0) {
            const long long r = t / p.E;
            for (int n = 0; n < p.nb; ++n) {
                if (message_dropped(p.seed, r, i, p.drop_thr, n)) continue;
                const int peer = det ? peer_deterministic(p.seed, r, i, p.W, n) : peer_free(p.seed, r, i, p.W, n);
                const int spar = det ? (int)(r & 1) : 0;
                if (sync && r >= 2) {
                    // the buffer still holds the message of round r - 2 until the peer has passed merge point r - 1
                    if (tid == 0 && !s_wait_failed && !mf_wait_flag(p.consumed + peer, (int)(r - 1), true, &s_wait_budget)) {
                        s_wait_failed = 1;
                        __hip_atomic_store(p.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // host memory
                    }
                    __syncthreads();
                }
                float4 *dst = reinterpret_cast<float4 *>(p.slot + exchange_buffer(spar, p.nb, n, p.W, peer) * kd);
                const float4 *src = reinterpret_cast<const float4 *>(wst);
                if (p.parts == 1) {
                    for (size_t e = tid; e < kd / 4; e += MF_THREADS) dst[e] = src[e];
                } else {
                    // only the rows of the part travel: row c = part + P * m, float4 column q4 (d is a multiple of 4)
                    const int part = message_part(r, peer, n, p.parts), row4 = d / 4;
                    const int nrows = part_rows(k, part, p.parts);
                    for (int e = tid; e < nrows * row4; e += MF_THREADS) {
                        const size_t o = (size_t)part_row(part, p.parts, e / row4) * row4 + e % row4;
                        dst[o] = src[o];
                    }
                }
                __threadfence();
                __syncthreads();
                if (tid == 0) __hip_atomic_store(p.stamp + exchange_buffer(spar, p.nb, n, p.W, peer), (int)r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (tid == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
        }
        __syncthreads();
        }
    }

    rechecks = (long long)wave_sum_d((double)rechecks);
    if (lane == 0 && rechecks)
        atomicAdd((unsigned long long *)&p.counters[(size_t)i * CNT_STRIDE + CNT_RECHECK], (unsigned long long)rechecks);
}

// Eq. 8 for the contraction shapes: the same matrix-core scores as phase 1 of the step kernel, for ONE state and
// all N samples.  The centroid with the largest score x.w_c - |w_c|^2/2 is the nearest one: only the running
// maximum per sample is kept, with the place it came from in its low mantissa bits, and the distance to that
// centroid is then formed directly as sum_j (x_j - w_cj)^2 (no cancellation).  A workgroup (8 waves) walks tiles of 256 samples with a fixed stride, every lane pair adds its samples
// in fp64 in a fixed order, the partials are added in a fixed order: the result does not depend on scheduling.
// RES: the whole padded state fits LDS and is staged once per launch (no barriers in the loop over the samples); then a
// last half-block of at most eight centroids goes to 4x4 matrix tiles as in the step kernel.
template <int NCH, bool RES>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void quant_error_mfma_kernel(
    const float *__restrict__ x, long long N, int k, int d, const float *__restrict__ w, double *partials)
{
    constexpr int NWV = 8, MF_THREADS = 512, TM = 256;
    constexpr int DP8 = NCH * 8, DP = DP8 + 4, ROW4 = NCH * 2, NVEC = WB * ROW4;
    constexpr int NST = (NVEC + MF_THREADS - 1) / MF_THREADS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ double red[NWV];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int kpad = (k + WB - 1) / WB * WB, nblocks = kpad / WB;
    float *Ws = reinterpret_cast<float *>(smem_raw);                      // (RES ? kpad : 2 x WB) x DP
    float *hs = Ws + (size_t)(RES ? kpad : 2 * WB) * DP;                  // kpad
    constexpr bool TAILOK = RES && NCH <= 13;
    const int tail_groups = (TAILOK && (k & 31) >= 1 && (k & 31) <= 8 && ((k >> 5) & 1)) ? ((k & 31) + 3) / 4 : 0;
    const int tail_row0 = k & ~31;

    for (int c0 = wave * RB; c0 < kpad; c0 += NWV * RB) {                 // h_c = -|w_c|^2 / 2
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            const int c = c0 + q;
            float sq = 0.0f;
            for (int j = lane; j < d; j += 64) {
                const float v = w[(size_t)(c < k ? c : 0) * d + j];
                sq = fmaf(v, v, sq);
            }
            sq = wave_sum_f(sq);
            if (lane == 0) hs[c] = c < k ? -0.5f * sq : PAD_SCORE;
        }
    }
    const int col0 = (half && d >= 8) ? 4 : 0;
    const int collim = half ? (d >= 8 ? (d - 8) / 8 * 8 + 4 : 0) : (d - 4) / 8 * 8;
    auto fetch_block = [&](float4(&st)[NST], int cb) {
#pragma unroll
        for (int q = 0; q < NST; ++q) {
            const int e = tid + q * MF_THREADS;
            const int r = (e < NVEC ? e : 0) / ROW4, c4 = (e < NVEC ? e : 0) - r * ROW4;
            const int c = cb * WB + r, col = 4 * c4;
            const bool ok = c < k && col < d;
            float4 v = *reinterpret_cast<const float4 *>(w + (size_t)(ok ? c : 0) * d + (ok ? col : 0));
            if (!ok) v = make_float4(0.f, 0.f, 0.f, 0.f);
            st[q] = v;
        }
    };
    auto store_block = [&](const float4(&st)[NST], float *dst) {
#pragma unroll
        for (int q = 0; q < NST; ++q) {
            const int e = tid + q * MF_THREADS;
            if (e < NVEC) {
                const int r = e / ROW4, c4 = e - r * ROW4;
                *reinterpret_cast<float4 *>(&dst[r * DP + 4 * c4]) = st[q];
            }
        }
    };

    if constexpr (RES) {
        float4 st[NST];
        for (int cb = 0; cb < nblocks; ++cb) {
            fetch_block(st, cb);
            store_block(st, Ws + (size_t)cb * WB * DP);
        }
        __syncthreads();                 // state rows and hs complete
    }
    double sum = 0.0;
    for (long long tile0 = (long long)blockIdx.x * TM; tile0 < N; tile0 += (long long)gridDim.x * TM) {
        const long long n = tile0 + wave * 32 + l32;
        const bool ok = n < N;
        const float *row = x + (size_t)(ok ? n : 0) * d;
        float4 xf[NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int col = ch * 8 + col0;
            xf[ch] = *reinterpret_cast<const float4 *>(row + (col < collim ? col : collim));
        }
        float4 st[NST];
        if constexpr (!RES) {
            __syncthreads();             // nobody still reads the stage (and hs is complete)
            fetch_block(st, 0);
            store_block(st, Ws);
        }
        float best = -INFINITY;         // largest score so far, the number of its accumulator register in its low 5 bits
        int bestcb = 0;                 // ... and the block it came from
        for (int cb = 0; cb < nblocks; ++cb) {
            if constexpr (!RES) __syncthreads();
            const float *Wc = Ws + (size_t)(RES ? cb : (cb & 1)) * WB * DP;
            const bool more = !RES && cb + 1 < nblocks;
            const bool tailb = TAILOK && tail_groups > 0 && cb + 1 == nblocks;
            floatx16 acc0, acc1;
            {
                const float4 *hp = reinterpret_cast<const float4 *>(hs + cb * WB + 4 * half);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 h0 = hp[2 * q], h1 = hp[8 + 2 * q];
                    acc0[4 * q + 0] = h0.x; acc0[4 * q + 1] = h0.y; acc0[4 * q + 2] = h0.z; acc0[4 * q + 3] = h0.w;
                    acc1[4 * q + 0] = h1.x; acc1[4 * q + 1] = h1.y; acc1[4 * q + 2] = h1.z; acc1[4 * q + 3] = h1.w;
                }
            }
            const float *w0row = Wc + l32 * DP + 4 * half;
            const float *w1row = Wc + (32 + l32) * DP + 4 * half;
            if (tailb) {
                if constexpr (TAILOK) {
                    // rows 32 + (lane mod 4) (+ 4): a column of four state rows per block of four lanes
                    const float *wt = Wc + (32 + (lane & 3)) * DP + 4 * half;
                    floatx4 te = {0.0f, 0.0f, 0.0f, 0.0f}, to = te, t2 = te;
                    float4 a0 = *reinterpret_cast<const float4 *>(w0row);
                    float4 at = *reinterpret_cast<const float4 *>(wt);
                    float4 a2 = at;
                    if (tail_groups > 1) a2 = *reinterpret_cast<const float4 *>(wt + 4 * DP);
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {
                        float4 n0 = a0, nt = at, n2 = a2;
                        if (ch + 1 < NCH) {
                            n0 = *reinterpret_cast<const float4 *>(w0row + (ch + 1) * 8);
                            nt = *reinterpret_cast<const float4 *>(wt + (ch + 1) * 8);
                            if (tail_groups > 1) n2 = *reinterpret_cast<const float4 *>(wt + 4 * DP + (ch + 1) * 8);
                        }
                        const float4 xv = xf[ch];
                        floatx4 &t = (ch & 1) ? to : te;
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, xv.x, acc0, 0, 0, 0);
                        t = __builtin_amdgcn_mfma_f32_4x4x1f32(at.x, xv.x, t, 0, 0, 0);
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, xv.y, acc0, 0, 0, 0);
                        t = __builtin_amdgcn_mfma_f32_4x4x1f32(at.y, xv.y, t, 0, 0, 0);
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, xv.z, acc0, 0, 0, 0);
                        t = __builtin_amdgcn_mfma_f32_4x4x1f32(at.z, xv.z, t, 0, 0, 0);
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, xv.w, acc0, 0, 0, 0);
                        t = __builtin_amdgcn_mfma_f32_4x4x1f32(at.w, xv.w, t, 0, 0, 0);
                        if (tail_groups > 1) {
                            t2 = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.x, xv.x, t2, 0, 0, 0);
                            t2 = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.y, xv.y, t2, 0, 0, 0);
                            t2 = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.z, xv.z, t2, 0, 0, 0);
                            t2 = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.w, xv.w, t2, 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        a0 = n0; at = nt; a2 = n2;
                    }
                    // both halves' sums: rows 0..3 to the lower half-wave, rows 4..7 to the upper one, where a 32x32 tile
                    // would have left them (registers 0..3); the other registers of this accumulator hold padding
                    const float4 hv = *reinterpret_cast<const float4 *>(hs + tail_row0 + 4 * half);
                    const float hq[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(te[r] + to[r]), __float_as_uint(t2[r]), false, false);
                        acc1[r] = (__uint_as_float(sw[0]) + __uint_as_float(sw[1])) + hq[r];
                    }
#pragma unroll
                    for (int r = 4; r < 16; ++r) acc1[r] = PAD_SCORE;
                }
            } else {
                float4 a0 = *reinterpret_cast<const float4 *>(w0row);
                float4 a1 = *reinterpret_cast<const float4 *>(w1row);
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    float4 n0 = a0, n1 = a1;
                    if (ch + 1 < NCH) {
                        n0 = *reinterpret_cast<const float4 *>(w0row + (ch + 1) * 8);
                        n1 = *reinterpret_cast<const float4 *>(w1row + (ch + 1) * 8);
                    }
                    const float4 xv = xf[ch];
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, xv.x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, xv.x, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, xv.y, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, xv.y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, xv.z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, xv.z, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, xv.w, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, xv.w, acc1, 0, 0, 0);
                    if (ch == 0 && more) fetch_block(st, cb + 1);
                    __builtin_amdgcn_sched_barrier(0);
                    a0 = n0; a1 = n1;
                }
            }
            if (more) store_block(st, Ws + ((cb + 1) & 1) * WB * DP);
            float bm = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float t0 = __uint_as_float((__float_as_uint(acc0[r]) & 0xFFFFFFE0u) | (unsigned)r);
                const float t1 = __uint_as_float((__float_as_uint(acc1[r]) & 0xFFFFFFE0u) | (unsigned)(16 + r));
                bm = fmaxf(bm, fmaxf(t0, t1));
            }
            if (bm > best) { best = bm; bestcb = cb; }
        }
        // The scores only pick the centroid; the distance to it is formed directly, sum_j (x_j - w_cj)^2, so that no
        // |x|^2/2 - score cancellation enters the sum (tight clusters far from the origin).  Among scores that agree to
        // the rounding error (and the 5 tag bits) any may win: their distances differ by less than that error.
        int c;
        {
            const int r = (int)(__float_as_uint(best) & 31u);
            // accumulator register r of half-wave h holds row 8*((r & 15) / 4) + 4*h + (r & 3) of the block (+32: second accumulator)
            c = bestcb * WB + (r & 16) * 2 + 8 * ((r & 15) >> 2) + 4 * half + (r & 3);
            const float ob = __shfl_xor(best, 32, 64);       // the other half-wave saw the other centroid rows
            const int oc = __shfl_xor(c, 32, 64);
            if (ob > best || (ob == best && oc < c)) c = oc;
            c = c < k ? c : k - 1;
        }
        float d2 = 0.0f;
        const float *wrow = w + (size_t)c * d;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            if (ch * 8 + 4 * half < d) {            // a real column (clamped ones repeat data)
                const float4 wv4 = *reinterpret_cast<const float4 *>(wrow + ch * 8 + col0);
                const float e0 = xf[ch].x - wv4.x, e1 = xf[ch].y - wv4.y, e2 = xf[ch].z - wv4.z, e3 = xf[ch].w - wv4.w;
                d2 = fmaf(e0, e0, d2); d2 = fmaf(e1, e1, d2); d2 = fmaf(e2, e2, d2); d2 = fmaf(e3, e3, d2);
            }
        }
        d2 += __shfl_xor(d2, 32, 64);                       // the other half-wave holds the other half of the dimensions
        if (half == 0 && ok) sum += (double)(0.5f * d2);
    }
    sum = wave_sum_d(sum);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int v = 0; v < NWV; ++v) tot += red[v];
        partials[blockIdx.x] = tot;
    }
}

constexpr size_t MF_LDS_BUDGET = 150 * 1024;

template <int NCH>
hipError_t launch_qe_nch(const float *x, long long N, int d, int k, const float *w, double *partials, int nblocks, hipStream_t s)
{
    const int kpad = (k + WB - 1) / WB * WB;
    const size_t lds_res = ((size_t)kpad * (NCH * 8 + 4) + kpad) * sizeof(float);
    if (lds_res <= MF_LDS_BUDGET) {
        hipError_t e = hipFuncSetAttribute((const void *)quant_error_mfma_kernel<NCH, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_res);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((quant_error_mfma_kernel<NCH, true>), dim3(nblocks), dim3(512), lds_res, s, x, N, k, d, w, partials);
        return hipGetLastError();
    }
    const size_t lds = ((size_t)2 * WB * (NCH * 8 + 4) + kpad) * sizeof(float);
    hipError_t e = hipFuncSetAttribute((const void *)quant_error_mfma_kernel<NCH, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((quant_error_mfma_kernel<NCH, false>), dim3(nblocks), dim3(512), lds, s, x, N, k, d, w, partials);
    return hipGetLastError();
}
template <int NCH, bool RES, int NWV, int FSM = 0>
hipError_t launch_variant(const StepParams &p, long long t0, long long t1, const float *xnorm2max, hipStream_t s, bool persistent)
{
    const size_t lds = mfma_geom(p.k, p.b, NCH, RES, NWV, FSM == 1 ? 1 : (FSM == 3 ? 2 : 0)).bytes;
    const void *kern = (const void *)mfma_steps_kernel<NCH, RES, NWV, FSM>;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (!persistent) {
        hipLaunchKernelGGL((mfma_steps_kernel<NCH, RES, NWV, FSM>), dim3(p.W), dim3(64 * NWV), lds, s, p, t0, t1, xnorm2max, 0);
        return hipGetLastError();
    }
    // one launch with waits inside: every workgroup must be resident
    int dev = 0, cus = 0, per_cu = 0;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 64 * NWV, lds);
    if (e != hipSuccess) return e;
    if ((long long)per_cu * cus < p.W) return hipErrorCooperativeLaunchTooLarge;
    StepParams pp = p;
    long long a0 = t0, a1 = t1;
    const float *xn = xnorm2max;
    int sync = 1;
    void *args[] = {&pp, &a0, &a1, &xn, &sync};
    if (p.cooperative) return hipLaunchCooperativeKernel(kern, dim3(p.W), dim3(64 * NWV), args, (unsigned)lds, s);
    hipLaunchKernelGGL((mfma_steps_kernel<NCH, RES, NWV, FSM>), dim3(p.W), dim3(64 * NWV), lds, s, pp, a0, a1, xn, sync);
    return hipGetLastError();
}
template <int NCH>
hipError_t launch_nch(const StepParams &p, long long t0, long long t1, const float *xnorm2max, hipStream_t s, bool persistent)
{
    // tune bit 0 forces 8 waves, bit 1 forces 4 waves (resident variant only); bit 2 (host side) forces one launch per
    // round, bit 3 one launch with waits also for 8 waves
    const size_t half_cu = 78 * 1024;      // two workgroups per CU must fit 160 KB, a little is reserved
    // Fused sums (the mini-batch is read once): eight waves, resident state and the fixed-point sums in LDS, which
    // leaves room for ONE workgroup per CU.  Measured on the k = d = 100 workload: 6.5 ms per epoch against 7.2 ms for
    // the same shape with sort and gather, but 6.1 ms for two four-wave workgroups per CU with sort and gather, whose
    // memory phases hide behind each other's matrix work; so it is not the default.  tune bit 5 asks for it.
    if constexpr (NCH <= 13) {             // (d = 128 would spill registers with two sets of fragments)
        const bool fits = mfma_geom(p.k, p.b, NCH, true, 8, 1).bytes <= MF_LDS_BUDGET;
        if (fits && (p.tune & 32)) {
            if (persistent && !(p.tune & 8)) return hipErrorNotSupported;      // one workgroup per CU: one launch per round
            return launch_variant<NCH, true, 8, 1>(p, t0, t1, xnorm2max, s, persistent);
        }
    }
    if (mfma_geom(p.k, p.b, NCH, true, 4).bytes <= half_cu && ((p.W > 256 && !(p.tune & 1)) || (p.tune & 2))) {
        // d <= 104 (d = 128 has no registers for it): the next tile's samples go to a second set of registers a whole
        // tile ahead, and the gradient sums are formed in a second pass over the mini-batch in memory order (on the
        // k = d = 100 workload 1.2 % and another 9 % of an epoch).  tune bit 7: sort and gather instead of the second
        // pass; bit 6: neither
        if constexpr (NCH <= 13) {
            if (!(p.tune & (64 | 128))) return launch_variant<NCH, true, 4, 3>(p, t0, t1, xnorm2max, s, persistent);
            if (!(p.tune & 64)) return launch_variant<NCH, true, 4, 2>(p, t0, t1, xnorm2max, s, persistent);
        }
        return launch_variant<NCH, true, 4>(p, t0, t1, xnorm2max, s, persistent);
    }
    // One workgroup per CU: the workers keep pace by themselves, and for a call of a single round one launch per round
    // measured 1 % faster than the waits inside one launch (two workgroups per CU drift apart and gain 3 % from not
    // meeting at every round).  A call that covers several rounds is better off as one launch here too: the start and
    // the tail of a launch are paid once (k = 1024, d = 128 workload, ten rounds per call: 9.88 -> 9.49 ms per round).
    const long long rounds_in_call = p.E > 0 ? (t1 - t0) / p.E : 0;
    if (persistent && !(p.tune & 8) && rounds_in_call < 2) return hipErrorNotSupported;
    if (mfma_geom(p.k, p.b, NCH, true, 8).bytes <= MF_LDS_BUDGET)
        return launch_variant<NCH, true, 8>(p, t0, t1, xnorm2max, s, persistent);
    return launch_variant<NCH, false, 8>(p, t0, t1, xnorm2max, s, persistent);
}

}  // namespace

bool mfma_kernel_supports(int k, int d, int b, const void *x)
{
    if (d % 4 != 0 || d > 128 || k < 2 || k > 32768 || b > 65535 || (((uintptr_t)x) & 15u) != 0) return false;
    return mfma_geom(k, b, mfma_chunks(d), false, 8).bytes <= MF_LDS_BUDGET;
}

bool mfma_quant_error_supports(int k, int d, const void *x)
{
    if (d % 4 != 0 || d < 16 || d > 128 || k < 32 || k > 32768 || (((uintptr_t)x) & 15u) != 0) return false;
    const int kpad = (k + WB - 1) / WB * WB;
    return ((size_t)2 * WB * (mfma_chunks(d) * 8 + 4) + kpad) * sizeof(float) <= MF_LDS_BUDGET;
}

hipError_t launch_quant_error_mfma(const float *x, long long N, int d, int k, const float *w, double *partials,
                                   int nblocks, hipStream_t s)
{
    switch (mfma_chunks(d)) {
        case 4: return launch_qe_nch<4>(x, N, d, k, w, partials, nblocks, s);
        case 8: return launch_qe_nch<8>(x, N, d, k, w, partials, nblocks, s);
        case 13: return launch_qe_nch<13>(x, N, d, k, w, partials, nblocks, s);
        default: return launch_qe_nch<16>(x, N, d, k, w, partials, nblocks, s);
    }
}

hipError_t launch_rownorm2max(const float *x, long long rows, int d, float *out, hipStream_t s)
{
    const int nblocks = 1024;
    float *partial = nullptr;
    hipError_t e = hipMalloc((void **)&partial, nblocks * sizeof(float));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rownorm2_partial_kernel, dim3(nblocks), dim3(256), 0, s, x, rows, d, partial);
    hipLaunchKernelGGL(rownorm2_final_kernel, dim3(1), dim3(64), 0, s, partial, nblocks, out);
    e = hipGetLastError();
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(partial);
    return e != hipSuccess ? e : e2;
}

hipError_t launch_mfma_steps(const StepParams &p, long long t0, long long t1, const float *xnorm2max, hipStream_t s,
                             bool persistent)
{
    switch (mfma_chunks(p.d)) {
        case 4: return launch_nch<4>(p, t0, t1, xnorm2max, s, persistent);
        case 8: return launch_nch<8>(p, t0, t1, xnorm2max, s, persistent);
        case 13: return launch_nch<13>(p, t0, t1, xnorm2max, s, persistent);
        default: return launch_nch<16>(p, t0, t1, xnorm2max, s, persistent);
    }
}

}  // namespace asgd
