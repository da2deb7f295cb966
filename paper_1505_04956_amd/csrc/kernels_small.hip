// Step kernel for small states (k*d of the order of 100): the streaming workloads.
//
// One workgroup of NW wavefronts per worker.  A lane takes one sample at a time:
//   - the sample's d floats come straight from HBM into registers (the next group of 64
//     samples is requested before the current one is processed);
//   - the k scores x.w_k - |w_k|^2/2 (largest score = nearest centroid, the |x|^2 term is
//     common to all k) are fused multiply-add chains against a wave-uniform copy of the state
//     held in registers;
//   - the two best scores are tracked; when they are closer than a rigorous bound on the fp32
//     rounding error of the scores, the lane recomputes its assignment exactly (fp64, direct
//     form), so the assignment is the exact-arithmetic nearest centroid of the fp32 state;
//   - the gradient sums of Eq. 9 go to a private accumulator column per lane in LDS
//     (bank = lane, so the LDS adds never conflict); a fixed-order reduction over the 64
//     columns and the NW waves follows once per step.
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

template <int K, int D, int NW, int PF>
__global__ __launch_bounds__(64 * NW) void small_steps_kernel(StepParams p, long long t0, long long t1)
{
    constexpr int KD = K * D;
    constexpr int NV = KD + K;                 // per-lane accumulator column: k*d sums, then k counts
    constexpr int NSLOT = (NV + 63) / 64;      // values a lane owns in the lane-distributed layout

    __shared__ __attribute__((aligned(16))) float acc[NW][NV][64];
    __shared__ float part[2][NW][NSLOT * 64];  // per-wave step totals, double-buffered by step parity
    __shared__ __attribute__((aligned(16))) float wbc[NW][KD];   // state, one copy per wave

    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int b = p.b;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);
    const float inv_b = 1.0f / (float)b;

    // lane-distributed state: element e = slot*64 + lane
    float wl[NSLOT];
#pragma unroll
    for (int q = 0; q < NSLOT; ++q) {
        const int e = q * 64 + lane;
        wl[q] = e < KD ? p.w[(size_t)i * KD + e] : 0.0f;
    }
    float xmax[D];
#pragma unroll
    for (int j = 0; j < D; ++j) xmax[j] = p.xabsmax[j];

    // clear this wave's accumulator columns
    {
        float4 *a4 = reinterpret_cast<float4 *>(&acc[wave][0][0]);
        for (int q = lane; q < NV * 16; q += 64) a4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    long long rechecks = 0;
    const int ngroups = (b + 63) / 64;

    for (long long t = t0; t < t1; ++t) {
        // ---- wave-uniform copy of the state and of -|w_k|^2/2 ----
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int e = q * 64 + lane;
            if (e < KD) wbc[wave][e] = wl[q];
        }
        __syncthreads();
        float wv[KD];
#pragma unroll
        for (int e = 0; e < KD; ++e) wv[e] = wbc[wave][e];
        float hn[K];
        float bound = 0.0f, hmax = 0.0f;
#pragma unroll
        for (int c = 0; c < K; ++c) {
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) s = fmaf(wv[c * D + j], wv[c * D + j], s);
            hn[c] = -0.5f * s;
            hmax = fmaxf(hmax, 0.5f * s);
        }
#pragma unroll
        for (int j = 0; j < D; ++j) {
            float m = 0.0f;
#pragma unroll
            for (int c = 0; c < K; ++c) m = fmaxf(m, fabsf(wv[c * D + j]));
            bound = fmaf(xmax[j], m, bound);
        }
        // Each score is a chain of D fused multiply-adds started from hn (itself D of them), so its
        // rounding error is below (2D+1) * 2^-24 * (sum_j max|x_j| max_k|w_kj| + max_k |hn_k|).  Two
        // scores that differ by more than twice that (here with a factor 1.5 to spare) are ordered
        // correctly.
        const float thr = 3.0f * (float)(2 * D + 1) * 5.9604645e-8f * (bound + hmax);

        const long long s = t % p.S;
        const float *xb = p.x + ((size_t)i * p.H + (size_t)s * b) * D;

        // ---- stream the mini-batch: groups of 64 samples, wave v takes groups v, v+NW, ... ----
        // PF groups are in flight per wave: buffer u is refilled (for the group PF turns ahead) as
        // soon as it has been consumed.  Loads past the end of the mini-batch are clamped to its
        // last row and never used; keeping them unconditional lets the hardware counters tell the
        // compiler exactly how many younger loads may still be outstanding.
        float xr[PF][D];
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int n = (wave + u * NW) * 64 + lane;
            load_row<D>(xr[u], xb + (size_t)(n < b ? n : b - 1) * D);
        }
        for (int g0 = wave; g0 < ngroups; g0 += NW * PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int g = g0 + u * NW;
                const int n = g * 64 + lane;
                float xc[D];
#pragma unroll
                for (int j = 0; j < D; ++j) xc[j] = xr[u][j];
                {
                    const int nn = (g + PF * NW) * 64 + lane;
                    load_row<D>(xr[u], xb + (size_t)(nn < b ? nn : b - 1) * D);
                }
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
                    double dbest = INFINITY;
                    int darg = 0;
                    for (int c = 0; c < K; ++c) {
                        double sd = 0.0;
#pragma unroll
                        for (int j = 0; j < D; ++j) {
                            double diff = (double)xc[j] - (double)wbc[wave][c * D + j];
                            sd += diff * diff;
                        }
                        if (sd < dbest) { dbest = sd; darg = c; }
                    }
                    arg = darg;
                    rechecks += 1;
                }
                if (valid) {
                    float *col = &acc[wave][arg * D][lane];
#pragma unroll
                    for (int j = 0; j < D; ++j)
                        __hip_atomic_fetch_add(col + j * 64, xc[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_fetch_add(&acc[wave][KD + arg][lane], 1.0f, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (p.dump) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;
                }
            }
        }

        // ---- reduce the 64 accumulator columns of this wave (fixed order), clear them ----
        __syncthreads();
        const int par = (int)(t & 1);
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int v = q * 64 + lane;
            float tot = 0.0f;
            if (v < NV) {
                float4 *row = reinterpret_cast<float4 *>(&acc[wave][v][0]);
                float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int cq = (lane + r) & 15;            // rotated start: conflict-free banks
                    float4 a = row[cq];
                    row[cq] = make_float4(0.f, 0.f, 0.f, 0.f);
                    s0 += a.x; s1 += a.y; s2 += a.z; s3 += a.w;
                }
                tot = (s0 + s1) + (s2 + s3);
            }
            part[par][wave][q * 64 + lane] = tot;
        }
        __syncthreads();
        // totals over the waves, in wave order; count of the centroid each owned element belongs to
        float S[NSLOT], cntv[NSLOT];
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int e = q * 64 + lane;
            float sv = 0.0f, cv = 0.0f;
            if (e < KD) {
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    sv += part[par][v][e];
                    cv += part[par][v][KD + e / D];
                }
            }
            S[q] = sv;
            cntv[q] = cv;
        }

        // ---- merge point? (a buffer is looked at once, at the first step of a round) ----
        const bool merge_point = (p.E > 0 && t > 0 && (t % p.E) == 0);
        const long long r_now = p.E > 0 ? t / p.E : 0;
        const int rpar = det ? (int)((r_now - 1) & 1) : 0;
        bool has_ext = false;
        if (merge_point) {
            const int st = p.stamp[(size_t)rpar * p.W + i];
            has_ext = det ? (st == (int)(r_now - 1)) : (st >= 0);
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
                we[q] = ext[e];
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
                if (tid == 0) {
                    long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                    cn[CNT_RECEIVED] += 1;
                    cn[CNT_ACCEPTED] += delta;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                }
            }
        }
        if (merge_point) {
            __syncthreads();     // every wave has read the stamp and the buffer
            if (tid == 0) p.stamp[(size_t)rpar * p.W + i] = -1;
        }
        // Eq. 7 and Alg. 5 line 8
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            float step = G[q];
            if (delta) step += wl[q] - 0.5f * (wl[q] + we[q]);
            wl[q] = wl[q] - p.eps * step;
        }

        // ---- send (Alg. 5 line 9) ----
        if (p.E > 0 && p.W > 1 && ((t + 1) % p.E) == 0) {
            const long long r = t / p.E;
            if (wave == 0) {
                if (!message_dropped(p.seed, r, i, p.drop_thr)) {
                    const int peer = det ? peer_deterministic(p.seed, r, i, p.W) : peer_free(p.seed, r, i, p.W);
                    const int spar = det ? (int)(r & 1) : 0;
                    float *dst = p.slot + ((size_t)spar * p.W + peer) * KD;
#pragma unroll
                    for (int q = 0; q < NSLOT; ++q) {
                        const int e = q * 64 + lane;
                        if (e < KD) dst[e] = wl[q];
                    }
                    __threadfence();
                    if (lane == 0) p.stamp[(size_t)spar * p.W + peer] = (int)r;
                }
                if (lane == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
            }
        }
    }

    if (wave == 0) {
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            const int e = q * 64 + lane;
            if (e < KD) p.w[(size_t)i * KD + e] = wl[q];
        }
    }
    for (int off = 32; off > 0; off >>= 1) rechecks += __shfl_xor(rechecks, off, 64);
    if (lane == 0 && rechecks)
        atomicAdd((unsigned long long *)&p.counters[(size_t)i * CNT_STRIDE + CNT_RECHECK], (unsigned long long)rechecks);
}

}  // namespace

bool small_kernel_supports(int k, int d, int b)
{
    (void)b;
    return k == 10 && d == 10;
}

hipError_t launch_small_steps(const StepParams &p, long long t0, long long t1, hipStream_t s)
{
    if (p.k == 10 && p.d == 10) {
        switch (p.tune) {
            case 1: hipLaunchKernelGGL((small_steps_kernel<10, 10, 1, 2>), dim3(p.W), dim3(64), 0, s, p, t0, t1); break;
            case 2: hipLaunchKernelGGL((small_steps_kernel<10, 10, 1, 4>), dim3(p.W), dim3(64), 0, s, p, t0, t1); break;
            case 3: hipLaunchKernelGGL((small_steps_kernel<10, 10, 2, 2>), dim3(p.W), dim3(128), 0, s, p, t0, t1); break;
            case 4: hipLaunchKernelGGL((small_steps_kernel<10, 10, 2, 3>), dim3(p.W), dim3(128), 0, s, p, t0, t1); break;
            default: hipLaunchKernelGGL((small_steps_kernel<10, 10, 1, 3>), dim3(p.W), dim3(64), 0, s, p, t0, t1); break;
        }
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace asgd
