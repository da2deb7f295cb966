// Step kernel for large states (k*d too large for registers/LDS): the contraction-bound workloads
// (k = 100, d = 100 and k = 1024, d = 128).
//
// One workgroup of 4 wavefronts per worker.  A step has two phases.
//
// Phase 1, assignment: the scores x.w_c - |w_c|^2/2 of a tile of 128 samples against all centroids
// are a dense contraction over d and run on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32).
//   - The state is kept a second time in "augmented" form W' (kpad x daug8, row c = [w_c, h_c, 0..],
//     h_c = -|w_c|^2/2) and a sample row as [x, 1, 0..], so the offset is part of the contraction.
//   - The sample tile sits in LDS for the whole pass over the centroids; blocks of 64 centroid rows
//     of W' stream through a double-buffered LDS stage (W' itself stays in L2 / Infinity Cache).
//   - Wave v owns 32 samples (matrix columns); rows are centroids.  A lane then holds, for ONE
//     sample, 16 centroid scores per 32x32 tile, so the running arg-max is lane-local; the two
//     half-waves (which see different centroid rows of the same sample) are merged once per tile.
//   - Operands are fetched as float4 (4 consecutive dimensions) with the same (row, 4*half) pattern
//     for both matrices; the matrix instruction number r of a group of four contracts dimensions
//     r and r+4 of an 8-dimension chunk.  The order of the contraction over d is therefore a fixed
//     permutation of 0..d-1; no transposition is needed.  LDS rows are padded to a stride that is an
//     odd multiple of 4 floats, which keeps the 128-bit reads free of bank conflicts.
//   - The three largest scores and the indices of the two largest are tracked.  If the first two are
//     closer than a bound on the fp32 rounding error, the sample is decided exactly in fp64 (pair
//     comparison, or all k distances when the third is close too), lowest index on ties.
// Phase 2, gradient and update: every centroid is owned by one wave (c mod 4), which scans the
// assignments in sample order, adds the matching samples (lanes = dimensions) and updates the
// centroid row: all sums have one fixed order, nothing is accumulated with atomics.
#include "asgd_internal.h"

namespace asgd {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int MF_THREADS = 256;
constexpr int MF_WAVES = 4;
constexpr int TM = 128;          // samples per tile (32 per wave)
constexpr int WB = 64;           // centroid rows per W' block (2 matrix tiles of 32)
constexpr float PAD_SCORE = -1.0e30f;   // offset of the padding rows of W': never the nearest

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

__device__ __forceinline__ double wave_sum_d(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Geometry shared by host and device.
struct MfmaGeom {
    int daug8;     // d + 1 rounded up to a multiple of 8: row length of W'
    int DP;        // LDS row stride in floats (daug8 + 4: an odd multiple of 4)
    int kpad;      // k rounded up to a multiple of WB
    int nblocks;   // kpad / WB
};
__host__ __device__ inline MfmaGeom mfma_geom(int k, int d)
{
    MfmaGeom g;
    g.daug8 = (d + 1 + 7) / 8 * 8;
    g.DP = g.daug8 + 4;
    g.kpad = (k + WB - 1) / WB * WB;
    g.nblocks = g.kpad / WB;
    return g;
}

// max over rows of |x|^2 (one value), used by the rounding-error bound
__global__ void rownorm2_partial_kernel(const float *__restrict__ x, long long rows, int d, float *partial)
{
    __shared__ float red[256];
    float m = 0.0f;
    for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += (long long)gridDim.x * blockDim.x) {
        const float *xr = x + (size_t)r * d;
        float s = 0.0f;
        for (int j = 0; j < d; ++j) s = fmaf(xr[j], xr[j], s);
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

// NJ = ceil(d / 64): dimensions per lane in the per-centroid passes (lane l owns l, l+64, ...)
template <int NJ>
__global__ __launch_bounds__(MF_THREADS) void mfma_steps_kernel(StepParams p, long long t0, long long t1, float *waug_all,
                                                                 const float *xnorm2max_ptr)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ double red_d[3][MF_WAVES];
    __shared__ float red_f[MF_WAVES];
    __shared__ int s_has_ext;

    const int i = blockIdx.x;                       // worker
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int half = lane >> 5, l32 = lane & 31;
    const int k = p.k, d = p.d, b = p.b;
    const MfmaGeom g = mfma_geom(k, d);
    const size_t kd = (size_t)k * d;
    const int det = (p.mode == ASGD_MODE_DETERMINISTIC);

    float *Xs = smem;                                   // TM x DP
    float *Ws = Xs + TM * g.DP;                         // 2 x WB x DP
    unsigned short *idx = reinterpret_cast<unsigned short *>(Ws + 2 * WB * g.DP);   // b assignments

    float *wst = p.w + (size_t)i * kd;                  // state of this worker
    float *waug = waug_all + (size_t)i * g.kpad * g.daug8;
    float *gsc = p.acc + (size_t)i * kd;                // gradient scratch
    const float xn2 = *xnorm2max_ptr;

    // ---- augmented copy of the state, and max_c |w_c|^2 ----
    float wn2max = 0.0f;
    for (int c = wave; c < g.kpad; c += MF_WAVES) {
        float *row = waug + (size_t)c * g.daug8;
        float s = 0.0f;
        for (int j = lane; j < g.daug8; j += 64) {
            float v = 0.0f;
            if (c < k && j < d) {
                v = wst[(size_t)c * d + j];
                s = fmaf(v, v, s);
            }
            if (j != d) row[j] = v;
        }
        s = wave_sum_f(s);
        if (lane == 0) row[d] = c < k ? -0.5f * s : PAD_SCORE;
        wn2max = fmaxf(wn2max, s);
    }
    if (lane == 0) red_f[wave] = wn2max;
    __syncthreads();
    wn2max = fmaxf(fmaxf(red_f[0], red_f[1]), fmaxf(red_f[2], red_f[3]));
    __syncthreads();

    long long rechecks = 0;

    for (long long t = t0; t < t1; ++t) {
        const long long s_ep = t % p.S;
        const float *xb = p.x + ((size_t)i * p.H + (size_t)s_ep * b) * d;
        // Rounding-error bound of a score: daug8 products and sums on the matrix core plus the d roundings
        // inside h_c, all relative to |x||w_c| + |h_c| <= sqrt(max|x|^2 max|w|^2) + max|w|^2/2.
        const float Bb = sqrtf(xn2) * sqrtf(wn2max) + 0.5f * wn2max;
        const float thr = 3.0f * (float)(2 * g.daug8 + 4) * 5.9604645e-8f * Bb;

        // ================= phase 1: assignment =================
        for (int tile0 = 0; tile0 < b; tile0 += TM) {
            __syncthreads();        // previous tile's readers of Xs are done
            // sample tile -> LDS, as [x, 1, 0...]; rows past the mini-batch are zero
            {
                const int d4 = d >> 2;
                for (int e = tid; e < TM * d4; e += MF_THREADS) {
                    const int r = e / d4, c4 = e - r * d4;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (tile0 + r < b) v = reinterpret_cast<const float4 *>(xb + (size_t)(tile0 + r) * d)[c4];
                    *reinterpret_cast<float4 *>(&Xs[r * g.DP + 4 * c4]) = v;
                }
                for (int e = tid; e < TM * (g.daug8 - d); e += MF_THREADS) {
                    const int r = e / (g.daug8 - d), c = d + e % (g.daug8 - d);
                    Xs[r * g.DP + c] = (c == d && tile0 + r < b) ? 1.0f : 0.0f;
                }
            }
            // first block of W' -> LDS buffer 0
            {
                const int row4 = g.daug8 >> 2;
                for (int e = tid; e < WB * row4; e += MF_THREADS) {
                    const int r = e / row4, c4 = e - r * row4;
                    *reinterpret_cast<float4 *>(&Ws[r * g.DP + 4 * c4]) =
                        reinterpret_cast<const float4 *>(waug + (size_t)r * g.daug8)[c4];
                }
            }
            Top3 top;
            top.v1 = top.v2 = top.v3 = -INFINITY;
            top.i1 = top.i2 = 0;

            for (int cb = 0; cb < g.nblocks; ++cb) {
                __syncthreads();                        // Ws[cb & 1] (and Xs) complete; Ws[(cb+1) & 1] free
                const float *Wc = Ws + (cb & 1) * WB * g.DP;
                float *Wn = Ws + ((cb + 1) & 1) * WB * g.DP;
                // next block: global -> registers now, -> LDS after the matrix work (at most 3 float4 per thread
                // per pass of the loop below keeps the register need small)
                const bool more = cb + 1 < g.nblocks;
                const float *wsrc = waug + (size_t)(cb + 1) * WB * g.daug8;
                const int row4 = g.daug8 >> 2, nvec = WB * row4;

                floatx16 acc0, acc1;
#pragma unroll
                for (int r = 0; r < 16; ++r) { acc0[r] = 0.0f; acc1[r] = 0.0f; }
                const float *xrow = Xs + (wave * 32 + l32) * g.DP + 4 * half;
                const float *w0row = Wc + l32 * g.DP + 4 * half;
                const float *w1row = Wc + (32 + l32) * g.DP + 4 * half;
                int e_next = tid;
                for (int ch = 0; ch < g.daug8; ch += 8) {
                    const float4 xv = *reinterpret_cast<const float4 *>(xrow + ch);
                    const float4 a0 = *reinterpret_cast<const float4 *>(w0row + ch);
                    const float4 a1 = *reinterpret_cast<const float4 *>(w1row + ch);
                    // one vector of the next block per chunk, spread over the matrix work
                    float4 nv = make_float4(0.f, 0.f, 0.f, 0.f);
                    const bool ld = more && e_next < nvec;
                    int nr = 0, nc4 = 0;
                    if (ld) {
                        nr = e_next / row4; nc4 = e_next - nr * row4;
                        nv = reinterpret_cast<const float4 *>(wsrc + (size_t)nr * g.daug8)[nc4];
                    }
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, xv.x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, xv.x, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, xv.y, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, xv.y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, xv.z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, xv.z, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, xv.w, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, xv.w, acc1, 0, 0, 0);
                    if (ld) {
                        *reinterpret_cast<float4 *>(&Wn[nr * g.DP + 4 * nc4]) = nv;
                        e_next += MF_THREADS;
                    }
                }
                // rest of the next block (when it has more vectors than there were chunks)
                if (more) {
                    for (; e_next < nvec; e_next += MF_THREADS) {
                        const int nr = e_next / row4, nc4 = e_next - nr * row4;
                        *reinterpret_cast<float4 *>(&Wn[nr * g.DP + 4 * nc4]) =
                            reinterpret_cast<const float4 *>(wsrc + (size_t)nr * g.daug8)[nc4];
                    }
                }
                // running arg-max of this lane's sample over the 32 centroid rows it sees in this block:
                // row of register r in a 32x32 tile is 8*(r/4) + 4*half + r%4, visited in increasing order
                const int cbase = cb * WB + 4 * half;
#pragma unroll
                for (int r = 0; r < 16; ++r) top3_insert(top, acc0[r], cbase + 8 * (r >> 2) + (r & 3));
#pragma unroll
                for (int r = 0; r < 16; ++r) top3_insert(top, acc1[r], cbase + 32 + 8 * (r >> 2) + (r & 3));
            }
            // merge the two half-waves (same sample, other centroid rows)
            {
                const float pv1 = __shfl_xor(top.v1, 32, 64), pv2 = __shfl_xor(top.v2, 32, 64), pv3 = __shfl_xor(top.v3, 32, 64);
                const int pi1 = __shfl_xor(top.i1, 32, 64), pi2 = __shfl_xor(top.i2, 32, 64);
                top3_insert(top, pv1, pi1);
                top3_insert(top, pv2, pi2);
                top.v3 = fmaxf(top.v3, pv3);
            }
            const int n = tile0 + wave * 32 + l32;       // this lane pair's sample
            const bool mine = half == 0 && n < b;
            int arg = top.i1;
            const bool close2 = mine && !(top.v1 - top.v2 > thr);
            // exact decisions, one flagged sample at a time, the whole wave working on it
            unsigned long long fm = __ballot(close2);
            while (fm) {
                const int L = __builtin_ctzll(fm);
                fm &= fm - 1;
                const int ca = __builtin_amdgcn_readlane(top.i1, L), cb2 = __builtin_amdgcn_readlane(top.i2, L);
                const float v1L = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(top.v1), L));
                const float v3L = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(top.v3), L));
                const float *xl = Xs + (wave * 32 + L) * g.DP;       // the sample (L < 32)
                int res;
                if (v1L - v3L > thr) {
                    // two candidates: |x - w_a|^2 - |x - w_b|^2 = sum_j (w_aj - w_bj)(w_aj + w_bj - 2 x_j), in fp64
                    double dd = 0.0;
                    for (int j = lane; j < d; j += 64) {
                        const double wa = (double)wst[(size_t)ca * d + j], wb = (double)wst[(size_t)cb2 * d + j];
                        dd += (wa - wb) * ((wa + wb) - 2.0 * (double)xl[j]);
                    }
                    dd = wave_sum_d(dd);
                    const int lo = ca < cb2 ? ca : cb2;
                    res = dd < 0.0 ? ca : (dd > 0.0 ? cb2 : lo);
                } else {
                    // all k distances in fp64, direct form; lane l takes centroids l, l+64, ...
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
                    res = barg;
                }
                if (lane == L) arg = res;
                rechecks += (lane == 0);
            }
            if (mine) {
                idx[n] = (unsigned short)arg;
                if (p.dump) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;
            }
        }
        __syncthreads();

        // ================= phase 2: gradient, merge, update =================
        const bool merge_point = (p.E > 0 && p.W > 1 && t > 0 && (t % p.E) == 0);
        const long long r_now = p.E > 0 ? t / p.E : 0;
        const int rpar = det ? (int)((r_now - 1) & 1) : 0;
        if (tid == 0) {
            int has = 0;
            if (merge_point) {
                const int st = p.stamp[(size_t)rpar * p.W + i];
                has = det ? (st == (int)(r_now - 1)) : (st >= 0);
                p.stamp[(size_t)rpar * p.W + i] = -1;
            }
            s_has_ext = has;
        }
        __syncthreads();
        const bool has_ext = s_has_ext != 0;
        const float *ext = p.slot + ((size_t)rpar * p.W + i) * kd;

        // pass A: per centroid, sums of the assigned samples in sample order -> gradient; Parzen sums
        double lhs = 0.0, rhs = 0.0, nrm = 0.0;
        for (int c = wave; c < k; c += MF_WAVES) {
            float S[NJ];
#pragma unroll
            for (int q = 0; q < NJ; ++q) S[q] = 0.0f;
            int cnt = 0;
            for (int n0 = 0; n0 < b; n0 += 64) {
                const int nn = n0 + lane;
                unsigned long long m = __ballot(nn < b && (int)idx[nn < b ? nn : 0] == c);
                while (m) {
                    int ns[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (m) { ns[q] = n0 + __builtin_ctzll(m); m &= m - 1; ++cnt; }
                        else ns[q] = -1;
                    }
                    float v[4][NJ];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
#pragma unroll
                        for (int jq = 0; jq < NJ; ++jq) {
                            const int j = lane + 64 * jq;
                            v[q][jq] = (ns[q] >= 0 && j < d) ? xb[(size_t)ns[q] * d + j] : 0.0f;
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
#pragma unroll
                        for (int jq = 0; jq < NJ; ++jq) S[jq] += v[q][jq];
                    }
                }
            }
#pragma unroll
            for (int jq = 0; jq < NJ; ++jq) {
                const int j = lane + 64 * jq;
                if (j < d) {
                    const size_t e = (size_t)c * d + j;
                    const float w = wst[e];
                    const float gq = ((float)cnt * w - S[jq]) / (float)b;      // descent gradient of Eq. 9
                    gsc[e] = gq;
                    if (has_ext) {
                        const double we = (double)ext[e];
                        const double a = ((double)w - (double)p.eps * (double)gq) - we;
                        const double c2 = (double)w - we;
                        lhs += a * a; rhs += c2 * c2; nrm += we * we;
                    }
                }
            }
        }
        int delta = 0;
        if (has_ext) {       // uniform over the workgroup
            lhs = wave_sum_d(lhs); rhs = wave_sum_d(rhs); nrm = wave_sum_d(nrm);
            if (lane == 0) { red_d[0][wave] = lhs; red_d[1][wave] = rhs; red_d[2][wave] = nrm; }
            __syncthreads();
            lhs = ((red_d[0][0] + red_d[0][1]) + red_d[0][2]) + red_d[0][3];
            rhs = ((red_d[1][0] + red_d[1][1]) + red_d[1][2]) + red_d[1][3];
            nrm = ((red_d[2][0] + red_d[2][1]) + red_d[2][2]) + red_d[2][3];
            if (nrm > 0.0) {                          // lambda of Eq. 3
                delta = p.parzen ? (lhs < rhs) : 1;   // Eq. 4
                if (tid == 0) {
                    long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                    cn[CNT_RECEIVED] += 1;
                    cn[CNT_ACCEPTED] += delta;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                }
            }
        }
        // pass B: Eq. 7, Alg. 5 line 8; refresh the augmented copy and max |w_c|^2
        wn2max = 0.0f;
        for (int c = wave; c < k; c += MF_WAVES) {
            float s = 0.0f;
#pragma unroll
            for (int jq = 0; jq < NJ; ++jq) {
                const int j = lane + 64 * jq;
                if (j < d) {
                    const size_t e = (size_t)c * d + j;
                    const float w = wst[e];
                    float step = gsc[e];
                    if (delta) step += w - 0.5f * (w + ext[e]);
                    const float wn = w - p.eps * step;
                    wst[e] = wn;
                    waug[(size_t)c * g.daug8 + j] = wn;
                    s = fmaf(wn, wn, s);
                }
            }
            s = wave_sum_f(s);
            if (lane == 0) waug[(size_t)c * g.daug8 + d] = -0.5f * s;
            wn2max = fmaxf(wn2max, s);
        }
        if (lane == 0) red_f[wave] = wn2max;
        __threadfence_block();
        __syncthreads();
        wn2max = fmaxf(fmaxf(red_f[0], red_f[1]), fmaxf(red_f[2], red_f[3]));

        // ---- send (Alg. 5 line 9) ----
        if (p.E > 0 && p.W > 1 && ((t + 1) % p.E) == 0) {
            const long long r = t / p.E;
            if (!message_dropped(p.seed, r, i, p.drop_thr)) {
                const int peer = det ? peer_deterministic(p.seed, r, i, p.W) : peer_free(p.seed, r, i, p.W);
                const int spar = det ? (int)(r & 1) : 0;
                float *dst = p.slot + ((size_t)spar * p.W + peer) * kd;
                for (size_t e = tid; e < kd; e += MF_THREADS) dst[e] = wst[e];
                __threadfence();
                __syncthreads();
                if (tid == 0) p.stamp[(size_t)spar * p.W + peer] = (int)r;
            }
            if (tid == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
        }
        __syncthreads();
    }

    rechecks = (long long)wave_sum_d((double)rechecks);
    if (lane == 0 && rechecks)
        atomicAdd((unsigned long long *)&p.counters[(size_t)i * CNT_STRIDE + CNT_RECHECK], (unsigned long long)rechecks);
}

size_t mfma_lds_bytes(int k, int d, int b)
{
    const MfmaGeom g = mfma_geom(k, d);
    return ((size_t)TM * g.DP + 2 * (size_t)WB * g.DP) * sizeof(float) + ((size_t)b * sizeof(unsigned short) + 15) / 16 * 16;
}

}  // namespace

bool mfma_kernel_supports(int k, int d, int b, const void *x)
{
    if (d % 4 != 0 || d > 128 || k < 2 || k > 65535 || (((uintptr_t)x) & 15u) != 0) return false;
    return mfma_lds_bytes(k, d, b) <= 150 * 1024;
}

size_t mfma_waug_floats(int k, int d, int W)
{
    const MfmaGeom g = mfma_geom(k, d);
    return (size_t)W * g.kpad * g.daug8;
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

hipError_t launch_mfma_steps(const StepParams &p, long long t0, long long t1, float *waug, const float *xnorm2max,
                             hipStream_t s)
{
    const size_t lds = mfma_lds_bytes(p.k, p.d, p.b);
    hipError_t e;
    if (p.d <= 64) {
        e = hipFuncSetAttribute((const void *)mfma_steps_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((mfma_steps_kernel<1>), dim3(p.W), dim3(MF_THREADS), lds, s, p, t0, t1, waug, xnorm2max);
    } else {
        e = hipFuncSetAttribute((const void *)mfma_steps_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((mfma_steps_kernel<2>), dim3(p.W), dim3(MF_THREADS), lds, s, p, t0, t1, waug, xnorm2max);
    }
    return hipGetLastError();
}

}  // namespace asgd
