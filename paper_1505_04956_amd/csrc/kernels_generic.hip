// Shape-agnostic kernels: worker initialisation, the generic step kernel (any k, d, b),
// the quantization error (Eq. 8) and the mean of the worker states (Sec. 4.3).
//
// The generic step kernel is the reference implementation inside the library: one
// workgroup of 256 threads per worker, direct-form fp32 distances, and a gradient-sum
// pass in which every centroid row is owned by exactly one wavefront, so that all sums are
// formed in a fixed order and a run is reproducible bit for bit.
#include "asgd_internal.h"

namespace asgd {

namespace {

constexpr int GEN_THREADS = 256;
constexpr int GEN_WAVES = GEN_THREADS / 64;
constexpr int GEN_ASG_LDS = 4096;   // assignments of a mini-batch stay in LDS up to this b

// s_i(w) in fp64, direct form, lowest index on ties (Sec. 5.1, text after Eq. 8).
__device__ int exact_nearest(const float *__restrict__ x, const float *w, int k, int d)
{
    int arg = 0;
    double best = INFINITY;
    for (int c = 0; c < k; ++c) {
        double s = 0.0;
        for (int j = 0; j < d; ++j) {
            double diff = (double)x[j] - (double)w[(size_t)c * d + j];
            s += diff * diff;
        }
        if (s < best) { best = s; arg = c; }
    }
    return arg;
}

// Deterministic block-wide sum of three doubles (fixed tree).
__device__ void block_sum3(double &a, double &b, double &c, double (*red)[GEN_THREADS])
{
    const int tid = threadIdx.x;
    red[0][tid] = a; red[1][tid] = b; red[2][tid] = c;
    __syncthreads();
    for (int off = GEN_THREADS / 2; off > 0; off >>= 1) {
        if (tid < off) {
            red[0][tid] += red[0][tid + off];
            red[1][tid] += red[1][tid + off];
            red[2][tid] += red[2][tid + off];
        }
        __syncthreads();
    }
    a = red[0][0]; b = red[1][0]; c = red[2][0];
    __syncthreads();
}

// Sum of a double over the 64 lanes of a wave, same value and same order in every lane.
__device__ __forceinline__ double gen_wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ void init_first_k_kernel(StepParams p)
{
    // Worker i starts from the first k rows of its own shard.
    const size_t kd = (size_t)p.k * p.d;
    const int i = blockIdx.x;
    for (size_t e = threadIdx.x; e < kd; e += blockDim.x)
        p.w[i * kd + e] = p.x[(size_t)i * p.H * p.d + e];
}

__global__ void absmax_partial_kernel(const float *__restrict__ x, long long n, int d, float *partial)
{
    // partial[block][j] = max |x[row][j]| over the elements this block visits.  The flat array
    // is walked with a stride that is a multiple of d, so a thread always sees one dimension.
    extern __shared__ float sm[];
    const long long total = n * d;
    const long long threads = (long long)gridDim.x * blockDim.x;
    const long long stride = threads / d * d;          // host guarantees threads >= d
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    for (int j = threadIdx.x; j < d; j += blockDim.x) sm[j] = 0.0f;
    __syncthreads();
    if (g < stride) {
        float m = 0.0f;
        long long e = g;
        for (; e + 7 * stride < total; e += 8 * stride) {      // eight independent loads in flight per thread
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = x[e + q * stride];
#pragma unroll
            for (int q = 0; q < 8; ++q) m = fmaxf(m, fabsf(v[q]));
        }
        for (; e < total; e += stride) m = fmaxf(m, fabsf(x[e]));
        // max is order independent; |x| >= 0, so the integer order of the bit patterns is the
        // floating-point order and an integer atomic is exact
        atomicMax((unsigned int *)&sm[g % d], __float_as_uint(m));
    }
    __syncthreads();
    for (int j = threadIdx.x; j < d; j += blockDim.x) partial[(size_t)blockIdx.x * d + j] = sm[j];
}

__global__ void absmax_final_kernel(const float *partial, int nblocks, int d, float *out)
{
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < d; j += gridDim.x * blockDim.x) {
        float m = 0.0f;
        for (int bidx = 0; bidx < nblocks; ++bidx) m = fmaxf(m, partial[(size_t)bidx * d + j]);
        out[j] = m;
    }
}

// ------------------------------------------------------------------------------------------
// Generic step kernel: steps [t0, t1) of worker blockIdx.x.
//   w_in_lds   state kept in LDS for the duration of the launch (else in global memory)
//   acc_in_lds gradient sums and counts kept in LDS (else in the global scratch)
// In deterministic mode the host splits runs at multiples of E, so that a message read here
// was written by an earlier launch.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(GEN_THREADS) void generic_steps_kernel(StepParams p, long long t0, long long t1,
                                                                     int w_in_lds, int acc_in_lds)
{
    extern __shared__ float smem[];
    __shared__ double red[3][GEN_THREADS];
    __shared__ int s_has_ext;
    __shared__ int s_ext_round[MAX_BUFFERS];   // round of the message in buffer n (free-running mode: any earlier one)
    __shared__ int s_rowflags[3];          // partial messages: buffers with a non-empty row, with an accepted row, near-ties
    __shared__ long long s_recheck;
    __shared__ int s_asg[GEN_ASG_LDS];

    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int k = p.k, d = p.d, b = p.b;
    const size_t kd = (size_t)k * d;

    float *wp = w_in_lds ? smem : p.w + (size_t)i * kd;
    float *sp = acc_in_lds ? smem + (w_in_lds ? kd : 0) : p.acc + (size_t)i * kd;
    int *cntp = acc_in_lds ? (int *)(smem + (w_in_lds ? 2 * kd : kd)) : p.cnt + (size_t)i * k;
    int *asg = b <= GEN_ASG_LDS ? s_asg : p.assign_tmp + (size_t)i * b;

    if (w_in_lds) {
        for (size_t e = tid; e < kd; e += GEN_THREADS) wp[e] = p.w[(size_t)i * kd + e];
    }
    if (tid == 0) s_recheck = 0;
    __syncthreads();

    long long my_recheck = 0;
    const float redecide = fmaxf(1e-5f, 4.0f * (float)(d + 2) * 5.9604645e-8f);
    for (long long t = t0; t < t1; ++t) {
        const long long s = t % p.S;
        const float *xb = p.x + ((size_t)i * p.H + (size_t)s * b) * d;   // this step's mini-batch

        for (size_t e = tid; e < kd; e += GEN_THREADS) sp[e] = 0.0f;
        for (int c = tid; c < k; c += GEN_THREADS) cntp[c] = 0;

        // ---- assignment under the state the step started with (Alg. 4, gradient step) ----
        for (int n = tid; n < b; n += GEN_THREADS) {
            const float *xr = xb + (size_t)n * d;
            float best = INFINITY, second = INFINITY;
            int arg = 0;
            for (int c = 0; c < k; ++c) {
                const float *wc = wp + (size_t)c * d;
                float acc = 0.0f;
                for (int j = 0; j < d; ++j) {
                    float diff = xr[j] - wc[j];
                    acc = fmaf(diff, diff, acc);
                }
                if (acc < best) { second = best; best = acc; arg = c; }
                else if (acc < second) { second = acc; }
            }
            // A direct-form distance in fp32 (one rounding per difference, one per fused multiply-add, all terms
            // non-negative) is off by at most (d + 2) * 2^-24 of its value, the difference of two of them by at most
            // 2 (d + 2) 2^-24 of the larger one.  Closer than twice that (and never less than 1e-5): decide in fp64.
            if (!(second - best > redecide * second)) {
                arg = exact_nearest(xr, wp, k, d);
                my_recheck += 1;
            }
            asg[n] = arg;
            if (p.dump) p.dump[((size_t)(t - p.t_dump0) * p.W + i) * b + n] = arg;
        }
        __syncthreads();

        // ---- gradient sums (Eq. 9): wave v owns the centroids c with c % GEN_WAVES == v and
        //      visits the samples in order, so every sum has one fixed order ----
        for (int n = 0; n < b; ++n) {
            const int a = asg[n];
            if ((a % GEN_WAVES) == wave) {
                const float *xr = xb + (size_t)n * d;
                float *sr = sp + (size_t)a * d;
                for (int j = lane; j < d; j += 64) sr[j] += xr[j];
                if (lane == 0) cntp[a] += 1;
            }
        }
        __syncthreads();

        if (p.lr_mode == ASGD_LR_INV_COUNT) {
            // per-centroid 1/count step: w_k becomes the mean of everything ever assigned to k
            long long *nc = p.ncum + (size_t)i * k;
            for (int c = tid; c < k; c += GEN_THREADS) nc[c] += cntp[c];
            __syncthreads();
            for (size_t e = tid; e < kd; e += GEN_THREADS) {
                const int c = (int)(e / d);
                const int cc = cntp[c];
                if (cc > 0) wp[e] = wp[e] + (sp[e] - (float)cc * wp[e]) / (float)nc[c];
            }
            __syncthreads();
            continue;
        }

        // ---- merge point? (a buffer is looked at once, at the first step of a round) ----
        const bool merge_point = (p.E > 0 && t > 0 && (t % p.E) == 0);
        const long long r_now = p.E > 0 ? t / p.E : 0;
        const int det = (p.mode == ASGD_MODE_DETERMINISTIC);
        const int rpar = det ? (int)((r_now - 1) & 1) : 0;
        if (tid == 0) {
            int has = 0;                       // bit n: buffer n holds a message for this merge point
            for (int n = 0; merge_point && n < p.nb; ++n) {
                int *stp = p.stamp + exchange_buffer(rpar, p.nb, n, p.W, i);
                const int st = *stp;
                if (det ? (st == (int)(r_now - 1)) : (st >= 0)) has |= 1 << n;
                s_ext_round[n] = st;
                *stp = -1;
            }
            s_has_ext = has;
        }
        __syncthreads();
        const int has_mask = s_has_ext;        // uniform over the block
        const float *ext[MAX_BUFFERS];
        for (int n = 0; n < MAX_BUFFERS; ++n) ext[n] = p.slot + exchange_buffer(rpar, p.nb, n < p.nb ? n : 0, p.W, i) * kd;
        // descent gradient of Eq. 9, G = (c_k * w_k - S_k) / b, stored over the sums
        for (size_t e = tid; e < kd; e += GEN_THREADS) {
            const int c = (int)(e / d);
            sp[e] = ((float)cntp[c] * wp[e] - sp[e]) / (float)b;
        }
        if (p.parts > 1) {
            // Partial messages (Sec. 4.4): copy n for this worker carries the centroid rows c with
            // c mod P = (round + worker + n) mod P; lambda, Eq. 4 and Eq. 6 row by row.  A wave takes a row
            // through gate and update in one pass (no sum over the whole state is needed).
            if (tid < 3) s_rowflags[tid] = 0;
            __syncthreads();
            int nz = 0, acc = 0, near = 0;
            for (int c = wave; c < k; c += GEN_THREADS / 64) {
                int rowmask = 0;
                for (int n = 0; n < p.nb; ++n) {
                    if (!(has_mask >> n & 1) || !row_travels(c, s_ext_round[n], i, n, p.parts)) continue;
                    double lhs = 0.0, rhs = 0.0, nrm = 0.0;
                    for (int j = lane; j < d; j += 64) {
                        const size_t e = (size_t)c * d + j;
                        const double we = (double)ext[n][e];
                        const double a = ((double)wp[e] - (double)p.eps * (double)sp[e]) - we;
                        const double c2 = (double)wp[e] - we;
                        lhs += a * a; rhs += c2 * c2; nrm += we * we;
                    }
                    lhs = gen_wave_sum(lhs); rhs = gen_wave_sum(rhs); nrm = gen_wave_sum(nrm);
                    if (!(nrm > 0.0)) continue;
                    nz |= 1 << n;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) near = 1;
                    if (p.parzen ? (lhs < rhs) : 1) rowmask |= 1 << n;
                }
                acc |= rowmask;
                const float inv = 1.0f / (float)(__builtin_popcount(rowmask) + 1);
                for (int j = lane; j < d; j += 64) {
                    const size_t e = (size_t)c * d + j;
                    float step = sp[e];
                    if (rowmask) {
                        float sum = wp[e];
                        for (int n = 0; n < p.nb; ++n)
                            if (rowmask >> n & 1) sum += ext[n][e];
                        step += wp[e] - inv * sum;
                    }
                    wp[e] = wp[e] - p.eps * step;
                }
            }
            if (lane == 0) {
                if (nz) atomicOr(&s_rowflags[0], nz);
                if (acc) atomicOr(&s_rowflags[1], acc);
                if (near) atomicOr(&s_rowflags[2], near);
            }
            __syncthreads();
            if (tid == 0) {
                long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                cn[CNT_RECEIVED] += __builtin_popcount(s_rowflags[0]);
                cn[CNT_ACCEPTED] += __builtin_popcount(s_rowflags[1]);
                cn[CNT_PARZEN_NEAR] += s_rowflags[2];
            }
        }
        int delta_mask = 0, ndelta = 0;
        for (int n = 0; n < p.nb && p.parts == 1; ++n) {
            if (!(has_mask >> n & 1)) continue;
            double lhs = 0.0, rhs = 0.0, nrm = 0.0;
            for (size_t e = tid; e < kd; e += GEN_THREADS) {
                const double we = (double)ext[n][e];
                const double a = ((double)wp[e] - (double)p.eps * (double)sp[e]) - we;
                const double c2 = (double)wp[e] - we;
                lhs += a * a; rhs += c2 * c2; nrm += we * we;
            }
            block_sum3(lhs, rhs, nrm, red);
            if (nrm > 0.0) {                      // lambda of Eq. 3: an all-zero buffer is empty
                const int delta = p.parzen ? (lhs < rhs) : 1;   // Eq. 4, every buffer on its own (Eq. 6)
                delta_mask |= delta << n;
                ndelta += delta;
                if (tid == 0) {
                    long long *cn = p.counters + (size_t)i * CNT_STRIDE;
                    cn[CNT_RECEIVED] += 1;
                    cn[CNT_ACCEPTED] += delta;
                    if (rhs > 0.0 && fabs(lhs - rhs) / rhs < 1e-6) cn[CNT_PARZEN_NEAR] += 1;
                }
            }
        }
        // Eq. 6 (one buffer: Eq. 7) and Alg. 5, update
        const float inv = 1.0f / (float)(ndelta + 1);
        for (size_t e = tid; p.parts == 1 && e < kd; e += GEN_THREADS) {
            float step = sp[e];
            if (ndelta) {
                float sum = wp[e];
                for (int n = 0; n < p.nb; ++n)
                    if (delta_mask >> n & 1) sum += ext[n][e];
                step += wp[e] - inv * sum;
            }
            wp[e] = wp[e] - p.eps * step;
        }
        __syncthreads();

        // ---- send (Alg. 5, send) ----
        if (p.E > 0 && p.W > 1 && ((t + 1) % p.E) == 0) {
            const long long r = t / p.E;
            for (int n = 0; n < p.nb; ++n) {
                if (message_dropped(p.seed, r, i, p.drop_thr, n)) continue;
                const int peer = det ? peer_deterministic(p.seed, r, i, p.W, n) : peer_free(p.seed, r, i, p.W, n);
                const int spar = det ? (int)(r & 1) : 0;
                float *dst = p.slot + exchange_buffer(spar, p.nb, n, p.W, peer) * kd;
                const int part = message_part(r, peer, n, p.parts);         // only the rows of this part travel
                for (size_t e = tid; e < kd; e += GEN_THREADS)
                    if (p.parts == 1 || (int)(e / d) % p.parts == part) dst[e] = wp[e];
                __threadfence();
                __syncthreads();
                if (tid == 0) p.stamp[exchange_buffer(spar, p.nb, n, p.W, peer)] = (int)r;
            }
            if (tid == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_SENT] += 1;
        }
        __syncthreads();
    }

    if (my_recheck) atomicAdd((unsigned long long *)&s_recheck, (unsigned long long)my_recheck);
    __syncthreads();
    if (tid == 0) p.counters[(size_t)i * CNT_STRIDE + CNT_RECHECK] += s_recheck;
    if (w_in_lds) {
        for (size_t e = tid; e < kd; e += GEN_THREADS) p.w[(size_t)i * kd + e] = wp[e];
    }
}

// ------------------------------------------------------------------------------------------
// Eq. 8.  Thread per sample, grid-stride; fp32 direct-form distances, fp64 sums.
// ------------------------------------------------------------------------------------------
constexpr int QE_THREADS = 256;
constexpr int QE_BLOCKS = 2048;

__global__ __launch_bounds__(QE_THREADS) void quant_error_kernel(const float *__restrict__ x, long long N, int d, int k,
                                                                  const float *__restrict__ w, int w_in_lds,
                                                                  double *partials)
{
    extern __shared__ float smem[];
    __shared__ double red[QE_THREADS];
    const size_t kd = (size_t)k * d;
    const float *wp = w;
    if (w_in_lds) {
        for (size_t e = threadIdx.x; e < kd; e += QE_THREADS) smem[e] = w[e];
        __syncthreads();
        wp = smem;
    }
    double sum = 0.0;
    for (long long n = (long long)blockIdx.x * QE_THREADS + threadIdx.x; n < N; n += (long long)gridDim.x * QE_THREADS) {
        const float *xr = x + (size_t)n * d;
        float best = INFINITY;
        for (int c = 0; c < k; ++c) {
            const float *wc = wp + (size_t)c * d;
            float acc = 0.0f;
            for (int j = 0; j < d; ++j) {
                float diff = xr[j] - wc[j];
                acc = fmaf(diff, diff, acc);
            }
            best = fminf(best, acc);
        }
        sum += 0.5 * (double)best;
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int off = QE_THREADS / 2; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0];
}

__global__ void quant_error_final_kernel(const double *partials, int n, double *out)
{
    // One wave, fixed order: lane l adds the partials l, l + 64, ... in that order, then the 64 sums are added in lane
    // order.  The result does not depend on scheduling.
    __shared__ double red[64];
    double s = 0.0;
    for (int q = threadIdx.x; q < n; q += 64) s += partials[q];
    red[threadIdx.x] = s;
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double t = 0.0;
        for (int l = 0; l < 64; ++l) t += red[l];
        *out = t;
    }
}

__global__ void mean_state_kernel(const float *w, int W, int kd, float *out)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= kd) return;
    double s = 0.0;
    for (int i = 0; i < W; ++i) s += (double)w[(size_t)i * kd + e];
    out[e] = (float)(s / (double)W);
}

}  // namespace

// ------------------------------------------------------------------------------------------
hipError_t launch_init_first_k(const StepParams &p, hipStream_t s)
{
    hipLaunchKernelGGL(init_first_k_kernel, dim3(p.W), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_absmax(const float *x, long long rows, int d, float *out, hipStream_t s)
{
    // out: d floats; uses a temporary of nblocks*d floats that is freed before returning
    const int nblocks = 1024;
    float *partial = nullptr;
    hipError_t e = hipMalloc((void **)&partial, (size_t)nblocks * d * sizeof(float));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(absmax_partial_kernel, dim3(nblocks), dim3(256), (size_t)d * sizeof(float), s, x, rows, d, partial);
    hipLaunchKernelGGL(absmax_final_kernel, dim3(1), dim3(256), 0, s, partial, nblocks, d, out);
    e = hipGetLastError();
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(partial);
    return e != hipSuccess ? e : e2;
}

hipError_t launch_generic_steps(const StepParams &p, long long t0, long long t1, hipStream_t s)
{
    const size_t kd = (size_t)p.k * p.d;
    const size_t budget = 40 * 1024;                    // dynamic LDS next to the static arrays
    const int w_in_lds = kd * sizeof(float) <= budget;
    const size_t wbytes = w_in_lds ? kd * sizeof(float) : 0;
    const int acc_in_lds = wbytes + kd * sizeof(float) + (size_t)p.k * sizeof(int) <= budget;
    const size_t lds = wbytes + (acc_in_lds ? kd * sizeof(float) + (size_t)p.k * sizeof(int) : 0);
    hipLaunchKernelGGL(generic_steps_kernel, dim3(p.W), dim3(GEN_THREADS), lds, s, p, t0, t1, w_in_lds, acc_in_lds);
    return hipGetLastError();
}

int quant_partials_count() { return QE_BLOCKS; }

hipError_t launch_quant_error(const float *x, long long N, int d, int k, const float *w, double *partials, double *out,
                              hipStream_t s)
{
    const size_t kd = (size_t)k * d;
    int nparts = QE_BLOCKS;
    hipError_t e = hipSuccess;
    if (small_kernel_supports(k, d, 1)) {
        e = launch_quant_error_small(x, N, d, k, w, partials, nparts, s);           // streaming shape: HBM bound
    } else if (mfma_quant_error_supports(k, d, x)) {
        nparts = 256;                                                           // one workgroup per CU
        e = launch_quant_error_mfma(x, N, d, k, w, partials, nparts, s);       // contraction shape: matrix cores
    } else {
        const int w_in_lds = kd * sizeof(float) <= 60 * 1024;
        hipLaunchKernelGGL(quant_error_kernel, dim3(QE_BLOCKS), dim3(QE_THREADS), w_in_lds ? kd * sizeof(float) : 0, s, x,
                           N, d, k, w, w_in_lds, partials);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(quant_error_final_kernel, dim3(1), dim3(64), 0, s, partials, nparts, out);
    return hipGetLastError();
}

__global__ void schedule_table_kernel(uint64_t seed, long long r0, int n, int W, int *shift_tab)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n) shift_tab[q] = (int)(1 + round_hash(seed, r0 + q) % (uint64_t)(W - 1));
}

hipError_t launch_schedule_table(uint64_t seed, long long r0, int n, int W, int *shift_tab, hipStream_t s)
{
    hipLaunchKernelGGL(schedule_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, seed, r0, n, W, shift_tab);
    return hipGetLastError();
}

hipError_t launch_mean_state(const float *w, int W, int kd, float *out, hipStream_t s)
{
    hipLaunchKernelGGL(mean_state_kernel, dim3((kd + 255) / 256), dim3(256), 0, s, w, W, kd, out);
    return hipGetLastError();
}

}  // namespace asgd
