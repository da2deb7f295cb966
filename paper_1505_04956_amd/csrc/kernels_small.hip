// Small-state step kernel: the shapes it is built for, the host side of its message format, and the dispatch to the
// per-shape translation units (small_shape_KxD.hip, each an instantiation of the templates in small_steps.h).
#include <string.h>

#include "asgd_internal.h"

namespace asgd {

// k x d shapes with a build of the kernel; the first is the streaming workload's own
#define ASGD_SMALL_SHAPES(X) X(10, 10) X(4, 4) X(8, 8) X(8, 16) X(16, 8) X(16, 12)

#define DECLARE_SHAPE(K, D)                                                                                            \
    hipError_t launch_small_steps_##K##x##D(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent); \
    hipError_t launch_quant_error_small_##K##x##D(const float *x, long long N, const float *w, double *partials, int nblocks, hipStream_t s);
ASGD_SMALL_SHAPES(DECLARE_SHAPE)
#undef DECLARE_SHAPE

bool small_kernel_supports(int k, int d, int b)
{
    (void)b;
#define TEST_SHAPE(K, D) if (k == K && d == D) return true;
    ASGD_SMALL_SHAPES(TEST_SHAPE)
#undef TEST_SHAPE
    return false;
}

size_t small_kernel_message_bytes(int k, int d)
{
    if (!small_kernel_supports(k, d, 1)) return 0;
    return (size_t)k * ((d + 1 + 3) / 4) * 4 * sizeof(unsigned long long);      // k padded rows of (value, stamp) pairs
}

// A message is k padded rows of RW = 4 * NQ pairs: pair c * RW + j holds element j of row c (j < d), zero beyond.
void small_kernel_unpack_message(int k, int d, const void *msg, float *rows, int *row_round)
{
    const unsigned long long *pairs = static_cast<const unsigned long long *>(msg);
    const int rw = 4 * ((d + 1 + 3) / 4);
    for (int c = 0; c < k; ++c) {
        const int st = (int)(pairs[(size_t)c * rw] >> 32);
        bool same = true;
        for (int j = 0; j < rw; ++j) {
            const unsigned long long pr = pairs[(size_t)c * rw + j];
            same = same && (int)(pr >> 32) == st;
            if (j < d) {
                const unsigned bits = (unsigned)(pr & 0xffffffffull);
                memcpy(&rows[(size_t)c * d + j], &bits, sizeof(float));
            }
        }
        row_round[c] = (same && st >= 0) ? st : -1;
    }
}

void small_kernel_pack_message(int k, int d, const float *rows, const int *row_round, void *msg)
{
    unsigned long long *pairs = static_cast<unsigned long long *>(msg);
    const int rw = 4 * ((d + 1 + 3) / 4);
    for (int c = 0; c < k; ++c)
        for (int j = 0; j < rw; ++j) {
            unsigned bits = 0;
            if (j < d) memcpy(&bits, &rows[(size_t)c * d + j], sizeof(float));
            pairs[(size_t)c * rw + j] = row_round[c] < 0 ? ~0ull
                                                         : (((unsigned long long)(unsigned)row_round[c] << 32) | bits);
        }
}

hipError_t launch_small_steps(const StepParams &p, long long t0, long long t1, hipStream_t s, bool persistent)
{
    // (32-bit bookkeeping in the kernel: steps of a launch, steps per epoch, rounds, rows of a shard)
    if (t1 - t0 > 0x7fffffffLL || p.S > 0x7fffffffLL || (p.E > 0 && t1 / p.E > 0x7ffffff0LL) || p.H > 0xffffffffLL)
        return hipErrorInvalidValue;
#define LAUNCH_SHAPE(K, D) if (p.k == K && p.d == D) return launch_small_steps_##K##x##D(p, t0, t1, s, persistent);
    ASGD_SMALL_SHAPES(LAUNCH_SHAPE)
#undef LAUNCH_SHAPE
    return hipErrorInvalidValue;
}

hipError_t launch_quant_error_small(const float *x, long long N, int d, int k, const float *w, double *partials, int nblocks,
                                    hipStream_t s)
{
#define LAUNCH_SHAPE(K, D) if (k == K && d == D) return launch_quant_error_small_##K##x##D(x, N, w, partials, nblocks, s);
    ASGD_SMALL_SHAPES(LAUNCH_SHAPE)
#undef LAUNCH_SHAPE
    return hipErrorInvalidValue;
}

}  // namespace asgd
