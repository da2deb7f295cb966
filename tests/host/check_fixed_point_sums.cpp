// Host-only check of the fixed-point gradient sums (csrc/fixed_point_sums.h), built with the plain C++ compiler:
//   - the scale of a column keeps a sum of b terms below 2^30 and (with the cap) a term below 2^22;
//   - the bit pattern added for a term is FX_BIAS + the term rounded to nearest (ties to even), negative terms included;
//   - a cell that wraps around many times still gives back the exact integer sum once count * FX_BIAS is taken off;
//   - the sum does not depend on the order of the additions;
//   - the value the row passes form, sum / scale, is within b * 0.5 / scale of the fp64 sum of the samples.
#include <cinttypes>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "fixed_point_sums.h"

using namespace asgd;

#define REQUIRE(c, ...) do { if (!(c)) { printf("FAIL line %d: ", __LINE__); printf(__VA_ARGS__); printf("\n"); return 1; } } while (0)

int main(int argc, char **argv)
{
    const int b = argc > 1 ? atoi(argv[1]) : 2000;
    const double xmax_d = argc > 2 ? atof(argv[2]) : 13.7;
    const unsigned seed = argc > 3 ? (unsigned)atoi(argv[3]) : 1u;
    const float xmax = (float)xmax_d;
    std::mt19937_64 rng(seed);
    std::uniform_real_distribution<double> uni(-xmax_d, xmax_d);

    int e = 0;
    REQUIRE(fx_scale_exponent(b, xmax, true, &e), "no scale for b = %d, xmax = %g", b, xmax_d);
    const float scale = ldexpf(1.0f, e), inv = ldexpf(1.0f, -e);
    REQUIRE((double)b * xmax_d * scale < 1073741824.0, "sum bound: b xmax scale = %g", (double)b * xmax_d * scale);
    REQUIRE(xmax_d * scale < 4194304.0, "term bound: xmax scale = %g", xmax_d * scale);
    int e_nocap = 0;
    REQUIRE(fx_scale_exponent(b, xmax, false, &e_nocap) && e <= e_nocap, "cap raises the exponent");
    if (b >= 256) REQUIRE(e == e_nocap, "cap active for b = %d", b);
    REQUIRE(e_nocap == 96 || (double)b * xmax_d * ldexp(1.0, e_nocap) >= 536870912.0, "scale not the largest power of two");
    int dummy = 0;
    REQUIRE(!fx_scale_exponent(b, 0.0f, true, &dummy) && !fx_scale_exponent(b, INFINITY, true, &dummy), "zero / infinite column");

    // single terms: bit pattern = bias + round to nearest even, at the extremes and at ties
    const float probes[] = {0.0f, xmax, -xmax, 0.5f * inv, -0.5f * inv, 1.5f * inv, 2.5f * inv, -2.5f * inv, 0.49999f * inv,
                            1.0f * inv, -1.0f * inv, 0.75f * xmax, -0.3f * xmax};
    for (float x : probes) {
        const uint32_t bits = fx_term_bits(x, scale);
        const long long want = llrint((double)x * (double)scale);       // round to nearest even (default mode)
        REQUIRE((int32_t)(bits - FX_BIAS) == (int32_t)want, "term %g: got %d, want %lld", x, (int32_t)(bits - FX_BIAS), want);
    }

    // sums of b random terms, many trials: exact integer sum after unbiasing, any order, close to the fp64 sum
    std::vector<float> xs((size_t)b);
    for (int trial = 0; trial < 200; ++trial) {
        const int n = trial == 0 ? b : 1 + (int)(rng() % (uint64_t)b);
        long long exact = 0;
        double real = 0.0;
        for (int i = 0; i < n; ++i) {
            double v = uni(rng);
            if (trial % 3 == 1) v = -fabs(v);                  // one-sided sums reach the bounds
            if (trial % 3 == 2) v = (i & 1) ? xmax_d : -xmax_d;
            xs[(size_t)i] = (float)v;
            exact += llrint((double)xs[(size_t)i] * (double)scale);
            real += (double)xs[(size_t)i];
        }
        uint32_t fwd = 0, bwd = 0;
        for (int i = 0; i < n; ++i) fwd += fx_term_bits(xs[(size_t)i], scale);
        for (int i = n - 1; i >= 0; --i) bwd += fx_term_bits(xs[(size_t)i], scale);
        REQUIRE(fwd == bwd, "order dependence in trial %d", trial);
        const int32_t got = fx_unbias(fwd, (uint32_t)n);
        REQUIRE((long long)got == exact, "trial %d (n = %d): got %d, exact %lld", trial, n, got, exact);
        const double back = (double)((float)got * inv);
        REQUIRE(fabs(back - real) <= (double)n * 0.5 * (double)inv + fabs(real) * 6.0e-8 + 1e-30,
                "trial %d: %g against %g (bound %g)", trial, back, real, (double)n * 0.5 * (double)inv);
    }
    printf("ok %d\n", e);
    return 0;
}
