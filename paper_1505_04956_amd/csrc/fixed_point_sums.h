// Fixed-point gradient sums of the streaming and the matrix-core kernel (Eq. 9: the sum of the samples assigned to a
// centroid), in one place: the kernels and a host-only check (tests/host/check_fixed_point_sums.cpp, plain C++
// compiler) use these.
//
// A column j of the samples gets a power-of-two scale; a term x * scale is rounded to an integer and added to a 32-bit
// cell with an integer atomic.  Integer addition is associative, so the sum does not depend on the order of the
// additions.  The variant that rounds with the magic constant adds the BIT PATTERN of the float (x * scale + 1.5 * 2^23),
// which is FX_BIAS + round(x * scale) as long as |x * scale| < 2^22; the count of the terms times FX_BIAS comes off
// when the cell is read, all modulo 2^32.  Plain C++, no HIP types.
#pragma once

#include <math.h>
#include <stdint.h>
#include <string.h>

#include "exchange_index.h"      // ASGD_HD

namespace asgd {

constexpr uint32_t FX_BIAS = 0x4B400000u;      // bit pattern of 1.5 * 2^23 = 12582912.0f
constexpr float FX_MAGIC = 12582912.0f;

// Exponent e of the scale 2^e of a column whose largest magnitude is xmax, for sums of at most b terms:
// b * xmax * 2^e in [2^29, 2^30) (e at most 96), so that a sum cannot overflow 32 bits; term_cap: also xmax * 2^e < 2^22, so that a
// single term can be rounded inside a float.  valid = false: the column is all zero or not finite (scale 0).
ASGD_HD inline bool fx_scale_exponent(int b, float xmax, bool term_cap, int *e)
{
    const float m = (float)b * xmax;
    if (!(m > 0.0f && m < 1.0e30f)) return false;
    int q = 0;
    (void)frexpf(m, &q);              // m = f * 2^q, f in [0.5, 1)
    int ex = 30 - q;
    if (term_cap) {
        int q1 = 0;
        (void)frexpf(xmax, &q1);
        ex = ex < 22 - q1 ? ex : 22 - q1;
    }
    *e = ex < 96 ? ex : 96;      // (columns of denormal size: the scale itself stays a normal float)
    return true;
}

// what is added to a cell for the value x of a column with the given scale (magic-constant form)
ASGD_HD inline uint32_t fx_term_bits(float x, float scale)
{
    const float t = fmaf(x, scale, FX_MAGIC);
    uint32_t u;
#if defined(__HIP_DEVICE_COMPILE__)
    u = __float_as_uint(t);
#else
    memcpy(&u, &t, sizeof(u));
#endif
    return u;
}

// the integer sum of the rounded terms from the content of a cell that took `count` of them
ASGD_HD inline int32_t fx_unbias(uint32_t cell, uint32_t count) { return (int32_t)(cell - count * FX_BIAS); }

}  // namespace asgd
