// LDS layout of the matrix-core step kernel: what lies where in the dynamic LDS allocation of a workgroup.  The kernel,
// its launcher and a host-only check (tests/host/check_exchange_index.cpp) use it.  Plain C++, no HIP types.
#pragma once

#include <stddef.h>

#include "exchange_index.h"      // ASGD_HD

namespace asgd {

enum { MFMA_WB = 64 };           // centroid rows per block (2 matrix tiles of 32)

// LDS layout, shared by host and device
struct MfmaGeom {
    int kpad;      // k rounded up to a multiple of MFMA_WB
    int nblocks;   // kpad / MFMA_WB
    int kq;        // centroids per owner wave (c % nwv), rounded up
    int ns;        // nwv * kq sort slots: slot(c) = (c % nwv) * kq + c / nwv
    int nr;        // shares of the mini-batch in the counting sort (waves that count and place): a power of two <= nwv
    size_t off_h, off_cstart, off_cursor, off_idx, off_perm, off_flist, off_sums, off_scale, bytes;
};
// sums: 0 = none in LDS, 1 = fixed-point sums and column scales behind the lists (fused sums), 2 = column scales only (the
// fixed-point sums take the place of the resident state once the assignments are done)
ASGD_HD inline MfmaGeom mfma_geom(int k, int b, int nch, bool resident, int nwv, int sums = 0)
{
    MfmaGeom g;
    const int DP = nch * 8 + 4;
    g.kpad = (k + MFMA_WB - 1) / MFMA_WB * MFMA_WB;
    g.nblocks = g.kpad / MFMA_WB;
    g.kq = (k + nwv - 1) / nwv;
    g.ns = nwv * g.kq;
    g.nr = nwv;
    while (g.nr > 1 && (size_t)g.ns * g.nr * sizeof(int) > 32768) g.nr /= 2;     // the counters stay within 32 KB
    size_t o = (size_t)(resident ? g.kpad : 2 * MFMA_WB) * DP * sizeof(float);
    g.off_h = o;            o += (size_t)g.kpad * sizeof(float);
    g.off_cstart = o;       o += ((size_t)g.ns + 4) / 4 * 4 * sizeof(int);
    g.off_cursor = o;       o += ((size_t)g.ns * g.nr + 3) / 4 * 4 * sizeof(int);
    g.off_idx = o;          o += ((size_t)b + 7) / 8 * 8 * sizeof(unsigned short);
    g.off_perm = o;         o += ((size_t)b + 7) / 8 * 8 * sizeof(unsigned short);
    g.off_flist = o;        // resident variant: per-wave lists of samples to re-decide, 32 * ceil(b / (32 nwv)) each
    if (resident) o += (size_t)nwv * 32 * ((b + 32 * nwv - 1) / (32 * nwv)) * sizeof(unsigned short);
    o = (o + 15) / 16 * 16;
    g.off_sums = sums == 2 ? 0 : o;      // k rows of 8 * nch fixed-point sums, then scale and inverse scale per column
    if (sums == 1) o += (size_t)k * nch * 8 * sizeof(int);
    g.off_scale = o;
    if (sums != 0) o += (size_t)2 * nch * 8 * sizeof(float);
    g.bytes = (o + 15) / 16 * 16;
    return g;
}
ASGD_HD inline int mfma_chunks(int d) { return d <= 32 ? 4 : d <= 64 ? 8 : d <= 104 ? 13 : 16; }

}  // namespace asgd
