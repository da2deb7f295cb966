// Host-only check of every offset the kernels with plain-row messages form in the exchange buffers, for given
// shapes: all rounds of a run, all workers, all copies, both modes' schedules, with and without partial messages.
// Built with the plain C++ compiler against csrc/exchange_index.h (the functions the kernels call); no GPU, no HIP.
// Also the LDS layout of the matrix-core kernel (csrc/mfma_geom.h) for the shape: every region holds what the kernel
// puts there, the regions do not overlap, every slot and counter index the kernel forms lies inside its region.
// usage: check_exchange_index k d W nb parts rounds seed b   -> prints "ok <number of checks>" or the first violation
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "exchange_index.h"
#include "mfma_geom.h"

using namespace asgd;

static long long checks = 0;
#define REQUIRE(cond, ...)                                      \
    do {                                                        \
        ++checks;                                               \
        if (!(cond)) {                                          \
            printf("violation: " __VA_ARGS__);                  \
            printf("\n");                                       \
            return 1;                                           \
        }                                                       \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 9) return 2;
    const int k = atoi(argv[1]), d = atoi(argv[2]), W = atoi(argv[3]), nb = atoi(argv[4]), parts = atoi(argv[5]);
    const long long rounds = atoll(argv[6]);
    const uint64_t seed = strtoull(argv[7], nullptr, 10);
    const int b = atoi(argv[8]);
    const size_t kd = (size_t)k * d;
    const size_t nbuf = exchange_buffers_total(nb, W);          // buffers in the slot allocation, ints in the stamp allocation
    const size_t slot_floats = nbuf * kd;
    std::vector<int> hits((size_t)nb * W);
    for (long long r = 0; r < rounds; ++r) {
        for (int free_mode = 0; free_mode < 2; ++free_mode) {
            const int spar = free_mode ? 0 : (int)(r & 1);
            std::fill(hits.begin(), hits.end(), 0);
            for (int i = 0; i < W; ++i)
                for (int n = 0; n < nb; ++n) {
                    // ---- sender side (Alg. 5, send) ----
                    const int peer = free_mode ? peer_free(seed, r, i, W, n) : peer_deterministic(seed, r, i, W, n);
                    REQUIRE(peer >= 0 && peer < W && peer != i, "peer %d of worker %d round %lld copy %d", peer, i, r, n);
                    const size_t buf = exchange_buffer(spar, nb, n, W, peer);
                    REQUIRE(buf < nbuf, "stamp index %zu >= %zu", buf, nbuf);
                    const int part = message_part(r, peer, n, parts);
                    REQUIRE(part >= 0 && part < parts, "part %d", part);
                    const int nrows = parts == 1 ? k : part_rows(k, part, parts);
                    int travelling = 0;
                    for (int c = 0; c < k; ++c) travelling += row_travels(c, r, peer, n, parts);
                    REQUIRE(nrows == travelling, "part %d of %d: %d rows by formula, %d by the row test", part, parts, nrows, travelling);
                    for (int e = 0; e < nrows; ++e) {
                        const int row = parts == 1 ? e : part_row(part, parts, e);
                        REQUIRE(row >= 0 && row < k && row_travels(row, r, peer, n, parts), "row %d of part %d", row, part);
                        const size_t first = buf * kd + (size_t)row * d, last = first + d - 1;
                        REQUIRE(last < slot_floats, "slot offset %zu >= %zu (worker %d round %lld copy %d row %d)", last, slot_floats, i, r, n, row);
                    }
                    if (!free_mode) hits[(size_t)n * W + peer] += 1;
                    // ---- recipient side at the merge point of round r + 1: buffer n of worker `peer`, same parity ----
                    const int rpar = free_mode ? 0 : (int)(((r + 1) - 1) & 1);
                    REQUIRE(exchange_buffer(rpar, nb, n, W, peer) == buf, "recipient looks at another buffer than the sender wrote");
                    if (!free_mode) {
                        const int from = (peer - shift_deterministic(seed, r, W, n) + W) % W;     // whom the recipient waits for
                        REQUIRE(from == i, "recipient %d expects sender %d, message came from %d", peer, from, i);
                    }
                }
            if (!free_mode)
                for (size_t q = 0; q < hits.size(); ++q) REQUIRE(hits[q] == 1, "buffer %zu written %d times in round %lld", q, hits[q], r);
        }
    }
    // ---- LDS layout of the matrix-core kernel for this shape, all the forms it is launched in ----
    if (d % 4 == 0 && d <= 128 && k >= 2 && b <= 65535) {
        const int nch = mfma_chunks(d), DP = nch * 8 + 4;
        for (int variant = 0; variant < 5; ++variant) {
            // 0: state streamed; 1: resident, four waves; 2: resident, eight waves; 3: fused sums; 4: four waves with
            // the fixed-point sums of the second pass in place of the state rows
            const bool resident = variant != 0, fused = variant == 3, streamed_sums = variant == 4;
            const int nwv = (variant == 1 || variant == 4) ? 4 : 8;
            const MfmaGeom g = mfma_geom(k, b, nch, resident, nwv, fused ? 1 : (streamed_sums ? 2 : 0));
            REQUIRE(g.kpad >= k && g.kpad % MFMA_WB == 0 && g.nblocks * MFMA_WB == g.kpad, "kpad %d", g.kpad);
            REQUIRE(nch * 8 >= d, "chunks %d for d = %d", nch, d);
            // regions in order, each large enough for what the kernel keeps there
            REQUIRE((size_t)(resident ? g.kpad : 2 * MFMA_WB) * DP * sizeof(float) <= g.off_h, "state stage");
            REQUIRE(g.off_h + (size_t)g.kpad * sizeof(float) <= g.off_cstart, "offsets h_c");
            REQUIRE(g.off_cstart + ((size_t)g.ns + 1) * sizeof(int) <= g.off_cursor, "list starts");
            REQUIRE(g.off_cursor + (size_t)g.ns * g.nr * sizeof(int) <= g.off_idx, "counters");
            REQUIRE(g.off_idx + (size_t)b * sizeof(unsigned short) <= g.off_perm, "assignments");
            REQUIRE(g.off_perm + (size_t)b * sizeof(unsigned short) <= g.off_flist, "permutation");
            const int TM = 32 * nwv;
            const size_t flist = resident ? (size_t)nwv * 32 * ((b + TM - 1) / TM) * sizeof(unsigned short) : 0;
            if (streamed_sums) {
                REQUIRE(g.off_sums == 0 && (size_t)k * nch * 8 * sizeof(int) <= g.off_h, "fixed-point sums in place of the state rows");
                REQUIRE(g.off_flist + flist <= g.off_scale, "lists of samples to re-decide");
            } else {
                REQUIRE(g.off_flist + flist <= g.off_sums, "lists of samples to re-decide");
                REQUIRE(g.off_sums + (fused ? (size_t)k * nch * 8 * sizeof(int) : 0) <= g.off_scale, "fixed-point sums");
            }
            REQUIRE(g.off_scale + ((fused || streamed_sums) ? (size_t)2 * nch * 8 * sizeof(float) : 0) <= g.bytes, "scales");
            REQUIRE(g.off_h % 16 == 0 && g.off_sums % 16 == 0 && g.off_scale % 16 == 0 && g.off_cstart % 4 == 0, "alignment");
            // slots of the counting sort: a bijection of the centroids into [0, ns), counters inside their region
            REQUIRE(g.nr >= 1 && g.nr <= nwv && (g.nr & (g.nr - 1)) == 0, "shares %d", g.nr);
            std::vector<int> seen((size_t)g.ns, 0);
            for (int c = 0; c < k; ++c) {
                const int sl = (c % nwv) * g.kq + c / nwv;
                REQUIRE(sl >= 0 && sl < g.ns, "slot %d of centroid %d (ns %d)", sl, c, g.ns);
                seen[sl] += 1;
                REQUIRE(seen[sl] == 1, "slot %d used twice", sl);
                REQUIRE((size_t)sl * g.nr + (g.nr - 1) < (size_t)g.ns * g.nr, "counter index");
            }
            // a wave's list of samples to re-decide: 32 per tile row it scans
            if (resident) {
                const int per_wave = 32 * ((b + TM - 1) / TM);
                int most = 0;
                for (int tile0 = 0; tile0 < b; tile0 += TM) most += 32;
                REQUIRE(most <= per_wave, "list of a wave: %d entries, room for %d", most, per_wave);
            }
        }
    }
    printf("ok %lld\n", checks);
    return 0;
}
