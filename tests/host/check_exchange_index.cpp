// Host-only check of every offset the kernels with plain-row messages form in the exchange buffers, for given
// shapes: all rounds of a run, all workers, all copies, both modes' schedules, with and without partial messages.
// Built with the plain C++ compiler against csrc/exchange_index.h (the functions the kernels call); no GPU, no HIP.
// usage: check_exchange_index k d W nb parts rounds seed   -> prints "ok <number of checks>" or the first violation
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "exchange_index.h"

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
    if (argc != 8) return 2;
    const int k = atoi(argv[1]), d = atoi(argv[2]), W = atoi(argv[3]), nb = atoi(argv[4]), parts = atoi(argv[5]);
    const long long rounds = atoll(argv[6]);
    const uint64_t seed = strtoull(argv[7], nullptr, 10);
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
                    // ---- sender side (Alg. 5 line 9) ----
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
    printf("ok %lld\n", checks);
    return 0;
}
