// Index arithmetic of the exchange buffers, in one place: the kernels that keep messages as plain rows (the
// shape-agnostic and the matrix-core kernel), the host side of the library and a host-only check of all the offsets a
// run can form (tests/host/check_exchange_index.cpp, built with the plain C++ compiler) use these functions.
// Plain C++, no HIP types.
#pragma once

#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define ASGD_HD __host__ __device__
#else
#define ASGD_HD
#endif

namespace asgd {

// ---- counter-based integer generator (published splitmix64 finaliser) --------------------
// Used for the peer schedule and the message-loss test hook.  Integer only, so host and
// device agree bit for bit.
ASGD_HD inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
ASGD_HD inline uint64_t round_hash(uint64_t seed, int64_t r)
{
    return mix64(seed + 0x9E3779B97F4A7C15ULL * (uint64_t)(r + 1));
}
// Deterministic schedule: one cyclic shift per round and copy, shared by all senders, so that every
// worker receives exactly one message per round in each of its buffers (Alg. 5, send asks only for
// "a random node other than i").  Copy n of a message (0 <= n < number of buffers < W) goes into the
// recipient's buffer n; the shifts of one round differ, so a worker's senders differ.
ASGD_HD inline int shift_deterministic(uint64_t seed, int64_t r, int W, int n = 0)
{
    return (int)(1 + (round_hash(seed, r) % (uint64_t)(W - 1) + (uint64_t)n) % (uint64_t)(W - 1));
}
ASGD_HD inline int peer_deterministic(uint64_t seed, int64_t r, int i, int W, int n = 0)
{
    return (int)(((uint64_t)i + (uint64_t)shift_deterministic(seed, r, W, n)) % (uint64_t)W);
}
// Free-running schedule: every sender draws its own recipients; collisions are the data race
// of Fig. 2 (III) and are allowed.
ASGD_HD inline int peer_free(uint64_t seed, int64_t r, int i, int W, int n = 0)
{
    uint64_t h = mix64(round_hash(seed, r) + 0x9E3779B97F4A7C15ULL * (uint64_t)(i + 1) + 0x5851F42D4C957F2DULL +
                       0xD1B54A32D192ED03ULL * (uint64_t)n);
    return (int)(((uint64_t)i + 1 + h % (uint64_t)(W - 1)) % (uint64_t)W);
}
ASGD_HD inline bool message_dropped(uint64_t seed, int64_t r, int sender, uint32_t thr, int n = 0)
{
    uint64_t u = mix64(round_hash(seed, r) + 0x9E3779B97F4A7C15ULL * (uint64_t)(sender + 1) +
                       0xD1B54A32D192ED03ULL * (uint64_t)n) >> 40;
    return u < (uint64_t)thr;
}
// Buffers are ordered (parity of the sending round, buffer n, recipient); `units` per buffer (k*d floats, or 1 for
// the stamps).  The allocation holds 2 * nb * W buffers.
ASGD_HD inline size_t exchange_buffer(int parity, int nb, int n, int W, int worker)
{
    return (size_t)(parity * nb + n) * (size_t)W + (size_t)worker;
}
ASGD_HD inline size_t exchange_buffers_total(int nb, int W) { return (size_t)2 * nb * W; }

// Partial messages (Sec. 4.4): copy n of the message of round r to recipient q carries the centroid rows c with
// c mod P = (r + q + n) mod P.
ASGD_HD inline int message_part(long long round, int recipient, int n, int parts)
{
    return (int)((round + recipient + n) % parts);
}
ASGD_HD inline bool row_travels(int row, long long round, int recipient, int n, int parts)
{
    return parts == 1 || row % parts == message_part(round, recipient, n, parts);
}
// number of rows of part `part` among k rows, and the e-th of them
ASGD_HD inline int part_rows(int k, int part, int parts) { return (k - part + parts - 1) / parts; }
ASGD_HD inline int part_row(int part, int parts, int e) { return part + parts * e; }

}  // namespace asgd
