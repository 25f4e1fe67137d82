// Cost model of one cp_eval call: the divisors of every vertex cost (device
// speeds) and of every transfer cost (bandwidth matrix), as plain divisors and,
// where it is provably exact, as 32-bit multiply-shift constants.
#include "cpeval_internal.hpp"

namespace cpeval {
namespace {

// ceil(a/d) for all 0 <= a <= amax through ((N*mul + N) >> 32) with N = a + d - 1,
// mul = M - 1, M = ceil(2^32/d).  Writing M*d = 2^32 + r (0 <= r < d) and
// N = q*d + rem:  N*M/2^32 = q + rem/d + N*r/(d*2^32), whose floor is q as long as
// N*r < 2^32.  N itself must fit 32 bits.
bool magic_for(int64_t d, int64_t amax, Magic &out) {
    if (d < 1 || d >= (int64_t)1 << 32) return false;
    uint64_t nmax = (uint64_t)amax + (uint64_t)d - 1;
    if (nmax >= (1ull << 32)) return false;
    uint64_t M = ((1ull << 32) + (uint64_t)d - 1) / (uint64_t)d;
    uint64_t r = M * (uint64_t)d - (1ull << 32);
    if (r != 0 && nmax >= ((1ull << 32) + r - 1) / r) return false;  // nmax * r >= 2^32
    out.mul = (uint32_t)(M - 1);
    out.dm1 = (uint32_t)(d - 1);
    return true;
}

// The 4-byte form: ceil(a/d) = (N * M' - N * 0 + ...) >> 32 with N = a + d - 1 and
// M' = 256 * ceil(2^24 / d), a multiple of 256 (the kernels take the entry's low byte, which
// holds d - 1, as all ones: multiplier M' - 1, plus N).  With M' * d = 2^32 + r the floor is
// exact as long as N * r < 2^32, as above.
bool magic4_for(int64_t d, int64_t amax, uint32_t &out) {
    if (d < 1 || d > 256) return false;
    const uint64_t nmax = (uint64_t)amax + (uint64_t)d - 1;
    if (nmax >= (1ull << 32)) return false;
    const uint64_t m24 = ((1ull << 24) + (uint64_t)d - 1) / (uint64_t)d;     // <= 2^24
    const uint64_t r = 256 * m24 * (uint64_t)d - (1ull << 32);
    if (r != 0 && nmax >= ((1ull << 32) + r - 1) / r) return false;          // nmax * r >= 2^32
    out = (uint32_t)((m24 - 1) << 8) | (uint32_t)(d - 1);
    return true;
}

}  // namespace

int build_cost_tables(int32_t k, const int64_t *speeds, const int64_t *bandwidth,
                      bool narrow, int64_t max_c, int64_t max_t, CostTables &out) {
    for (int i = 0; i < k; ++i)
        if (speeds[i] < 1) return CP_ERR_SPEED;
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j)
            if (i != j && bandwidth[(size_t)i * k + j] < 1) return CP_ERR_BANDWIDTH;

    const size_t kk = (size_t)k * k;
    out.k = k;
    out.divisor.assign(table_entries(k), 0);
    out.magic.assign(table_entries(k), Magic{0, 0});
    out.tab4.assign(table_entries(k), 0u);
    bool ok = narrow && k <= kMagicMaxK;
    // a free transfer's entry 0 multiplies by 255: 0 ticks only while the volume is below 2^24
    bool ok4 = ok && max_t < ((int64_t)1 << 24) && max_c < ((int64_t)1 << 24);

    for (int own = 0; own < k; ++own)
        for (int nbr = 0; nbr < k; ++nbr) {
            if (own == nbr) continue;  // same device: free, stays {0,0} / divisor 0
            // b sweep: own = device of the edge's source vertex, nbr = device of its target
            int64_t db = bandwidth[(size_t)own * k + nbr];
            // t sweep: own = device of the edge's target vertex, nbr = device of its source
            int64_t dt = bandwidth[(size_t)nbr * k + own];
            out.divisor[(size_t)own * k + nbr] = db;
            out.divisor[kk + (size_t)own * k + nbr] = dt;
            if (ok) ok = magic_for(db, max_t, out.magic[(size_t)own * k + nbr]);
            if (ok) ok = magic_for(dt, max_t, out.magic[kk + (size_t)own * k + nbr]);
            if (ok4) ok4 = magic4_for(db, max_t, out.tab4[(size_t)own * k + nbr]);
            if (ok4) ok4 = magic4_for(dt, max_t, out.tab4[kk + (size_t)own * k + nbr]);
        }
    for (int i = 0; i < k; ++i) {
        out.divisor[2 * kk + i] = speeds[i];
        if (ok) ok = magic_for(speeds[i], max_c, out.magic[2 * kk + i]);
        if (ok4) ok4 = magic4_for(speeds[i], max_c, out.tab4[2 * kk + i]);
    }
    out.magic_ok = ok;
    out.tab4_ok = ok && ok4;
    return CP_OK;
}

}  // namespace cpeval
