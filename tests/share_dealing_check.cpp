// Host-only check of the functions that deal a call's units to the workers of the persistent
// grid (paper_2405_01814_amd/csrc/lamina_shares.h).  Compiled and run by
// tests/test_share_dealing.py with the host compiler; prints "ok <cases>" or the first
// violated property.  The properties are the ones the kernels rely on:
//   * the shares are contiguous, in order, and cover [0, U) exactly;
//   * share_owner(u) is the one worker whose share holds u;
//   * without a skew the shares are equal to within one unit and the empty ones come last, so
//     that every worker between a row's first and last piece holds a piece of it;
//   * with a skew no share is empty and every share lies within two units of its ideal
//     (64 + skew) / 64 or (64 - skew) / 64 of an even share;
//   * share_skew is zero wherever a share could be empty.
#include <cstdio>
#include <cstdlib>

#include "lamina_shares.h"

static long long g_cases = 0;

#define REQUIRE(cond, ...)                                                                     \
    do {                                                                                       \
        if (!(cond)) {                                                                         \
            std::printf("FAILED %s: ", #cond);                                                 \
            std::printf(__VA_ARGS__);                                                          \
            std::printf("\n");                                                                 \
            std::exit(1);                                                                      \
        }                                                                                      \
    } while (0)

static void check(unsigned U, unsigned n, int skew, bool every_owner)
{
    ++g_cases;
    REQUIRE(share_begin(U, n, 0, skew) == 0, "U=%u n=%u skew=%d", U, n, skew);
    REQUIRE(share_begin(U, n, n, skew) == U, "U=%u n=%u skew=%d", U, n, skew);
    unsigned lo = ~0u, hi = 0, even_sum = 0, odd_sum = 0;
    bool seen_empty = false;
    for (unsigned j = 0; j < n; ++j) {
        const unsigned b = share_begin(U, n, j, skew), e = share_begin(U, n, j + 1, skew);
        REQUIRE(b <= e, "U=%u n=%u skew=%d j=%u", U, n, skew, j);
        const unsigned len = e - b;
        if (len == 0)
            seen_empty = true;
        else
            REQUIRE(!seen_empty, "a share with work after an empty one: U=%u n=%u j=%u", U, n, j);
        lo = len < lo ? len : lo;
        hi = len > hi ? len : hi;
        (j & 1 ? odd_sum : even_sum) += len;
        if (len > 0) {                                    // first and last unit of the share
            REQUIRE(share_owner(U, n, b, skew) == (int)j, "U=%u n=%u skew=%d j=%u", U, n, skew, j);
            REQUIRE(share_owner(U, n, e - 1, skew) == (int)j, "U=%u n=%u skew=%d j=%u", U, n, skew, j);
        }
        if (every_owner)
            for (unsigned u = b; u < e; ++u)
                REQUIRE(share_owner(U, n, u, skew) == (int)j, "U=%u n=%u skew=%d u=%u", U, n, skew, u);
    }
    if (skew == 0) {
        REQUIRE(hi - lo <= 1, "uneven: U=%u n=%u lo=%u hi=%u", U, n, lo, hi);
    } else {
        REQUIRE(lo > 0, "empty share under a skew: U=%u n=%u skew=%d", U, n, skew);
        // every share within two units of its ideal (64 +- skew) / 64 of U / n
        for (unsigned j = 0; j < n; ++j) {
            const double ideal = (double)U / n * (64.0 + (j & 1 ? -skew : skew)) / 64.0 *
                                 (64.0 * n) / (64.0 * n + (double)skew * (n & 1));
            const double len = (double)share_begin(U, n, j + 1, skew) - share_begin(U, n, j, skew);
            REQUIRE(len > ideal - 2.0 && len < ideal + 2.0, "U=%u n=%u skew=%d j=%u len=%.0f ideal=%.2f",
                    U, n, skew, j, len, ideal);
        }
        if (n % 2 == 0 && U >= 64 * n)                    // beyond the rounding of whole units
            REQUIRE(even_sum > odd_sum, "U=%u n=%u skew=%d", U, n, skew);
    }
}

int main()
{
    const unsigned ns[] = {1, 2, 3, 7, 8, 63, 64, 255, 256, 511, 512, 608, 1023, 1024};
    for (unsigned n : ns) {
        // the rule the library applies, on either side of its thresholds and far beyond
        for (unsigned U = 0; U <= 40 * n + 3; U += (n > 64 ? 1 + n / 37 : 1)) {
            const int skew = share_skew(true, U, n);
            REQUIRE(share_skew(false, U, n) == 0, "U=%u n=%u", U, n);
            REQUIRE(skew == 0 || U >= 2 * n, "a skew where a share could be empty: U=%u n=%u", U, n);
            REQUIRE(skew >= 0 && skew <= kParitySkew, "U=%u n=%u", U, n);
            check(U, n, skew, n <= 64 || U % 97 == 0);
            check(U, n, 0, n <= 64 || U % 89 == 0);
        }
        const unsigned big[] = {1000003u, 16777259u, 1u << 30};
        for (unsigned U : big)
            if (U >= 24u * n) {
                check(U, n, share_skew(true, U, n), false);
                check(U, n, 0, false);
                // owners of units spread over the whole stream
                const int skew = share_skew(true, U, n);
                for (unsigned k = 0; k < 4096; ++k) {
                    const unsigned u = (unsigned)(((unsigned long long)U - 1) * k / 4095);
                    const int j = share_owner(U, n, u, skew);
                    REQUIRE(j >= 0 && (unsigned)j < n && share_begin(U, n, j, skew) <= u &&
                                u < share_begin(U, n, j + 1, skew),
                            "U=%u n=%u skew=%d u=%u j=%d", U, n, skew, u, j);
                }
            }
        // every skew the functions accept, not only the ones the rule picks
        for (int skew = 1; skew <= 8; ++skew)
            for (unsigned U = 2 * n; U <= 30 * n; U += 1 + n / 5)
                check(U, n, skew, n <= 64);
    }
    std::printf("ok %lld\n", g_cases);
    return 0;
}
