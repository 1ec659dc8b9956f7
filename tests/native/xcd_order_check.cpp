// xcd_order(b, n, g) must be a permutation of [0, n) for every launch size and run length, and the
// workgroups that one XCD receives (b mod 8 equal, consecutive in b) must take consecutive positions.
// Behind the last complete round the run length halves until it fits: also checked, through the
// largest run that fits a launch shorter than one round.
#include "xcd_order.h"
#include <cstdio>
#include <vector>
using ffsnap::xcd_order;
int main()
{
    // 2^28 is the longest run the plan flags can ask for: 8 * g still fits 32 bits
    const uint32_t gs[] = {0, 1, 2, 3, 4, 8, 16, 100, 1u << 20, 1u << 28};
    for (uint32_t g : gs) {
        for (uint32_t n = 0; n <= 700; n++) {
            std::vector<int> seen(n, 0);
            for (uint32_t b = 0; b < n; b++) {
                const uint32_t t = xcd_order(b, n, g);
                if (t >= n || seen[t]++) { std::printf("not a permutation: g=%u n=%u b=%u -> %u\n", g, n, b, t); return 1; }
            }
            if (g == 0) {
                for (uint32_t b = 0; b < n; b++) if (xcd_order(b, n, 0) != b) { std::printf("g=0 must be the identity\n"); return 1; }
                continue;
            }
            // inside complete rounds: the next workgroup of the same XCD (b + 8) takes the next position
            const uint32_t span = 8 * g, full = n / span * span;
            for (uint32_t b = 0; b + 8 < full; b++) {
                if ((b % span) + 8 >= span) continue;  // last of this XCD's run in the round
                if (xcd_order(b + 8, n, g) != xcd_order(b, n, g) + 1) { std::printf("run broken: g=%u n=%u b=%u\n", g, n, b); return 1; }
            }
            // every round maps onto itself
            for (uint32_t b = 0; b < full; b++)
                if (xcd_order(b, n, g) / span != b / span) { std::printf("round left: g=%u n=%u b=%u\n", g, n, b); return 1; }
        }
    }
    // a launch shorter than one round of the requested run length still gets runs: the longest
    // power of two that fits, from workgroup 0 on
    for (uint32_t n = 8; n <= 3000; n += 37) {
        const uint32_t g = 1u << 11;
        uint32_t fit = g;
        while (8 * fit > n) fit >>= 1;
        for (uint32_t b = 0; b + 8 < 8 * fit; b++) {
            if ((b % (8 * fit)) + 8 >= 8 * fit) continue;
            if (xcd_order(b + 8, n, g) != xcd_order(b, n, g) + 1) { std::printf("short launch: n=%u b=%u\n", n, b); return 1; }
        }
    }
    // a large launch, spot-checked through its inverse
    {
        const uint32_t n = 3000000007u, g = 8, span = 64;
        for (uint32_t b = 0; b < n; b += 9973) {
            const uint32_t t = xcd_order(b, n, g);
            if (t >= n) { std::printf("range\n"); return 1; }
            if (b < n / span * span) {
                const uint32_t in = t % span, back = t / span * span + (in % g) * 8 + in / g;
                if (back != b) { std::printf("inverse: b=%u t=%u back=%u\n", b, t, back); return 1; }
            }
        }
    }
    std::printf("ok\n");
    return 0;
}
