// Order in which the workgroups of a launch take their tiles on a GPU with 8 XCDs.  No HIP
// dependency: the host tests include this file as well.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FF_XCD_HD __host__ __device__
#else
#define FF_XCD_HD
#endif

namespace ffsnap {

// Workgroups are dealt to the 8 XCDs round-robin by launch index.  Within every complete round
// of 8 * g workgroups, workgroup b takes position (b mod 8) * g + b div 8 of the round, so the
// g workgroups that land on one XCD take g consecutive positions.  What is left behind the last
// complete round is divided the same way with runs of g / 2, then g / 4, ... so that a launch
// shorter than a round still gets the longest runs that fit.  A bijection on [0, n); the identity
// when g == 0.  g <= 2^28, so that 8 * g fits.
FF_XCD_HD inline uint32_t xcd_order(uint32_t b, uint32_t n, uint32_t g)
{
    constexpr uint32_t kXcds = 8;
    uint32_t start = 0;  // workgroups in front of the rounds of the current run length
    for (; g; g >>= 1) {
        const uint32_t span = kXcds * g;  // workgroups in one round over the XCDs
        const uint32_t full = (n - start) / span * span;
        if (b - start < full) {
            const uint32_t round = (b - start) / span, in = (b - start) % span;
            return start + round * span + (in % kXcds) * g + in / kXcds;
        }
        start += full;
    }
    return b;
}

}  // namespace ffsnap
