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
// g workgroups that land on one XCD take g consecutive positions.  A bijection on [0, n);
// the identity when g == 0 and on the incomplete last round.  g <= 2^28, so that 8 * g fits.
FF_XCD_HD inline uint32_t xcd_order(uint32_t b, uint32_t n, uint32_t g)
{
    constexpr uint32_t kXcds = 8;
    if (g == 0) return b;
    const uint32_t span = kXcds * g;       // workgroups in one round over the XCDs
    if (b >= n / span * span) return b;    // the incomplete last round keeps its order
    const uint32_t round = b / span, in = b % span;
    return round * span + (in % kXcds) * g + in / kXcds;
}

}  // namespace ffsnap
