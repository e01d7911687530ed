// Visibility of four consecutive cache positions for a query row of a draft tree.
//
// A row sees the whole context in front of its request's new tokens, and of the new tokens those
// its mask word names (bit j = new token j, at cache position ctx + j).  Plain integer code with no
// device dependency, so that a host test can sweep it over every offset a kernel can produce.
#pragma once

#include <stdint.h>

#ifndef SS_HOST_DEVICE
#define SS_HOST_DEVICE __host__ __device__
#endif

namespace ss {

// rel = (first of the four positions) - ctx; may be negative (old context) or reach past the 32 mask bits
// (slots behind the last new token in the request's last cache block).  Bit e of the result: position
// rel + e is visible.
SS_HOST_DEVICE inline uint32_t tree_visible4(uint32_t newmask, int rel)
{
    // A 64-position window: 32 positions of old context (all visible) below the 32 mask bits,
    // shifted so that bit e is position rel + e.  Shift counts of 64 and more would wrap: nothing is
    // visible there (no mask bit lies that far out).
    const int sh = rel + 32;
    if (sh < 0) return 0xfu;
    if (sh >= 64) return 0u;
    const uint64_t window = ((uint64_t)newmask << 32) | 0xffffffffull;
    return (uint32_t)(window >> sh) & 0xfu;
}

}  // namespace ss
