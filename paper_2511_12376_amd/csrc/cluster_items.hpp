// Lookup in the device-side item list of the batched cluster entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bitsnap.h"

namespace bitsnap {

// The item that holds list-wide group gg: the last one whose first_group <= gg (binary search;
// every operand is wave-uniform, so this runs on the scalar unit).
__device__ __forceinline__ int64_t find_item(const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t gg)
{
    int64_t lo = 0, hi = count - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (items[mid].first_group <= gg)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

}  // namespace bitsnap
