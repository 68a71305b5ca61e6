// Ancestor masks of a draft tree: device helpers shared by the kernels that build or check them.
#pragma once
#include "device_utils.h"

namespace adaspec {

// A parent index as the kernels use it: the root has none (-1); anything else is forced into
// [0, j) so that malformed input cannot send a kernel out of the request.
__device__ __forceinline__ int sane_parent(int p, int j) { return j == 0 ? -1 : min(max(p, 0), j - 1); }

// The masks of the n nodes of one request whose first row is r0, by one wavefront (lane j = node j).
// Pointer jumping: after s rounds lane j holds the nodes up to 2^s levels above it and points 2^s
// levels up; six rounds cover 64 nodes.
__device__ __forceinline__ void tree_masks_of_request(const int32_t *__restrict__ parents, int r0, int n, int lane,
                                                      unsigned long long *__restrict__ anc)
{
    const int j = lane;
    const int p = j < n ? sane_parent(j > 0 ? parents[r0 + j] : -1, j) : -1;
    int up = p < 0 ? j : p;                             // the root, and idle lanes, point at themselves
    unsigned long long a = j < n ? 1ull << j : 0ull;
#pragma unroll
    for (int s = 0; s < 6; ++s) {
        a |= __shfl(a, up, kWave);
        up = __shfl(up, up, kWave);
    }
    if (j < n) anc[r0 + j] = a;
}

// Batches up to this size have their masks built by extra workgroups of the metadata kernel (each
// wavefront adds up the rows of the requests before its own: quadratic, fine for a few thousand).
constexpr int kFusedMaskMaxBatch = 2048;

}  // namespace adaspec
