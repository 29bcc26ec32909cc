// XCD-aware split of a kernel's work items over its workgroups (device code, gfx950: 8 XCDs).
#pragma once
#include <hip/hip_runtime.h>

namespace gleam {

// XCD-aware work split.  Workgroups are dealt to the 8 XCDs round-robin by their linear id, and each XCD
// has its own L2.  Work items (pixel tiles or chunks) that re-read each other's rows - the row taps of a
// convolution - should therefore run on the same XCD at about the same time: XCD x owns one contiguous
// eighth of the items and its workgroups walk that range with stride = workgroups per XCD.
// gridDim.x must be a multiple of 8 (launchers round up; surplus workgroups get an empty range).
struct XcdRange {
    long long first, end, stride;
};
__device__ __forceinline__ XcdRange xcd_range(long long n_items) {
    const long long per_xcd = (n_items + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    XcdRange r;
    r.first = xcd * per_xcd + slot;
    r.end = (xcd + 1) * per_xcd < n_items ? (xcd + 1) * per_xcd : n_items;
    r.stride = gridDim.x >> 3;
    return r;
}

}  // namespace gleam
