// Work-item order that keeps neighbouring items on one XCD (gfx950: 8 XCDs, each with an L2 of its own;
// consecutive workgroup ids are dealt to the XCDs in turn).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gad {

constexpr int kXcds = 8;

// Workgroup id (or position in a grid-stride sequence) -> work item, such that the items handled on one XCD are
// consecutive; a bijection on [0, total).
__device__ __forceinline__ int64_t xcd_order(int64_t bid, int64_t total) {
  const int64_t per = total / kXcds, rem = total % kXcds;
  const int64_t x = bid % kXcds, slot = bid / kXcds;
  return x * per + (x < rem ? x : rem) + slot;
}

}  // namespace gad
