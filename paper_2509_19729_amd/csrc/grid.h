// Launch-grid arithmetic shared by the launchers (host only).
//
// HIP refuses a launch whose gridDim.x * blockDim.x exceeds 2^32 - 1 work-items (each
// dimension of the dispatch packet is a 32-bit count of work-items), so a grid is clamped
// to that and the kernels stride over what is left.  The clamped count is kept a multiple
// of 8 so that a striding workgroup stays on the XCD (workgroup id mod 8) whose chunk of
// the work order it started in.
#pragma once
#include <stdint.h>

#include <algorithm>

namespace amoeba {

constexpr uint64_t kMaxWorkItemsPerDim = (uint64_t(1) << 32) - 1;

inline uint32_t clamp_grid_x(uint64_t want, uint32_t threads) {
  uint64_t cap = kMaxWorkItemsPerDim / threads;
  cap -= cap % 8;
  return uint32_t(std::max<uint64_t>(1, std::min<uint64_t>(want, cap)));
}

// A grid of `want` workgroups for `items` work items: all of them if it covers them, else
// a multiple of 8 (rounded up), for the same reason.
inline uint64_t grid_for_items(uint64_t want, uint64_t items) {
  if (want >= items) return items;
  return std::min<uint64_t>((want + 7) / 8 * 8, items);
}

// What a launcher decided, for amoeba_plan_launch_shape().
struct LaunchShape {
  uint32_t grid_x = 0, grid_y = 0, threads = 0;
  uint64_t items = 0;  // work items (tiles) the grid covers per grid.y slice
};

}  // namespace amoeba
