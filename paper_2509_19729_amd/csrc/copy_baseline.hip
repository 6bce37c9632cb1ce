// Plain streaming copy with the same access shape as the reshard kernels
// (16 bytes per lane, UNROLL loads in flight, 256-lane workgroups).  It is a
// measurement aid: the achievable copy rate of the machine to set beside the
// reshard rates, and a transfer of known size to calibrate the HBM traffic
// counters with.
#include <algorithm>
#include <string>

#include "device_common.h"
#include "launch.h"

namespace amoeba {

template <int UNROLL, bool NT>
__global__ void __launch_bounds__(kThreads)
copy_kernel(char* __restrict__ dst, const char* __restrict__ src, uint64_t n_vecs, uint64_t n_tiles) {
  constexpr uint64_t kTileVecs = uint64_t(kThreads) * UNROLL;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t v0 = t * kTileVecs + threadIdx.x;
    u32x4 val[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (v0 + u * kThreads < n_vecs) val[u] = ld<NT, u32x4>(src + (v0 + u * kThreads) * 16);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (v0 + u * kThreads < n_vecs) st<NT, u32x4>(dst + (v0 + u * kThreads) * 16, val[u]);
  }
}

int launch_copy_baseline(void* dst, const void* src, size_t bytes, int unroll, int grid, bool nt,
                         hipStream_t stream, std::string* err) {
  if ((reinterpret_cast<uint64_t>(dst) | reinterpret_cast<uint64_t>(src) | bytes) & 15) {
    *err = "copy baseline needs 16-byte aligned pointers and size";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (bytes == 0) return AMOEBA_OK;
  if (unroll != 1 && unroll != 2 && unroll != 8) unroll = 4;
  const uint64_t n_vecs = bytes / 16, tile = uint64_t(kThreads) * unroll;
  const uint64_t n_tiles = (n_vecs + tile - 1) / tile;
  uint64_t g = std::min<uint64_t>(n_tiles, (uint64_t(1) << 31) - 1);
  if (grid > 0) g = std::min<uint64_t>(g, uint64_t(grid));
  char* d = static_cast<char*>(dst);
  const char* s = static_cast<const char*>(src);
#define AMOEBA_COPY(U)                                                                          \
  if (nt) hipLaunchKernelGGL((copy_kernel<U, true>), dim3(uint32_t(g)), dim3(kThreads), 0,      \
                             stream, d, s, n_vecs, n_tiles);                                    \
  else hipLaunchKernelGGL((copy_kernel<U, false>), dim3(uint32_t(g)), dim3(kThreads), 0,        \
                          stream, d, s, n_vecs, n_tiles)
  switch (unroll) {
    case 1: AMOEBA_COPY(1); break;
    case 2: AMOEBA_COPY(2); break;
    case 8: AMOEBA_COPY(8); break;
    default: AMOEBA_COPY(4); break;
  }
#undef AMOEBA_COPY
  const hipError_t rc = hipGetLastError();
  if (rc != hipSuccess) {
    *err = std::string("copy kernel launch failed: ") + hipGetErrorString(rc);
    return AMOEBA_ERR_HIP;
  }
  return AMOEBA_OK;
}

}  // namespace amoeba
