// Plain streaming copy with the same access shape as the reshard kernels
// (16 bytes per lane, UNROLL loads in flight, 64- or 256-lane workgroups).  It is a
// measurement aid: the achievable copy rate of the machine to set beside the
// reshard rates, and a transfer of known size to calibrate the HBM traffic
// counters with.
#include <algorithm>
#include <string>

#include "device_common.h"
#include "launch.h"

namespace amoeba {

template <int THREADS, int UNROLL, bool NT>
__global__ void __launch_bounds__(THREADS)
copy_kernel(char* __restrict__ dst, const char* __restrict__ src, uint64_t n_vecs, uint64_t n_tiles) {
  constexpr uint64_t kTileVecs = uint64_t(THREADS) * UNROLL;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t v0 = t * kTileVecs + threadIdx.x;
    u32x4 val[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (v0 + u * THREADS < n_vecs) val[u] = ld<NT, u32x4>(src + (v0 + u * THREADS) * 16);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (v0 + u * THREADS < n_vecs) st<NT, u32x4>(dst + (v0 + u * THREADS) * 16, val[u]);
  }
}

namespace {

template <int THREADS, int UNROLL>
void launch(bool nt, uint32_t grid, hipStream_t stream, char* d, const char* s, uint64_t n_vecs,
            uint64_t n_tiles) {
  if (nt)
    hipLaunchKernelGGL((copy_kernel<THREADS, UNROLL, true>), dim3(grid), dim3(THREADS), 0, stream,
                       d, s, n_vecs, n_tiles);
  else
    hipLaunchKernelGGL((copy_kernel<THREADS, UNROLL, false>), dim3(grid), dim3(THREADS), 0, stream,
                       d, s, n_vecs, n_tiles);
}

template <int THREADS>
void launch_unroll(int unroll, bool nt, uint32_t grid, hipStream_t stream, char* d, const char* s,
                   uint64_t n_vecs, uint64_t n_tiles) {
  switch (unroll) {
    case 2: launch<THREADS, 2>(nt, grid, stream, d, s, n_vecs, n_tiles); break;
    case 4: launch<THREADS, 4>(nt, grid, stream, d, s, n_vecs, n_tiles); break;
    case 8: launch<THREADS, 8>(nt, grid, stream, d, s, n_vecs, n_tiles); break;
    default: launch<THREADS, 1>(nt, grid, stream, d, s, n_vecs, n_tiles); break;
  }
}

}  // namespace

int launch_copy_baseline(void* dst, const void* src, size_t bytes, int threads, int unroll, int grid,
                         bool nt, hipStream_t stream, std::string* err) {
  if ((reinterpret_cast<uint64_t>(dst) | reinterpret_cast<uint64_t>(src) | bytes) & 15) {
    *err = "copy baseline needs 16-byte aligned pointers and size";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (bytes == 0) return AMOEBA_OK;
  if (unroll != 2 && unroll != 4 && unroll != 8) unroll = 1;
  if (threads != 64) threads = 256;
  const uint64_t n_vecs = bytes / 16, tile = uint64_t(threads) * unroll;
  const uint64_t n_tiles = (n_vecs + tile - 1) / tile;
  uint64_t g = n_tiles;
  if (grid > 0) g = std::min<uint64_t>(g, uint64_t(grid));
  g = clamp_grid_x(g, uint32_t(threads));
  char* d = static_cast<char*>(dst);
  const char* s = static_cast<const char*>(src);
  if (threads == 64) launch_unroll<64>(unroll, nt, uint32_t(g), stream, d, s, n_vecs, n_tiles);
  else launch_unroll<256>(unroll, nt, uint32_t(g), stream, d, s, n_vecs, n_tiles);
  const hipError_t rc = hipGetLastError();
  if (rc != hipSuccess) {
    *err = std::string("copy kernel launch failed: ") + hipGetErrorString(rc);
    return AMOEBA_ERR_HIP;
  }
  return AMOEBA_OK;
}

}  // namespace amoeba
