// Weight reshard kernel: one launch gathers the target rank's shard for all layers.
//
// What it computes (paper Sec. 2.2 and Sec. 3.2 Eq. (1)): the target rank's slice
// of q/k/v/gate/up (cut along stored rows) and of o/down (cut along stored
// columns), taken from whichever source ranks hold it.  The host planner has
// already expressed that as a short per-layer table of strided byte rectangles;
// this kernel is a table-driven streaming gather.
//
// Mapping to the machine.  The work is HBM-bound (every byte is read once and
// written once), so: each lane moves 16 bytes per access, a workgroup of THREADS
// lanes (one wavefront by default) owns a tile of UNROLL x THREADS x 16 B that is
// contiguous in the destination,
// all loads of a tile are issued before its first store, and accesses carry the
// non-temporal hint because nothing is reused.  Measured on MI355X the best shape
// is the smallest one: one 16-byte vector per lane and one workgroup per tile,
// leaving the overlap of reads and writes to the many short-lived wavefronts in
// flight (larger tiles or persistent grid-stride loops cost 5-15 %).  Tiles are numbered in
// destination order (layer, segment, position) and each of the 8 XCDs takes its own
// contiguous eighth of them, so that the workgroups in flight at any time sweep eight
// contiguous windows of the destination, one per XCD and L2.  Within a strided
// rectangle the lane's vector index n is split into (row, column) with a
// multiply-high division by the row length.
#include <algorithm>
#include <string>
#include <vector>

#include "device_common.h"
#include "grid.h"
#include "launch.h"
#include "plan.h"

namespace amoeba {

constexpr int kMaxSegs = 64;  // segments per launch (kernel arguments are limited to 4 KiB)

struct WSeg {
  const char* src;      // layer 0 address of the segment's first vector
  int64_t dst_off;      // byte offset of its first vector in the target shard, layer 0
  uint32_t src_pitch;   // bytes between rows, source side
  uint32_t dst_pitch;   // bytes between rows, target side
  uint32_t total_vecs;  // rows * row_vecs
  FastDiv row_vecs;     // vectors per row
};

struct WArgs {
  WSeg seg[kMaxSegs];
  uint32_t tile_begin[kMaxSegs];  // first tile of each segment within a layer
  char* dst;
  int64_t src_layer_stride, dst_layer_stride;  // bytes
  uint32_t n_seg;
  uint32_t total_tiles;  // tiles_per_layer * n_layers
  FastDiv tiles_per_layer;
};

template <int VEC, int THREADS, int UNROLL, bool NT>
__global__ void __launch_bounds__(THREADS) reshard_weights_kernel(const WArgs a) {
  using V = typename VecOf<VEC>::type;
  constexpr uint32_t kTileVecs = THREADS * UNROLL;
  const uint32_t tid = threadIdx.x;

  // Tiles are taken in the XCD-chunked order (see xcd_item()): every XCD sweeps its own
  // contiguous eighth of the (layer, tile) space; measured +2-3 % over the plain order here.
  const uint32_t n_loop = xcd_loop_bound(a.total_tiles);
  for (uint32_t wi = blockIdx.x; wi < n_loop; wi += gridDim.x) {
    const uint32_t w = xcd_item(wi, a.total_tiles);
    if (w >= a.total_tiles) continue;
    const uint32_t layer = fd_div(w, a.tiles_per_layer);
    const uint32_t t = w - layer * a.tiles_per_layer.d;
    // last segment whose first tile is <= t (uniform across the workgroup)
    uint32_t lo = 0, hi = a.n_seg;
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (a.tile_begin[mid] <= t) lo = mid; else hi = mid;
    }
    const WSeg& s = a.seg[lo];
    const char* src = s.src + int64_t(layer) * a.src_layer_stride;
    char* dst = a.dst + s.dst_off + int64_t(layer) * a.dst_layer_stride;
    const uint32_t n0 = (t - a.tile_begin[lo]) * kTileVecs + tid;

    V val[UNROLL];
    uint64_t doff[UNROLL];
    bool live[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const uint32_t n = n0 + u * THREADS;
      live[u] = n < s.total_vecs;
      const uint32_t row = fd_div(n, s.row_vecs);
      const uint32_t col = n - row * s.row_vecs.d;
      const uint64_t soff = uint64_t(row) * s.src_pitch + uint64_t(col) * VEC;
      doff[u] = uint64_t(row) * s.dst_pitch + uint64_t(col) * VEC;
      if (live[u]) val[u] = s.src ? ld<NT, V>(src + soff) : V(0);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (live[u]) st<NT, V>(dst + doff[u], val[u]);
  }
}

namespace {

template <int VEC, int THREADS, int UNROLL>
void launch_one(bool nt, dim3 grid, hipStream_t stream, const WArgs& a) {
  if (nt)
    hipLaunchKernelGGL((reshard_weights_kernel<VEC, THREADS, UNROLL, true>), grid, dim3(THREADS),
                       0, stream, a);
  else
    hipLaunchKernelGGL((reshard_weights_kernel<VEC, THREADS, UNROLL, false>), grid, dim3(THREADS),
                       0, stream, a);
}

template <int THREADS>
void dispatch_unroll(int unroll, bool nt, dim3 grid, hipStream_t stream, const WArgs& a) {
  switch (unroll) {
    case 2: launch_one<16, THREADS, 2>(nt, grid, stream, a); break;
    case 4: launch_one<16, THREADS, 4>(nt, grid, stream, a); break;
    case 8: launch_one<16, THREADS, 8>(nt, grid, stream, a); break;
    default: launch_one<16, THREADS, 1>(nt, grid, stream, a); break;
  }
}

void dispatch(int vec, int threads, int unroll, bool nt, dim3 grid, hipStream_t stream,
              const WArgs& a) {
  if (vec == 16) {
    if (threads == 64) dispatch_unroll<64>(unroll, nt, grid, stream, a);
    else if (threads == 128) dispatch_unroll<128>(unroll, nt, grid, stream, a);
    else dispatch_unroll<256>(unroll, nt, grid, stream, a);
  } else if (vec == 8) {
    launch_one<8, 256, 1>(nt, grid, stream, a);
  } else if (vec == 4) {
    launch_one<4, 256, 1>(nt, grid, stream, a);
  } else if (vec == 2) {
    launch_one<2, 256, 1>(nt, grid, stream, a);
  } else {
    launch_one<1, 256, 1>(nt, grid, stream, a);
  }
}

}  // namespace

// Tile geometry of one launch over `chosen` segments: fills the kernel's segment table
// (sources left null when src_shards is null) and returns the tiles per layer, or -1.
namespace {

struct WShape {
  int vec, threads, unroll;
  bool nt;
};

WShape weights_shape(const amoeba_plan_s* p, int vec) {
  WShape w;
  w.vec = vec;
  w.unroll = p->tune.w_unroll;
  w.threads = p->tune.w_threads;
  if (vec != 16 || (w.unroll != 2 && w.unroll != 4 && w.unroll != 8)) w.unroll = 1;
  if (vec != 16) w.threads = 256;
  else if (w.threads != 128 && w.threads != 256) w.threads = 64;  // one wavefront per 1 KiB tile
  w.nt = p->tune.nontemporal != 2;
  return w;
}

// Alignment every offset, run and pitch of the plan's segments allows (with the layer strides).
uint64_t plan_alignment_bits(const amoeba_plan_s* p) {
  uint64_t bits = uint64_t(p->src_layer_bytes) | uint64_t(p->dst_layer_bytes);
  for (const Segment& g : p->segments) {
    bits |= uint64_t(g.dst_off) | uint64_t(g.run);
    if (g.src_rank >= 0) bits |= uint64_t(g.src_off);
    if (g.rows > 1) bits |= uint64_t(g.src_pitch) | uint64_t(g.dst_pitch);
  }
  return bits;
}

std::vector<Segment> chosen_segments(const amoeba_plan_s* p, int part) {
  std::vector<Segment> chosen;
  for (const Segment& g : p->segments)
    if (part == AMOEBA_PART_ALL || part == g.part + 1) chosen.push_back(g);
  return chosen;
}

// Fills the tile table of segments [first, first + n_seg) and returns the tiles of one layer;
// false if a segment does not fit 32-bit tile indexing.
bool tile_table(const std::vector<Segment>& chosen, size_t first, uint32_t n_seg, const WShape& w,
                const void* const* src_shards, WArgs* a, uint64_t* tiles_out, std::string* err) {
  const uint64_t tile_vecs = uint64_t(w.threads) * w.unroll;
  uint64_t tiles = 0;
  for (uint32_t i = 0; i < n_seg; ++i) {
    const Segment& g = chosen[first + i];
    const uint64_t row_vecs = uint64_t(g.run) / w.vec, total = row_vecs * uint64_t(g.rows);
    const bool strided = g.rows > 1;
    if (total >= (uint64_t(1) << 32) - 65536 ||
        (strided && (uint64_t(g.src_pitch) >= (uint64_t(1) << 32) ||
                     uint64_t(g.dst_pitch) >= (uint64_t(1) << 32)))) {
      *err = "a weight segment is too large for 32-bit tile indexing";
      return false;
    }
    WSeg& s = a->seg[i];
    s.src = (g.src_rank < 0 || !src_shards)
                ? nullptr  // a gap of a padded target: zeros
                : static_cast<const char*>(src_shards[g.src_rank]) + g.src_off;
    s.dst_off = g.dst_off;
    s.src_pitch = strided ? uint32_t(g.src_pitch) : 0;  // a single row never uses its pitch
    s.dst_pitch = strided ? uint32_t(g.dst_pitch) : 0;
    s.total_vecs = uint32_t(total);
    s.row_vecs = make_fastdiv(uint32_t(row_vecs));
    a->tile_begin[i] = uint32_t(tiles);
    tiles += (total + tile_vecs - 1) / tile_vecs;
  }
  *tiles_out = tiles;
  return true;
}

// One workgroup per tile, up to what one grid dimension holds; past it the workgroups stride.
bool weights_grid(const amoeba_plan_s* p, uint64_t tiles_per_layer, const WShape& w,
                  uint64_t* total_tiles, uint32_t* grid, std::string* err) {
  *total_tiles = tiles_per_layer * uint64_t(p->shape.n_layers);
  // Tile ids are 32-bit and a striding workgroup adds the grid size to one: both stay below
  // 2^32 with at most 2^31 tiles (2 TiB of 1 KiB tiles) and a grid of at most 2^26.
  if (*total_tiles >= (uint64_t(1) << 31)) {
    *err = "too many tiles for one launch";
    return false;
  }
  uint64_t want = *total_tiles;
  if (p->tune.w_grid > 0) want = std::min<uint64_t>(want, uint64_t(p->tune.w_grid));
  *grid = clamp_grid_x(want, uint32_t(w.threads));  // (a sweep's grid is taken as given)
  return true;
}

}  // namespace

bool weights_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                             std::string* err) {
  const WShape w = weights_shape(p, common_alignment(plan_alignment_bits(p) | uint64_t(align_bytes)));
  const std::vector<Segment> chosen = chosen_segments(p, AMOEBA_PART_ALL);
  WArgs a;
  uint64_t tiles = 0, total = 0;
  uint32_t grid = 0;
  const uint32_t n_seg = uint32_t(std::min<size_t>(kMaxSegs, chosen.size()));
  if (!tile_table(chosen, 0, n_seg, w, nullptr, &a, &tiles, err)) return false;
  if (!weights_grid(p, tiles, w, &total, &grid, err)) return false;
  out->grid_x = total ? grid : 0;
  out->grid_y = 1;
  out->threads = uint32_t(w.threads);
  out->items = total;
  return true;
}

int launch_reshard_weights(const amoeba_plan_s* p, const void* const* src_shards, void* dst,
                           int part, hipStream_t stream, std::string* err) {
  const int64_t src_layer = p->src_layer_bytes, dst_layer = p->dst_layer_bytes;
  const uint64_t src_bytes = uint64_t(src_layer) * p->shape.n_layers,
                 dst_bytes = uint64_t(dst_layer) * p->shape.n_layers;

  // widest access every address of this call is aligned to
  uint64_t bits = plan_alignment_bits(p) | reinterpret_cast<uint64_t>(dst);
  const uint64_t d0 = reinterpret_cast<uint64_t>(dst);
  for (int r = 0; r < p->k; ++r) {
    if (!(p->weight_rank_mask >> r & 1)) continue;
    const uint64_t s0 = reinterpret_cast<uint64_t>(src_shards[r]);
    if (!s0) { *err = "a needed source shard pointer is NULL"; return AMOEBA_ERR_INVALID_ARG; }
    if (s0 < d0 + dst_bytes && d0 < s0 + src_bytes) {
      *err = "dst overlaps a source shard (the reshard is out of place)";
      return AMOEBA_ERR_INVALID_ARG;
    }
    bits |= s0;
  }
  const WShape w = weights_shape(p, common_alignment(bits));

  const std::vector<Segment> chosen = chosen_segments(p, part);
  const size_t n = chosen.size();
  for (size_t first = 0; first < n; first += kMaxSegs) {
    WArgs a;
    a.dst = static_cast<char*>(dst);
    a.src_layer_stride = src_layer;
    a.dst_layer_stride = dst_layer;
    a.n_seg = uint32_t(std::min<size_t>(kMaxSegs, n - first));
    uint64_t tiles = 0, total_tiles = 0;
    uint32_t grid = 0;
    if (!tile_table(chosen, first, a.n_seg, w, src_shards, &a, &tiles, err)) return AMOEBA_ERR_INVALID_ARG;
    if (!weights_grid(p, tiles, w, &total_tiles, &grid, err)) return AMOEBA_ERR_INVALID_ARG;
    if (total_tiles == 0) continue;
    a.total_tiles = uint32_t(total_tiles);
    a.tiles_per_layer = make_fastdiv(uint32_t(tiles));
    dispatch(w.vec, w.threads, w.unroll, w.nt, dim3(grid), stream, a);
    const hipError_t rc = hipGetLastError();
    if (rc != hipSuccess) {
      *err = std::string("weight kernel launch failed: ") + hipGetErrorString(rc);
      return AMOEBA_ERR_HIP;
    }
  }
  return AMOEBA_OK;
}

}  // namespace amoeba
