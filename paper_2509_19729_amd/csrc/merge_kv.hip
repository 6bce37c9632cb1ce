// In-place merge of m instances at TP=k into one instance at TP=k*m (KV cache).
//
// What it computes (paper Sec. 3.1, base solution and Improvement 1).  Each instance
// holds the whole cache of its own ("local") requests.  After the merge worker
// r' = s*m + g, hosted where rank s of instance g was, owns a 1/m slice of the heads of
// that rank, for the requests of ALL instances.  With the header-centric block
// [head][K/V][token][d] that slice is one contiguous sub-block, so a block of n_kv/k
// heads is re-read as m blocks of n_kv/(k*m) heads ("block reshaping"): old block b
// becomes new blocks b*m .. b*m+m-1.  A local request keeps its slice where it is (new
// id b*m + g); the slices the worker gives away leave holes, and the slice of a request
// of instance g2 lands in hole b*m + g2 of ITS block id b.  Ids of different instances
// never collide (id = g2 mod m), the table is the same on every worker, no block is
// moved twice and no memory beyond the pool is needed.
//
// Kernels (no host round trip):
//   merge_check_kernel    one workgroup: validates every sequence length of every instance.
//   merge_clear_kernel    clears one flag per new block id of the pool.
//   merge_table_kernel    one lane per cell of the merged table: new id = old*m + g2,
//                         range check, and flag[id] = 1 if the block is remote.
//   merge_count / offsets / scatter
//                         stream compaction of the flags into the ascending list of new
//                         ids to fill: per-chunk counts by wavefront ballots, a scan of
//                         the counts, then ballot-prefix scatter.  Ascending ids matter:
//                         block b of instance g2 is read at pool offset ~b and written
//                         at offset ~b as well, so both sides sweep their pools
//                         monotonically; in table order (random ids) the scattered
//                         16-64 KiB writes cost 12-25 % of the rate.
//   merge_copy_kernel     one wavefront per 1 KiB tile of a remote sub-block, layer on
//                         grid.y, 16 bytes per lane, non-temporal.
#include <algorithm>
#include <string>

#include "device_common.h"
#include "grid.h"
#include "launch.h"
#include "plan.h"

namespace amoeba {

constexpr int kWide = 1024;  // lanes of the single-workgroup and per-chunk kernels
constexpr int kWideWaves = kWide / 64;

struct MergeInputs {
  const int32_t* lens[AMOEBA_MAX_TP];
  const int32_t* tables[AMOEBA_MAX_TP];
};

__global__ void __launch_bounds__(kWide)
merge_check_kernel(const MergeInputs in, uint32_t n_inst, FastDiv seqs, uint32_t row_width,
                   uint32_t block_tokens, int32_t* __restrict__ ws) {
  __shared__ unsigned int err_s;
  if (threadIdx.x == 0) err_s = 0;
  __syncthreads();
  const uint32_t n = n_inst * seqs.d;
  unsigned int e = 0;
  for (uint32_t i = threadIdx.x; i < n; i += kWide) {
    const uint32_t inst = fd_div(i, seqs);
    const long long len = in.lens[inst][i - inst * seqs.d];
    if (len < 0) e |= kErrNegativeLen;
    else if ((len + block_tokens - 1) / block_tokens > (long long)row_width) e |= kErrRowTooShort;
  }
  if (e) atomicOr(&err_s, e);
  __syncthreads();
  if (threadIdx.x == 0) {
    ws[kWsTotal] = 0;
    ws[kWsError] = (int32_t)err_s;
  }
}

__global__ void __launch_bounds__(kThreads)
merge_clear_kernel(int32_t* __restrict__ flags, uint32_t n) {
  const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) flags[i] = 0;
}

__global__ void __launch_bounds__(kThreads)
merge_table_kernel(const MergeInputs in, int32_t* __restrict__ dst_table, uint32_t n_inst,
                   uint32_t local_inst, FastDiv seqs, FastDiv row_width, uint32_t block_tokens,
                   int64_t pool_blocks, int32_t* __restrict__ ws, int32_t* __restrict__ flags) {
  const uint64_t cell = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
  const uint64_t cells = uint64_t(n_inst) * seqs.d * row_width.d;
  if (cell >= cells) return;
  const uint32_t row = fd_div(uint32_t(cell), row_width);  // merged sequence index
  const uint32_t j = uint32_t(cell) - row * row_width.d;
  const uint32_t inst = fd_div(row, seqs);
  const uint32_t i = row - inst * seqs.d;
  const bool failed = (ws[kWsError] & (kErrNegativeLen | kErrRowTooShort)) != 0;
  int32_t out = -1;
  if (!failed) {
    const long long len = in.lens[inst][i];
    const long long nb = (len + block_tokens - 1) / block_tokens;
    if ((long long)j < nb) {
      const int32_t b = in.tables[inst][uint64_t(i) * row_width.d + j];
      if (b < 0 || (int64_t)b >= pool_blocks) {
        atomicOr(reinterpret_cast<unsigned int*>(ws + kWsError), (unsigned int)kErrBlockId);
      } else {
        out = b * (int32_t)n_inst + (int32_t)inst;  // < pool_blocks * m <= INT32_MAX (plan check)
        if (inst != local_inst) flags[out] = 1;
      }
    }
  }
  dst_table[cell] = out;
}

// Number of set flags in each chunk of kWide new-block ids.
__global__ void __launch_bounds__(kWide)
merge_count_kernel(const int32_t* __restrict__ flags, uint32_t n, int32_t* __restrict__ counts) {
  __shared__ int wave_count[kWideWaves];
  const uint32_t i = blockIdx.x * kWide + threadIdx.x;
  const bool f = i < n && flags[i] != 0;
  const unsigned long long mask = __ballot(f);
  if ((threadIdx.x & 63) == 0) wave_count[threadIdx.x >> 6] = __popcll(mask);
  __syncthreads();
  if (threadIdx.x == 0) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < kWideWaves; ++w) c += wave_count[w];
    counts[blockIdx.x] = c;
  }
}

// Exclusive scan of the chunk counts, in place; the grand total goes to the header.
__global__ void __launch_bounds__(kWide)
merge_offsets_kernel(int32_t* __restrict__ counts, uint32_t n_chunks, int32_t* __restrict__ ws) {
  __shared__ int wave_total[kWideWaves];
  __shared__ int carry_s;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (uint32_t c0 = 0; c0 < n_chunks; c0 += kWide) {
    const uint32_t i = c0 + tid;
    const int v = i < n_chunks ? counts[i] : 0;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off, 64);
      if (lane >= (uint32_t)off) incl += up;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int before = 0, chunk = 0;
#pragma unroll
    for (int w = 0; w < kWideWaves; ++w) {
      const int t = wave_total[w];
      if ((uint32_t)w < wave) before += t;
      chunk += t;
    }
    const int carry = carry_s;
    if (i < n_chunks) counts[i] = carry + before + incl - v;
    __syncthreads();
    if (tid == 0) carry_s = carry + chunk;
    __syncthreads();
  }
  if (tid == 0) {
    const bool failed = (ws[kWsError] & (kErrNegativeLen | kErrRowTooShort)) != 0;
    ws[kWsTotal] = failed ? 0 : carry_s;
  }
}

// worklist[rank of id among the set flags] = id, ascending.
__global__ void __launch_bounds__(kWide)
merge_scatter_kernel(const int32_t* __restrict__ flags, uint32_t n,
                     const int32_t* __restrict__ offsets, int32_t* __restrict__ worklist) {
  __shared__ int wave_count[kWideWaves];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t i = blockIdx.x * kWide + tid;
  const bool f = i < n && flags[i] != 0;
  const unsigned long long mask = __ballot(f);
  if (lane == 0) wave_count[wave] = __popcll(mask);
  __syncthreads();
  if (!f) return;
  int pos = offsets[blockIdx.x] + __popcll(mask & ((1ull << lane) - 1ull));
#pragma unroll
  for (int w = 0; w < kWideWaves; ++w)
    if ((uint32_t)w < wave) pos += wave_count[w];
  worklist[pos] = (int32_t)i;
}

struct MergeCopyArgs {
  const char* remote[AMOEBA_MAX_TP];
  char* local;
  uint64_t layer_stride;     // bytes between layers of a pool (same geometry everywhere)
  uint64_t old_block_bytes;  // m * sub_bytes
  uint64_t sub_bytes;        // one new block
  uint32_t sub_vecs;
  uint32_t local_inst;
  FastDiv n_inst;
  FastDiv tiles_per_sub;
};

// WAVES wavefronts per workgroup, each with a tile of its own: the tile shape stays one
// wavefront per 1 KiB while the number of workgroups to dispatch drops by WAVES.
template <int VEC, bool NT, int WAVES>
__global__ void __launch_bounds__(64 * WAVES)
merge_copy_kernel(const MergeCopyArgs a, const int32_t* __restrict__ ws,
                  const int32_t* __restrict__ worklist) {
  using V = typename VecOf<VEC>::type;
  const uint32_t layer = blockIdx.y;
  const uint32_t total = (uint32_t)ws[kWsTotal];
  const uint32_t n_items = total * a.tiles_per_sub.d;
  const uint32_t wave = WAVES > 1 ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) : 0;
  // (the XCD-chunked order of xcd_item() measured no different here: the sources are
  // several pools already and the ids ascend)
  for (uint32_t w = blockIdx.x * WAVES + wave; w < n_items; w += gridDim.x * WAVES) {
    const uint32_t n = fd_div(w, a.tiles_per_sub);
    const uint32_t tile = w - n * a.tiles_per_sub.d;
    const uint32_t id = (uint32_t)worklist[n];  // new block id = old id * m + instance
    const uint32_t sb = fd_div(id, a.n_inst);
    const uint32_t inst = id - sb * a.n_inst.d;
    const uint32_t v = tile * 64 + (threadIdx.x & 63);
    if (v >= a.sub_vecs) continue;
    const uint64_t lo = uint64_t(layer) * a.layer_stride;
    const char* from = a.remote[inst] + lo + uint64_t(sb) * a.old_block_bytes +
                       uint64_t(a.local_inst) * a.sub_bytes + uint64_t(v) * VEC;
    char* to = a.local + lo + uint64_t(id) * a.sub_bytes + uint64_t(v) * VEC;
    st<NT, V>(to, ld<NT, V>(from));
  }
}

namespace {

bool launched(const char* what, std::string* err) {
  const hipError_t rc = hipGetLastError();
  if (rc == hipSuccess) return true;
  *err = std::string(what) + ": " + hipGetErrorString(rc);
  return false;
}

template <int VEC>
void launch_copy(bool nt, int waves, dim3 grid, hipStream_t stream, const MergeCopyArgs& a,
                 const int32_t* ws, const int32_t* worklist) {
  if (waves == 4) {
    grid.x = (grid.x + 3) / 4;
    if (nt)
      hipLaunchKernelGGL((merge_copy_kernel<VEC, true, 4>), grid, dim3(256), 0, stream, a, ws,
                         worklist);
    else
      hipLaunchKernelGGL((merge_copy_kernel<VEC, false, 4>), grid, dim3(256), 0, stream, a, ws,
                         worklist);
  } else {
    if (nt)
      hipLaunchKernelGGL((merge_copy_kernel<VEC, true, 1>), grid, dim3(64), 0, stream, a, ws,
                         worklist);
    else
      hipLaunchKernelGGL((merge_copy_kernel<VEC, false, 1>), grid, dim3(64), 0, stream, a, ws,
                         worklist);
  }
}

}  // namespace

namespace {

struct MergeLaunch {
  uint64_t tiles;   // 1 KiB tiles of one new block
  uint32_t grid_x;  // tiles the grid covers per layer (launch_copy packs `waves` per workgroup)
  int waves;        // wavefronts per workgroup
};

// One wavefront per tile.  The number of remote blocks is only known on the device, so
// the grid covers the pool's capacity unless the caller gave a bound on the blocks in use
// (amoeba_model_shape.kv_blocks_bound); past the grid, workgroups stride.
bool merge_launch_shape(const amoeba_plan_s* p, int vec, MergeLaunch* out, std::string* err) {
  const amoeba_model_shape& s = p->shape;
  const uint64_t m = uint64_t(p->merge_factor);
  const uint64_t slots = uint64_t(s.src_pool_blocks) * m;
  const uint64_t sub_vecs = uint64_t(p->block_bytes_dst) / uint64_t(vec);
  const uint64_t tiles = (sub_vecs + 63) / 64;
  const uint64_t max_items = slots * tiles;
  // item ids are 32-bit and a striding workgroup adds the grid size (at most 2^27) to one
  if (sub_vecs >= (uint64_t(1) << 32) - 64 || max_items >= (uint64_t(1) << 31) ||
      s.kv_layers > 65535) {
    *err = "KV pool too large for 32-bit work indexing";
    return false;
  }
  const int64_t bound = p->tune.kv_blocks_hint > 0 ? p->tune.kv_blocks_hint : s.kv_blocks_bound;
  uint64_t grid = std::max<uint64_t>(uint64_t(1) << 16, (uint64_t(1) << 27) / uint64_t(s.kv_layers));
  if (p->tune.kv_grid > 0) grid = uint64_t(p->tune.kv_grid);
  if (bound > 0) grid = std::min<uint64_t>(grid, std::max<uint64_t>(1, uint64_t(bound) * tiles));
  grid = std::min<uint64_t>(grid, max_items);
  // one wavefront per workgroup when the grid is tight, four when it covers the capacity
  out->waves = p->tune.kv_threads == 256 ? 4 : p->tune.kv_threads == 64 ? 1 : (bound > 0 ? 1 : 4);
  out->tiles = tiles;
  out->grid_x = clamp_grid_x(std::max<uint64_t>(grid, 1), 64u);  // in tiles; <= 2^26 workgroups
  return true;
}

}  // namespace

bool merge_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                           std::string* err) {
  if (p->merge_factor < 2) { *err = "the plan is not an in-place merge"; return false; }
  MergeLaunch L;
  const int vec = common_alignment(uint64_t(p->block_bytes_dst) | uint64_t(align_bytes));
  if (!merge_launch_shape(p, vec, &L, err)) return false;
  out->grid_x = L.waves == 4 ? (L.grid_x + 3) / 4 : L.grid_x;
  out->grid_y = uint32_t(p->shape.kv_layers);
  out->threads = uint32_t(64 * L.waves);
  out->items = uint64_t(p->shape.src_pool_blocks) * uint64_t(p->merge_factor) * L.tiles;
  return true;
}

size_t merge_workspace_ints(int64_t pool_blocks, int m) {
  const size_t slots = size_t(pool_blocks) * size_t(m);
  return size_t(kWsHeader) + (slots + kWide - 1) / kWide + 1 + 2 * slots;
}

int launch_merge_kv_inplace(const amoeba_plan_s* p, void* local_pool,
                            const void* const* remote_pools,
                            const int32_t* const* src_block_tables,
                            const int32_t* const* seq_lens, int32_t* dst_block_tables,
                            hipStream_t stream, std::string* err) {
  const amoeba_model_shape& s = p->shape;
  if (p->merge_factor < 2) {
    *err = "the plan is not an in-place merge (needs dst_tp = m * src_tp, m >= 2, header-centric "
           "layout on both sides, src_pool_blocks * m < 2^31)";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (!p->merge_workspace) {
    *err = "the plan has no device workspace (it was created without a GPU)";
    return AMOEBA_ERR_HIP;
  }
  int current_device = -1;
  if (hipGetDevice(&current_device) != hipSuccess || current_device != p->device) {
    *err = "the current device is not the one the plan's workspace was allocated on";
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint32_t m = uint32_t(p->merge_factor), g = uint32_t(p->rp) % m;
  const uint64_t S = uint64_t(s.num_seqs), W = uint64_t(s.max_blocks_per_seq);
  const uint64_t cells = uint64_t(m) * S * W;
  if (cells >= (uint64_t(1) << 32) - kThreads) {
    *err = "merged block table has 2^32 cells or more";
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint64_t layer_stride = uint64_t(s.src_pool_blocks) * uint64_t(p->block_bytes_src);
  const uint64_t pool_bytes = layer_stride * uint64_t(s.kv_layers);
  const uint64_t l0 = reinterpret_cast<uint64_t>(local_pool);
  if (!l0 && pool_bytes) { *err = "local_pool is NULL"; return AMOEBA_ERR_INVALID_ARG; }
  MergeInputs in;
  MergeCopyArgs a;
  uint64_t bits = l0 | uint64_t(p->block_bytes_dst);
  for (uint32_t i = 0; i < AMOEBA_MAX_TP; ++i) {
    in.lens[i] = in.tables[i] = nullptr;
    a.remote[i] = nullptr;
  }
  for (uint32_t i = 0; i < m; ++i) {
    if (S && (!seq_lens || !seq_lens[i])) { *err = "a seq_lens pointer is NULL"; return AMOEBA_ERR_INVALID_ARG; }
    if (cells && (!src_block_tables || !src_block_tables[i] || !dst_block_tables)) {
      *err = "a block table pointer is NULL";
      return AMOEBA_ERR_INVALID_ARG;
    }
    in.lens[i] = S ? seq_lens[i] : nullptr;
    in.tables[i] = cells ? src_block_tables[i] : nullptr;
    if (i == g) continue;
    const uint64_t r0 = reinterpret_cast<uint64_t>(remote_pools ? remote_pools[i] : nullptr);
    if (!r0 && pool_bytes) { *err = "a remote pool pointer is NULL"; return AMOEBA_ERR_INVALID_ARG; }
    if (r0 < l0 + pool_bytes && l0 < r0 + pool_bytes) {
      *err = "a remote pool overlaps the local pool";
      return AMOEBA_ERR_INVALID_ARG;
    }
    bits |= r0;
    a.remote[i] = reinterpret_cast<const char*>(r0);
  }
  const int vec = common_alignment(bits);
  const bool nt = p->tune.nontemporal != 2;
  const uint32_t slots = uint32_t(uint64_t(s.src_pool_blocks) * m);  // new block ids of the pool
  const uint32_t n_chunks = (slots + kWide - 1) / kWide;
  int32_t* ws = p->merge_workspace;
  int32_t* counts = ws + kWsHeader;
  int32_t* flags = counts + n_chunks + 1;
  int32_t* worklist = flags + slots;

  hipLaunchKernelGGL(merge_check_kernel, dim3(1), dim3(kWide), 0, stream, in, m,
                     make_fastdiv(uint32_t(std::max<uint64_t>(S, 1))), uint32_t(W),
                     uint32_t(s.kv_block_tokens), ws);
  if (!launched("merge check kernel launch failed", err)) return AMOEBA_ERR_HIP;
  if (cells == 0 || slots == 0) return AMOEBA_OK;
  hipLaunchKernelGGL(merge_clear_kernel, dim3((slots + kThreads - 1) / kThreads), dim3(kThreads),
                     0, stream, flags, slots);
  hipLaunchKernelGGL(merge_table_kernel, dim3(uint32_t((cells + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, stream, in, dst_block_tables, m, g,
                     make_fastdiv(uint32_t(S)), make_fastdiv(uint32_t(W)),
                     uint32_t(s.kv_block_tokens), int64_t(s.src_pool_blocks), ws, flags);
  hipLaunchKernelGGL(merge_count_kernel, dim3(n_chunks), dim3(kWide), 0, stream, flags, slots,
                     counts);
  hipLaunchKernelGGL(merge_offsets_kernel, dim3(1), dim3(kWide), 0, stream, counts, n_chunks, ws);
  hipLaunchKernelGGL(merge_scatter_kernel, dim3(n_chunks), dim3(kWide), 0, stream, flags, slots,
                     counts, worklist);
  if (!launched("merge table/compaction kernel launch failed", err)) return AMOEBA_ERR_HIP;

  a.local = static_cast<char*>(local_pool);
  a.layer_stride = layer_stride;
  a.old_block_bytes = uint64_t(p->block_bytes_src);
  a.sub_bytes = uint64_t(p->block_bytes_dst);
  a.sub_vecs = uint32_t(a.sub_bytes / uint64_t(vec));
  a.n_inst = make_fastdiv(m);
  a.local_inst = g;
  MergeLaunch L;
  if (!merge_launch_shape(p, vec, &L, err)) return AMOEBA_ERR_INVALID_ARG;
  a.tiles_per_sub = make_fastdiv(uint32_t(L.tiles));
  const dim3 gr(L.grid_x, uint32_t(s.kv_layers));
  const int waves = L.waves;
  switch (vec) {
    case 16: launch_copy<16>(nt, waves, gr, stream, a, ws, worklist); break;
    case 8: launch_copy<8>(nt, waves, gr, stream, a, ws, worklist); break;
    case 4: launch_copy<4>(nt, waves, gr, stream, a, ws, worklist); break;
    case 2: launch_copy<2>(nt, waves, gr, stream, a, ws, worklist); break;
    default: launch_copy<1>(nt, waves, gr, stream, a, ws, worklist); break;
  }
  if (!launched("merge copy kernel launch failed", err)) return AMOEBA_ERR_HIP;
  return AMOEBA_OK;
}

}  // namespace amoeba
