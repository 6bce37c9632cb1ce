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
//   merge_scan_kernel   one workgroup; blocks per sequence over all m*S sequences,
//                       wavefront scans joined through LDS, counting remote ones only
//                       -> position of every remote block in a flat work list.
//   merge_table_kernel  one lane per cell of the merged table: new id = old*m + g2,
//                       range check, work-list entry (source id, instance) if remote.
//   merge_copy_kernel   one wavefront per 1 KiB tile of a remote sub-block, layer on
//                       grid.y, 16 bytes per lane, non-temporal.
#include <algorithm>
#include <string>

#include "device_common.h"
#include "launch.h"
#include "plan.h"

namespace amoeba {

constexpr int kMergeScanThreads = 1024;
constexpr int kMergeScanWaves = kMergeScanThreads / 64;

struct MergeInputs {
  const int32_t* lens[AMOEBA_MAX_TP];
  const int32_t* tables[AMOEBA_MAX_TP];
};

__global__ void __launch_bounds__(kMergeScanThreads)
merge_scan_kernel(const MergeInputs in, uint32_t n_inst, uint32_t local_inst, FastDiv seqs,
                  uint32_t row_width, uint32_t block_tokens, int64_t max_remote,
                  int32_t* __restrict__ ws) {
  __shared__ long long wave_total[kMergeScanWaves];
  __shared__ long long carry_s;
  __shared__ unsigned int err_s;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t n = n_inst * seqs.d;
  int32_t* base = ws + kWsHeader;
  if (tid == 0) { carry_s = 0; err_s = 0; }
  __syncthreads();
  for (uint32_t c0 = 0; c0 < n; c0 += kMergeScanThreads) {
    const uint32_t i = c0 + tid;
    long long nb = 0;
    unsigned int e = 0;
    if (i < n) {
      const uint32_t inst = fd_div(i, seqs);
      const long long len = in.lens[inst][i - inst * seqs.d];
      if (len < 0) {
        e = kErrNegativeLen;
      } else {
        nb = (len + block_tokens - 1) / block_tokens;
        if (nb > (long long)row_width) e = kErrRowTooShort;
        if (inst == local_inst) nb = 0;  // local blocks stay where they are
      }
    }
    long long incl = nb;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const long long up = __shfl_up(incl, off, 64);
      if (lane >= (uint32_t)off) incl += up;
    }
    if (lane == 63) wave_total[wave] = incl;
    if (e) atomicOr(&err_s, e);
    __syncthreads();
    long long before = 0, chunk = 0;
#pragma unroll
    for (int wv = 0; wv < kMergeScanWaves; ++wv) {
      const long long t = wave_total[wv];
      if ((uint32_t)wv < wave) before += t;
      chunk += t;
    }
    const long long carry = carry_s;
    if (i < n) {
      const long long b = carry + before + incl - nb;
      base[i] = b > INT32_MAX ? INT32_MAX : (int32_t)b;
    }
    __syncthreads();
    if (tid == 0) carry_s = carry + chunk;
    __syncthreads();
  }
  if (tid == 0) {
    unsigned int e = err_s;
    const long long total = carry_s;
    if (total > max_remote) e |= kErrPoolTooSmall;  // only possible with repeated block ids
    ws[kWsTotal] = e ? 0 : (int32_t)total;
    ws[kWsError] = (int32_t)e;
  }
}

__global__ void __launch_bounds__(kThreads)
merge_table_kernel(const MergeInputs in, int32_t* __restrict__ dst_table, uint32_t n_inst,
                   uint32_t local_inst, FastDiv seqs, FastDiv row_width, uint32_t block_tokens,
                   int64_t pool_blocks, uint32_t max_remote, int32_t* __restrict__ ws) {
  const uint64_t cell = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
  const uint64_t cells = uint64_t(n_inst) * seqs.d * row_width.d;
  if (cell >= cells) return;
  const uint32_t row = fd_div(uint32_t(cell), row_width);  // merged sequence index
  const uint32_t j = uint32_t(cell) - row * row_width.d;
  const uint32_t inst = fd_div(row, seqs);
  const uint32_t i = row - inst * seqs.d;
  const bool failed = (ws[kWsError] & (kErrNegativeLen | kErrRowTooShort | kErrPoolTooSmall)) != 0;
  int32_t out = -1;
  if (!failed) {
    const long long len = in.lens[inst][i];
    const long long nb = (len + block_tokens - 1) / block_tokens;
    if ((long long)j < nb) {
      int32_t b = in.tables[inst][uint64_t(i) * row_width.d + j];
      if (b < 0 || (int64_t)b >= pool_blocks) {
        atomicOr(reinterpret_cast<unsigned int*>(ws + kWsError), (unsigned int)kErrBlockId);
        b = -1;
      } else {
        out = b * (int32_t)n_inst + (int32_t)inst;  // < pool_blocks * m <= INT32_MAX (host check)
      }
      if (inst != local_inst) {
        const uint32_t n = uint32_t(ws[kWsHeader + row]) + j;
        int32_t* wl = ws + kWsHeader + n_inst * seqs.d;
        wl[n] = b;
        wl[max_remote + n] = (int32_t)inst;
      }
    }
  }
  dst_table[cell] = out;
}

struct MergeCopyArgs {
  const char* remote[AMOEBA_MAX_TP];
  char* local;
  uint64_t layer_stride;     // bytes between layers of a pool (same geometry everywhere)
  uint64_t old_block_bytes;  // m * sub_bytes
  uint64_t sub_bytes;        // one new block
  uint32_t sub_vecs;
  uint32_t n_inst, local_inst, n_seqs_total, max_remote;
  FastDiv tiles_per_sub;
};

template <int VEC, bool NT>
__global__ void __launch_bounds__(64)
merge_copy_kernel(const MergeCopyArgs a, const int32_t* __restrict__ ws) {
  using V = typename VecOf<VEC>::type;
  const uint32_t layer = blockIdx.y;
  const uint32_t total = (uint32_t)ws[kWsTotal];
  const int32_t* __restrict__ wl = ws + kWsHeader + a.n_seqs_total;
  const uint32_t n_items = total * a.tiles_per_sub.d;
  for (uint32_t w = blockIdx.x; w < n_items; w += gridDim.x) {
    const uint32_t n = fd_div(w, a.tiles_per_sub);
    const uint32_t tile = w - n * a.tiles_per_sub.d;
    const int32_t sb = wl[n];
    const uint32_t inst = (uint32_t)wl[a.max_remote + n];
    const uint32_t v = tile * 64 + threadIdx.x;
    if (sb < 0 || v >= a.sub_vecs) continue;
    const uint64_t lo = uint64_t(layer) * a.layer_stride;
    const char* from = a.remote[inst] + lo + uint64_t(sb) * a.old_block_bytes +
                       uint64_t(a.local_inst) * a.sub_bytes + uint64_t(v) * VEC;
    char* to = a.local + lo + (uint64_t(sb) * a.n_inst + inst) * a.sub_bytes + uint64_t(v) * VEC;
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
void launch_copy(bool nt, dim3 grid, hipStream_t stream, const MergeCopyArgs& a,
                 const int32_t* ws) {
  if (nt) hipLaunchKernelGGL((merge_copy_kernel<VEC, true>), grid, dim3(64), 0, stream, a, ws);
  else hipLaunchKernelGGL((merge_copy_kernel<VEC, false>), grid, dim3(64), 0, stream, a, ws);
}

}  // namespace

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
  const uint32_t max_remote = uint32_t(uint64_t(s.src_pool_blocks) * m);

  hipLaunchKernelGGL(merge_scan_kernel, dim3(1), dim3(kMergeScanThreads), 0, stream, in, m, g,
                     make_fastdiv(uint32_t(std::max<uint64_t>(S, 1))), uint32_t(W),
                     uint32_t(s.kv_block_tokens), int64_t(max_remote), p->merge_workspace);
  if (!launched("merge scan kernel launch failed", err)) return AMOEBA_ERR_HIP;
  if (cells == 0) return AMOEBA_OK;
  hipLaunchKernelGGL(merge_table_kernel, dim3(uint32_t((cells + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, stream, in, dst_block_tables, m, g,
                     make_fastdiv(uint32_t(S)), make_fastdiv(uint32_t(W)),
                     uint32_t(s.kv_block_tokens), int64_t(s.src_pool_blocks), max_remote,
                     p->merge_workspace);
  if (!launched("merge table kernel launch failed", err)) return AMOEBA_ERR_HIP;

  a.local = static_cast<char*>(local_pool);
  a.layer_stride = layer_stride;
  a.old_block_bytes = uint64_t(p->block_bytes_src);
  a.sub_bytes = uint64_t(p->block_bytes_dst);
  a.sub_vecs = uint32_t(a.sub_bytes / uint64_t(vec));
  a.n_inst = m;
  a.local_inst = g;
  a.n_seqs_total = uint32_t(m * S);
  a.max_remote = max_remote;
  const uint64_t tiles = (uint64_t(a.sub_vecs) + 63) / 64;
  a.tiles_per_sub = make_fastdiv(uint32_t(tiles));
  const uint64_t max_items = uint64_t(max_remote) * tiles;
  if (a.sub_bytes / uint64_t(vec) >= (uint64_t(1) << 32) - 64 ||
      max_items >= (uint64_t(1) << 32) - (1 << 24) || s.kv_layers > 65535) {
    *err = "KV pool too large for 32-bit work indexing";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (max_items == 0) return AMOEBA_OK;
  uint64_t grid = std::max<uint64_t>(uint64_t(1) << 16, (uint64_t(1) << 27) / uint64_t(s.kv_layers));
  if (p->tune.kv_grid > 0) grid = uint64_t(p->tune.kv_grid);
  grid = std::min<uint64_t>(grid, max_items);
  const dim3 gr(uint32_t(grid), uint32_t(s.kv_layers));
  switch (vec) {
    case 16: launch_copy<16>(nt, gr, stream, a, p->merge_workspace); break;
    case 8: launch_copy<8>(nt, gr, stream, a, p->merge_workspace); break;
    case 4: launch_copy<4>(nt, gr, stream, a, p->merge_workspace); break;
    case 2: launch_copy<2>(nt, gr, stream, a, p->merge_workspace); break;
    default: launch_copy<1>(nt, gr, stream, a, p->merge_workspace); break;
  }
  if (!launched("merge copy kernel launch failed", err)) return AMOEBA_ERR_HIP;
  return AMOEBA_OK;
}

}  // namespace amoeba
