// KV cache reshard: sequence scan, block-table rewrite and block regroup by head.
//
// What it computes (paper Sec. 3.1).  When the TP degree changes, the KV cache of
// every token is redistributed by attention head: rank r of a TP group owns the
// contiguous head range [r*H/TP, (r+1)*H/TP).  The target rank therefore gathers,
// for every block in use, its heads from the source ranks that own them, and the
// blocks get new, compact ids (an exclusive prefix sum of blocks per sequence, in
// sequence order).  Two block layouts are understood on either side: the
// header-centric one ([head][K/V][token][d]) whose head sub-ranges are contiguous,
// and the token-first one ([K/V][token][head][d]).
//
// Three kernels, no host round trip:
//   kv_scan_kernel   one workgroup; nb_i = ceil(len_i / B), wavefront-level
//                    inclusive scans joined through LDS, carried across chunks of
//                    1024 sequences; validates lengths / row width / pool size.
//   kv_table_kernel  one lane per table cell: writes the new table and a flat list
//                    "new block id -> source block id" (ids range-checked here).
//   kv_regroup_kernel persistent workgroups stride over work items
//                    (layer group, new block, tile); a tile is a run of 16-byte
//                    vectors contiguous in the destination block.  A lane turns its
//                    vector index into (head, K/V*token, d-offset) for the
//                    destination layout with multiply-high divisions, maps the head
//                    to (source rank, local head) and rebuilds the index for the
//                    source layout.  All loads of a tile are issued before its
//                    stores; accesses are 16 bytes per lane and non-temporal.
#include <algorithm>
#include <string>

#include "device_common.h"
#include "launch.h"
#include "plan.h"

namespace amoeba {

constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;

__global__ void __launch_bounds__(kScanThreads)
kv_scan_kernel(const int32_t* __restrict__ seq_lens, uint32_t num_seqs, uint32_t row_width,
               uint32_t block_tokens, int64_t dst_pool_blocks, int32_t* __restrict__ ws) {
  __shared__ long long wave_total[kScanWaves];
  __shared__ long long carry_s;
  __shared__ unsigned int err_s;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t* base = ws + kWsHeader;
  if (tid == 0) { carry_s = 0; err_s = 0; }
  __syncthreads();

  for (uint32_t c0 = 0; c0 < num_seqs; c0 += kScanThreads) {
    const uint32_t i = c0 + tid;
    long long nb = 0;
    unsigned int e = 0;
    if (i < num_seqs) {
      const long long len = seq_lens[i];
      if (len < 0) {
        e = kErrNegativeLen;
      } else {
        nb = (len + block_tokens - 1) / block_tokens;
        if (nb > (long long)row_width) e = kErrRowTooShort;
      }
    }
    long long incl = nb;  // inclusive scan inside the wavefront
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
    for (int wv = 0; wv < kScanWaves; ++wv) {
      const long long t = wave_total[wv];
      if ((uint32_t)wv < wave) before += t;
      chunk += t;
    }
    const long long carry = carry_s;
    if (i < num_seqs) {
      const long long b = carry + before + incl - nb;
      base[i] = b > INT32_MAX ? INT32_MAX : (int32_t)b;  // only reachable on an error path
    }
    __syncthreads();
    if (tid == 0) carry_s = carry + chunk;
    __syncthreads();
  }
  if (tid == 0) {
    unsigned int e = err_s;
    const long long total = carry_s;
    if (total > dst_pool_blocks) e |= kErrPoolTooSmall;
    ws[kWsTotal] = e ? 0 : (int32_t)total;
    ws[kWsError] = (int32_t)e;
  }
}

__global__ void __launch_bounds__(kThreads)
kv_table_kernel(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ src_table,
                int32_t* __restrict__ dst_table, uint32_t num_seqs, FastDiv row_width,
                uint32_t block_tokens, int64_t src_pool_blocks, int32_t* __restrict__ ws) {
  const uint64_t cell = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
  const uint64_t cells = uint64_t(num_seqs) * row_width.d;
  if (cell >= cells) return;
  const uint32_t i = fd_div(uint32_t(cell), row_width);  // cells < 2^32 is checked on the host
  const uint32_t j = uint32_t(cell) - i * row_width.d;
  const bool failed = (ws[kWsError] & (kErrNegativeLen | kErrRowTooShort | kErrPoolTooSmall)) != 0;
  int32_t out = -1;
  if (!failed) {
    const long long len = seq_lens[i];
    const long long nb = (len + block_tokens - 1) / block_tokens;
    if ((long long)j < nb) {
      out = ws[kWsHeader + i] + (int32_t)j;
      int32_t sb = src_table[cell];
      if (sb < 0 || (int64_t)sb >= src_pool_blocks) {
        atomicOr(reinterpret_cast<unsigned int*>(ws + kWsError), (unsigned int)kErrBlockId);
        sb = -1;
      }
      ws[kWsHeader + num_seqs + out] = sb;
    }
  }
  dst_table[cell] = out;
}

struct KVArgs {
  const char* src[AMOEBA_MAX_TP];
  char* dst;
  const int32_t* ws;
  uint64_t src_layer_stride, dst_layer_stride;  // bytes between layers of a pool
  uint64_t src_block_bytes, dst_block_bytes;
  uint32_t num_seqs;
  uint32_t layers, layers_per_item, layer_groups;
  uint32_t block_vecs;       // vectors in one destination block
  FastDiv tiles_per_block;
  uint32_t head0;            // first global head the target rank owns
  FastDiv heads_src;         // heads per source rank
  FastDiv heads_dst;         // heads per target rank
  FastDiv head_vecs;         // vectors of one head in a header-centric block: 2 * B * dv
  FastDiv dv;                // vectors of one head vector (d * elem_bytes / VEC)
};

template <int SL, int DL, int VEC, int UNROLL, bool NT>
__global__ void __launch_bounds__(kThreads) kv_regroup_kernel(const KVArgs a) {
  using V = typename VecOf<VEC>::type;
  constexpr uint32_t kTileVecs = kThreads * UNROLL;
  __shared__ const char* src_s[AMOEBA_MAX_TP];
  const uint32_t tid = threadIdx.x;
  if (tid < AMOEBA_MAX_TP) src_s[tid] = a.src[tid];
  __syncthreads();

  const uint32_t total = (uint32_t)a.ws[kWsTotal];
  const int32_t* worklist = a.ws + kWsHeader + a.num_seqs;
  const uint32_t per_group = total * a.tiles_per_block.d;
  const uint32_t n_items = per_group * a.layer_groups;  // < 2^32, bounded on the host

  for (uint32_t w = blockIdx.x; w < n_items; w += gridDim.x) {
    const uint32_t lg = w / per_group;
    const uint32_t r = w - lg * per_group;
    const uint32_t b = fd_div(r, a.tiles_per_block);
    const uint32_t tile = r - b * a.tiles_per_block.d;
    const int32_t sb = worklist[b];
    if (sb < 0) continue;  // source id was out of range: leave the block alone

    const char* sp[UNROLL];
    uint32_t dvec[UNROLL];
    bool live[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const uint32_t v = tile * kTileVecs + u * kThreads + tid;
      live[u] = v < a.block_vecs;
      dvec[u] = v;
      uint32_t hp, within, ct = 0, x = 0;  // within: index inside one header-centric head
      if (DL == AMOEBA_KV_HEAD_MAJOR) {
        hp = fd_div(v, a.head_vecs);
        within = v - hp * a.head_vecs.d;
        if (SL != AMOEBA_KV_HEAD_MAJOR) {
          ct = fd_div(within, a.dv);
          x = within - ct * a.dv.d;
        }
      } else {
        const uint32_t q = fd_div(v, a.dv);
        x = v - q * a.dv.d;
        ct = fd_div(q, a.heads_dst);
        hp = q - ct * a.heads_dst.d;
        within = ct * a.dv.d + x;
      }
      const uint32_t h = a.head0 + hp;
      const uint32_t s = fd_div(h, a.heads_src);
      const uint32_t hs = h - s * a.heads_src.d;
      const uint32_t svec = (SL == AMOEBA_KV_HEAD_MAJOR)
                                ? hs * a.head_vecs.d + within
                                : (ct * a.heads_src.d + hs) * a.dv.d + x;
      sp[u] = src_s[live[u] ? s : 0] + uint64_t(sb) * a.src_block_bytes + uint64_t(svec) * VEC;
    }
    char* dp = a.dst + uint64_t(b) * a.dst_block_bytes;

    const uint32_t l0 = lg * a.layers_per_item;
    const uint32_t l1 = min(a.layers, l0 + a.layers_per_item);
    for (uint32_t l = l0; l < l1; ++l) {
      const uint64_t so = uint64_t(l) * a.src_layer_stride, dof = uint64_t(l) * a.dst_layer_stride;
      V val[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (live[u]) val[u] = ld<NT, V>(sp[u] + so);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (live[u]) st<NT, V>(dp + dof + uint64_t(dvec[u]) * VEC, val[u]);
    }
  }
}

namespace {

template <int SL, int DL, int VEC, int UNROLL>
void launch_nt(bool nt, dim3 grid, hipStream_t stream, const KVArgs& a) {
  if (nt)
    hipLaunchKernelGGL((kv_regroup_kernel<SL, DL, VEC, UNROLL, true>), grid, dim3(kThreads), 0,
                       stream, a);
  else
    hipLaunchKernelGGL((kv_regroup_kernel<SL, DL, VEC, UNROLL, false>), grid, dim3(kThreads), 0,
                       stream, a);
}

template <int SL, int DL>
void launch_vec(int vec, int unroll, bool nt, dim3 grid, hipStream_t stream, const KVArgs& a) {
  if (vec == 16) {
    switch (unroll) {
      case 1: launch_nt<SL, DL, 16, 1>(nt, grid, stream, a); break;
      case 2: launch_nt<SL, DL, 16, 2>(nt, grid, stream, a); break;
      case 8: launch_nt<SL, DL, 16, 8>(nt, grid, stream, a); break;
      default: launch_nt<SL, DL, 16, 4>(nt, grid, stream, a); break;
    }
  } else if (vec == 8) {
    launch_nt<SL, DL, 8, 4>(nt, grid, stream, a);
  } else if (vec == 4) {
    launch_nt<SL, DL, 4, 4>(nt, grid, stream, a);
  } else if (vec == 2) {
    launch_nt<SL, DL, 2, 4>(nt, grid, stream, a);
  } else {
    launch_nt<SL, DL, 1, 4>(nt, grid, stream, a);
  }
}

bool hip_ok(const char* what, std::string* err) {
  const hipError_t rc = hipGetLastError();
  if (rc == hipSuccess) return true;
  *err = std::string(what) + ": " + hipGetErrorString(rc);
  return false;
}

}  // namespace

int launch_reshard_kv(const amoeba_plan_s* p, const void* const* src_blocks,
                      const int32_t* src_block_tables, const int32_t* seq_lens, void* dst_blocks,
                      int32_t* dst_block_tables, hipStream_t stream, std::string* err) {
  const amoeba_model_shape& s = p->shape;
  if (!p->workspace) {
    *err = "the plan has no device workspace (it was created without a GPU)";
    return AMOEBA_ERR_HIP;
  }
  const uint64_t cells = uint64_t(s.num_seqs) * uint64_t(s.max_blocks_per_seq);
  if (cells >= (uint64_t(1) << 32) - kThreads) {
    *err = "block table has 2^32 cells or more";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (cells && (!src_block_tables || !seq_lens || !dst_block_tables)) {
    *err = "table or length pointer is NULL";
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint64_t src_layer = uint64_t(s.src_pool_blocks) * p->block_bytes_src,
                 dst_layer = uint64_t(s.dst_pool_blocks) * p->block_bytes_dst;
  const uint64_t src_bytes = src_layer * s.kv_layers, dst_bytes = dst_layer * s.kv_layers;
  const uint64_t d0 = reinterpret_cast<uint64_t>(dst_blocks);
  if (!d0 && dst_bytes) { *err = "dst_blocks is NULL"; return AMOEBA_ERR_INVALID_ARG; }

  const uint64_t head_vec_bytes = uint64_t(s.head_dim) * s.elem_bytes;
  uint64_t bits = head_vec_bytes | d0;
  KVArgs a;
  for (int r = 0; r < AMOEBA_MAX_TP; ++r) a.src[r] = nullptr;
  for (int r = 0; r < p->k; ++r) {
    if (!(p->kv_rank_mask >> r & 1)) continue;
    const uint64_t s0 = reinterpret_cast<uint64_t>(src_blocks[r]);
    if (!s0 && src_bytes) { *err = "a needed source pool pointer is NULL"; return AMOEBA_ERR_INVALID_ARG; }
    if (s0 < d0 + dst_bytes && d0 < s0 + src_bytes) {
      *err = "dst_blocks overlaps a source pool (the regroup is out of place)";
      return AMOEBA_ERR_INVALID_ARG;
    }
    bits |= s0;
    a.src[r] = static_cast<const char*>(src_blocks[r]);
  }
  const int vec = common_alignment(bits);
  int unroll = p->tune.kv_unroll;
  if (vec != 16 || (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8)) unroll = 4;
  const bool nt = p->tune.nontemporal != 2;

  // 1. scan
  hipLaunchKernelGGL(kv_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, seq_lens,
                     uint32_t(s.num_seqs), uint32_t(s.max_blocks_per_seq),
                     uint32_t(s.kv_block_tokens), int64_t(s.dst_pool_blocks), p->workspace);
  if (!hip_ok("kv scan kernel launch failed", err)) return AMOEBA_ERR_HIP;
  // 2. tables
  if (cells) {
    const uint32_t grid = uint32_t((cells + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(kv_table_kernel, dim3(grid), dim3(kThreads), 0, stream, seq_lens,
                       src_block_tables, dst_block_tables, uint32_t(s.num_seqs),
                       make_fastdiv(uint32_t(s.max_blocks_per_seq)), uint32_t(s.kv_block_tokens),
                       int64_t(s.src_pool_blocks), p->workspace);
    if (!hip_ok("kv table kernel launch failed", err)) return AMOEBA_ERR_HIP;
  }
  // 3. regroup
  const uint64_t block_vecs = uint64_t(p->block_bytes_dst) / vec;
  const uint64_t tile_vecs = uint64_t(kThreads) * unroll;
  const uint64_t tiles_per_block = (block_vecs + tile_vecs - 1) / tile_vecs;
  uint32_t lpi = p->tune.kv_layers > 0 ? uint32_t(p->tune.kv_layers) : 1;
  lpi = std::min<uint32_t>(lpi, uint32_t(s.kv_layers));
  const uint32_t groups = (uint32_t(s.kv_layers) + lpi - 1) / lpi;
  const uint64_t max_items = uint64_t(s.dst_pool_blocks) * tiles_per_block * groups;
  if (block_vecs >= (uint64_t(1) << 32) - 65536 || max_items >= (uint64_t(1) << 32)) {
    *err = "KV pool too large for 32-bit work indexing";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (max_items == 0 || cells == 0) return AMOEBA_OK;
  a.dst = static_cast<char*>(dst_blocks);
  a.ws = p->workspace;
  a.src_layer_stride = src_layer;
  a.dst_layer_stride = dst_layer;
  a.src_block_bytes = uint64_t(p->block_bytes_src);
  a.dst_block_bytes = uint64_t(p->block_bytes_dst);
  a.num_seqs = uint32_t(s.num_seqs);
  a.layers = uint32_t(s.kv_layers);
  a.layers_per_item = lpi;
  a.layer_groups = groups;
  a.block_vecs = uint32_t(block_vecs);
  a.tiles_per_block = make_fastdiv(uint32_t(tiles_per_block));
  a.head0 = uint32_t(p->rp * p->heads_dst);
  a.heads_src = make_fastdiv(uint32_t(p->heads_src));
  a.heads_dst = make_fastdiv(uint32_t(p->heads_dst));
  const uint32_t dv = uint32_t(head_vec_bytes / vec);
  a.dv = make_fastdiv(dv);
  a.head_vecs = make_fastdiv(uint32_t(2u * uint32_t(s.kv_block_tokens) * dv));

  uint64_t grid = uint64_t(p->n_cu > 0 ? p->n_cu : 256) * 8;
  if (p->tune.kv_grid > 0) grid = uint64_t(p->tune.kv_grid);
  grid = std::min<uint64_t>(grid, max_items);
  const dim3 g{uint32_t(grid)};
  const bool sh = s.kv_layout_src == AMOEBA_KV_HEAD_MAJOR, dh = s.kv_layout_dst == AMOEBA_KV_HEAD_MAJOR;
  if (sh && dh)
    launch_vec<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_HEAD_MAJOR>(vec, unroll, nt, g, stream, a);
  else if (sh && !dh)
    launch_vec<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_TOKEN_MAJOR>(vec, unroll, nt, g, stream, a);
  else if (!sh && dh)
    launch_vec<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_HEAD_MAJOR>(vec, unroll, nt, g, stream, a);
  else
    launch_vec<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_TOKEN_MAJOR>(vec, unroll, nt, g, stream, a);
  if (!hip_ok("kv regroup kernel launch failed", err)) return AMOEBA_ERR_HIP;
  return AMOEBA_OK;
}

}  // namespace amoeba
