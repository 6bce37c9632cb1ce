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
// Three kernels, no host round trip (one when the table is small, see kv_small_kernel):
//   kv_scan_kernel   one workgroup; nb_i = ceil(len_i / B), wavefront-level
//                    inclusive scans joined through LDS, carried across chunks of
//                    1024 sequences; validates lengths / row width / pool size.
//   kv_table_kernel  one lane per table cell: writes the new table and a flat list
//                    "new block id -> source block id" (ids range-checked here).
//   kv_regroup_kernel one workgroup per (layer, new block, tile), layer on grid.y;
//                    a tile is a run of 16-byte vectors contiguous in the
//                    destination block.  The number of blocks in use is only
//                    known on the device, so the grid covers the pool's capacity
//                    (or the caller's bound on the blocks in use) and idle
//                    workgroups leave at once.  A lane turns its
//                    vector index into (head, K/V*token, d-offset) for the
//                    destination layout with multiply-high divisions, maps the head
//                    to (source rank, local head) and rebuilds the index for the
//                    source layout.  All loads of a tile are issued before its
//                    stores; accesses are 16 bytes per lane and non-temporal.
#include <algorithm>
#include <string>

#include <mutex>

#include "device_common.h"
#include "grid.h"
#include "launch.h"
#include "plan.h"

// Workspace of amoeba_reshard_kv_static(), for callers that cannot allocate: 4 MiB of
// device memory that every GPU the library runs on holds from the moment the code object
// is loaded there until the process ends.  This name is a host-side stand-in, not a device
// address: host code only ever uses the address static_kv_workspace() looks up.
constexpr size_t kScratchInts = size_t(1) << 20;
static __device__ __align__(256) int32_t scratch[kScratchInts];

namespace amoeba {

size_t static_kv_workspace_ints() { return kScratchInts; }

// Device address of `scratch` on the current device, looked up once per device (each GPU has
// its own copy of the array at its own address).  nullptr and a message on failure.
int32_t* static_kv_workspace(std::string* err) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static int32_t* ptr[kMaxDevices] = {};
  int dev = -1;
  hipError_t rc = hipGetDevice(&dev);
  if (rc != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *err = rc != hipSuccess ? std::string("hipGetDevice: ") + hipGetErrorString(rc)
                            : std::string("device index outside [0, 64)");
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    rc = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (rc != hipSuccess || !p) {
      *err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(rc);
      return nullptr;
    }
    ptr[dev] = static_cast<int32_t*>(p);
  }
  return ptr[dev];
}

constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;

// Lengths and tables of the sequences a call works on: one instance for the reshard, m
// instances (instance-major) for the merge of Sec. 3.1.  Sequence q of the merged list is
// sequence q mod seqs of instance q / seqs.
struct SeqInputs {
  const int32_t* lens[AMOEBA_MAX_TP];
  const int32_t* tables[AMOEBA_MAX_TP];
  FastDiv seqs;         // sequences per instance
  uint32_t n_inst;      // instances (1: a plain reshard)
  uint32_t local_inst;  // the instance hosted where the target rank is (merge only)
};

__global__ void __launch_bounds__(kScanThreads)
kv_scan_kernel(const SeqInputs in, uint32_t row_width, uint32_t block_tokens,
               int64_t dst_pool_blocks, int32_t* __restrict__ ws) {
  __shared__ long long wave_total[kScanWaves];
  __shared__ long long carry_s;
  __shared__ unsigned int err_s;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t num_seqs = in.n_inst * in.seqs.d;
  int32_t* base = ws + kWsHeader;
  if (tid == 0) { carry_s = 0; err_s = 0; }
  __syncthreads();

  for (uint32_t c0 = 0; c0 < num_seqs; c0 += kScanThreads) {
    const uint32_t i = c0 + tid;
    long long nb = 0;
    unsigned int e = 0;
    if (i < num_seqs) {
      const uint32_t inst = fd_div(i, in.seqs);
      const long long len = in.lens[inst][i - inst * in.seqs.d];
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
    // the id range of the local instance's blocks (the bases were written by this workgroup
    // before the barriers above)
    int32_t lo = 0, n = 0;
    if (!e && in.n_inst > 1 && in.seqs.d > 0) {
      lo = base[in.local_inst * in.seqs.d];
      const int32_t hi = in.local_inst + 1 < in.n_inst ? base[(in.local_inst + 1) * in.seqs.d]
                                                        : (int32_t)total;
      n = hi - lo;
    }
    ws[kWsLocalBase] = lo;
    ws[kWsLocalCount] = n;
  }
}

// One lane per cell of the (merged) table: the new id of the cell's block, and the flat list
// new id -> source block id (for a merge: source id * instances + instance).
__global__ void __launch_bounds__(kThreads)
kv_table_kernel(const SeqInputs in, int32_t* __restrict__ dst_table, FastDiv row_width,
                uint32_t block_tokens, int64_t src_pool_blocks, int32_t* __restrict__ ws) {
  const uint32_t num_seqs = in.n_inst * in.seqs.d;
  const uint64_t cell = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
  const uint64_t cells = uint64_t(num_seqs) * row_width.d;
  if (cell >= cells) return;
  const uint32_t q = fd_div(uint32_t(cell), row_width);  // cells < 2^32 is checked on the host
  const uint32_t j = uint32_t(cell) - q * row_width.d;
  const uint32_t inst = fd_div(q, in.seqs);
  const uint32_t i = q - inst * in.seqs.d;
  const bool failed = (ws[kWsError] & (kErrNegativeLen | kErrRowTooShort | kErrPoolTooSmall)) != 0;
  int32_t out = -1;
  if (!failed) {
    const long long len = in.lens[inst][i];
    const long long nb = (len + block_tokens - 1) / block_tokens;
    if ((long long)j < nb) {
      out = ws[kWsHeader + q] + (int32_t)j;
      int32_t sb = in.tables[inst][uint64_t(i) * row_width.d + j];
      if (sb < 0 || (int64_t)sb >= src_pool_blocks) {
        atomicOr(reinterpret_cast<unsigned int*>(ws + kWsError), (unsigned int)kErrBlockId);
        sb = -1;
      } else if (in.n_inst > 1) {
        sb = sb * (int32_t)in.n_inst + (int32_t)inst;  // < 2^31, checked on the host
      }
      ws[kWsHeader + num_seqs + out] = sb;
    }
  }
  dst_table[cell] = out;
}

struct KVArgs {
  const char* src[AMOEBA_MAX_TP];
  const char* src_lo;        // == src[rank_lo]
  const char* src_hi;        // == src[rank_hi]
  char* dst;
  const int32_t* ws;
  uint64_t src_layer_stride, dst_layer_stride;  // bytes between layers of a pool
  uint64_t src_block_bytes, dst_block_bytes;
  uint32_t num_seqs;
  uint32_t block_vecs;       // vectors in one destination block
  FastDiv tiles_per_block;
  uint32_t head0;            // first global head the target rank owns
  uint32_t rank_lo, rank_hi; // first and last source rank that own one of those heads
  uint32_t n_src;            // rank_hi - rank_lo + 1
  FastDiv heads_src;         // heads per source rank
  FastDiv heads_dst;         // heads per target rank
  FastDiv head_vecs;         // vectors of one head in a header-centric block: 2 * B * dv
  FastDiv dv;                // vectors of one head vector (d * elem_bytes / VEC)
  // merge of m instances (base solution of Sec. 3.1); n_inst.d <= 1: a plain reshard
  FastDiv n_inst;            // m: a work-list entry is source id * m + instance, src[] holds
                             // the instances' pools and head0 is relative to the old block
  uint32_t pass;             // 0: migration (blocks of the other instances), 1: de-fragmentation
                             // (blocks of the local instance)
};

// Moves one tile (THREADS * UNROLL vectors, contiguous in the destination block) of new
// block b, whose source block id is sb (negative: the id was out of range, nothing moves).
// A lane turns its vector index into (head, K/V * token, d-offset) for the destination
// layout, maps the head to (source rank, local head) and rebuilds the index for the source
// layout; all loads of the tile are issued before its stores.
template <int SL, int DL, int VEC, int THREADS, int UNROLL, bool NT>
__device__ __forceinline__ void regroup_tile(const KVArgs& a, uint32_t layer, uint32_t b,
                                             uint32_t tile, int32_t sb, uint32_t tid,
                                             const char* one_pool = nullptr) {
  using V = typename VecOf<VEC>::type;
  constexpr uint32_t kTileVecs = THREADS * UNROLL;
  if (sb < 0) return;  // uniform: the block's source id was out of range
  const char* sp[UNROLL];
  uint32_t dvec[UNROLL];
  bool live[UNROLL];
  const char* const pool_lo = uniform_ptr(a.src_lo);
  const char* const pool_hi = uniform_ptr(a.src_hi);
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    // Lanes past the end of a ragged last tile are clamped to the block's last vector for
    // the load (valid memory, value unused) and only masked for the store: loads inside
    // per-lane branches are separated by waits, which would serialise the UNROLL loads.
    const uint32_t v_raw = tile * kTileVecs + u * THREADS + tid;
    live[u] = v_raw < a.block_vecs;
    const uint32_t v = min(v_raw, a.block_vecs - 1);
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
    // Source pool of the owning rank.  Nearly always one or two ranks feed a target
    // rank; then the choice is a select between two pointers held in scalar registers
    // and costs no memory access.
    const char* pool;
    if (one_pool)  // merge: every head of the block comes from the block's instance
      pool = one_pool;
    else if (a.n_src <= 2)
      pool = (s == a.rank_lo) ? pool_lo : pool_hi;
    else
      pool = a.src[s];  // s < src_tp: v is a vector of the block
    sp[u] = pool + uint64_t(svec) * VEC;
  }
  const uint64_t soff = uint64_t(layer) * a.src_layer_stride + uint64_t(sb) * a.src_block_bytes;
  char* dp = a.dst + uint64_t(layer) * a.dst_layer_stride + uint64_t(b) * a.dst_block_bytes;
  V val[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) val[u] = ld<NT, V>(sp[u] + soff);
  if constexpr (VEC == 16) {
    // pin the loads here, unconditional and back to back (otherwise the compiler sinks each
    // one into the masked block of its store)
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) asm volatile("" : "+v"(val[u]));
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u)
    if (live[u]) st<NT, V>(dp + uint64_t(dvec[u]) * VEC, val[u]);
}

// blockIdx.y = layer; blockIdx.x strides over (new block, tile) of that layer.
// `ws` is only read here (the scan and table kernels that fill it have finished),
// which lets the uniform lookups go through scalar loads.
// MERGE: the two passes of the base solution of Sec. 3.1 over m instances' pools (a
// template parameter, not a run-time branch: even uniform scalar work in this kernel's
// short prologue costs 1-2 % of the rate).
template <int SL, int DL, int VEC, int THREADS, int UNROLL, bool NT, bool MERGE>
__global__ void __launch_bounds__(THREADS)
kv_regroup_kernel(const KVArgs a, const int32_t* __restrict__ ws) {
  const uint32_t layer = blockIdx.y;
  const uint32_t total = (uint32_t)ws[kWsTotal];
  const int32_t* __restrict__ worklist = ws + kWsHeader + a.num_seqs;
  // the migration pass takes the blocks outside the local instance's id range
  // [local_base, local_base + local_n), the de-fragmentation pass the ones inside
  const uint32_t local_base = MERGE ? (uint32_t)ws[kWsLocalBase] : 0u;
  const uint32_t local_n = MERGE ? (uint32_t)ws[kWsLocalCount] : 0u;
  const uint32_t n_blocks = !MERGE ? total : (a.pass ? local_n : total - local_n);
  const uint32_t n_items = n_blocks * a.tiles_per_block.d;  // < 2^31, bounded on the host
  // Items are taken in the XCD-chunked order (see xcd_item()): +4 % for workgroups of four
  // wavefronts, +1-2 % for single-wavefront ones on the block gather (a plain copy with
  // single-wavefront workgroups does not gain from it).
  const uint32_t n_loop = xcd_loop_bound(n_items);

  for (uint32_t wi = blockIdx.x; wi < n_loop; wi += gridDim.x) {
    const uint32_t w = xcd_item(wi, n_items);
    if (w >= n_items) continue;
    uint32_t b = fd_div(w, a.tiles_per_block);
    const uint32_t tile = w - b * a.tiles_per_block.d;
    if (MERGE) b = a.pass ? local_base + b : (b < local_base ? b : b + local_n);
    int32_t sb = worklist[b];  // -1: the source id was out of range, block is skipped
    const char* one_pool = nullptr;
    if (MERGE) {  // a work-list entry is source id * m + instance
      const uint32_t id = sb < 0 ? 0u : (uint32_t)sb;
      const uint32_t old_block = fd_div(id, a.n_inst);
      one_pool = a.src[id - old_block * a.n_inst.d];
      if (sb >= 0) sb = (int32_t)old_block;
    }
    regroup_tile<SL, DL, VEC, THREADS, UNROLL, NT>(a, layer, b, tile, sb, threadIdx.x, one_pool);
  }
}

// The whole KV path in one launch, for small tables (at most 64 sequences and kSmallCells
// table cells): a configuration of a few short sequences is bound by launch latency, and
// three dependent launches cost three times one.  Every workgroup is one wavefront and
// redoes the scan itself: lane i takes sequence i, the inclusive scan is six __shfl_up
// steps, the sequence that owns new block b is found with one ballot.  Workgroup (0, 0)
// alone writes the new table, checks every source id and writes the status words, so no
// word is written by two workgroups and nothing has to be cleared beforehand.
constexpr uint32_t kSmallSeqs = 64;
constexpr uint32_t kSmallCells = 4096;

template <int SL, int DL>
__global__ void __launch_bounds__(64)
kv_small_kernel(const KVArgs a, const int32_t* __restrict__ seq_lens,
                const int32_t* __restrict__ src_table, int32_t* __restrict__ dst_table,
                uint32_t row_width, uint32_t block_tokens, int64_t src_pool_blocks,
                int64_t dst_pool_blocks, int32_t* __restrict__ ws) {
  __shared__ int32_t base_s[kSmallSeqs], nb_s[kSmallSeqs];
  const uint32_t lane = threadIdx.x;
  const bool has_seq = lane < a.num_seqs;
  const long long len = has_seq ? seq_lens[lane] : 0;
  const bool negative = len < 0;
  long long nb = negative ? 0 : (len + block_tokens - 1) / block_tokens;
  const bool too_long = nb > (long long)row_width;
  long long incl = nb;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long up = __shfl_up(incl, off, 64);
    if (lane >= (uint32_t)off) incl += up;
  }
  const long long total = __shfl(incl, 63, 64);
  unsigned int err = (__ballot(negative) ? kErrNegativeLen : 0u) |
                     (__ballot(too_long) ? kErrRowTooShort : 0u) |
                     (total > dst_pool_blocks ? kErrPoolTooSmall : 0u);
  if (!err) {  // then nb <= row_width and every base is below dst_pool_blocks < 2^31
    base_s[lane] = (int32_t)(incl - nb);
    nb_s[lane] = (int32_t)nb;
  }
  __syncthreads();

  if (blockIdx.x == 0 && blockIdx.y == 0) {
    const uint32_t cells = a.num_seqs * row_width;
    bool bad = false;
    for (uint32_t cell = lane; cell < cells; cell += 64) {
      const uint32_t i = cell / row_width, j = cell - i * row_width;
      int32_t out = -1;
      if (!err && (int32_t)j < nb_s[i]) {
        out = base_s[i] + (int32_t)j;
        const int32_t sb = src_table[cell];
        if (sb < 0 || (int64_t)sb >= src_pool_blocks) bad = true;
      }
      dst_table[cell] = out;
    }
    const bool any_bad = __ballot(bad) != 0;
    if (lane == 0) {
      ws[kWsTotal] = err ? 0 : (int32_t)total;
      ws[kWsError] = (int32_t)(err | (any_bad ? (unsigned int)kErrBlockId : 0u));
    }
  }
  if (err) return;

  const uint32_t layer = blockIdx.y;
  const uint32_t n_items = (uint32_t)total * a.tiles_per_block.d;
  const uint32_t my_base = has_seq ? (uint32_t)(incl - nb) : 0u, my_nb = has_seq ? (uint32_t)nb : 0u;
  for (uint32_t w = blockIdx.x; w < n_items; w += gridDim.x) {
    const uint32_t b = fd_div(w, a.tiles_per_block);
    const uint32_t tile = w - b * a.tiles_per_block.d;
    // the one sequence whose id range [base, base + nb) holds b
    const unsigned long long owner = __ballot(b >= my_base && b - my_base < my_nb);
    if (!owner) continue;  // cannot happen for b < total; keeps the lookup below in bounds
    const uint32_t i = (uint32_t)__ffsll((long long)owner) - 1u;
    int32_t sb = src_table[i * row_width + (b - (uint32_t)base_s[i])];
    if (sb < 0 || (int64_t)sb >= src_pool_blocks) sb = -1;
    sb = __builtin_amdgcn_readfirstlane(sb);
    regroup_tile<SL, DL, 16, 64, 1, true>(a, layer, b, tile, sb, lane);
  }
}

// Layout-converting regroup through LDS (token-first <-> header-centric).
//
// Between the two layouts a block is transposed at the granularity of one head vector
// (d * elem_bytes bytes): in the token-first block the heads of a token are adjacent, in
// the header-centric block the tokens of a head are.  Gathering directly, one side of
// the copy is touched in pieces of one head vector; when that is less than a 128-byte
// cache line (d = 32 at 16 bits: 64 bytes) every line is fetched twice (FETCH_SIZE
// doubles, the rate drops to about 4 TB/s).  Here a workgroup owns a tile of
// (tile_tokens x tile_heads) head vectors of one K-or-V plane: it reads the tile in the
// source's storage order, parks it in LDS, and writes it in the destination's order, so
// both sides see runs of tile_heads (or tile_tokens) head vectors.
struct KVStagedGeom {
  uint32_t tile_tokens, tile_heads;  // tile extent; tile_tokens divides block_tokens
  uint32_t block_tokens;
  uint32_t tile_vecs;                // tile_tokens * tile_heads * dv
  FastDiv token_groups;              // block_tokens / tile_tokens
  FastDiv fd_tile_tokens, fd_tile_heads;
};

template <int LAYOUT>
__device__ __forceinline__ void staged_split(uint32_t e, const KVStagedGeom& g, uint32_t& t,
                                             uint32_t& h) {
  if (LAYOUT == AMOEBA_KV_TOKEN_MAJOR) {  // storage order: token outer, head inner
    t = fd_div(e, g.fd_tile_heads);
    h = e - t * g.tile_heads;
  } else {                                // head outer, token inner
    h = fd_div(e, g.fd_tile_tokens);
    t = e - h * g.tile_tokens;
  }
}

template <int LAYOUT>
__device__ __forceinline__ uint32_t block_vec(uint32_t h, uint32_t c, uint32_t t, uint32_t x,
                                              uint32_t heads, uint32_t B, uint32_t dv) {
  if (LAYOUT == AMOEBA_KV_HEAD_MAJOR) return ((h * 2 + c) * B + t) * dv + x;
  return ((c * B + t) * heads + h) * dv + x;
}

// THREADS lanes per workgroup, ITERS vectors per lane: the tile has at most THREADS * ITERS
// vectors.  All global loads of a tile are issued before the first LDS write and all LDS
// reads before the first global store, so a lane has ITERS accesses in flight on each side.
template <int SL, int DL, bool NT, int THREADS, int ITERS>
__global__ void __launch_bounds__(THREADS)
kv_regroup_staged_kernel(const KVArgs a, const KVStagedGeom g, const int32_t* __restrict__ ws) {
  extern __shared__ u32x4 tile_lds[];  // [tile_tokens][tile_heads][dv]
  const uint32_t tid = threadIdx.x;
  const uint32_t layer = blockIdx.y;
  const uint32_t total = (uint32_t)ws[kWsTotal];
  const int32_t* __restrict__ worklist = ws + kWsHeader + a.num_seqs;
  const uint32_t n_items = total * a.tiles_per_block.d;
  const uint32_t dv = a.dv.d, B = g.block_tokens;
  const uint32_t n_loop = xcd_loop_bound(n_items);  // XCD-chunked order, see xcd_item()
  const char* const pool_lo = uniform_ptr(a.src_lo);
  const char* const pool_hi = uniform_ptr(a.src_hi);

  for (uint32_t wi = blockIdx.x; wi < n_loop; wi += gridDim.x) {
    const uint32_t w = xcd_item(wi, n_items);
    if (w >= n_items) continue;  // uniform over the workgroup: no barrier is skipped by part of it
    const uint32_t b = fd_div(w, a.tiles_per_block);
    const uint32_t tile = w - b * a.tiles_per_block.d;
    const int32_t sb = worklist[b];
    // tile -> (head group, K/V plane, token group), token group fastest
    const uint32_t r = fd_div(tile, g.token_groups);
    const uint32_t t0 = (tile - r * g.token_groups.d) * g.tile_tokens;
    const uint32_t c = r & 1, h0 = (r >> 1) * g.tile_heads;
    const uint64_t soff = uint64_t(layer) * a.src_layer_stride + uint64_t(sb) * a.src_block_bytes;
    char* dp = a.dst + uint64_t(layer) * a.dst_layer_stride + uint64_t(b) * a.dst_block_bytes;

    u32x4 val[ITERS];
    uint32_t slot[ITERS];  // index in LDS; ~0u: nothing to move
#pragma unroll
    for (int u = 0; u < ITERS; ++u) {  // source order -> registers
      const uint32_t v = u * THREADS + tid;
      const uint32_t e = fd_div(v, a.dv), x = v - e * dv;
      uint32_t t, h;
      staged_split<SL>(e, g, t, h);
      const uint32_t hp = h0 + h;
      slot[u] = ~0u;
      if (v < g.tile_vecs && hp < a.heads_dst.d && sb >= 0) {
        const uint32_t hg = a.head0 + hp;
        const uint32_t s = fd_div(hg, a.heads_src);
        const uint32_t hs = hg - s * a.heads_src.d;
        const char* pool = (a.n_src <= 2) ? ((s == a.rank_lo) ? pool_lo : pool_hi) : a.src[s];
        const uint32_t sv = block_vec<SL>(hs, c, t0 + t, x, a.heads_src.d, B, dv);
        val[u] = ld<NT, u32x4>(pool + soff + uint64_t(sv) * 16);
        slot[u] = (t * g.tile_heads + h) * dv + x;
      }
    }
#pragma unroll
    for (int u = 0; u < ITERS; ++u)
      if (slot[u] != ~0u) tile_lds[slot[u]] = val[u];
    __syncthreads();
    uint32_t dvi[ITERS];
#pragma unroll
    for (int u = 0; u < ITERS; ++u) {  // LDS -> registers, destination order
      const uint32_t v = u * THREADS + tid;
      const uint32_t e = fd_div(v, a.dv), x = v - e * dv;
      uint32_t t, h;
      staged_split<DL>(e, g, t, h);
      const uint32_t hp = h0 + h;
      slot[u] = ~0u;
      if (v < g.tile_vecs && hp < a.heads_dst.d && sb >= 0) {
        slot[u] = (t * g.tile_heads + h) * dv + x;
        dvi[u] = block_vec<DL>(hp, c, t0 + t, x, a.heads_dst.d, B, dv);
        val[u] = tile_lds[slot[u]];
      }
    }
#pragma unroll
    for (int u = 0; u < ITERS; ++u)
      if (slot[u] != ~0u) st<NT, u32x4>(dp + uint64_t(dvi[u]) * 16, val[u]);
    __syncthreads();  // the next tile reuses the LDS buffer
  }
}

namespace {

template <int SL, int DL, int VEC, int THREADS, int UNROLL, bool MERGE>
void launch_nt(bool nt, dim3 grid, hipStream_t stream, const KVArgs& a) {
  if (nt)
    hipLaunchKernelGGL((kv_regroup_kernel<SL, DL, VEC, THREADS, UNROLL, true, MERGE>), grid,
                       dim3(THREADS), 0, stream, a, a.ws);
  else
    hipLaunchKernelGGL((kv_regroup_kernel<SL, DL, VEC, THREADS, UNROLL, false, MERGE>), grid,
                       dim3(THREADS), 0, stream, a, a.ws);
}

template <int SL, int DL, int THREADS>
void launch_unroll(int unroll, bool nt, dim3 grid, hipStream_t stream, const KVArgs& a) {
  switch (unroll) {
    case 2: launch_nt<SL, DL, 16, THREADS, 2, false>(nt, grid, stream, a); break;
    case 4: launch_nt<SL, DL, 16, THREADS, 4, false>(nt, grid, stream, a); break;
    default: launch_nt<SL, DL, 16, THREADS, 1, false>(nt, grid, stream, a); break;
  }
}

// merge: one vector per lane only (the launch shape that measured best)
template <int SL, int DL>
void launch_vec(int vec, int threads, int unroll, bool nt, bool merge, dim3 grid,
                hipStream_t stream, const KVArgs& a) {
  if (merge) {
    if (vec == 16) {
      if (threads == 64) launch_nt<SL, DL, 16, 64, 1, true>(nt, grid, stream, a);
      else launch_nt<SL, DL, 16, 256, 1, true>(nt, grid, stream, a);
    } else if (vec == 8) {
      launch_nt<SL, DL, 8, 256, 1, true>(true, grid, stream, a);
    } else if (vec == 4) {
      launch_nt<SL, DL, 4, 256, 1, true>(true, grid, stream, a);
    } else if (vec == 2) {
      launch_nt<SL, DL, 2, 256, 1, true>(true, grid, stream, a);
    } else {
      launch_nt<SL, DL, 1, 256, 1, true>(true, grid, stream, a);
    }
    return;
  }
  if (vec == 16) {
    if (threads == 64) launch_unroll<SL, DL, 64>(unroll, nt, grid, stream, a);
    else launch_unroll<SL, DL, 256>(unroll, nt, grid, stream, a);
  } else if (vec == 8) {
    launch_nt<SL, DL, 8, 256, 1, false>(true, grid, stream, a);
  } else if (vec == 4) {
    launch_nt<SL, DL, 4, 256, 1, false>(true, grid, stream, a);
  } else if (vec == 2) {
    launch_nt<SL, DL, 2, 256, 1, false>(true, grid, stream, a);
  } else {
    launch_nt<SL, DL, 1, 256, 1, false>(true, grid, stream, a);
  }
}

bool hip_ok(const char* what, std::string* err) {
  const hipError_t rc = hipGetLastError();
  if (rc == hipSuccess) return true;
  *err = std::string(what) + ": " + hipGetErrorString(rc);
  return false;
}

// Everything the host decides about the regroup launch, from the plan and the common
// alignment of the call's pointers.
struct KVLaunch {
  bool staged = false;   // layout conversion through LDS
  bool small = false;    // scan, table and regroup in one launch (kv_small_kernel)
  int vec = 16, threads = 64, unroll = 1;  // unroll: vectors per lane (staged: per side)
  uint64_t tiles_per_block = 0;
  uint64_t basis = 0;    // items per layer the grid was sized for (capacity, or the bound)
  dim3 grid;
  KVStagedGeom g;
  size_t lds = 0;
};

// multi: the merge of several instances (always the three-kernel direct gather).
bool kv_launch_shape(const amoeba_plan_s* p, int vec, bool multi, KVLaunch* out,
                     std::string* err) {
  const amoeba_model_shape& s = p->shape;
  const uint64_t head_vec_bytes = uint64_t(s.head_dim) * s.elem_bytes;
  const uint32_t B = uint32_t(s.kv_block_tokens);
  const uint32_t dv = uint32_t(head_vec_bytes / vec);  // vectors of one head vector
  const uint64_t block_vecs = uint64_t(p->block_bytes_dst) / vec;
  const uint64_t cells = uint64_t(s.num_seqs) * uint64_t(s.max_blocks_per_seq);
  // the caller's bound on the blocks in use (the shape's, unless a sweep overrides it)
  const int64_t bound = p->tune.kv_blocks_hint > 0 ? p->tune.kv_blocks_hint : s.kv_blocks_bound;
  KVLaunch L;
  L.vec = vec;
  int unroll = p->tune.kv_unroll, threads = p->tune.kv_threads;
  if (vec != 16 || multi || (unroll != 2 && unroll != 4)) unroll = 1;
  if (vec != 16) threads = 256;
  else if (threads != 256 && threads != 64)
    // One wavefront per 1 KiB tile is fastest when the grid is tight (6.45 TB/s against 6.4
    // for four wavefronts in the XCD-chunked order, 6.15 in plain order), but with the grid
    // sized by the pool's capacity every idle workgroup costs dispatch time; 4 KiB tiles cut
    // that cost by four.  So: small tiles when the caller bounded the blocks in use, large
    // ones otherwise.
    threads = bound > 0 ? 64 : 256;

  // Grid: one workgroup per tile of the pool's capacity (workgroups that stride over several
  // tiles measured 8 % slower), or of the caller's bound on the blocks in use; capped at 2^27
  // workgroups over all layers so that a huge, mostly empty pool does not pay for idle
  // workgroups without limit, and at the work-items one grid dimension can hold.  Past the
  // grid, workgroups stride.
  auto grid_for = [&](uint64_t tiles_per_block, uint32_t lanes, dim3* g) {
    const uint64_t max_items = uint64_t(s.dst_pool_blocks) * tiles_per_block;  // per layer
    // item ids are 32-bit and a striding workgroup adds the grid size (at most 2^27) to one
    if (block_vecs >= (uint64_t(1) << 32) - 65536 || max_items >= (uint64_t(1) << 31) ||
        s.kv_layers > 65535)
      return false;
    uint64_t grid =
        std::max<uint64_t>(uint64_t(1) << 16, (uint64_t(1) << 27) / uint64_t(s.kv_layers));
    if (p->tune.kv_grid > 0) grid = uint64_t(p->tune.kv_grid);
    uint64_t basis = max_items;
    if (bound > 0)
      basis = std::min<uint64_t>(basis, std::max<uint64_t>(1, uint64_t(bound) * tiles_per_block));
    grid = grid_for_items(std::min(grid, basis), max_items);
    *g = dim3(clamp_grid_x(grid, lanes), uint32_t(s.kv_layers));
    L.basis = basis;
    return true;
  };

  // Converting between the layouts goes through LDS when one head vector is at most one
  // 128-byte cache line (see kv_regroup_staged_kernel): below a line the direct gather
  // fetches every line twice (4.0 against 6.3 TB/s), at exactly one line it moves whole
  // lines but in single-line pieces (6.0 against 6.3).  With 256-byte head vectors the
  // direct gather measured the same or faster.
  const bool convert = s.kv_layout_src != s.kv_layout_dst;
  const bool want_staged =
      p->tune.kv_staged == 1 || (p->tune.kv_staged == 0 && head_vec_bytes <= 128);
  if (convert && vec == 16 && want_staged && head_vec_bytes <= 4096 && !multi) {
    // Tile: 1 KiB runs on the destination's side first (scattered writes cost more than
    // scattered reads), then as much of the other axis as the lanes' vectors allow.
    // Measured best: 256 lanes x 2 vectors (8 KiB); 4 vectors per lane lose 3-8 %.
    const int st_threads = p->tune.kv_threads == 64 ? 64 : 256;
    int st_iters = p->tune.kv_unroll;
    if (st_iters != 1 && st_iters != 2 && st_iters != 4) st_iters = 2;
    while (uint32_t(st_threads * st_iters) < dv) st_iters *= 2;  // dv <= 256 = 64 * 4
    const uint32_t cap = uint32_t(st_threads * st_iters);  // vectors of a tile at most
    const uint32_t run = std::max<uint32_t>(1, 1024u / uint32_t(head_vec_bytes));
    uint32_t tt, th;
    if (s.kv_layout_dst == AMOEBA_KV_HEAD_MAJOR) {
      // the destination's contiguous runs are tokens of a head: 1 KiB of them first
      tt = std::min(run, B);
      while (B % tt || tt * dv > cap) --tt;  // tokens per tile divide the block; dv <= cap
      th = std::min<uint32_t>(std::max<uint32_t>(1, cap / (tt * dv)), uint32_t(p->heads_dst));
    } else {
      // the destination's contiguous runs are heads of a token
      th = std::min<uint32_t>(run, uint32_t(p->heads_dst));
      while (th * dv > cap) --th;
      tt = std::min<uint32_t>(std::max<uint32_t>(1, cap / (th * dv)), B);
      while (B % tt) --tt;
    }
    L.staged = true;
    L.threads = st_threads;
    L.unroll = st_iters;
    L.g.tile_tokens = tt;
    L.g.tile_heads = th;
    L.g.block_tokens = B;
    L.g.tile_vecs = tt * th * dv;
    L.g.token_groups = make_fastdiv(B / tt);
    L.g.fd_tile_tokens = make_fastdiv(tt);
    L.g.fd_tile_heads = make_fastdiv(th);
    const uint64_t head_groups = (uint64_t(p->heads_dst) + th - 1) / th;
    L.tiles_per_block = head_groups * 2 * (B / tt);
    L.lds = size_t(L.g.tile_vecs) * 16;
    if (!grid_for(L.tiles_per_block, uint32_t(st_threads), &L.grid)) {
      *err = "KV pool too large for 32-bit work indexing";
      return false;
    }
    *out = L;
    return true;
  }

  // A small table: scan, table and regroup in one launch of single-wavefront workgroups.
  if (vec == 16 && !multi && p->tune.kv_small != 1 && p->tune.kv_unroll == 0 && p->tune.kv_threads == 0 &&
      p->tune.nontemporal != 2 && cells > 0 && cells <= kSmallCells &&
      uint32_t(s.num_seqs) <= kSmallSeqs && s.dst_pool_blocks > 0) {
    L.small = true;
    threads = 64;
    unroll = 1;
  }
  L.threads = threads;
  L.unroll = unroll;
  const uint64_t tile_vecs = uint64_t(threads) * unroll;
  L.tiles_per_block = (block_vecs + tile_vecs - 1) / tile_vecs;
  if (!grid_for(L.tiles_per_block, uint32_t(threads), &L.grid)) {
    *err = "KV pool too large for 32-bit work indexing";
    return false;
  }
  *out = L;
  return true;
}

}  // namespace

bool kv_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                        std::string* err) {
  const uint64_t head_vec_bytes = uint64_t(p->shape.head_dim) * p->shape.elem_bytes;
  const int vec = common_alignment(head_vec_bytes | uint64_t(align_bytes));
  KVLaunch L;
  if (!kv_launch_shape(p, vec, false, &L, err)) return false;
  out->grid_x = L.grid.x;
  out->grid_y = L.grid.y;
  out->threads = uint32_t(L.threads);
  out->items = uint64_t(p->shape.dst_pool_blocks) * L.tiles_per_block;
  return true;
}

namespace {

// Geometry fields of the regroup arguments that follow from the plan and the vector width.
void fill_geometry(KVArgs* a, const amoeba_plan_s* p, int vec, const KVLaunch& L) {
  const amoeba_model_shape& s = p->shape;
  const uint32_t B = uint32_t(s.kv_block_tokens);
  const uint32_t dv = uint32_t(uint64_t(s.head_dim) * s.elem_bytes / vec);
  a->src_layer_stride = uint64_t(s.src_pool_blocks) * p->block_bytes_src;
  a->dst_layer_stride = uint64_t(s.dst_pool_blocks) * p->block_bytes_dst;
  a->src_block_bytes = uint64_t(p->block_bytes_src);
  a->dst_block_bytes = uint64_t(p->block_bytes_dst);
  a->heads_src = make_fastdiv(uint32_t(p->heads_src));
  a->heads_dst = make_fastdiv(uint32_t(p->heads_dst));
  a->dv = make_fastdiv(dv);
  a->head_vecs = make_fastdiv(2u * B * dv);
  a->block_vecs = uint32_t(uint64_t(p->block_bytes_dst) / vec);
  a->tiles_per_block = make_fastdiv(uint32_t(L.tiles_per_block));
  a->n_inst = make_fastdiv(1);
  a->pass = 0;
}

// Scan of the (merged) sequence lengths, then the (merged) table and the work list.
int launch_scan_and_table(const amoeba_plan_s* p, const SeqInputs& in, int32_t* dst_block_tables,
                          int32_t* ws, hipStream_t stream, std::string* err) {
  const amoeba_model_shape& s = p->shape;
  hipLaunchKernelGGL(kv_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, in,
                     uint32_t(s.max_blocks_per_seq), uint32_t(s.kv_block_tokens),
                     int64_t(s.dst_pool_blocks), ws);
  if (!hip_ok("kv scan kernel launch failed", err)) return AMOEBA_ERR_HIP;
  const uint64_t cells = uint64_t(in.n_inst) * in.seqs.d * uint64_t(s.max_blocks_per_seq);
  if (cells) {
    const uint32_t grid = uint32_t((cells + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(kv_table_kernel, dim3(grid), dim3(kThreads), 0, stream, in,
                       dst_block_tables, make_fastdiv(uint32_t(s.max_blocks_per_seq)),
                       uint32_t(s.kv_block_tokens), int64_t(s.src_pool_blocks), ws);
    if (!hip_ok("kv table kernel launch failed", err)) return AMOEBA_ERR_HIP;
  }
  return AMOEBA_OK;
}

void launch_direct(const amoeba_model_shape& s, const KVLaunch& L, dim3 grid, bool nt, bool merge,
                   hipStream_t stream, const KVArgs& a) {
  const bool sh = s.kv_layout_src == AMOEBA_KV_HEAD_MAJOR, dh = s.kv_layout_dst == AMOEBA_KV_HEAD_MAJOR;
  if (sh && dh)
    launch_vec<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_HEAD_MAJOR>(L.vec, L.threads, L.unroll, nt, merge, grid, stream, a);
  else if (sh && !dh)
    launch_vec<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_TOKEN_MAJOR>(L.vec, L.threads, L.unroll, nt, merge, grid, stream, a);
  else if (!sh && dh)
    launch_vec<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_HEAD_MAJOR>(L.vec, L.threads, L.unroll, nt, merge, grid, stream, a);
  else
    launch_vec<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_TOKEN_MAJOR>(L.vec, L.threads, L.unroll, nt, merge, grid, stream, a);
}

}  // namespace

int launch_merge_kv_base(const amoeba_plan_s* p, int32_t* ws, const void* const* pools,
                         const int32_t* const* src_block_tables, const int32_t* const* seq_lens,
                         void* new_pool, int32_t* dst_block_tables, int64_t local_blocks_bound,
                         hipStream_t stream, std::string* err) {
  const amoeba_model_shape& s = p->shape;
  if (p->kp % p->k || p->kp / p->k < 2 ||
      uint64_t(s.src_pool_blocks) * uint64_t(p->kp / p->k) > uint64_t(INT32_MAX)) {
    *err = "the plan is not a merge of instances (needs dst_tp = m * src_tp, m >= 2, "
           "src_pool_blocks * m < 2^31)";
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint32_t m = uint32_t(p->kp / p->k), g = uint32_t(p->rp) % m;
  const uint64_t S = uint64_t(s.num_seqs), W = uint64_t(s.max_blocks_per_seq);
  const uint64_t cells = uint64_t(m) * S * W;
  if (cells >= (uint64_t(1) << 32) - kThreads) {
    *err = "merged block table has 2^32 cells or more";
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (!pools || (S && !seq_lens) || (cells && (!src_block_tables || !dst_block_tables))) {
    *err = "a pools, seq_lens or table argument is NULL";
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint64_t src_layer = uint64_t(s.src_pool_blocks) * p->block_bytes_src,
                 dst_layer = uint64_t(s.dst_pool_blocks) * p->block_bytes_dst;
  const uint64_t src_bytes = src_layer * s.kv_layers, dst_bytes = dst_layer * s.kv_layers;
  const uint64_t d0 = reinterpret_cast<uint64_t>(new_pool);
  if (!d0 && dst_bytes) { *err = "new_pool is NULL"; return AMOEBA_ERR_INVALID_ARG; }
  SeqInputs in;
  KVArgs a;
  uint64_t bits = uint64_t(s.head_dim) * s.elem_bytes | d0;
  for (uint32_t i = 0; i < AMOEBA_MAX_TP; ++i) {
    in.lens[i] = in.tables[i] = nullptr;
    a.src[i] = nullptr;
  }
  for (uint32_t i = 0; i < m; ++i) {
    if ((S && !seq_lens[i]) || (cells && !src_block_tables[i])) {
      *err = "a seq_lens or block table pointer is NULL";
      return AMOEBA_ERR_INVALID_ARG;
    }
    in.lens[i] = S ? seq_lens[i] : nullptr;
    in.tables[i] = cells ? src_block_tables[i] : nullptr;
    const uint64_t s0 = reinterpret_cast<uint64_t>(pools[i]);
    if (!s0 && src_bytes) { *err = "a pool pointer is NULL"; return AMOEBA_ERR_INVALID_ARG; }
    if (s0 < d0 + dst_bytes && d0 < s0 + src_bytes) {
      *err = "new_pool overlaps a source pool (the base solution needs a second pool)";
      return AMOEBA_ERR_INVALID_ARG;
    }
    bits |= s0;
    a.src[i] = static_cast<const char*>(pools[i]);
  }
  in.seqs = make_fastdiv(uint32_t(std::max<uint64_t>(S, 1)));
  in.n_inst = S ? m : 0;   // no sequences: nothing to scan
  in.local_inst = g;
  const int vec = common_alignment(bits);
  KVLaunch L;
  if (!kv_launch_shape(p, vec, true, &L, err)) return AMOEBA_ERR_INVALID_ARG;
  const bool nt = p->tune.nontemporal != 2;

  const int rc = launch_scan_and_table(p, in, dst_block_tables, ws, stream, err);
  if (rc != AMOEBA_OK) return rc;
  if (cells == 0 || s.dst_pool_blocks == 0) return AMOEBA_OK;

  fill_geometry(&a, p, vec, L);
  a.dst = static_cast<char*>(new_pool);
  a.ws = ws;
  a.num_seqs = uint32_t(m * S);
  // rank r' = s*m + g keeps heads [g * heads_dst, (g + 1) * heads_dst) of an old block
  a.head0 = g * uint32_t(p->heads_dst);
  a.rank_lo = a.rank_hi = 0;
  a.n_src = 1;
  a.src_lo = a.src_hi = nullptr;  // the pool comes from the block's instance
  a.n_inst = make_fastdiv(m);
  // Pass 1, migration: the blocks of the other instances.  Pass 2, de-fragmentation: the
  // local blocks.  Idle workgroups cost dispatch time (a pass sized for all blocks that only
  // finds the local quarter takes almost as long as the whole), so each pass gets a grid of
  // its own: the bound on all blocks minus the bound on the local ones, and the local bound.
  // Without a local bound the passes share the whole bound evenly by instance count.  Past
  // its grid a pass strides, so any bounds are correct.
  const int64_t bound = p->tune.kv_blocks_hint > 0 ? p->tune.kv_blocks_hint : s.kv_blocks_bound;
  auto pass_grid = [&](uint64_t blocks) {
    dim3 g = L.grid;
    if (bound > 0) {
      const uint64_t want = std::max<uint64_t>(1, blocks) * L.tiles_per_block;
      g.x = clamp_grid_x(grid_for_items(std::min<uint64_t>(want, L.grid.x), uint64_t(L.grid.x)),
                         uint32_t(L.threads));
    }
    return g;
  };
  const uint64_t local_share = local_blocks_bound > 0 ? uint64_t(local_blocks_bound)
                                                      : (uint64_t(std::max<int64_t>(bound, 0)) + m - 1) / m;
  const uint64_t remote_share = uint64_t(bound) > local_share ? uint64_t(bound) - local_share : 1;
  a.pass = 0;
  launch_direct(s, L, pass_grid(remote_share), nt, true, stream, a);
  if (!hip_ok("kv migration kernel launch failed", err)) return AMOEBA_ERR_HIP;
  a.pass = 1;
  launch_direct(s, L, pass_grid(local_share), nt, true, stream, a);
  if (!hip_ok("kv de-fragmentation kernel launch failed", err)) return AMOEBA_ERR_HIP;
  return AMOEBA_OK;
}

int launch_reshard_kv(const amoeba_plan_s* p, int32_t* ws, const void* const* src_blocks,
                      const int32_t* src_block_tables, const int32_t* seq_lens, void* dst_blocks,
                      int32_t* dst_block_tables, hipStream_t stream, std::string* err) {
  const amoeba_model_shape& s = p->shape;
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
  KVLaunch L;
  if (!kv_launch_shape(p, vec, false, &L, err)) return AMOEBA_ERR_INVALID_ARG;
  const bool nt = p->tune.nontemporal != 2;

  const uint32_t B = uint32_t(s.kv_block_tokens);
  fill_geometry(&a, p, vec, L);
  a.dst = static_cast<char*>(dst_blocks);
  a.ws = ws;
  a.num_seqs = uint32_t(s.num_seqs);
  a.head0 = uint32_t(p->rp * p->heads_dst);
  a.rank_lo = a.head0 / uint32_t(p->heads_src);
  a.rank_hi = (a.head0 + uint32_t(p->heads_dst) - 1) / uint32_t(p->heads_src);
  a.n_src = a.rank_hi - a.rank_lo + 1;
  a.src_lo = a.src[a.rank_lo];
  a.src_hi = a.src[a.rank_hi];
  const bool sh = s.kv_layout_src == AMOEBA_KV_HEAD_MAJOR, dh = s.kv_layout_dst == AMOEBA_KV_HEAD_MAJOR;

  if (L.small) {
#define AMOEBA_SMALL(SLAY, DLAY)                                                                  \
  hipLaunchKernelGGL((kv_small_kernel<SLAY, DLAY>), L.grid, dim3(64), 0, stream, a, seq_lens,     \
                     src_block_tables, dst_block_tables, uint32_t(s.max_blocks_per_seq), B,       \
                     int64_t(s.src_pool_blocks), int64_t(s.dst_pool_blocks), ws)
    if (sh && dh) AMOEBA_SMALL(AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_HEAD_MAJOR);
    else if (sh) AMOEBA_SMALL(AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_TOKEN_MAJOR);
    else if (dh) AMOEBA_SMALL(AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_HEAD_MAJOR);
    else AMOEBA_SMALL(AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_TOKEN_MAJOR);
#undef AMOEBA_SMALL
    if (!hip_ok("kv small-table kernel launch failed", err)) return AMOEBA_ERR_HIP;
    return AMOEBA_OK;
  }

  // 1. scan, 2. tables
  SeqInputs in;
  for (int r = 0; r < AMOEBA_MAX_TP; ++r) in.lens[r] = in.tables[r] = nullptr;
  in.lens[0] = seq_lens;
  in.tables[0] = src_block_tables;
  in.seqs = make_fastdiv(uint32_t(std::max<int32_t>(s.num_seqs, 1)));
  in.n_inst = s.num_seqs > 0 ? 1 : 0;
  in.local_inst = 0;
  const int rc = launch_scan_and_table(p, in, dst_block_tables, ws, stream, err);
  if (rc != AMOEBA_OK) return rc;
  // 3. regroup
  if (cells == 0 || s.dst_pool_blocks == 0) return AMOEBA_OK;

  if (L.staged) {
    const KVStagedGeom& g = L.g;
    const dim3 grid = L.grid;
    const size_t lds = L.lds;
    const bool src_hm = sh;
#define AMOEBA_STAGED(T, I)                                                                       \
  do {                                                                                            \
    if (src_hm && nt)                                                                             \
      hipLaunchKernelGGL((kv_regroup_staged_kernel<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_TOKEN_MAJOR,   \
                                                   true, T, I>),                                  \
                         grid, dim3(T), lds, stream, a, g, a.ws);                                 \
    else if (src_hm)                                                                              \
      hipLaunchKernelGGL((kv_regroup_staged_kernel<AMOEBA_KV_HEAD_MAJOR, AMOEBA_KV_TOKEN_MAJOR,   \
                                                   false, T, I>),                                 \
                         grid, dim3(T), lds, stream, a, g, a.ws);                                 \
    else if (nt)                                                                                  \
      hipLaunchKernelGGL((kv_regroup_staged_kernel<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_HEAD_MAJOR,   \
                                                   true, T, I>),                                  \
                         grid, dim3(T), lds, stream, a, g, a.ws);                                 \
    else                                                                                          \
      hipLaunchKernelGGL((kv_regroup_staged_kernel<AMOEBA_KV_TOKEN_MAJOR, AMOEBA_KV_HEAD_MAJOR,   \
                                                   false, T, I>),                                 \
                         grid, dim3(T), lds, stream, a, g, a.ws);                                 \
  } while (0)
    if (L.threads == 64) {
      switch (L.unroll) {
        case 1: AMOEBA_STAGED(64, 1); break;
        case 2: AMOEBA_STAGED(64, 2); break;
        default: AMOEBA_STAGED(64, 4); break;
      }
    } else {
      switch (L.unroll) {
        case 1: AMOEBA_STAGED(256, 1); break;
        case 2: AMOEBA_STAGED(256, 2); break;
        default: AMOEBA_STAGED(256, 4); break;
      }
    }
#undef AMOEBA_STAGED
    if (!hip_ok("kv staged regroup kernel launch failed", err)) return AMOEBA_ERR_HIP;
    return AMOEBA_OK;
  }

  launch_direct(s, L, L.grid, nt, false, stream, a);
  if (!hip_ok("kv regroup kernel launch failed", err)) return AMOEBA_ERR_HIP;
  return AMOEBA_OK;
}

}  // namespace amoeba
