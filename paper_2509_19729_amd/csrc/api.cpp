// C ABI of the reshard library: argument checks, error text, plan lifetime.
// The entry points and their contracts are documented in include/amoeba.h.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <string>

#include "../../include/amoeba.h"
#include "../../include/amoeba_measure.h"
#include "launch.h"
#include "plan.h"

namespace {
thread_local std::string g_last_error;
}

namespace amoeba {
void set_error(const std::string& msg) { g_last_error = msg; }
}  // namespace amoeba

using amoeba::set_error;

namespace {

// Shared by the two status calls: copies the 2-word header back and decodes the flags.
int read_status(const char* who, const int32_t* ws, void* stream, int64_t* total) {
  int32_t head[2] = {0, 0};
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t rc = hipMemcpyAsync(head, ws, sizeof(head), hipMemcpyDeviceToHost, st);
  if (rc == hipSuccess) rc = hipStreamSynchronize(st);
  if (rc != hipSuccess) {
    set_error(std::string(who) + ": " + hipGetErrorString(rc));
    return AMOEBA_ERR_HIP;
  }
  if (total) *total = head[amoeba::kWsTotal];
  const int e = head[amoeba::kWsError];
  if (e & (amoeba::kErrNegativeLen | amoeba::kErrRowTooShort | amoeba::kErrPoolTooSmall)) {
    set_error(std::string(who) + ": " +
              ((e & amoeba::kErrNegativeLen) ? "negative sequence length; " : "") +
              ((e & amoeba::kErrRowTooShort) ? "a sequence needs more blocks than a table row holds; " : "") +
              ((e & amoeba::kErrPoolTooSmall) ? "destination pool too small; " : ""));
    return AMOEBA_ERR_OVERFLOW;
  }
  if (e & amoeba::kErrBlockId) {
    set_error(std::string(who) + ": a source block id lies outside the source pool");
    return AMOEBA_ERR_BLOCK_ID;
  }
  return AMOEBA_OK;
}

}  // namespace

extern "C" {

const char* amoeba_last_error(void) { return g_last_error.c_str(); }

amoeba_plan_t* amoeba_plan(const amoeba_model_shape* shape, int src_tp, int dst_tp,
                           int dst_rank) {
  amoeba_plan_s* p = new (std::nothrow) amoeba_plan_s();
  if (!p) { set_error("out of host memory"); return nullptr; }
  std::string err;
  if (!amoeba::build_plan(p, shape, src_tp, dst_tp, dst_rank, &err)) {
    set_error("amoeba_plan: " + err);
    delete p;
    return nullptr;
  }
  p->device = -1;
  p->n_cu = 0;
  p->workspace = nullptr;
  p->status_ws = nullptr;
  p->merge_workspace = nullptr;
  p->merge_workspace_bytes = 0;
  p->workspace_bytes = 0;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
      int cu = 0;
      if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
        p->n_cu = cu;
      // a merge of m = dst_tp / src_tp instances scans m * num_seqs sequences
      const size_t inst = (p->kp % p->k == 0 && p->kp > p->k) ? size_t(p->kp / p->k) : 1;
      const size_t bytes = sizeof(int32_t) * (size_t(amoeba::kWsHeader) +
                                              inst * size_t(p->shape.num_seqs) +
                                              size_t(p->shape.dst_pool_blocks));
      void* ws = nullptr;
      const hipError_t rc = hipMalloc(&ws, bytes);
      if (rc != hipSuccess) {
        set_error(std::string("amoeba_plan: workspace allocation failed: ") +
                  hipGetErrorString(rc));
        delete p;
        return nullptr;
      }
      // set-up time is when the static workspace's address on this device is looked up (the
      // first lookup may load the code object), so that amoeba_reshard_kv_static() itself
      // finds it cached; a failure is reported by that call, not here
      std::string ignored;
      (void)amoeba::static_kv_workspace(&ignored);
      p->device = dev;
      p->workspace = static_cast<int32_t*>(ws);
      p->workspace_bytes = bytes;
      if (p->merge_factor >= 2) {
        const size_t mbytes =
            sizeof(int32_t) *
            amoeba::merge_workspace_ints(p->shape.src_pool_blocks, p->merge_factor);
        void* mws = nullptr;
        const hipError_t mrc = hipMalloc(&mws, mbytes);
        if (mrc != hipSuccess) {
          set_error(std::string("amoeba_plan: merge workspace allocation failed: ") +
                    hipGetErrorString(mrc));
          (void)hipFree(ws);
          delete p;
          return nullptr;
        }
        p->merge_workspace = static_cast<int32_t*>(mws);
        p->merge_workspace_bytes = mbytes;
      }
    }
  } else {
    (void)hipGetLastError();  // no GPU: host-side planning only
  }
  g_last_error.clear();
  return p;
}

void amoeba_plan_destroy(amoeba_plan_t* plan) {
  if (!plan) return;
  if (plan->workspace) (void)hipFree(plan->workspace);
  if (plan->merge_workspace) (void)hipFree(plan->merge_workspace);
  delete plan;
}

int amoeba_reshard_weights_part(const amoeba_plan_t* plan, const void* const* src_shards,
                                void* dst, int part, void* stream) {
  if (!plan || !src_shards || !dst) {
    set_error("amoeba_reshard_weights: NULL plan, src_shards or dst");
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (part != AMOEBA_PART_ALL && part != AMOEBA_PART_ATTENTION && part != AMOEBA_PART_FFN) {
    set_error("amoeba_reshard_weights_part: part must be AMOEBA_PART_ALL, _ATTENTION or _FFN");
    return AMOEBA_ERR_INVALID_ARG;
  }
  std::string err;
  const int rc = amoeba::launch_reshard_weights(plan, src_shards, dst, part,
                                                static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_reshard_weights: " + err);
  return rc;
}

int amoeba_reshard_weights(const amoeba_plan_t* plan, const void* const* src_shards, void* dst,
                           void* stream) {
  return amoeba_reshard_weights_part(plan, src_shards, dst, AMOEBA_PART_ALL, stream);
}

int amoeba_reshard_kv(const amoeba_plan_t* plan, const void* const* src_blocks,
                      const int32_t* src_block_tables, const int32_t* seq_lens, void* dst_blocks,
                      int32_t* dst_block_tables, void* stream) {
  if (!plan || !src_blocks) {
    set_error("amoeba_reshard_kv: NULL plan or src_blocks");
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (!plan->workspace) {
    set_error("amoeba_reshard_kv: the plan has no device workspace (it was created without a GPU)");
    return AMOEBA_ERR_HIP;
  }
  int current_device = -1;
  if (hipGetDevice(&current_device) != hipSuccess || current_device != plan->device) {
    set_error("amoeba_reshard_kv: the current device is not the one the plan's workspace was "
              "allocated on");
    return AMOEBA_ERR_INVALID_ARG;
  }
  std::string err;
  const int rc = amoeba::launch_reshard_kv(plan, plan->workspace, src_blocks, src_block_tables,
                                           seq_lens, dst_blocks, dst_block_tables,
                                           static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_reshard_kv: " + err);
  else plan->status_ws = plan->workspace;
  return rc;
}

int amoeba_reshard_kv_static(const amoeba_plan_t* plan, const void* const* src_blocks,
                             const int32_t* src_block_tables, const int32_t* seq_lens,
                             void* dst_blocks, int32_t* dst_block_tables, void* stream) {
  if (!plan || !src_blocks) {
    set_error("amoeba_reshard_kv_static: NULL plan or src_blocks");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const uint64_t need = uint64_t(amoeba::kWsHeader) + uint64_t(plan->shape.num_seqs) +
                        uint64_t(plan->shape.dst_pool_blocks);
  if (need > amoeba::static_kv_workspace_ints()) {
    set_error("amoeba_reshard_kv_static: 8 + num_seqs + dst_pool_blocks = " +
              std::to_string(need) + " int32 words exceed the static workspace of " +
              std::to_string(amoeba::static_kv_workspace_ints()) +
              " words; use amoeba_reshard_kv()");
    return AMOEBA_ERR_INVALID_ARG;
  }
  std::string err;
  int32_t* ws = amoeba::static_kv_workspace(&err);
  if (!ws) {
    set_error("amoeba_reshard_kv_static: " + err);
    return AMOEBA_ERR_HIP;
  }
  const int rc = amoeba::launch_reshard_kv(plan, ws, src_blocks, src_block_tables, seq_lens,
                                           dst_blocks, dst_block_tables,
                                           static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_reshard_kv_static: " + err);
  else plan->status_ws = ws;
  return rc;
}

int amoeba_kv_status(const amoeba_plan_t* plan, void* stream, int64_t* total_blocks) {
  if (!plan || !plan->status_ws) {
    set_error("amoeba_kv_status: NULL plan, or no KV reshard was enqueued on it");
    return AMOEBA_ERR_INVALID_ARG;
  }
  return read_status("amoeba_kv_status", plan->status_ws, stream, total_blocks);
}

int amoeba_merge_kv_inplace(const amoeba_plan_t* plan, void* local_pool,
                            const void* const* remote_pools,
                            const int32_t* const* src_block_tables,
                            const int32_t* const* seq_lens, int32_t* dst_block_tables,
                            void* stream) {
  if (!plan) {
    set_error("amoeba_merge_kv_inplace: NULL plan");
    return AMOEBA_ERR_INVALID_ARG;
  }
  std::string err;
  const int rc = amoeba::launch_merge_kv_inplace(plan, local_pool, remote_pools, src_block_tables,
                                                 seq_lens, dst_block_tables,
                                                 static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_merge_kv_inplace: " + err);
  return rc;
}

int amoeba_merge_kv_base(const amoeba_plan_t* plan, const void* const* pools,
                         const int32_t* const* src_block_tables, const int32_t* const* seq_lens,
                         void* new_pool, int32_t* dst_block_tables, int64_t local_blocks_bound,
                         void* stream) {
  if (!plan || local_blocks_bound < 0) {
    set_error("amoeba_merge_kv_base: NULL plan or negative local_blocks_bound");
    return AMOEBA_ERR_INVALID_ARG;
  }
  if (!plan->workspace) {
    set_error("amoeba_merge_kv_base: the plan has no device workspace (it was created without a GPU)");
    return AMOEBA_ERR_HIP;
  }
  int current_device = -1;
  if (hipGetDevice(&current_device) != hipSuccess || current_device != plan->device) {
    set_error("amoeba_merge_kv_base: the current device is not the one the plan's workspace was "
              "allocated on");
    return AMOEBA_ERR_INVALID_ARG;
  }
  std::string err;
  const int rc = amoeba::launch_merge_kv_base(plan, plan->workspace, pools, src_block_tables,
                                              seq_lens, new_pool, dst_block_tables,
                                              local_blocks_bound,
                                              static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_merge_kv_base: " + err);
  else plan->status_ws = plan->workspace;
  return rc;
}

int amoeba_merge_kv_status(const amoeba_plan_t* plan, void* stream, int64_t* remote_blocks) {
  if (!plan || !plan->merge_workspace) {
    set_error("amoeba_merge_kv_status: NULL plan or no merge workspace");
    return AMOEBA_ERR_INVALID_ARG;
  }
  return read_status("amoeba_merge_kv_status", plan->merge_workspace, stream, remote_blocks);
}

int amoeba_plan_merge_factor(const amoeba_plan_t* plan) { return plan ? plan->merge_factor : 0; }

size_t amoeba_plan_shard_bytes(const amoeba_plan_t* plan, int side) {
  if (!plan) return 0;
  return size_t(side ? plan->dst_layer_bytes : plan->src_layer_bytes) * size_t(plan->shape.n_layers);
}

size_t amoeba_plan_kv_block_bytes(const amoeba_plan_t* plan, int side) {
  if (!plan) return 0;
  return size_t(side ? plan->block_bytes_dst : plan->block_bytes_src);
}

uint32_t amoeba_plan_src_rank_mask(const amoeba_plan_t* plan) {
  return plan ? plan->weight_rank_mask : 0;
}

uint32_t amoeba_plan_kv_rank_mask(const amoeba_plan_t* plan) {
  return plan ? plan->kv_rank_mask : 0;
}

int amoeba_plan_tensor_info(const amoeba_plan_t* plan, int side, int tensor, int64_t* elem_off,
                            int64_t* rows, int64_t* cols, int64_t* layer_elems) {
  if (!plan || tensor < 0 || tensor >= AMOEBA_T_COUNT || (side != 0 && side != 1)) {
    set_error("amoeba_plan_tensor_info: bad plan, side or tensor id");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const amoeba::ShardLayout& L = side ? plan->dst_layout : plan->src_layout;
  if (elem_off) *elem_off = L.off[tensor];
  if (rows) *rows = L.rows[tensor];
  if (cols) *cols = L.cols[tensor];
  if (layer_elems) *layer_elems = L.layer_elems;
  if (plan->shape.n_experts > 0) {  // gate/up/down: the first owned expert's tensors
    const amoeba::ExpertGeom& g = side ? plan->exp_dst : plan->exp_src;
    const int64_t e = plan->shape.elem_bytes;
    if (elem_off && tensor >= AMOEBA_T_GATE)
      *elem_off = (g.first + (tensor - AMOEBA_T_GATE) * g.tensor) / e;
    if (layer_elems) *layer_elems = g.layer / e;
  }
  return AMOEBA_OK;
}

int amoeba_plan_expert_info(const amoeba_plan_t* plan, int side, int64_t out[4]) {
  if (!plan || !out || (side != 0 && side != 1) || plan->shape.n_experts <= 0) {
    set_error("amoeba_plan_expert_info: bad plan, side or out, or the model has no experts");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const amoeba::ExpertGeom& g = side ? plan->exp_dst : plan->exp_src;
  out[0] = g.own; out[1] = g.first; out[2] = g.tensor; out[3] = g.slot;
  return AMOEBA_OK;
}

int amoeba_plan_padded_info(const amoeba_plan_t* plan, int side, int64_t out[6]) {
  if (!plan || !out || (side != 0 && side != 1) || !(side ? plan->dst_padded : plan->src_padded) ||
      plan->shape.n_experts > 0) {
    set_error("amoeba_plan_padded_info: bad plan, side or out, or that side is dense or expert-wise");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const amoeba::PaddedGeom& g = side ? plan->pad_dst : plan->pad_src;
  out[0] = g.attn; out[1] = g.attn_padded; out[2] = g.part; out[3] = g.part_padded;
  out[4] = g.stride; out[5] = g.layer;
  return AMOEBA_OK;
}

int amoeba_plan_ffn_view(const amoeba_plan_t* plan, int64_t out[4]) {
  if (!plan || !out || plan->kp % plan->k) return 0;
  if (plan->shape.n_experts > 0) {  // the target's experts inside their one source rank
    if (plan->src_padded != plan->dst_padded) return 0;
    const amoeba::ExpertGeom& S = plan->exp_src;
    const int64_t own = plan->exp_dst.own, host = int64_t(plan->rp) * plan->k / plan->kp;
    out[0] = host;
    out[1] = S.first + (int64_t(plan->rp) * own - host * S.own) * S.slot;
    out[2] = own * S.slot;
    out[3] = S.layer;
    return 1;
  }
  if (!plan->src_padded || !plan->dst_padded) return 0;
  const int64_t T = plan->shape.pad_max_tp;
  const int64_t host = int64_t(plan->rp) * plan->k / plan->kp;  // source rank holding the range
  const int64_t first = int64_t(plan->rp) * (T / plan->kp) - host * (T / plan->k);
  out[0] = host;
  out[1] = plan->pad_src.attn_padded + first * plan->pad_src.stride;
  out[2] = (T / plan->kp) * plan->pad_src.stride;
  out[3] = plan->pad_src.layer;
  return 1;
}

int amoeba_plan_kv_stride_order(const amoeba_plan_t* plan, int side, int64_t out[5]) {
  if (!plan || !out || (side != 0 && side != 1)) {
    set_error("amoeba_plan_kv_stride_order: bad plan, side or out");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const int64_t heads = side ? plan->heads_dst : plan->heads_src;
  const int layout = side ? plan->shape.kv_layout_dst : plan->shape.kv_layout_src;
  const int64_t B = plan->shape.kv_block_tokens, d = plan->shape.head_dim;
  if (layout == AMOEBA_KV_HEAD_MAJOR) {  // [head][K/V][token][d]
    out[0] = 2 * B * d; out[1] = B * d; out[2] = d; out[3] = 1;
  } else {                               // [K/V][token][head][d]
    out[0] = d; out[1] = B * heads * d; out[2] = heads * d; out[3] = 1;
  }
  out[4] = heads * 2 * B * d;
  return AMOEBA_OK;
}

int amoeba_plan_num_segments(const amoeba_plan_t* plan) {
  return plan ? int(plan->segments.size()) : 0;
}

int amoeba_plan_segment(const amoeba_plan_t* plan, int index, int64_t out[7]) {
  if (!plan || !out || index < 0 || index >= int(plan->segments.size())) {
    set_error("amoeba_plan_segment: bad plan, index or out");
    return AMOEBA_ERR_INVALID_ARG;
  }
  const amoeba::Segment& g = plan->segments[size_t(index)];
  out[0] = g.src_rank; out[1] = g.src_off; out[2] = g.src_pitch; out[3] = g.dst_off;
  out[4] = g.dst_pitch; out[5] = g.rows; out[6] = g.run;
  return AMOEBA_OK;
}

int amoeba_copy_baseline(void* dst, const void* src, size_t bytes, int threads, int unroll,
                         int grid, int nontemporal, void* stream) {
  if (!dst || !src) { set_error("amoeba_copy_baseline: NULL pointer"); return AMOEBA_ERR_INVALID_ARG; }
  std::string err;
  const int rc = amoeba::launch_copy_baseline(dst, src, bytes, threads, unroll, grid, nontemporal != 2,
                                              static_cast<hipStream_t>(stream), &err);
  if (rc != AMOEBA_OK) set_error("amoeba_copy_baseline: " + err);
  return rc;
}

int amoeba_plan_launch_shape(const amoeba_plan_t* plan, int kernel, int align_bytes,
                             int64_t out[4]) {
  if (!plan || !out || align_bytes < 1 || (align_bytes & (align_bytes - 1))) {
    set_error("amoeba_plan_launch_shape: bad plan or out, or align_bytes is not a power of two");
    return AMOEBA_ERR_INVALID_ARG;
  }
  amoeba::LaunchShape L;
  std::string err;
  bool ok = false;
  switch (kernel) {
    case 0: ok = amoeba::weights_launch_geometry(plan, align_bytes, &L, &err); break;
    case 1: ok = amoeba::kv_launch_geometry(plan, align_bytes, &L, &err); break;
    case 2: ok = amoeba::merge_launch_geometry(plan, align_bytes, &L, &err); break;
    default: err = "kernel must be 0 (weights), 1 (KV regroup) or 2 (merge copy)"; break;
  }
  if (!ok) {
    set_error("amoeba_plan_launch_shape: " + err);
    return AMOEBA_ERR_INVALID_ARG;
  }
  out[0] = L.grid_x; out[1] = L.grid_y; out[2] = L.threads; out[3] = int64_t(L.items);
  return AMOEBA_OK;
}

int amoeba_plan_tune(amoeba_plan_t* plan, int knob, int value) {
  if (!plan || value < 0) { set_error("amoeba_plan_tune: bad plan or value"); return AMOEBA_ERR_INVALID_ARG; }
  switch (knob) {
    case AMOEBA_TUNE_W_GRID: plan->tune.w_grid = value; break;
    case AMOEBA_TUNE_W_UNROLL: plan->tune.w_unroll = value; break;
    case AMOEBA_TUNE_KV_GRID: plan->tune.kv_grid = value; break;
    case AMOEBA_TUNE_KV_UNROLL: plan->tune.kv_unroll = value; break;
    case AMOEBA_TUNE_W_THREADS: plan->tune.w_threads = value; break;
    case AMOEBA_TUNE_KV_THREADS: plan->tune.kv_threads = value; break;
    case AMOEBA_TUNE_NONTEMPORAL: plan->tune.nontemporal = value; break;
    case AMOEBA_TUNE_KV_STAGED: plan->tune.kv_staged = value; break;
    case AMOEBA_TUNE_KV_BLOCKS_HINT: plan->tune.kv_blocks_hint = value; break;
    case AMOEBA_TUNE_KV_SMALL_TABLE:
      if (value > 1) { set_error("amoeba_plan_tune: AMOEBA_TUNE_KV_SMALL_TABLE takes 0 or 1"); return AMOEBA_ERR_INVALID_ARG; }
      plan->tune.kv_small = value;
      break;
    default: set_error("amoeba_plan_tune: unknown knob"); return AMOEBA_ERR_INVALID_ARG;
  }
  return AMOEBA_OK;
}

}  // extern "C"
