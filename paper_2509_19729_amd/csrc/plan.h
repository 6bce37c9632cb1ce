// Host-side plan of one TP=k -> TP=k' reshard for one target rank: where every
// tensor sits in a shard, which strided byte ranges move where, and the KV block
// geometry of both sides.  Pure host code; the kernels receive tables derived
// from it at call time.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/amoeba.h"

namespace amoeba {

// Position of the seven tensors inside one rank's per-layer shard (elements).
struct ShardLayout {
  int64_t off[AMOEBA_T_COUNT];
  int64_t rows[AMOEBA_T_COUNT];
  int64_t cols[AMOEBA_T_COUNT];
  int64_t layer_elems;
};

// A rectangle of bytes copied from one source rank into the target shard, within
// one layer: `rows` runs of `run` bytes, `*_pitch` bytes apart.  A contiguous copy
// has rows == 1.
struct Segment {
  int32_t src_rank;  // -1: fill with zeros
  int32_t part;      // 0: attention tensors (q, k, v, o and their gap), 1: FFN tensors
  int64_t src_off, src_pitch;
  int64_t dst_off, dst_pitch;
  int64_t rows, run;
};

// Padded partition-major FFN layout of one side, in bytes.
struct PaddedGeom {
  int64_t attn, attn_padded;  // dense attention part, rounded up to a page
  int64_t part, part_padded;  // one tensor-partition (gate, up and down are equal in size)
  int64_t stride;             // from one partition to the next: 3 padded tensor-partitions
  int64_t layer;
};

// Expert-wise FFN layout of one side of a mixture-of-experts plan, in bytes.
struct ExpertGeom {
  int64_t own;     // experts per rank
  int64_t first;   // offset of the first expert tensor in a layer
  int64_t tensor;  // one expert tensor (gate, up and down are equal in size)
  int64_t slot;    // from one expert to the next: 3 tensors, rounded up to a page if padded
  int64_t layer;
};

// Launch-shape overrides of the measurement interface (0 = the built-in choice).
struct Tuning {
  int w_grid = 0, w_unroll = 0, w_threads = 0, kv_grid = 0, kv_unroll = 0, kv_threads = 0,
      nontemporal = 0, kv_staged = 0, kv_blocks_hint = 0, kv_small = 0;
};

}  // namespace amoeba

struct amoeba_plan_s {
  amoeba_model_shape shape;
  int k, kp, rp;
  amoeba::ShardLayout src_layout, dst_layout;
  std::vector<amoeba::Segment> segments;  // one layer's worth, target order; src_rank -1 = zeros
  bool src_padded, dst_padded;
  amoeba::PaddedGeom pad_src, pad_dst;     // valid where the side is padded (dense FFN)
  amoeba::ExpertGeom exp_src, exp_dst;     // valid when shape.n_experts > 0
  int64_t src_layer_bytes, dst_layer_bytes;
  uint32_t weight_rank_mask, kv_rank_mask;
  // KV geometry
  int64_t heads_src, heads_dst;            // KV heads per rank on either side
  int64_t block_bytes_src, block_bytes_dst;
  // device side
  int device;           // device the workspace lives on, -1 if none
  int n_cu;             // compute units of that device
  int32_t* workspace;   // [8 header][num_seqs bases][dst_pool_blocks source ids]
  mutable const int32_t* status_ws;  // workspace of the last KV reshard enqueued on this plan
  size_t workspace_bytes;
  // in-place instance merge: m = dst_tp / src_tp when the plan qualifies, else 0
  int merge_factor;
  int32_t* merge_workspace;  // [8 header][chunk counts][P*m flags][P*m work list]
  size_t merge_workspace_bytes;
  amoeba::Tuning tune;
};

namespace amoeba {

// Fills every host-side field of `p` (not the device ones).  Returns false and
// writes a message to `err` when the shape or TP degrees are unsupported.
bool build_plan(amoeba_plan_s* p, const amoeba_model_shape* shape, int src_tp, int dst_tp,
                int dst_rank, std::string* err);

void set_error(const std::string& msg);

}  // namespace amoeba
