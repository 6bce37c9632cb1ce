// Host-side planning: shard geometry, copy segments, KV block geometry.
//
// The partition follows the paper's statement of tensor parallelism (Sec. 2.2:
// heads and FFN segments spread evenly over the workers) and of the FFN cut
// (Sec. 3.2, Eq. (1): up_proj by columns of U, down_proj by rows of D).  With
// [out, in] row-major storage the q/k/v/gate/up cuts fall on stored rows
// (contiguous ranges) and the o/down cuts on stored columns (strided ranges).
// Ownership is by contiguous index ranges (Sec. 3.1 head-range rule), so the
// target rank's range of each partitioned axis is intersected with every source
// rank's range; each non-empty intersection is one copy segment.
#include "plan.h"

#include <algorithm>

namespace amoeba {

namespace {

ShardLayout shard_layout(const amoeba_model_shape& s, int tp) {
  ShardLayout L;
  const int64_t H = s.hidden, d = s.head_dim;
  const bool moe = s.n_experts > 0;  // then gate/up/down describe the first owned expert
  const int64_t q = int64_t(s.n_q_heads) * d / tp, kv = int64_t(s.n_kv_heads) * d / tp,
                f = moe ? int64_t(s.ffn_dim) : int64_t(s.ffn_dim) / tp;
  const int64_t rows[AMOEBA_T_COUNT] = {q, kv, kv, H, f, f, H};
  const int64_t cols[AMOEBA_T_COUNT] = {H, H, H, q, H, H, f};
  int64_t at = 0;
  for (int t = 0; t < AMOEBA_T_COUNT; ++t) {
    L.off[t] = at;
    L.rows[t] = rows[t];
    L.cols[t] = cols[t];
    at += rows[t] * cols[t];
  }
  if (moe) at += (int64_t(s.n_experts) / tp - 1) * 3 * f * H;
  L.layer_elems = at;
  return L;
}

bool fail(std::string* err, const std::string& msg) {
  if (err) *err = msg;
  return false;
}

}  // namespace

bool build_plan(amoeba_plan_s* p, const amoeba_model_shape* shape, int k, int kp, int rp,
                std::string* err) {
  if (!shape) return fail(err, "shape is NULL");
  const amoeba_model_shape& s = *shape;
  if (s.n_layers <= 0 || s.hidden <= 0 || s.n_q_heads <= 0 || s.n_kv_heads <= 0 ||
      s.head_dim <= 0 || s.ffn_dim <= 0 || s.kv_block_tokens <= 0 || s.kv_layers <= 0)
    return fail(err, "model sizes must be positive");
  if (s.elem_bytes != 1 && s.elem_bytes != 2 && s.elem_bytes != 4)
    return fail(err, "elem_bytes must be 1, 2 or 4");
  if (s.n_q_heads % s.n_kv_heads) return fail(err, "n_q_heads must be a multiple of n_kv_heads");
  for (int lay : {s.kv_layout_src, s.kv_layout_dst})
    if (lay != AMOEBA_KV_HEAD_MAJOR && lay != AMOEBA_KV_TOKEN_MAJOR)
      return fail(err, "unknown KV layout");
  if (s.num_seqs < 0 || s.max_blocks_per_seq < 0 || s.src_pool_blocks < 0 ||
      s.dst_pool_blocks < 0)
    return fail(err, "negative table or pool size");
  if (s.kv_blocks_bound < 0) return fail(err, "kv_blocks_bound is negative");
  if (s.src_pool_blocks > INT32_MAX || s.dst_pool_blocks > INT32_MAX)
    return fail(err, "a pool has more than 2^31-1 blocks (block ids are int32)");
  for (int tp : {k, kp}) {
    if (tp < 1 || tp > AMOEBA_MAX_TP) return fail(err, "TP degree outside [1, 16]");
    if (s.n_q_heads % tp || s.n_kv_heads % tp)
      return fail(err, "TP degree must divide n_q_heads and n_kv_heads");
    if (s.n_experts > 0 ? s.n_experts % tp : s.ffn_dim % tp)
      return fail(err, s.n_experts > 0 ? "TP/EP degree must divide n_experts"
                                       : "TP degree must divide ffn_dim");
  }
  if (s.n_experts < 0) return fail(err, "n_experts is negative");
  const bool moe = s.n_experts > 0;
  if (rp < 0 || rp >= kp) return fail(err, "dst_rank outside [0, dst_tp)");
  for (int lay : {s.w_layout_src, s.w_layout_dst})
    if (lay != AMOEBA_W_DENSE && lay != AMOEBA_W_FFN_PADDED)
      return fail(err, "unknown weight layout");
  const bool any_padded = s.w_layout_src == AMOEBA_W_FFN_PADDED || s.w_layout_dst == AMOEBA_W_FFN_PADDED;
  if (any_padded) {
    if (!moe && (s.pad_max_tp < 1 || s.pad_max_tp > AMOEBA_MAX_TP || s.ffn_dim % s.pad_max_tp ||
        s.pad_max_tp % k || s.pad_max_tp % kp))
      return fail(err, "pad_max_tp must be in [1, 16], divide ffn_dim and be a multiple of both TP degrees");
    if (s.pad_page_bytes < s.elem_bytes || s.pad_page_bytes % s.elem_bytes)
      return fail(err, "pad_page_bytes must be a positive multiple of elem_bytes");
  }

  p->shape = s;
  p->k = k;
  p->kp = kp;
  p->rp = rp;
  p->src_layout = shard_layout(s, k);
  p->dst_layout = shard_layout(s, kp);
  p->segments.clear();
  p->weight_rank_mask = 0;

  const int64_t e = s.elem_bytes;
  const int64_t d = s.head_dim;
  p->src_padded = s.w_layout_src == AMOEBA_W_FFN_PADDED;
  p->dst_padded = s.w_layout_dst == AMOEBA_W_FFN_PADDED;
  p->src_layer_bytes = p->src_layout.layer_elems * e;
  p->dst_layer_bytes = p->dst_layout.layer_elems * e;
  if (any_padded && !moe) {
    const int64_t G = s.pad_page_bytes, T = s.pad_max_tp;
    auto pages = [G](int64_t bytes) { return (bytes + G - 1) / G * G; };
    auto padded_geom = [&](const ShardLayout& L, int tp) {
      PaddedGeom g;
      g.attn = L.off[AMOEBA_T_GATE] * e;  // q, k, v, o come first and stay dense
      g.attn_padded = pages(g.attn);
      g.part = int64_t(s.ffn_dim) / T * s.hidden * e;
      g.part_padded = pages(g.part);
      g.stride = 3 * g.part_padded;
      g.layer = g.attn_padded + (T / tp) * g.stride;
      return g;
    };
    p->pad_src = padded_geom(p->src_layout, k);
    p->pad_dst = padded_geom(p->dst_layout, kp);
    if (p->src_padded) p->src_layer_bytes = p->pad_src.layer;
    if (p->dst_padded) p->dst_layer_bytes = p->pad_dst.layer;
  }
  // extent of the partitioned axis of each tensor in the unsharded model
  const int64_t axis[AMOEBA_T_COUNT] = {int64_t(s.n_q_heads) * d, int64_t(s.n_kv_heads) * d,
                                        int64_t(s.n_kv_heads) * d, int64_t(s.n_q_heads) * d,
                                        s.ffn_dim,                 s.ffn_dim,
                                        s.ffn_dim};
  for (int t = 0; t < AMOEBA_T_COUNT; ++t) {
    if ((any_padded || moe) && t >= AMOEBA_T_GATE) break;  // FFN tensors: below
    const bool cut_on_rows = (t != AMOEBA_T_O && t != AMOEBA_T_DOWN);
    const int64_t N = axis[t], per_src = N / k, per_dst = N / kp;
    const int64_t want_lo = rp * per_dst, want_hi = want_lo + per_dst;
    for (int r = 0; r < k; ++r) {
      const int64_t lo = std::max(want_lo, r * per_src), hi = std::min(want_hi, (r + 1) * per_src);
      if (lo >= hi) continue;
      Segment g;
      g.src_rank = r;
      g.part = t >= AMOEBA_T_GATE;
      if (cut_on_rows) {
        const int64_t width = p->src_layout.cols[t];  // == hidden on both sides
        g.src_off = (p->src_layout.off[t] + (lo - r * per_src) * width) * e;
        g.dst_off = (p->dst_layout.off[t] + (lo - want_lo) * width) * e;
        g.rows = 1;
        g.run = (hi - lo) * width * e;
        g.src_pitch = g.dst_pitch = g.run;
      } else {
        g.src_off = (p->src_layout.off[t] + (lo - r * per_src)) * e;
        g.dst_off = (p->dst_layout.off[t] + (lo - want_lo)) * e;
        g.src_pitch = per_src * e;
        g.dst_pitch = per_dst * e;
        g.rows = p->src_layout.rows[t];  // == hidden on both sides
        g.run = (hi - lo) * e;
        if (g.run == g.src_pitch && g.run == g.dst_pitch) {  // whole rows: one contiguous range
          g.run *= g.rows;
          g.rows = 1;
          g.src_pitch = g.dst_pitch = g.run;
        }
      }
      p->segments.push_back(g);
      p->weight_rank_mask |= 1u << r;
    }
  }

  if (moe) {
    // Sec. 3.2, EP discussion: the FFN is stored expert by expert and whole experts change
    // owner.  The target's expert range is intersected with every source rank's range; the
    // experts of an intersection are equally spaced on both sides, so they form one
    // rectangle (one contiguous range when neither side has gaps).
    auto geom = [&](const ShardLayout& L, int tp, bool padded) {
      ExpertGeom g;
      const int64_t G = s.pad_page_bytes;
      g.own = int64_t(s.n_experts) / tp;
      g.first = L.off[AMOEBA_T_GATE] * e;
      g.tensor = int64_t(s.ffn_dim) * s.hidden * e;
      g.slot = 3 * g.tensor;
      if (padded) {
        g.first = (g.first + G - 1) / G * G;
        g.slot = (g.slot + G - 1) / G * G;
      }
      g.layer = g.first + g.own * g.slot;
      return g;
    };
    p->exp_src = geom(p->src_layout, k, p->src_padded);
    p->exp_dst = geom(p->dst_layout, kp, p->dst_padded);
    p->src_layer_bytes = p->exp_src.layer;
    p->dst_layer_bytes = p->exp_dst.layer;
    const ExpertGeom &S = p->exp_src, &D = p->exp_dst;
    const int64_t attn = p->dst_layout.off[AMOEBA_T_GATE] * e;
    if (D.first > attn) {
      Segment z{};
      z.src_rank = -1;
      z.part = 0;
      z.dst_off = attn;
      z.rows = 1;
      z.run = z.src_pitch = z.dst_pitch = D.first - attn;
      p->segments.push_back(z);
    }
    const int64_t want_lo = rp * D.own, want_hi = want_lo + D.own;
    for (int r = 0; r < k; ++r) {
      const int64_t lo = std::max(want_lo, r * S.own), hi = std::min(want_hi, (r + 1) * S.own);
      if (lo >= hi) continue;
      Segment g;
      g.src_rank = r;
      g.part = 1;
      g.src_off = S.first + (lo - r * S.own) * S.slot;
      g.dst_off = D.first + (lo - want_lo) * D.slot;
      g.rows = hi - lo;
      g.run = 3 * S.tensor;
      g.src_pitch = S.slot;
      g.dst_pitch = D.slot;
      if (g.run == g.src_pitch && g.run == g.dst_pitch) {
        g.run *= g.rows;
        g.rows = 1;
        g.src_pitch = g.dst_pitch = g.run;
      }
      p->segments.push_back(g);
      p->weight_rank_mask |= 1u << r;
      if (D.slot > 3 * D.tensor) {  // gaps behind every expert of a padded target
        Segment z{};
        z.src_rank = -1;
        z.part = 1;
        z.dst_off = g.dst_off + 3 * D.tensor;
        z.rows = hi - lo;
        z.run = D.slot - 3 * D.tensor;
        z.src_pitch = z.dst_pitch = D.slot;
        p->segments.push_back(z);
      }
    }
  } else if (any_padded) {
    // Sec. 3.2, Improvement 1.  Walk the finest partitions the target rank owns; each one
    // lives on exactly one source rank.  On a padded side a tensor-partition is one
    // contiguous, page-aligned range; on a dense side gate/up partitions are row ranges of
    // the fused tensor and a down partition is a column range (strided).
    const int64_t T = s.pad_max_tp, w = int64_t(s.ffn_dim) / T, H = s.hidden;
    const int64_t per_src = T / k, per_dst = T / kp;
    auto zero_fill = [&](int64_t off, int64_t bytes, int part) {
      if (bytes <= 0) return;
      Segment z;
      z.src_rank = -1;
      z.part = part;
      z.src_off = 0;
      z.dst_off = off;
      z.rows = 1;
      z.run = z.src_pitch = z.dst_pitch = bytes;
      p->segments.push_back(z);
    };
    if (p->dst_padded) zero_fill(p->pad_dst.attn, p->pad_dst.attn_padded - p->pad_dst.attn, 0);
    for (int64_t q = 0; q < per_dst; ++q) {
      const int64_t part = rp * per_dst + q;  // global partition index
      const int64_t r = part / per_src, qs = part - r * per_src;
      for (int t = AMOEBA_T_GATE; t <= AMOEBA_T_DOWN; ++t) {
        const int slot = t - AMOEBA_T_GATE;
        const bool is_down = t == AMOEBA_T_DOWN;
        Segment g;
        g.src_rank = int32_t(r);
        g.part = 1;
        // source side
        if (p->src_padded) {
          g.src_off = p->pad_src.attn_padded + qs * p->pad_src.stride + slot * p->pad_src.part_padded;
          g.src_pitch = w * e;
        } else if (!is_down) {
          g.src_off = (p->src_layout.off[t] + qs * w * H) * e;
          g.src_pitch = H * e;
        } else {
          g.src_off = (p->src_layout.off[t] + qs * w) * e;
          g.src_pitch = p->src_layout.cols[t] * e;
        }
        // target side
        if (p->dst_padded) {
          g.dst_off = p->pad_dst.attn_padded + q * p->pad_dst.stride + slot * p->pad_dst.part_padded;
          g.dst_pitch = w * e;
        } else if (!is_down) {
          g.dst_off = (p->dst_layout.off[t] + q * w * H) * e;
          g.dst_pitch = H * e;
        } else {
          g.dst_off = (p->dst_layout.off[t] + q * w) * e;
          g.dst_pitch = p->dst_layout.cols[t] * e;
        }
        if (!is_down || (g.src_pitch == w * e && g.dst_pitch == w * e)) {
          g.rows = 1;  // contiguous on both sides
          g.run = w * H * e;
          g.src_pitch = g.dst_pitch = g.run;
        } else {
          g.rows = H;
          g.run = w * e;
        }
        p->segments.push_back(g);
        p->weight_rank_mask |= 1u << r;
        if (p->dst_padded)
          zero_fill(g.dst_off + p->pad_dst.part, p->pad_dst.part_padded - p->pad_dst.part, 1);
      }
    }
  }

  // KV: contiguous head ranges again (Sec. 3.1); whole heads move, so only the
  // owning ranks are recorded here and the per-head mapping is done in the kernel.
  p->heads_src = s.n_kv_heads / k;
  p->heads_dst = s.n_kv_heads / kp;
  p->block_bytes_src = p->heads_src * 2 * s.kv_block_tokens * d * e;
  p->block_bytes_dst = p->heads_dst * 2 * s.kv_block_tokens * d * e;
  p->kv_rank_mask = 0;
  for (int64_t h = rp * p->heads_dst; h < (rp + 1) * p->heads_dst; ++h)
    p->kv_rank_mask |= 1u << (h / p->heads_src);

  // In-place merge of m = k'/k instances (Sec. 3.1, Improvement 1) needs the
  // header-centric block on both sides, where a rank's new head range is one
  // contiguous sub-block, and reshaped ids b*m + g that still fit an int32.
  p->merge_factor = 0;
  if (kp % k == 0 && kp / k >= 2 && s.kv_layout_src == AMOEBA_KV_HEAD_MAJOR &&
      s.kv_layout_dst == AMOEBA_KV_HEAD_MAJOR && s.src_pool_blocks * (kp / k) <= INT32_MAX)
    p->merge_factor = kp / k;
  return true;
}

}  // namespace amoeba
