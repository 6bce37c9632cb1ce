// CPU oracle (TEST INFRASTRUCTURE ONLY): per-element definition of the TP=k ->
// TP=k' reshard of decoder weights and of the paged KV cache.  Single thread,
// no blocking, no shared code with the HIP library.  See amoeba_oracle.h for
// the paper passages each part follows.
#include "amoeba_oracle.h"

#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

bool divides(int tp, int64_t n) { return tp > 0 && n % tp == 0; }

bool model_ok(const ao_model* m) {
  return m && m->n_layers > 0 && m->hidden > 0 && m->n_q_heads > 0 && m->n_kv_heads > 0 &&
         m->head_dim > 0 && m->ffn_dim > 0 &&
         (m->elem_bytes == 1 || m->elem_bytes == 2 || m->elem_bytes == 4) &&
         m->n_q_heads % m->n_kv_heads == 0;
}

bool tp_ok(const ao_model* m, int tp) {
  return divides(tp, m->n_q_heads) && divides(tp, m->n_kv_heads) && divides(tp, m->ffn_dim);
}

// Geometry of one rank's per-layer shard at TP=t (element offsets inside a layer).
struct ShardGeom {
  int64_t q_rows, kv_rows, ffn_rows;  // rows of Wq / Wk,Wv / Wg,Wu held by one rank
  int64_t o_cols, down_cols;          // columns of Wo / Wd held by one rank
  int64_t off_qkv, off_o, off_gate_up, off_down, layer_elems;
};

ShardGeom geom(const ao_model* m, int t) {
  ShardGeom g;
  const int64_t H = m->hidden, d = m->head_dim;
  g.q_rows = (int64_t)m->n_q_heads * d / t;
  g.kv_rows = (int64_t)m->n_kv_heads * d / t;
  g.ffn_rows = (int64_t)m->ffn_dim / t;
  g.o_cols = g.q_rows;
  g.down_cols = g.ffn_rows;
  g.off_qkv = 0;
  g.off_o = g.off_qkv + (g.q_rows + 2 * g.kv_rows) * H;
  g.off_gate_up = g.off_o + H * g.o_cols;
  g.off_down = g.off_gate_up + 2 * g.ffn_rows * H;
  g.layer_elems = g.off_down + H * g.down_cols;
  return g;
}

// Sec. 3.2: a tensor cut along stored rows (q, k, v, gate, up).  `rows_total`
// is the unsharded row count; the sub-block starts `sub_src` / `sub_dst`
// elements into the fused per-rank tensor on either side.
template <typename E>
void gather_row_cut(const E* const* src, E* dst, int64_t src_layer_base, int64_t dst_layer_base,
                    int64_t sub_src, int64_t sub_dst, int64_t rows_total, int64_t cols, int k,
                    int kp, int rp) {
  const int64_t rows_src = rows_total / k, rows_dst = rows_total / kp;
  for (int64_t rho = 0; rho < rows_dst; ++rho) {
    const int64_t g = (int64_t)rp * rows_dst + rho;  // row in the unsharded tensor
    const int64_t s = g / rows_src;                  // owning source rank
    const int64_t lr = g % rows_src;                 // row inside that rank's sub-block
    const E* from = src[s] + src_layer_base + sub_src + lr * cols;
    E* to = dst + dst_layer_base + sub_dst + rho * cols;
    for (int64_t j = 0; j < cols; ++j) to[j] = from[j];
  }
}

// Sec. 3.2: a tensor cut along stored columns (o_proj, down_proj).
template <typename E>
void gather_col_cut(const E* const* src, E* dst, int64_t src_layer_base, int64_t dst_layer_base,
                    int64_t t_src, int64_t t_dst, int64_t rows, int64_t cols_total, int k, int kp,
                    int rp) {
  const int64_t cols_src = cols_total / k, cols_dst = cols_total / kp;
  for (int64_t i = 0; i < rows; ++i) {
    for (int64_t c = 0; c < cols_dst; ++c) {
      const int64_t g = (int64_t)rp * cols_dst + c;  // column in the unsharded tensor
      const int64_t s = g / cols_src;
      const int64_t lc = g % cols_src;
      dst[dst_layer_base + t_dst + i * cols_dst + c] =
          src[s][src_layer_base + t_src + i * cols_src + lc];
    }
  }
}

template <typename E>
int reshard_weights_t(const ao_model* m, int k, int kp, int rp, const void* const* src_v,
                      void* dst_v) {
  const ShardGeom gs = geom(m, k), gd = geom(m, kp);
  const int64_t H = m->hidden, d = m->head_dim;
  const int64_t Nq = (int64_t)m->n_q_heads * d, Nkv = (int64_t)m->n_kv_heads * d, I = m->ffn_dim;

  // Which source ranks hold something of the target?  (Needed ones must be non-NULL.)
  const E* src[64];
  for (int s = 0; s < k; ++s) src[s] = static_cast<const E*>(src_v[s]);
  for (int s = 0; s < k; ++s) {
    bool needed = false;
    const int64_t tot[3] = {Nq, Nkv, I};
    for (int a = 0; a < 3; ++a) {
      const int64_t lo = rp * (tot[a] / kp), hi = lo + tot[a] / kp;
      const int64_t slo = s * (tot[a] / k), shi = slo + tot[a] / k;
      if (lo < shi && slo < hi) needed = true;
    }
    if (needed && !src[s]) return AO_ERR_ARG;
  }
  E* dst = static_cast<E*>(dst_v);

  for (int64_t l = 0; l < m->n_layers; ++l) {
    const int64_t sb = l * gs.layer_elems, db = l * gd.layer_elems;
    // fused qkv: [q_r ; k_r ; v_r], each cut along rows by head ranges
    gather_row_cut(src, dst, sb, db, gs.off_qkv, gd.off_qkv, Nq, H, k, kp, rp);
    gather_row_cut(src, dst, sb, db, gs.off_qkv + gs.q_rows * H, gd.off_qkv + gd.q_rows * H, Nkv,
                   H, k, kp, rp);
    gather_row_cut(src, dst, sb, db, gs.off_qkv + (gs.q_rows + gs.kv_rows) * H,
                   gd.off_qkv + (gd.q_rows + gd.kv_rows) * H, Nkv, H, k, kp, rp);
    // o_proj: cut along columns (input features = q heads)
    gather_col_cut(src, dst, sb, db, gs.off_o, gd.off_o, H, Nq, k, kp, rp);
    // fused gate_up: [g_r ; u_r], each cut along rows
    gather_row_cut(src, dst, sb, db, gs.off_gate_up, gd.off_gate_up, I, H, k, kp, rp);
    gather_row_cut(src, dst, sb, db, gs.off_gate_up + gs.ffn_rows * H,
                   gd.off_gate_up + gd.ffn_rows * H, I, H, k, kp, rp);
    // down_proj: cut along columns
    gather_col_cut(src, dst, sb, db, gs.off_down, gd.off_down, H, I, k, kp, rp);
  }
  return AO_OK;
}

bool kv_ok(const ao_kv* c) {
  return c && c->kv_layers > 0 && c->n_kv_heads > 0 && c->head_dim > 0 && c->block_tokens > 0 &&
         (c->elem_bytes == 1 || c->elem_bytes == 2 || c->elem_bytes == 4) &&
         (c->layout_src == AO_LAYOUT_HEAD_MAJOR || c->layout_src == AO_LAYOUT_TOKEN_MAJOR) &&
         (c->layout_dst == AO_LAYOUT_HEAD_MAJOR || c->layout_dst == AO_LAYOUT_TOKEN_MAJOR) &&
         c->num_seqs >= 0 && c->max_blocks_per_seq >= 0 && c->src_pool_blocks >= 0 &&
         c->dst_pool_blocks >= 0;
}

// Element index inside one block.  h: head local to the rank, c: 0 = K, 1 = V,
// t: token slot, x: position in the head vector, heads: heads per rank.
//   header-centric  [Header, K/V, Token, d]   (Sec. 3.1, Improvement 1)
//   token-first     [K/V, Token, Header, d]   (Sec. 3.1, base layout)
int64_t block_index(int layout, int64_t h, int64_t c, int64_t t, int64_t x, int64_t heads,
                    int64_t B, int64_t d) {
  if (layout == AO_LAYOUT_HEAD_MAJOR) return ((h * 2 + c) * B + t) * d + x;
  return ((c * B + t) * heads + h) * d + x;
}

template <typename E>
int reshard_kv_t(const ao_kv* c, int k, int kp, int rp, const void* const* src_v,
                 const int32_t* src_table, const int32_t* seq_lens, void* dst_v,
                 int32_t* dst_table, int64_t* total_out) {
  const int64_t S = c->num_seqs, W = c->max_blocks_per_seq, B = c->block_tokens, d = c->head_dim;
  const int64_t Hs = c->n_kv_heads / k, Hd = c->n_kv_heads / kp;
  const int64_t src_block = Hs * 2 * B * d, dst_block = Hd * 2 * B * d;

  const E* src[64];
  for (int s = 0; s < k; ++s) src[s] = static_cast<const E*>(src_v[s]);
  for (int64_t hp = 0; hp < Hd; ++hp)  // every rank owning a needed head must be present
    if (!src[((int64_t)rp * Hd + hp) / Hs]) return AO_ERR_ARG;

  if (total_out) *total_out = 0;
  for (int64_t i = 0; i < S * W; ++i) dst_table[i] = -1;

  // step 1: blocks per sequence and the exclusive prefix sum, with the checks
  bool overflow = false;
  int64_t total = 0;
  for (int64_t i = 0; i < S; ++i) {
    const int64_t len = seq_lens[i];
    if (len < 0) { overflow = true; continue; }
    const int64_t nb = (len + B - 1) / B;
    if (nb > W) overflow = true;
    total += nb;
  }
  if (total > c->dst_pool_blocks) overflow = true;
  if (overflow) return AO_ERR_OVERFLOW;

  // step 2: the new table, sequence-major compact ids
  int64_t base = 0;
  for (int64_t i = 0; i < S; ++i) {
    const int64_t nb = ((int64_t)seq_lens[i] + B - 1) / B;
    for (int64_t j = 0; j < nb; ++j) dst_table[i * W + j] = (int32_t)(base + j);
    base += nb;
  }
  if (total_out) *total_out = total;

  // step 3: move the heads the target rank owns
  E* dst = static_cast<E*>(dst_v);
  bool bad_id = false;
  for (int64_t l = 0; l < c->kv_layers; ++l) {
    for (int64_t i = 0; i < S; ++i) {
      const int64_t nb = ((int64_t)seq_lens[i] + B - 1) / B;
      for (int64_t j = 0; j < nb; ++j) {
        const int64_t sb = src_table[i * W + j];
        const int64_t db = dst_table[i * W + j];
        if (sb < 0 || sb >= c->src_pool_blocks) { bad_id = true; continue; }
        for (int64_t t = 0; t < B; ++t)
          for (int64_t kv = 0; kv < 2; ++kv)
            for (int64_t hp = 0; hp < Hd; ++hp) {
              const int64_t h = (int64_t)rp * Hd + hp;  // global KV head
              const int64_t s = h / Hs;                 // source rank that owns it
              const int64_t hs = h % Hs;                // its index on that rank
              const E* from = src[s] + (l * c->src_pool_blocks + sb) * src_block;
              E* to = dst + (l * c->dst_pool_blocks + db) * dst_block;
              for (int64_t x = 0; x < d; ++x)
                to[block_index(c->layout_dst, hp, kv, t, x, Hd, B, d)] =
                    from[block_index(c->layout_src, hs, kv, t, x, Hs, B, d)];
            }
      }
    }
  }
  return bad_id ? AO_ERR_BLOCK_ID : AO_OK;
}

template <typename E>
int merge_kv_inplace_t(const ao_kv* c, int k, int m, int rp, void* local_v,
                       const void* const* remote_v, const int32_t* const* tables,
                       const int32_t* const* lens, int32_t* dst_table, int64_t* remote_out) {
  const int64_t S = c->num_seqs, W = c->max_blocks_per_seq, B = c->block_tokens, d = c->head_dim;
  const int64_t P = c->src_pool_blocks;
  const int64_t g = rp % m;                            // instance hosted here
  const int64_t heads_new = c->n_kv_heads / ((int64_t)k * m);
  const int64_t sub = heads_new * 2 * B * d;           // elements of one new (sub-)block
  const int64_t old_block = sub * m;
  if (remote_out) *remote_out = 0;
  for (int64_t i = 0; i < (int64_t)m * S * W; ++i) dst_table[i] = -1;

  for (int64_t g2 = 0; g2 < m; ++g2)
    for (int64_t i = 0; i < S; ++i) {
      const int64_t len = lens[g2][i];
      if (len < 0 || (len + B - 1) / B > W) return AO_ERR_OVERFLOW;
    }

  E* local = static_cast<E*>(local_v);
  bool bad_id = false;
  // remote_blocks_out counts the slots of the reshaped pool that receive remote heads: one
  // per distinct new id.  An id outside the pool has no slot and is not counted; a block two
  // sequences of one instance share is one slot, filled (twice, with the same bytes) and
  // counted once.  It is the number the bytes moved follow from: count x sub-block x layers.
  std::vector<char> filled((size_t)(P * m), 0);
  int64_t copied = 0;
  for (int64_t g2 = 0; g2 < m; ++g2) {
    const E* remote = static_cast<const E*>(remote_v[g2]);
    for (int64_t i = 0; i < S; ++i) {
      const int64_t nb = ((int64_t)lens[g2][i] + B - 1) / B;
      for (int64_t j = 0; j < nb; ++j) {
        const int64_t b = tables[g2][i * W + j];
        if (b < 0 || b >= P) { bad_id = true; continue; }
        const int64_t id = b * m + g2;                 // reshaped id, same on every rank
        dst_table[(g2 * S + i) * W + j] = (int32_t)id;
        if (g2 == g) continue;                         // local heads stay where they are
        if (!filled[(size_t)id]) { filled[(size_t)id] = 1; ++copied; }
        for (int64_t l = 0; l < c->kv_layers; ++l) {
          const E* from = remote + (l * P + b) * old_block + g * sub;  // heads of r' in block b
          E* to = local + (l * P * m + id) * sub;
          for (int64_t x = 0; x < sub; ++x) to[x] = from[x];
        }
      }
    }
  }
  if (remote_out) *remote_out = copied;
  return bad_id ? AO_ERR_BLOCK_ID : AO_OK;
}

// ---- base solution of Sec. 3.1: migration, then de-fragmentation ---------------------------
//
// m instances at TP=k become one at TP=k*m without the in-place trick.  The worker that hosted
// rank s of instance g becomes rank r' = s*m + g.  It gets a second pool ("reserved pages" for
// what it receives, plus room for its own cache in compact form) and two passes fill it:
//   migration        for every request of every OTHER instance, the heads of r' are taken
//                    out of the sender's blocks and stored in reserved blocks;
//   de-fragmentation for every LOCAL request, the heads r' keeps are taken out of the old
//                    blocks (where they sit between the heads that were given away) and
//                    stored compactly; afterwards the old pool can be released.
// New ids are compact over the merged sequence list in instance-major order, so the table is
// the same on every worker and instance g2's blocks are the id range starting at the number
// of blocks of instances 0 .. g2-1.
template <typename E>
int merge_kv_base_t(const ao_kv* c, int k, int m, int rp, const void* const* pools_v,
                    const int32_t* const* tables, const int32_t* const* lens, void* new_pool_v,
                    int32_t* dst_table, int64_t* migrated_out, int64_t* defrag_out) {
  const int64_t S = c->num_seqs, W = c->max_blocks_per_seq, B = c->block_tokens, d = c->head_dim;
  const int64_t P = c->src_pool_blocks, Pn = c->dst_pool_blocks;
  const int64_t g = rp % m;                          // the instance hosted here
  const int64_t Hs = c->n_kv_heads / k;              // heads in an old block
  const int64_t Hd = c->n_kv_heads / ((int64_t)k * m);  // heads in a new block
  const int64_t old_block = Hs * 2 * B * d, new_block = Hd * 2 * B * d;
  if (migrated_out) *migrated_out = 0;
  if (defrag_out) *defrag_out = 0;
  for (int64_t i = 0; i < (int64_t)m * S * W; ++i) dst_table[i] = -1;

  // blocks per sequence, checks, compact ids
  int64_t total = 0;
  bool overflow = false;
  for (int64_t g2 = 0; g2 < m; ++g2)
    for (int64_t i = 0; i < S; ++i) {
      const int64_t len = lens[g2][i];
      if (len < 0) { overflow = true; continue; }
      const int64_t nb = (len + B - 1) / B;
      if (nb > W) overflow = true;
      total += nb;
    }
  if (total > Pn) overflow = true;
  if (overflow) return AO_ERR_OVERFLOW;
  int64_t next = 0;
  for (int64_t g2 = 0; g2 < m; ++g2)
    for (int64_t i = 0; i < S; ++i) {
      const int64_t nb = ((int64_t)lens[g2][i] + B - 1) / B;
      for (int64_t j = 0; j < nb; ++j) dst_table[(g2 * S + i) * W + j] = (int32_t)next++;
    }

  E* fresh = static_cast<E*>(new_pool_v);
  bool bad_id = false;
  // heads [g*Hd, (g+1)*Hd) of the old block are the ones rank r' owns: its global range
  // [r'*Hd, (r'+1)*Hd) starts at s*Hs + g*Hd and rank s's block starts at head s*Hs
  auto move_heads = [&](int64_t g2, int64_t* count) {
    const E* pool = static_cast<const E*>(pools_v[g2]);
    for (int64_t i = 0; i < S; ++i) {
      const int64_t nb = ((int64_t)lens[g2][i] + B - 1) / B;
      for (int64_t j = 0; j < nb; ++j) {
        const int64_t sb = tables[g2][i * W + j];
        const int64_t db = dst_table[(g2 * S + i) * W + j];
        if (sb < 0 || sb >= P) { bad_id = true; continue; }
        ++*count;
        for (int64_t l = 0; l < c->kv_layers; ++l) {
          const E* from = pool + (l * P + sb) * old_block;
          E* to = fresh + (l * Pn + db) * new_block;
          for (int64_t t = 0; t < B; ++t)
            for (int64_t kv = 0; kv < 2; ++kv)
              for (int64_t hp = 0; hp < Hd; ++hp)
                for (int64_t x = 0; x < d; ++x)
                  to[block_index(c->layout_dst, hp, kv, t, x, Hd, B, d)] =
                      from[block_index(c->layout_src, g * Hd + hp, kv, t, x, Hs, B, d)];
        }
      }
    }
  };
  int64_t migrated = 0, defragged = 0;
  for (int64_t g2 = 0; g2 < m; ++g2)  // pass 1: migration of the remote requests
    if (g2 != g) move_heads(g2, &migrated);
  move_heads(g, &defragged);          // pass 2: de-fragmentation of the local requests
  if (migrated_out) *migrated_out = migrated;
  if (defrag_out) *defrag_out = defragged;
  return bad_id ? AO_ERR_BLOCK_ID : AO_OK;
}

// ---- padded, partition-major FFN layout (Sec. 3.2, Improvement 1) ---------------------
//
// T = pad->max_tp is the finest TP degree of the model's TP set.  Every FFN tensor is cut in
// T partitions (gate/up by stored rows, down by stored columns, Eq. (1)); a rank at TP=t
// stores its T/t partitions one after the other, each tensor-partition starting on a
// multiple of page_bytes with zeros in the gap (U' = [U1,0,U2,0,..], D' likewise):
//   layer = [qkv_r | o_r | zeros to a page][gate_p | 0][up_p | 0][down_p | 0] for p = r*T/t ..
// with down_p stored as its own row-major [hidden][ffn/T] matrix.

struct PadGeom {
  int64_t attn, attn_padded;  // elements of the dense attention part, rounded up to a page
  int64_t part, part_padded;  // elements of one tensor-partition (gate, up and down alike)
  int64_t stride;             // elements from one partition to the next (3 padded tensors)
  int64_t layer;              // elements per layer
};

int64_t round_up(int64_t x, int64_t g) { return (x + g - 1) / g * g; }

PadGeom pad_geom(const ao_model* m, const ao_pad* pad, int tp) {
  PadGeom g;
  const int64_t page = pad->page_bytes / m->elem_bytes;
  const ShardGeom d = geom(m, tp);
  g.attn = d.off_gate_up;
  g.attn_padded = round_up(g.attn, page);
  g.part = (int64_t)m->ffn_dim / pad->max_tp * m->hidden;
  g.part_padded = round_up(g.part, page);
  g.stride = 3 * g.part_padded;
  g.layer = g.attn_padded + (int64_t)(pad->max_tp / tp) * g.stride;
  return g;
}

struct Loc { int64_t rank, off; };  // owning rank, element offset inside that rank's layer

// One side of a reshard: its TP degree, whether it uses the padded layout, its geometry.
struct Side {
  bool padded;
  int tp;
  ShardGeom g;
  PadGeom pg;
};

Side make_side(const ao_model* m, const ao_pad* pad, bool padded, int tp) {
  Side s;
  s.padded = padded;
  s.tp = tp;
  s.g = geom(m, tp);
  s.pg = pad_geom(m, pad, tp);
  return s;
}

// Where element (row, col) of unsharded tensor `t` (0..6 = q,k,v,o,gate,up,down) lives on a side.
Loc locate(const ao_model* m, const ao_pad* pad, const Side& sd, int t, int64_t row, int64_t col) {
  const int64_t H = m->hidden, d = m->head_dim, I = m->ffn_dim;
  const int64_t Nq = (int64_t)m->n_q_heads * d, Nkv = (int64_t)m->n_kv_heads * d;
  const ShardGeom& g = sd.g;
  const bool cut_rows = (t != 3 && t != 6);
  const int64_t axis[7] = {Nq, Nkv, Nkv, Nq, I, I, I};
  const int64_t per = axis[t] / sd.tp;
  const int64_t a = cut_rows ? row : col;     // index along the partitioned axis
  Loc L;
  L.rank = a / per;
  const int64_t la = a % per;                 // the same index inside the owner's share
  if (t <= 3 || !sd.padded) {
    switch (t) {
      case 0: L.off = g.off_qkv + la * H + col; break;
      case 1: L.off = g.off_qkv + g.q_rows * H + la * H + col; break;
      case 2: L.off = g.off_qkv + (g.q_rows + g.kv_rows) * H + la * H + col; break;
      case 3: L.off = g.off_o + row * g.o_cols + la; break;
      case 4: L.off = g.off_gate_up + la * H + col; break;
      case 5: L.off = g.off_gate_up + g.ffn_rows * H + la * H + col; break;
      default: L.off = g.off_down + row * g.down_cols + la; break;
    }
    return L;
  }
  const PadGeom& pg = sd.pg;
  const int64_t w = I / pad->max_tp;          // rows (gate/up) or columns (down) per partition
  const int64_t base = pg.attn_padded + (la / w) * pg.stride;
  const int64_t in = la % w;
  if (t == 4) L.off = base + in * H + col;
  else if (t == 5) L.off = base + pg.part_padded + in * H + col;
  else L.off = base + 2 * pg.part_padded + row * w + in;
  return L;
}

bool pad_ok(const ao_model* m, const ao_pad* pad, int tp) {
  return pad && pad->max_tp >= 1 && pad->page_bytes >= m->elem_bytes &&
         pad->page_bytes % m->elem_bytes == 0 && m->ffn_dim % pad->max_tp == 0 &&
         pad->max_tp % tp == 0;
}

template <typename E>
int reshard_weights_padded_t(const ao_model* m, const ao_pad* pad, int k, int kp, int rp,
                             const void* const* src_v, void* dst_v) {
  const bool sp = pad->src_padded != 0, dp = pad->dst_padded != 0;
  const Side src_side = make_side(m, pad, sp, k), dst_side = make_side(m, pad, dp, kp);
  const int64_t src_layer = sp ? src_side.pg.layer : src_side.g.layer_elems;
  const int64_t dst_layer = dp ? dst_side.pg.layer : dst_side.g.layer_elems;
  const int64_t H = m->hidden, d = m->head_dim, I = m->ffn_dim;
  const int64_t Nq = (int64_t)m->n_q_heads * d, Nkv = (int64_t)m->n_kv_heads * d;
  const int64_t rows[7] = {Nq, Nkv, Nkv, H, I, I, H}, cols[7] = {H, H, H, Nq, H, H, I};
  E* dst = static_cast<E*>(dst_v);
  if (dp)  // the gaps hold zeros
    for (int64_t i = 0; i < dst_layer * m->n_layers; ++i) dst[i] = 0;
  for (int64_t l = 0; l < m->n_layers; ++l)
    for (int t = 0; t < 7; ++t) {
      const bool cut_rows = (t != 3 && t != 6);
      const int64_t per = (cut_rows ? rows[t] : cols[t]) / kp;
      const int64_t r0 = cut_rows ? rp * per : 0, r1 = cut_rows ? r0 + per : rows[t];
      const int64_t c0 = cut_rows ? 0 : rp * per, c1 = cut_rows ? cols[t] : c0 + per;
      for (int64_t r = r0; r < r1; ++r)
        for (int64_t c = c0; c < c1; ++c) {
          const Loc to = locate(m, pad, dst_side, t, r, c);
          const Loc from = locate(m, pad, src_side, t, r, c);
          const E* src = static_cast<const E*>(src_v[from.rank]);
          if (!src) return AO_ERR_ARG;
          dst[l * dst_layer + to.off] = src[l * src_layer + from.off];
        }
    }
  return AO_OK;
}

// ---- mixture of experts (Sec. 3.2, EP discussion; TPkEPk of Sec. 4.3) ---------------------
// Attention tensors are cut by head as in the dense model; the FFN is stored expert by expert
// and rank r at degree t owns experts [r*E/t, (r+1)*E/t) whole.

bool moe_ok(const ao_model* m, const ao_moe* x, int tp) {
  return x && x->n_experts > 0 && divides(tp, m->n_q_heads) && divides(tp, m->n_kv_heads) &&
         divides(tp, x->n_experts) &&
         (x->page_bytes == 0 || (x->page_bytes >= m->elem_bytes && x->page_bytes % m->elem_bytes == 0));
}

struct MoeGeom {
  int64_t own;      // experts per rank
  int64_t first;    // element offset of the first expert tensor in a layer
  int64_t tensor;   // elements of one expert tensor (gate, up and down are equal in size)
  int64_t slot;     // elements from one expert to the next: 3 tensors, rounded up to a page
  int64_t layer;
};

MoeGeom moe_geom(const ao_model* m, const ao_moe* x, bool padded, int tp) {
  MoeGeom g;
  const int64_t page = padded ? x->page_bytes / m->elem_bytes : 1;  // in elements
  const int64_t attn = geom(m, tp).off_gate_up;                     // q, k, v, o of this rank
  g.own = x->n_experts / tp;
  g.first = (attn + page - 1) / page * page;
  g.tensor = (int64_t)m->ffn_dim * m->hidden;
  g.slot = (3 * g.tensor + page - 1) / page * page;
  g.layer = g.first + g.own * g.slot;
  return g;
}

template <typename E>
int reshard_weights_moe_t(const ao_model* m, const ao_moe* x, int k, int kp, int rp,
                          const void* const* src_v, void* dst_v) {
  const bool sp = x->src_padded && x->page_bytes, dp = x->dst_padded && x->page_bytes;
  const ShardGeom as = geom(m, k), ad = geom(m, kp);  // attention offsets only
  const MoeGeom gs = moe_geom(m, x, sp, k), gd = moe_geom(m, x, dp, kp);
  const int64_t H = m->hidden, d = m->head_dim;
  const int64_t Nq = (int64_t)m->n_q_heads * d, Nkv = (int64_t)m->n_kv_heads * d;
  const E* src[64];
  for (int s = 0; s < k; ++s) src[s] = static_cast<const E*>(src_v[s]);
  E* dst = static_cast<E*>(dst_v);
  // every source rank that owns a wanted head or expert must be present
  for (int s = 0; s < k; ++s) {
    bool needed = false;
    const int64_t tot[3] = {m->n_q_heads, m->n_kv_heads, x->n_experts};
    for (int a = 0; a < 3; ++a) {
      const int64_t lo = rp * (tot[a] / kp), hi = lo + tot[a] / kp;
      const int64_t slo = s * (tot[a] / k), shi = slo + tot[a] / k;
      if (lo < shi && slo < hi) needed = true;
    }
    if (needed && !src[s]) return AO_ERR_ARG;
  }
  if (dp)
    for (int64_t i = 0; i < gd.layer * m->n_layers; ++i) dst[i] = 0;
  for (int64_t l = 0; l < m->n_layers; ++l) {
    const int64_t sb = l * gs.layer, db = l * gd.layer;
    gather_row_cut(src, dst, sb, db, as.off_qkv, ad.off_qkv, Nq, H, k, kp, rp);
    gather_row_cut(src, dst, sb, db, as.off_qkv + as.q_rows * H, ad.off_qkv + ad.q_rows * H, Nkv,
                   H, k, kp, rp);
    gather_row_cut(src, dst, sb, db, as.off_qkv + (as.q_rows + as.kv_rows) * H,
                   ad.off_qkv + (ad.q_rows + ad.kv_rows) * H, Nkv, H, k, kp, rp);
    gather_col_cut(src, dst, sb, db, as.off_o, ad.off_o, H, Nq, k, kp, rp);
    for (int64_t j = 0; j < gd.own; ++j) {       // j-th expert of the target rank
      const int64_t ex = rp * gd.own + j;        // its index in the model
      const int64_t s = ex / gs.own;             // source rank that owns it
      const int64_t js = ex % gs.own;            // its position on that rank
      for (int64_t w = 0; w < 3; ++w)            // gate, up, down
        for (int64_t i = 0; i < gd.tensor; ++i)
          dst[db + gd.first + j * gd.slot + w * gd.tensor + i] =
              src[s][sb + gs.first + js * gs.slot + w * gs.tensor + i];
    }
  }
  return AO_OK;
}

}  // namespace

extern "C" {

int64_t ao_shard_elems(const ao_model* m, int tp) {
  if (!model_ok(m) || !tp_ok(m, tp)) return -1;
  return geom(m, tp).layer_elems * m->n_layers;
}

int64_t ao_kv_block_elems(const ao_kv* c, int tp) {
  if (!kv_ok(c) || !divides(tp, c->n_kv_heads)) return -1;
  return (int64_t)(c->n_kv_heads / tp) * 2 * c->block_tokens * c->head_dim;
}

int ao_reshard_weights(const ao_model* m, int src_tp, int dst_tp, int dst_rank,
                       const void* const* src_shards, void* dst) {
  if (!model_ok(m) || src_tp > 64 || !tp_ok(m, src_tp) || !tp_ok(m, dst_tp) || dst_rank < 0 ||
      dst_rank >= dst_tp || !src_shards || !dst)
    return AO_ERR_ARG;
  switch (m->elem_bytes) {
    case 1: return reshard_weights_t<uint8_t>(m, src_tp, dst_tp, dst_rank, src_shards, dst);
    case 2: return reshard_weights_t<uint16_t>(m, src_tp, dst_tp, dst_rank, src_shards, dst);
    default: return reshard_weights_t<uint32_t>(m, src_tp, dst_tp, dst_rank, src_shards, dst);
  }
}

int ao_reshard_kv(const ao_kv* c, int src_tp, int dst_tp, int dst_rank,
                  const void* const* src_pools, const int32_t* src_table,
                  const int32_t* seq_lens, void* dst_pool, int32_t* dst_table,
                  int64_t* total_blocks_out) {
  if (!kv_ok(c) || src_tp > 64 || !divides(src_tp, c->n_kv_heads) ||
      !divides(dst_tp, c->n_kv_heads) || dst_rank < 0 || dst_rank >= dst_tp || !src_pools ||
      !dst_pool || (c->num_seqs > 0 && (!seq_lens || !src_table || !dst_table)))
    return AO_ERR_ARG;
  switch (c->elem_bytes) {
    case 1:
      return reshard_kv_t<uint8_t>(c, src_tp, dst_tp, dst_rank, src_pools, src_table, seq_lens,
                                   dst_pool, dst_table, total_blocks_out);
    case 2:
      return reshard_kv_t<uint16_t>(c, src_tp, dst_tp, dst_rank, src_pools, src_table, seq_lens,
                                    dst_pool, dst_table, total_blocks_out);
    default:
      return reshard_kv_t<uint32_t>(c, src_tp, dst_tp, dst_rank, src_pools, src_table, seq_lens,
                                    dst_pool, dst_table, total_blocks_out);
  }
}

int ao_merge_kv_inplace(const ao_kv* c, int src_tp, int m, int dst_rank, void* local_pool,
                        const void* const* remote_pools, const int32_t* const* src_tables,
                        const int32_t* const* seq_lens, int32_t* dst_table,
                        int64_t* remote_blocks_out) {
  if (!kv_ok(c) || m < 1 || m > 64 || src_tp < 1 || !divides(src_tp * m, c->n_kv_heads) ||
      dst_rank < 0 || dst_rank >= src_tp * m || c->layout_src != AO_LAYOUT_HEAD_MAJOR ||
      c->layout_dst != AO_LAYOUT_HEAD_MAJOR || !local_pool || !remote_pools || !src_tables ||
      !seq_lens || !dst_table)
    return AO_ERR_ARG;
  for (int g2 = 0; g2 < m; ++g2) {
    if (!src_tables[g2] || !seq_lens[g2]) return AO_ERR_ARG;
    if (g2 != dst_rank % m && !remote_pools[g2]) return AO_ERR_ARG;
  }
  switch (c->elem_bytes) {
    case 1:
      return merge_kv_inplace_t<uint8_t>(c, src_tp, m, dst_rank, local_pool, remote_pools,
                                         src_tables, seq_lens, dst_table, remote_blocks_out);
    case 2:
      return merge_kv_inplace_t<uint16_t>(c, src_tp, m, dst_rank, local_pool, remote_pools,
                                          src_tables, seq_lens, dst_table, remote_blocks_out);
    default:
      return merge_kv_inplace_t<uint32_t>(c, src_tp, m, dst_rank, local_pool, remote_pools,
                                          src_tables, seq_lens, dst_table, remote_blocks_out);
  }
}

int ao_merge_kv_base(const ao_kv* c, int src_tp, int m, int dst_rank, const void* const* pools,
                     const int32_t* const* src_tables, const int32_t* const* seq_lens,
                     void* new_pool, int32_t* dst_table, int64_t* migrated_blocks_out,
                     int64_t* defrag_blocks_out) {
  if (!kv_ok(c) || m < 2 || m > 64 || src_tp < 1 || !divides(src_tp * m, c->n_kv_heads) ||
      dst_rank < 0 || dst_rank >= src_tp * m || !pools || !src_tables || !seq_lens ||
      !dst_table || (!new_pool && c->dst_pool_blocks > 0))
    return AO_ERR_ARG;
  for (int g2 = 0; g2 < m; ++g2)
    if (!src_tables[g2] || !seq_lens[g2] || !pools[g2]) return AO_ERR_ARG;
  switch (c->elem_bytes) {
    case 1:
      return merge_kv_base_t<uint8_t>(c, src_tp, m, dst_rank, pools, src_tables, seq_lens,
                                      new_pool, dst_table, migrated_blocks_out, defrag_blocks_out);
    case 2:
      return merge_kv_base_t<uint16_t>(c, src_tp, m, dst_rank, pools, src_tables, seq_lens,
                                       new_pool, dst_table, migrated_blocks_out, defrag_blocks_out);
    default:
      return merge_kv_base_t<uint32_t>(c, src_tp, m, dst_rank, pools, src_tables, seq_lens,
                                       new_pool, dst_table, migrated_blocks_out, defrag_blocks_out);
  }
}

int64_t ao_padded_shard_elems(const ao_model* m, const ao_pad* pad, int tp) {
  if (!model_ok(m) || !tp_ok(m, tp) || !pad_ok(m, pad, tp)) return -1;
  return pad_geom(m, pad, tp).layer * m->n_layers;
}

int ao_padded_geometry(const ao_model* m, const ao_pad* pad, int tp, int64_t out[6]) {
  if (!model_ok(m) || !tp_ok(m, tp) || !pad_ok(m, pad, tp) || !out) return AO_ERR_ARG;
  const PadGeom g = pad_geom(m, pad, tp);
  out[0] = g.attn; out[1] = g.attn_padded; out[2] = g.part; out[3] = g.part_padded;
  out[4] = g.stride; out[5] = g.layer;
  return AO_OK;
}

int ao_reshard_weights_padded(const ao_model* m, const ao_pad* pad, int src_tp, int dst_tp,
                              int dst_rank, const void* const* src_shards, void* dst) {
  if (!model_ok(m) || src_tp > 64 || !tp_ok(m, src_tp) || !tp_ok(m, dst_tp) || dst_rank < 0 ||
      dst_rank >= dst_tp || !src_shards || !dst || !pad_ok(m, pad, src_tp) ||
      !pad_ok(m, pad, dst_tp))
    return AO_ERR_ARG;
  switch (m->elem_bytes) {
    case 1: return reshard_weights_padded_t<uint8_t>(m, pad, src_tp, dst_tp, dst_rank, src_shards, dst);
    case 2: return reshard_weights_padded_t<uint16_t>(m, pad, src_tp, dst_tp, dst_rank, src_shards, dst);
    default: return reshard_weights_padded_t<uint32_t>(m, pad, src_tp, dst_tp, dst_rank, src_shards, dst);
  }
}

int64_t ao_moe_shard_elems(const ao_model* m, const ao_moe* x, int padded, int tp) {
  if (!model_ok(m) || !moe_ok(m, x, tp)) return -1;
  return moe_geom(m, x, padded && x->page_bytes, tp).layer * m->n_layers;
}

int ao_moe_geometry(const ao_model* m, const ao_moe* x, int padded, int tp, int64_t out[5]) {
  if (!model_ok(m) || !moe_ok(m, x, tp) || !out) return AO_ERR_ARG;
  const MoeGeom g = moe_geom(m, x, padded && x->page_bytes, tp);
  out[0] = g.own; out[1] = g.first; out[2] = g.tensor; out[3] = g.slot; out[4] = g.layer;
  return AO_OK;
}

int ao_reshard_weights_moe(const ao_model* m, const ao_moe* x, int src_tp, int dst_tp,
                           int dst_rank, const void* const* src_shards, void* dst) {
  if (!model_ok(m) || src_tp > 64 || !moe_ok(m, x, src_tp) || !moe_ok(m, x, dst_tp) ||
      dst_rank < 0 || dst_rank >= dst_tp || !src_shards || !dst)
    return AO_ERR_ARG;
  switch (m->elem_bytes) {
    case 1: return reshard_weights_moe_t<uint8_t>(m, x, src_tp, dst_tp, dst_rank, src_shards, dst);
    case 2: return reshard_weights_moe_t<uint16_t>(m, x, src_tp, dst_tp, dst_rank, src_shards, dst);
    default: return reshard_weights_moe_t<uint32_t>(m, x, src_tp, dst_tp, dst_rank, src_shards, dst);
  }
}

}  // extern "C"
