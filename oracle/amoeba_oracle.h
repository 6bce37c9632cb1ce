/*
 * CPU oracle for runtime Tensor-Parallel (TP) transformation of one instance's
 * state: TP=k shards -> target rank r' of TP=k'.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, single-threaded, per-element
 * definition of the result.  It shares no code, header, table or helper with
 * the HIP library; nothing in the product path may include, link or call it.
 *
 * What it follows (paper sections, restated):
 *   - Sec. 2.2 (TP): attention heads are spread evenly over the workers, FFN
 *     weights are cut in equal segments, one per worker.
 *   - Sec. 3.2, Eq. (1) and the definition of U', D': up_proj is cut by
 *     columns of the mathematical matrix U (FFN = f(I x U) x D), down_proj by
 *     rows of D.  With tensors stored row-major as [out_features, in_features]
 *     a column of U is a stored row of up_proj/gate_proj (contiguous cut) and
 *     a row of D is a stored column of down_proj (strided cut).  q/k/v behave
 *     like U, o_proj like D.
 *   - Sec. 3.1, head-range rule: worker i of a TP group (1-based) owns heads
 *     (H/TP)(i-1)+1 .. (H/TP)i, i.e. 0-based rank r owns [r*H/TP,(r+1)*H/TP).
 *   - Sec. 3.1, KV layouts: "page-friendly" token-first block and the
 *     header-centric block ordered [Block, Header, K/V, Token] with the head
 *     dimension innermost.
 *
 * Every function below is pinned by tests/test_oracle_*.py (worked example of
 * Sec. 3.1, brute-force enumeration, round trips, tiling of the unsharded
 * tensors, torch cat/chunk/index_select special cases, Eq. (1)/(2) identity).
 *
 * All pointers are HOST pointers.  Elements are opaque (never interpreted).
 */
#ifndef AMOEBA_ORACLE_H
#define AMOEBA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { AO_LAYOUT_HEAD_MAJOR = 0, AO_LAYOUT_TOKEN_MAJOR = 1 };

enum {
  AO_OK = 0,
  AO_ERR_ARG = 1,      /* bad shape / tp / rank / NULL pointer          */
  AO_ERR_OVERFLOW = 2, /* tables or pool too small, negative length     */
  AO_ERR_BLOCK_ID = 3  /* a source block id outside [0, src_pool_blocks) */
};

/* Decoder shape.  Unsharded tensors, row-major [out, in]:
 *   Wq[n_q*d, hidden] Wk[n_kv*d, hidden] Wv[n_kv*d, hidden] Wo[hidden, n_q*d]
 *   Wg[ffn, hidden]   Wu[ffn, hidden]    Wd[hidden, ffn]
 * Rank r of TP=t stores per layer, packed in this order:
 *   qkv_r     = [Wq rows of r's q heads; Wk rows of r's kv heads; Wv rows ...]
 *   o_r       = Wo[:, columns of r's q heads]
 *   gate_up_r = [Wg rows r*ffn/t ..; Wu rows r*ffn/t ..]
 *   down_r    = Wd[:, columns r*ffn/t ..]
 * and the layers follow each other without padding. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim;
  int32_t elem_bytes; /* 1, 2 or 4 */
} ao_model;

/* Paged KV cache.  A pool is [kv_layers][pool_blocks][block_elems(tp)];
 * block tables are [num_seqs][max_blocks_per_seq] int32, -1 padded. */
typedef struct {
  int32_t kv_layers, n_kv_heads, head_dim, elem_bytes;
  int32_t block_tokens;
  int32_t layout_src, layout_dst;
  int32_t num_seqs, max_blocks_per_seq;
  int64_t src_pool_blocks, dst_pool_blocks;
} ao_kv;

/* Elements of one rank's weight shard at TP=tp, all layers; -1 if tp does not
 * divide n_q_heads, n_kv_heads and ffn_dim. */
int64_t ao_shard_elems(const ao_model* m, int tp);

/* Elements of one KV block on a rank at TP=tp; -1 if tp does not divide heads. */
int64_t ao_kv_block_elems(const ao_kv* c, int tp);

/* dst <- rank dst_rank's shard at TP=dst_tp, gathered from the src_tp shards.
 * src_shards: src_tp host pointers; ranks that own nothing of the target may
 * be NULL.  dst must not overlap any source. */
int ao_reshard_weights(const ao_model* m, int src_tp, int dst_tp, int dst_rank,
                       const void* const* src_shards, void* dst);

/* Sequence scan + table rewrite + block regroup by KV head.
 *   nb_i = ceil(len_i / block_tokens); base_i = sum_{i'<i} nb_i';
 *   dst_table[i][j] = base_i + j (j < nb_i) else -1;
 *   every slot of every used block is copied for the heads dst_rank owns.
 * One src table serves all src ranks.  On AO_ERR_OVERFLOW nothing is written
 * to dst_pool and dst_table is all -1.  A block whose source id is out of
 * range is skipped and AO_ERR_BLOCK_ID is returned after the rest is done.
 * total_blocks_out (may be NULL) receives sum nb_i (0 on overflow). */
int ao_reshard_kv(const ao_kv* c, int src_tp, int dst_tp, int dst_rank,
                  const void* const* src_pools, const int32_t* src_table,
                  const int32_t* seq_lens, void* dst_pool, int32_t* dst_table,
                  int64_t* total_blocks_out);

/* In-place merge of m instances running at TP=src_tp into one instance at
 * TP=src_tp*m, header-centric layout on both sides (Sec. 3.1: every worker keeps,
 * for its local requests, the heads of its new range where they are; the heads it
 * gives away leave "bubbles" that are reused by reshaping blocks; Improvement 1).
 *
 * Target rank r' = s*m + g is hosted where rank s of instance g was.  local_pool is
 * that rank's pool [kv_layers][P][block(src_tp)], P = c->src_pool_blocks; afterwards
 * it is read as [kv_layers][P*m][block(src_tp*m)]: old block b is cut in m sub-blocks
 * of n_kv/(src_tp*m) heads, sub-block j living at new id b*m + j.
 *   - a block b of a local sequence keeps sub-block g where it is: new id b*m + g;
 *   - a block b of a sequence of instance g2 != g gets new id b*m + g2; its heads
 *     for r' are sub-block g of block b in remote_pools[g2] (rank s of instance g2)
 *     and are copied there.
 * No two blocks collide (ids of instance g2 are = g2 mod m) and no extra memory is
 * needed.  Every instance has c->num_seqs sequences and a table
 * [num_seqs][max_blocks_per_seq]; dst_table is [m*num_seqs][max_blocks_per_seq] in
 * instance-major order and is the same for every target rank.  remote_pools[g] is
 * ignored.  A negative length or a row that is too short gives AO_ERR_OVERFLOW
 * (nothing written, table all -1); an id outside [0, P) gives a -1 entry, skips the
 * block and returns AO_ERR_BLOCK_ID.  remote_blocks_out: the slots (distinct new ids) of
 * the reshaped pool that received remote heads, per layer: a skipped id has no slot and is
 * not counted, a block id two sequences of one instance share is one slot, counted once. */
int ao_merge_kv_inplace(const ao_kv* c, int src_tp, int m, int dst_rank, void* local_pool,
                        const void* const* remote_pools, const int32_t* const* src_tables,
                        const int32_t* const* seq_lens, int32_t* dst_table,
                        int64_t* remote_blocks_out);

/* The base solution of Sec. 3.1 for the same merge of m instances (TP=src_tp each) into one
 * at TP=src_tp*m: migration, then de-fragmentation, into a second pool.  Target rank
 * r' = s*m + g is hosted where rank s of instance g was.  pools[g2] is the pool of rank s of
 * instance g2, [kv_layers][P][block(src_tp)] in c->layout_src (all m entries are read; entry g
 * is the worker's own).  new_pool is [kv_layers][c->dst_pool_blocks][block(src_tp*m)] in
 * c->layout_dst: the reserved pages for what the worker receives plus room for its own
 * requests in compact form; the paper's base solution stores both sides token-first.
 *   pass 1 (migration): for every request of every other instance, the heads r' owns are
 *     taken out of the sender's blocks and stored in new blocks;
 *   pass 2 (de-fragmentation): for every local request the heads r' keeps, which sit between
 *     the heads it gave away, are stored compactly in new blocks.
 * New ids are compact over the merged sequence list, instance-major (exclusive prefix sum of
 * ceil(len / block_tokens)); dst_table is [m*num_seqs][max_blocks_per_seq], -1 padded, the
 * same for every target rank.  Negative length, short row or sum of blocks > dst_pool_blocks:
 * AO_ERR_OVERFLOW, nothing written, table all -1.  An id outside [0, P): that block is skipped
 * (its new block keeps its bytes), AO_ERR_BLOCK_ID.  migrated_blocks_out / defrag_blocks_out
 * (may be NULL): blocks moved by either pass, per layer. */
int ao_merge_kv_base(const ao_kv* c, int src_tp, int m, int dst_rank, const void* const* pools,
                     const int32_t* const* src_tables, const int32_t* const* seq_lens,
                     void* new_pool, int32_t* dst_table, int64_t* migrated_blocks_out,
                     int64_t* defrag_blocks_out);

/* Padded, partition-major FFN layout (Sec. 3.2, Improvement 1: padding at every potential
 * TP boundary so that each partition starts on an allocation granule and a split only has
 * to release pages).  max_tp = finest TP degree T; every FFN tensor is cut in T partitions;
 * a rank at TP=t stores, per layer,
 *   [qkv_r | o_r | zeros up to a page] then for each of its T/t partitions p:
 *   [gate_p | zeros][up_p | zeros][down_p | zeros],   each tensor-partition page-aligned,
 * gate_p/up_p = rows p*ffn/T.. of Wg/Wu ([ffn/T][hidden]), down_p = columns p*ffn/T.. of Wd
 * stored as a row-major [hidden][ffn/T] matrix.  src_padded / dst_padded say which side of
 * a reshard uses this layout (the other side is the dense shard). */
typedef struct {
  int32_t max_tp;
  int32_t src_padded, dst_padded;
  int64_t page_bytes;
} ao_pad;

/* Elements of one rank's padded shard at TP=tp (all layers); -1 if unsupported. */
int64_t ao_padded_shard_elems(const ao_model* m, const ao_pad* pad, int tp);
/* out = {attention elems, attention elems padded, tensor-partition elems, padded,
 *        partition stride, layer elems} at TP=tp. */
int ao_padded_geometry(const ao_model* m, const ao_pad* pad, int tp, int64_t out[6]);
/* Like ao_reshard_weights with either side in the padded layout; gaps of a padded
 * destination are zero-filled. */
int ao_reshard_weights_padded(const ao_model* m, const ao_pad* pad, int src_tp, int dst_tp,
                              int dst_rank, const void* const* src_shards, void* dst);

/* Mixture-of-experts model (Sec. 3.2, "Supporting EP transformation": the FFN is stored in an
 * expert-wise layout, so experts that leave a rank are released whole; Sec. 4.3 runs
 * 4 x (TP1 EP1) -> TP4 EP4).  m->ffn_dim is ONE expert's intermediate size f; every expert e
 * has Wg_e[f, hidden], Wu_e[f, hidden], Wd_e[hidden, f].  Attention tensors are cut by head
 * as in the dense model; rank r at degree t owns experts [r*E/t, (r+1)*E/t) (the paper does
 * not print the expert-to-rank rule; contiguous ranges, like its head rule).  Per layer a
 * rank stores [qkv_r | o_r] and then, for each owned expert in order, [gate_e][up_e][down_e].
 * On a padded side (page_bytes > 0 and the side's flag set) the attention part is rounded up
 * to a page and every expert starts on a page boundary (experts are released whole, so that
 * is the only boundary a release can fall on), the gaps holding zeros. */
typedef struct {
  int32_t n_experts;
  int32_t src_padded, dst_padded;
  int64_t page_bytes; /* 0: no padding anywhere */
} ao_moe;

/* Elements of one rank's shard at degree tp, all layers; -1 if unsupported. */
int64_t ao_moe_shard_elems(const ao_model* m, const ao_moe* x, int padded, int tp);
/* out = {experts per rank, offset of the first expert, expert tensor elems, stride between
 *        experts, layer elems}, in elements. */
int ao_moe_geometry(const ao_model* m, const ao_moe* x, int padded, int tp, int64_t out[5]);
/* dst <- rank dst_rank's shard at degree dst_tp (attention TP, experts EP), gathered from the
 * src_tp shards; gaps of a padded destination are zero-filled. */
int ao_reshard_weights_moe(const ao_model* m, const ao_moe* x, int src_tp, int dst_tp,
                           int dst_rank, const void* const* src_shards, void* dst);

#ifdef __cplusplus
}
#endif
#endif
