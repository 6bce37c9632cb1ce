/*
 * amoeba.h -- C ABI of the MI355X (gfx950) reshard library.
 *
 * Runtime Tensor-Parallel transformation of one serving instance, restated for
 * one GPU: all source shards of TP = src_tp sit in this GPU's HBM and the
 * library produces target rank dst_rank's share at TP = dst_tp.
 *
 *   weights : every decoder layer's fused QKV / O / gate_up / down tensors are
 *             re-sliced by attention head and by FFN column/row partition
 *             (paper Sec. 2.2; Sec. 3.2, Eq. (1) and the definition of U', D').
 *   KV cache: every paged block is regrouped by KV head under a compacted,
 *             rewritten block table (paper Sec. 3.1: each worker of a TP group owns
 *             one contiguous run of H/TP heads, in rank order; the token-first
 *             block layout of the base solution and the header-centric layout
 *             of Improvement 1).
 *
 * Everything is an opaque move of 1-, 2- or 4-byte elements: no arithmetic on
 * the payload.  All compute runs in HIP kernels; there is no CPU fallback.
 *
 * Storage convention (fixed by this library; the paper gives none).  Unsharded
 * tensors are row-major [out_features, in_features]:
 *     Wq[n_q*d, hidden] Wk[n_kv*d, hidden] Wv[n_kv*d, hidden] Wo[hidden, n_q*d]
 *     Wg[ffn, hidden]   Wu[ffn, hidden]    Wd[hidden, ffn]
 * Rank r of TP = t owns q heads [r*n_q/t, (r+1)*n_q/t), kv heads likewise and
 * FFN units [r*ffn/t, (r+1)*ffn/t).  Its shard is, per layer and packed in this
 * order with no padding, layers back to back:
 *     qkv_r     [(n_q + 2 n_kv) d / t, hidden] = [Wq rows; Wk rows; Wv rows] of its heads
 *     o_r       [hidden, n_q d / t]            = Wo[:, its q-head columns]
 *     gate_up_r [2 ffn / t, hidden]            = [Wg rows; Wu rows] of its FFN units
 *     down_r    [hidden, ffn / t]              = Wd[:, its FFN columns]
 *
 * A KV pool is [kv_layers][pool_blocks][block], one block holding
 * kv_block_tokens tokens of the rank's n_kv/t heads, K and V, in one of
 *     AMOEBA_KV_HEAD_MAJOR : [head][K/V][token][d]   (header-centric, Sec. 3.1 Improvement 1)
 *     AMOEBA_KV_TOKEN_MAJOR: [K/V][token][head][d]   (token-first, Sec. 3.1 base layout)
 * Block tables are int32 [num_seqs][max_blocks_per_seq], padded with -1.  One
 * source table serves all source ranks (one instance, one scheduler).
 *
 * Device memory and threading.  The host side of a plan is immutable after
 * amoeba_plan().  The plan owns two device workspaces, allocated once by
 * amoeba_plan() and freed by amoeba_plan_destroy(); the reshard calls themselves
 * never allocate, free or synchronise:
 *   - for amoeba_reshard_kv() and amoeba_merge_kv_base(): 4 * (8 + m * num_seqs +
 *     dst_pool_blocks) bytes, m = dst_tp / src_tp if that is an integer, else 1 (a status
 *     header, the scanned base of every sequence, and the source id of every new
 *     block, which the block-regroup kernel reads instead of searching the table);
 *   - for amoeba_merge_kv_inplace(), when the plan qualifies: about
 *     8 * m * src_pool_blocks bytes (a flag and a work-list entry per new block id).
 * The kernels of a call write these, so two amoeba_reshard_kv() calls (or two
 * amoeba_merge_kv_inplace() or amoeba_merge_kv_base() calls) on the same plan must not
 * overlap in time; use one plan per stream.  amoeba_reshard_weights() uses no workspace
 * and its calls may overlap freely.
 */
#ifndef AMOEBA_H
#define AMOEBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AMOEBA_MAX_TP 16

enum { AMOEBA_KV_HEAD_MAJOR = 0, AMOEBA_KV_TOKEN_MAJOR = 1 };

/*
 * AMOEBA_W_FFN_PADDED: the layout of Sec. 3.2, Improvement 1 (weight padding at the partition
 * boundaries).
 * Every FFN tensor is cut in T = pad_max_tp partitions (gate/up by stored rows, down by
 * stored columns) and padding is added at every potential TP boundary so that each
 * partition starts on a multiple of pad_page_bytes.  A rank at TP = t stores, per layer,
 *     [qkv_r | o_r | zeros up to a page]
 *     then for each of its T/t partitions p = r*T/t ..:  [gate_p | 0][up_p | 0][down_p | 0]
 * gate_p / up_p = rows p*ffn/T .. of Wg / Wu ([ffn/T][hidden]); down_p = columns p*ffn/T ..
 * of Wd as a row-major [hidden][ffn/T] matrix; every tensor-partition is page aligned and
 * its gap holds zeros, so the FFN computed on the padded operands equals the FFN (Eq. (2)).
 * A scale-up (t | t') then keeps a contiguous page range of each layer and releases the
 * rest without copying (amoeba_plan_ffn_view); building the layout from a dense shard and
 * gathering partitions on scale-down are amoeba_reshard_weights() calls on such a plan.
 */
enum { AMOEBA_W_DENSE = 0, AMOEBA_W_FFN_PADDED = 1 };

enum {
  AMOEBA_OK = 0,
  AMOEBA_ERR_INVALID_ARG = 1, /* NULL plan / pointer, misaligned or aliased buffers      */
  AMOEBA_ERR_HIP = 2,         /* a HIP call failed; text in amoeba_last_error()          */
  AMOEBA_ERR_OVERFLOW = 3,    /* device found: negative length, table row or pool small  */
  AMOEBA_ERR_BLOCK_ID = 4     /* device found: a source block id outside the source pool */
};

/* Tensor ids for amoeba_plan_tensor_info(). */
enum {
  AMOEBA_T_Q = 0, AMOEBA_T_K = 1, AMOEBA_T_V = 2, AMOEBA_T_O = 3,
  AMOEBA_T_GATE = 4, AMOEBA_T_UP = 5, AMOEBA_T_DOWN = 6, AMOEBA_T_COUNT = 7
};

/* Which tensors amoeba_reshard_weights_part() moves. */
enum { AMOEBA_PART_ALL = 0, AMOEBA_PART_ATTENTION = 1, AMOEBA_PART_FFN = 2 };

/* Caller-owned POD; amoeba_plan() copies it. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim;
  int32_t elem_bytes;      /* 1, 2 or 4; 2 = fp16/bf16, never interpreted                 */
  int32_t kv_block_tokens; /* tokens per KV block on both sides (16 in the paper's engines) */
  int32_t kv_layout_src, kv_layout_dst; /* AMOEBA_KV_*                                    */
  int32_t kv_layers;       /* layers held by each KV pool passed to amoeba_reshard_kv     */
  int32_t num_seqs, max_blocks_per_seq; /* block tables are [num_seqs][max_blocks_per_seq] */
  int64_t src_pool_blocks, dst_pool_blocks; /* blocks per layer in each pool              */
  /* Weight shard layout of either side: AMOEBA_W_DENSE (0, the packing described above) or
   * AMOEBA_W_FFN_PADDED, the padded partition-major FFN layout (see below).  With both 0
   * the three pad_* fields are ignored. */
  int32_t w_layout_src, w_layout_dst;
  int32_t pad_max_tp;      /* T: finest TP degree of the model's TP set; src_tp, dst_tp | T */
  int32_t n_experts;       /* 0: dense FFN; E > 0: mixture of experts, see below           */
  int64_t pad_page_bytes;  /* allocation granule the partitions are aligned to (2 MiB)    */
  /* Upper bound on the KV blocks in use (sum over sequences of ceil(len / kv_block_tokens)),
   * as the scheduler that owns the block tables knows it when it asks for the transform;
   * 0 = unknown.  The lengths themselves are device data, so without the bound the regroup
   * grid has to cover dst_pool_blocks and the workgroups past the blocks in use cost
   * dispatch time (up to 30 % with a pool far from full).  A bound that turns out too
   * small is still correct: the workgroups stride over the rest, only slower. */
  int64_t kv_blocks_bound;
} amoeba_model_shape;

/*
 * Mixture-of-experts models (Sec. 3.2, "Supporting EP transformation"; the TPkEPk
 * configurations of Sec. 4.3).  With n_experts = E > 0 the attention tensors are cut by
 * head as above and the FFN is stored expert by expert: ffn_dim is one expert's
 * intermediate size f, every expert has Wg_e[f, hidden], Wu_e[f, hidden], Wd_e[hidden, f],
 * and rank r at degree t owns the whole experts [r*E/t, (r+1)*E/t) (contiguous ranges, the
 * head rule applied to experts).  Its shard is, per layer,
 *     AMOEBA_W_DENSE     : [qkv_r | o_r] then [gate_e | up_e | down_e] for each owned e
 *     AMOEBA_W_FFN_PADDED: [qkv_r | o_r | 0 up to a page] then [gate_e | up_e | down_e | 0],
 *                          every expert starting on a multiple of pad_page_bytes: experts
 *                          are released whole, so no other boundary needs a page
 *                          (pad_max_tp is ignored)
 * so a target rank's experts are one contiguous byte range of one source rank whenever
 * src_tp divides dst_tp (amoeba_plan_ffn_view: release the rest, copy nothing), and whole
 * experts are gathered from several ranks otherwise.  Replicated tensors (router, norms)
 * are on every rank already and are not part of a shard.  The degrees must divide E; they
 * need not divide ffn_dim.
 */

typedef struct amoeba_plan_s amoeba_plan_t;

/*
 * Host-side planning (Sec. 3.2: partition boundaries are fixed per model and TP
 * set, so they are computed once).  Builds the per-layer table of strided copy
 * segments for the weights and the stride description of both KV layouts (the
 * role of the paper's kv_stride_order(), Sec. 3.1), and allocates the device
 * workspaces described at the top of this file on the current device (skipped,
 * without error, when no GPU is present; then amoeba_reshard_kv() fails with
 * AMOEBA_ERR_HIP).
 * Returns NULL and sets amoeba_last_error() if: a size is not positive (num_seqs,
 * max_blocks_per_seq and the pool sizes may be 0), dst_rank is outside
 * [0, dst_tp), either TP degree exceeds AMOEBA_MAX_TP or does not divide
 * n_q_heads, n_kv_heads and ffn_dim (n_experts instead of ffn_dim for a
 * mixture-of-experts model; fewer KV heads than ranks, i.e. head
 * replication, is unsupported), n_q_heads is not a multiple of n_kv_heads,
 * a layout or elem_bytes is unknown, a pool has more than 2^31-1 blocks, or
 * kv_blocks_bound is negative.
 */
amoeba_plan_t* amoeba_plan(const amoeba_model_shape* shape, int src_tp, int dst_tp, int dst_rank);

/* Frees the plan and its device workspace.  NULL is ignored. */
void amoeba_plan_destroy(amoeba_plan_t* plan);

/*
 * Weights (Sec. 2.2; Sec. 3.2 Eq. (1)): dst <- rank dst_rank's shard at dst_tp.
 *   src_shards : HOST array of src_tp DEVICE pointers, entry s = rank s's shard
 *                (amoeba_plan_shard_bytes(plan, 0) bytes).  Entries whose bit is
 *                clear in amoeba_plan_src_rank_mask() are never read, may be NULL.
 *   dst        : DEVICE buffer of amoeba_plan_shard_bytes(plan, 1) bytes; must not
 *                overlap a source that is read (checked; AMOEBA_ERR_INVALID_ARG).
 *   stream     : hipStream_t (NULL = default stream).
 * Enqueues one kernel over all layers; does not synchronise, allocate or keep
 * any pointer.  Any alignment works; 16-byte aligned buffers take the fast path.
 */
int amoeba_reshard_weights(const amoeba_plan_t* plan, const void* const* src_shards, void* dst,
                           void* stream);

/* The same with a choice of tensors: AMOEBA_PART_ALL (what amoeba_reshard_weights() does),
 * AMOEBA_PART_ATTENTION (q, k, v, o and, in a padded layout, the zero gap behind them) or
 * AMOEBA_PART_FFN (gate, up, down or the experts).  For the scale-up of Sec. 3.2,
 * Improvement 1: when amoeba_plan_ffn_view() says the target's FFN partitions are a page
 * range of a source buffer that is kept in place, only the attention part is re-sliced.
 * Bytes of `dst` outside the chosen part are not touched. */
int amoeba_reshard_weights_part(const amoeba_plan_t* plan, const void* const* src_shards,
                                void* dst, int part, void* stream);

/*
 * KV cache (Sec. 3.1): scan sequence lengths, rewrite the block table, regroup
 * every used block by KV head.
 *   src_blocks       : HOST array of src_tp DEVICE pool pointers
 *                      [kv_layers][src_pool_blocks][amoeba_plan_kv_block_bytes(plan,0)];
 *                      ranks outside amoeba_plan_kv_rank_mask() may be NULL.
 *   src_block_tables : DEVICE int32 [num_seqs][max_blocks_per_seq].
 *   seq_lens         : DEVICE int32 [num_seqs], tokens per sequence.
 *   dst_blocks       : DEVICE pool [kv_layers][dst_pool_blocks][amoeba_plan_kv_block_bytes(plan,1)].
 *   dst_block_tables : DEVICE int32 [num_seqs][max_blocks_per_seq], fully overwritten:
 *                      row i = base_i, base_i+1, .. for ceil(len_i/kv_block_tokens)
 *                      entries, then -1; base = exclusive prefix sum in sequence order.
 * Whole blocks move (all kv_block_tokens slots).  Enqueues three kernels on
 * `stream`; no host synchronisation.  Conditions found on the device are reported
 * by amoeba_kv_status(): on AMOEBA_ERR_OVERFLOW the pool is untouched and the
 * table is all -1; a source block id outside [0, src_pool_blocks) skips that
 * block (its destination block is left as it was) and yields AMOEBA_ERR_BLOCK_ID.
 */
int amoeba_reshard_kv(const amoeba_plan_t* plan, const void* const* src_blocks,
                      const int32_t* src_block_tables, const int32_t* seq_lens, void* dst_blocks,
                      int32_t* dst_block_tables, void* stream);

/*
 * amoeba_reshard_kv() for callers that cannot allocate device memory or let a library do
 * it: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same result, same kernels, but the kernels' workspace (the status
 * header, the scanned bases and the new-block -> source-block list) is a static device
 * array inside the library instead of the plan's allocation, so the call allocates and
 * frees nothing and calls no allocating routine.  Limits and rules:
 *   - 8 + num_seqs + dst_pool_blocks must not exceed 2^20 int32 words (the array is
 *     4 MiB, held by every GPU the library is loaded on until the process ends); beyond
 *     that the call returns AMOEBA_ERR_INVALID_ARG and amoeba_last_error() says so;
 *   - every call on one GPU shares that GPU's array, whatever the plan or stream: calls
 *     that overlap in time on one GPU race, and amoeba_kv_status() reports the last such
 *     call enqueued on that GPU if it is read after another one was enqueued;
 *   - the array keeps the last call's contents; nothing needs clearing between calls
 *     (every word a call reads was written by that call's own kernels first).
 * The address of the array on a device is looked up when the first plan is created with
 * that device current (or, failing that, on the first call there).
 */
int amoeba_reshard_kv_static(const amoeba_plan_t* plan, const void* const* src_blocks,
                             const int32_t* src_block_tables, const int32_t* seq_lens,
                             void* dst_blocks, int32_t* dst_block_tables, void* stream);

/* Synchronises `stream`, then returns what the last amoeba_reshard_kv() (or
 * amoeba_reshard_kv_static()) enqueued on this plan found: AMOEBA_OK, AMOEBA_ERR_OVERFLOW
 * or AMOEBA_ERR_BLOCK_ID (AMOEBA_ERR_HIP if the copy back fails).  total_blocks (may be
 * NULL) receives sum_i nb_i. */
int amoeba_kv_status(const amoeba_plan_t* plan, void* stream, int64_t* total_blocks);

/*
 * In-place merge of m = dst_tp / src_tp instances into one (Sec. 3.1: the paper's
 * 4 x TP1 -> TP4 scenario, base solution + Improvement 1 "in-place migration with
 * header-centric layout").  Each instance runs at TP = src_tp with its own sequences,
 * block table and pools.  Target rank dst_rank = s*m + g is hosted where rank s of
 * instance g was and reuses that rank's pool:
 *   local_pool       : DEVICE, in/out.  In : [kv_layers][src_pool_blocks][block(src_tp)].
 *                      Out: the same bytes read as [kv_layers][src_pool_blocks*m][block(dst_tp)]
 *                      ("block reshaping": old block b = new blocks b*m .. b*m+m-1, one per
 *                      m-th of the heads).  Heads of local sequences that dst_rank keeps are
 *                      not moved; the sub-blocks it gives away are overwritten by the heads
 *                      it receives: new block b*m + g2 <- heads of dst_rank in block b of
 *                      remote_pools[g2], for every block b of every sequence of instance g2.
 *   remote_pools     : HOST array of m DEVICE pointers, entry g2 = pool of rank s of
 *                      instance g2 (same geometry, read only; entry g is ignored).
 *   src_block_tables : HOST array of m DEVICE int32 [num_seqs][max_blocks_per_seq].
 *   seq_lens         : HOST array of m DEVICE int32 [num_seqs].
 *   dst_block_tables : DEVICE int32 [m*num_seqs][max_blocks_per_seq], instance-major;
 *                      entry = old id * m + instance, -1 padded; identical for every dst_rank.
 * The plan must have kv_layout_src = kv_layout_dst = AMOEBA_KV_HEAD_MAJOR and
 * amoeba_plan_merge_factor(plan) = m >= 2 (dst_pool_blocks is not used).  Enqueues three
 * kernels, no host synchronisation, no extra device memory beyond the plan's workspace
 * (about 8*m*src_pool_blocks bytes: a flag and a work-list entry per new block id).
 * For this call the shape's kv_blocks_bound, if set, bounds the blocks that move, i.e. those
 * of the other instances (the local ones stay where they are).  Device-found conditions are read
 * with amoeba_merge_kv_status(): AMOEBA_ERR_OVERFLOW (negative length / row too short:
 * nothing written, table all -1), AMOEBA_ERR_BLOCK_ID (an id outside the pool: entry -1,
 * block skipped).  Calls on one plan must not overlap in time.
 */
int amoeba_merge_kv_inplace(const amoeba_plan_t* plan, void* local_pool,
                            const void* const* remote_pools,
                            const int32_t* const* src_block_tables,
                            const int32_t* const* seq_lens, int32_t* dst_block_tables,
                            void* stream);

/*
 * The same merge of m = dst_tp / src_tp instances the base way (Sec. 3.1, base solution:
 * migration and de-fragmentation), for comparison with the in-place merge and for engines
 * whose blocks are token-first.  The worker gets a second pool; two passes fill it:
 *   migration       : for every request of every other instance, the heads dst_rank owns
 *                     are taken out of the sender's blocks and stored in new blocks (the
 *                     reserved pages of the paper);
 *   de-fragmentation: for every local request, the heads dst_rank keeps (which sit between
 *                     the heads it gave away) are stored compactly in new blocks; the old
 *                     pool can be released afterwards.
 *   pools            : HOST array of m DEVICE pointers, entry g2 = pool of rank s of instance
 *                      g2, [kv_layers][src_pool_blocks][block(src_tp)] in kv_layout_src, read
 *                      only (dst_rank = s*m + g; entry g is the worker's own pool).
 *   src_block_tables : HOST array of m DEVICE int32 [num_seqs][max_blocks_per_seq].
 *   seq_lens         : HOST array of m DEVICE int32 [num_seqs].
 *   new_pool         : DEVICE [kv_layers][dst_pool_blocks][block(dst_tp)] in kv_layout_dst;
 *                      must not overlap any source pool.
 *   dst_block_tables : DEVICE int32 [m*num_seqs][max_blocks_per_seq], instance-major: compact
 *                      ids over the merged sequence list (exclusive prefix sum of
 *                      ceil(len / kv_block_tokens)), -1 padded; identical for every dst_rank.
 * Any layout pair works (the paper's base solution is token-first on both sides).  Enqueues
 * four kernels (scan, table, one block gather per pass), no host synchronisation, no memory
 * beyond the plan's workspace (4 * (8 + m*num_seqs + dst_pool_blocks) bytes) and new_pool
 * itself.  Grid sizing: the shape's kv_blocks_bound bounds the blocks of all instances
 * together and local_blocks_bound (0 = unknown) those of the local instance g; with both
 * given, the migration pass is sized for their difference and the de-fragmentation pass
 * for the local bound (exact counts make both grids tight; any values are correct, since
 * workgroups stride over what a grid does not cover).  Device-found conditions are read
 * with amoeba_kv_status() (total_blocks = blocks of all instances) and are those of
 * amoeba_reshard_kv().  Calls on one plan must not overlap in time.
 */
int amoeba_merge_kv_base(const amoeba_plan_t* plan, const void* const* pools,
                         const int32_t* const* src_block_tables, const int32_t* const* seq_lens,
                         void* new_pool, int32_t* dst_block_tables, int64_t local_blocks_bound,
                         void* stream);

/* Like amoeba_kv_status() for the last amoeba_merge_kv_inplace() on this plan;
 * remote_blocks (may be NULL) receives the blocks copied per layer. */
int amoeba_merge_kv_status(const amoeba_plan_t* plan, void* stream, int64_t* remote_blocks);

/* ---- queries (host only) ------------------------------------------------- */

/* Bytes of one rank's weight shard, all layers.  side: 0 = source TP, 1 = target TP. */
size_t amoeba_plan_shard_bytes(const amoeba_plan_t* plan, int side);
/* m if the plan can be used with amoeba_merge_kv_inplace(), else 0. */
int amoeba_plan_merge_factor(const amoeba_plan_t* plan);
/* Bytes of one KV block on one rank. */
size_t amoeba_plan_kv_block_bytes(const amoeba_plan_t* plan, int side);
/* Bit s set: source rank s holds weights the target rank needs. */
uint32_t amoeba_plan_src_rank_mask(const amoeba_plan_t* plan);
/* Bit s set: source rank s holds KV heads the target rank needs. */
uint32_t amoeba_plan_kv_rank_mask(const amoeba_plan_t* plan);
/* Where tensor `tensor` (AMOEBA_T_*) sits in a rank's per-layer shard: element offset
 * from the layer start, rows, columns; *layer_elems = elements per layer.  Any out
 * pointer may be NULL.  Returns AMOEBA_OK or AMOEBA_ERR_INVALID_ARG. */
int amoeba_plan_tensor_info(const amoeba_plan_t* plan, int side, int tensor, int64_t* elem_off,
                            int64_t* rows, int64_t* cols, int64_t* layer_elems);
/* Geometry of the padded layout of one side (bytes): out = {attention part, attention part
 * padded, one tensor-partition, one tensor-partition padded, partition stride, layer}.
 * AMOEBA_ERR_INVALID_ARG if that side is dense. */
int amoeba_plan_padded_info(const amoeba_plan_t* plan, int side, int64_t out[6]);
/* Zero-copy scale-up (Sec. 3.2, Improvement 1: with the padding in place a split only has to
 * release pages).  If both sides are padded
 * and src_tp divides dst_tp, the target's FFN partitions are one page-aligned byte range of
 * every layer of source rank out[0]: out = {source rank, byte offset of the range inside a
 * source layer, bytes of the range, source layer bytes}.  Returns 1 if such a view exists,
 * else 0.  (The attention part is re-sliced by head and is not a view.)  For a
 * mixture-of-experts plan the view is the target's expert range and exists whenever src_tp
 * divides dst_tp and both sides use the same weight layout (Sec. 3.2, EP discussion:
 * unused experts are freed directly); it is page aligned in the padded layout. */
int amoeba_plan_ffn_view(const amoeba_plan_t* plan, int64_t out[4]);
/* Expert geometry of one side of a mixture-of-experts plan (bytes): out = {experts per
 * rank, offset of the first expert in a layer, one expert tensor, stride from one expert
 * to the next}; an expert is three such tensors back to back (gate, up, down) and the
 * stride is their size, rounded up to a page in the padded layout.
 * AMOEBA_ERR_INVALID_ARG for a dense model. */
int amoeba_plan_expert_info(const amoeba_plan_t* plan, int side, int64_t out[4]);
/* Strides, in elements, of (head, K/V, token, d) inside one block, and the block
 * size: what an attention kernel needs to read either layout unchanged
 * (Sec. 3.1, kv_stride_order()).  out[0..3] = strides, out[4] = block elements. */
int amoeba_plan_kv_stride_order(const amoeba_plan_t* plan, int side, int64_t out[5]);
/* Weight copy segments of one layer (for inspection and host-side tests).
 * out = {src_rank, src_byte_off, src_pitch, dst_byte_off, dst_pitch, rows, run_bytes};
 * src_rank = -1 marks a zero fill (a gap of a padded destination). */
int amoeba_plan_num_segments(const amoeba_plan_t* plan);
int amoeba_plan_segment(const amoeba_plan_t* plan, int index, int64_t out[7]);

/* Text of the calling thread's last error ("" if none). */
const char* amoeba_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
