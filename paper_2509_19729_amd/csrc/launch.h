// Internal: host launchers of the two reshard paths (defined in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include <string>

#include "../../include/amoeba.h"
#include "grid.h"

struct amoeba_plan_s;

namespace amoeba {

// Workspace header (int32 words) shared by the KV kernels and the status call.
enum { kWsTotal = 0, kWsError = 1, kWsLocalBase = 2, kWsLocalCount = 3, kWsHeader = 8 };
enum { kErrNegativeLen = 1, kErrRowTooShort = 2, kErrPoolTooSmall = 4, kErrBlockId = 8 };

// part: AMOEBA_PART_ALL, _ATTENTION or _FFN.
int launch_reshard_weights(const amoeba_plan_s* p, const void* const* src_shards, void* dst,
                           int part, hipStream_t stream, std::string* err);

// ws: the workspace the kernels use, 8 + num_seqs + dst_pool_blocks int32 words on the
// current device (the plan's own, or the static one of the entry point that allocates nothing).
int launch_reshard_kv(const amoeba_plan_s* p, int32_t* ws, const void* const* src_blocks,
                      const int32_t* src_block_tables, const int32_t* seq_lens, void* dst_blocks,
                      int32_t* dst_block_tables, hipStream_t stream, std::string* err);

// The static workspace of amoeba_reshard_kv_static(): its address on the current device
// (nullptr and a message on failure; the first call on a device looks it up) and its size.
int32_t* static_kv_workspace(std::string* err);
size_t static_kv_workspace_ints();

// Base solution of Sec. 3.1 (migration pass, de-fragmentation pass) for m = dst_tp / src_tp
// instances; ws: 8 + m * num_seqs + dst_pool_blocks int32 words.
int launch_merge_kv_base(const amoeba_plan_s* p, int32_t* ws, const void* const* pools,
                         const int32_t* const* src_block_tables, const int32_t* const* seq_lens,
                         void* new_pool, int32_t* dst_block_tables, int64_t local_blocks_bound,
                         hipStream_t stream, std::string* err);

// Launch geometry of the three copy kernels for pointers aligned to align_bytes (host only).
bool weights_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                             std::string* err);
bool kv_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                        std::string* err);
bool merge_launch_geometry(const amoeba_plan_s* p, int align_bytes, LaunchShape* out,
                           std::string* err);

// int32 words of the merge workspace: header, chunk counts, one flag and one work-list
// entry per new block id of the pool.
size_t merge_workspace_ints(int64_t pool_blocks, int m);

int launch_merge_kv_inplace(const amoeba_plan_s* p, void* local_pool,
                            const void* const* remote_pools,
                            const int32_t* const* src_block_tables,
                            const int32_t* const* seq_lens, int32_t* dst_block_tables,
                            hipStream_t stream, std::string* err);

int launch_copy_baseline(void* dst, const void* src, size_t bytes, int threads, int unroll, int grid,
                         bool nt, hipStream_t stream, std::string* err);

}  // namespace amoeba
