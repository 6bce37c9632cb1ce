/*
 * amoeba_measure.h -- measurement and inspection interface of the reshard library.
 *
 * Not part of the reshard boundary (include/amoeba.h does not include this file and no
 * call here is needed to run a transform): launch-shape overrides for sweeps, a plain
 * streaming copy that gives the rate this GPU reaches on a read-once/write-once stream and
 * a transfer of known size for calibrating HBM traffic counters, and a query of the launch
 * geometry the library would use.  Used by the benchmark, the profiling runs and the tests
 * that force every launch shape.
 */
#ifndef AMOEBA_MEASURE_H
#define AMOEBA_MEASURE_H

#include "amoeba.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Knobs for amoeba_plan_tune(); 0 restores the built-in choice. */
enum {
  AMOEBA_TUNE_W_GRID = 0,      /* workgroups of the weight kernel (0: one per tile)          */
  AMOEBA_TUNE_W_UNROLL = 1,    /* 16-byte vectors per lane per tile: 1, 2, 4 or 8            */
  AMOEBA_TUNE_W_THREADS = 2,   /* lanes per workgroup: 64, 128 or 256                        */
  AMOEBA_TUNE_KV_GRID = 3,     /* workgroups per layer of the KV regroup kernel              */
  AMOEBA_TUNE_KV_UNROLL = 4,   /* vectors per lane per tile: 1, 2 or 4                       */
  AMOEBA_TUNE_KV_THREADS = 5,  /* lanes per workgroup: 64 or 256                             */
  AMOEBA_TUNE_NONTEMPORAL = 6, /* 1: streaming (nt) loads/stores, 2: plain                   */
  AMOEBA_TUNE_KV_STAGED = 7,   /* 1: LDS-staged layout-converting regroup, 2: direct         */
  AMOEBA_TUNE_KV_BLOCKS_HINT = 8, /* overrides amoeba_model_shape.kv_blocks_bound (0: use the
                                  shape's value)                                             */
  AMOEBA_TUNE_KV_SMALL_TABLE = 9  /* 1: never take the one-launch path of small block tables
                                  (at most 64 sequences and 4096 cells), always the
                                  three-kernel scan / table / regroup path                  */
};

/* Launch-shape overrides, for measurement sweeps and for tests that must reach every launch
 * shape.  Not thread-safe against concurrent reshard calls on the same plan. */
int amoeba_plan_tune(amoeba_plan_t* plan, int knob, int value);

/* Launch geometry the library uses for this plan (and its current overrides) when every
 * pointer of the call is aligned to `align_bytes` (16 takes the fast path).
 *   kernel 0: weight kernel (first launch), 1: KV block regroup, 2: in-place merge copy.
 *   out = {grid.x, grid.y, lanes per workgroup, work items (tiles) the grid covers per
 *          grid.y slice}.
 * HIP limits grid.x * lanes to 2^32 - 1 work-items per dimension; past the grid the
 * workgroups stride.  Host only.  Returns AMOEBA_OK or AMOEBA_ERR_INVALID_ARG. */
int amoeba_plan_launch_shape(const amoeba_plan_t* plan, int kernel, int align_bytes,
                             int64_t out[4]);

/* A plain device-to-device streaming copy with the same access shape as the reshard
 * kernels (16 B per lane, `threads` lanes per workgroup: 64 or 256; `unroll` loads in
 * flight per lane: 1, 2, 4 or 8; `grid` workgroups, 0 = one per tile; nontemporal as in
 * AMOEBA_TUNE_NONTEMPORAL).  dst, src: DEVICE pointers, 16-byte aligned, non-overlapping;
 * bytes a multiple of 16. */
int amoeba_copy_baseline(void* dst, const void* src, size_t bytes, int threads, int unroll,
                         int grid, int nontemporal, void* stream);

#ifdef __cplusplus
}
#endif
#endif
