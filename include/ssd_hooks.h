/*
 * ssd_hooks.h -- hooks of libssd_hip.so for its own tests and benchmarks.
 *
 * Nothing here is a step of the method or part of the interface a model uses
 * (that is ssd.h).  These calls expose host-side arithmetic for checks that
 * need no GPU, override launch shapes that the library otherwise chooses by
 * itself, and time the memory system without the method's arithmetic.
 */
#ifndef SSD_HOOKS_H
#define SSD_HOOKS_H

#include "ssd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * With enable == 0 every later call on this cache does all of its checking and
 * counter updates but enqueues nothing (for exercising the host logic on a
 * machine without a GPU).  Default: enabled.
 */
int ssd_cache_set_launch(ssd_cache *cache, int enable);

/*
 * The slot arithmetic (host only, nothing is enqueued): the same functions the
 * kernels evaluate.
 *   ssd_cache_head_runs    : the up to three runs of consecutive valid slots of
 *                            one head's unit at the layer's current counters,
 *                            in the order the attention streams them
 *                            (start[k], len[k]; unused runs have len 0)
 *   ssd_cache_spatial_slot : slot that holds `position` in a spatial head's
 *                            unit (sink slot, else ring slot S + (p-S) mod ring
 *                            size); SSD_ERR_INVALID_ARG for a semantic head
 */
int ssd_cache_head_runs(const ssd_cache *cache, int layer, int head, int32_t start[3], int32_t len[3]);
int ssd_cache_spatial_slot(const ssd_cache *cache, int layer, int head, int position, int32_t *slot);

/*
 * Override, for this cache only, the launch shape of the attention / step
 * kernel, which the library otherwise picks from the launch size.  Results
 * change by rounding only: ch and the number of wavefronts per unit set the
 * order of the fp32 softmax sums (the library's own choice is ch = 4 and one
 * wavefront, two or four as the launch size says); units per workgroup and
 * new_rows change nothing.  (0, 0, 0) restores the library's choice.
 *   ch       : wave-wide loads of K (and of V) per chunk: 0, 1, 2, 4
 *   wpb      : units per workgroup: 0, 1, 2, 4; 12 / 14 = one unit per workgroup
 *              shared by 2 / 4 wavefronts
 *   new_rows : fused step: 1 / 2 = store the new token's rows at the start of /
 *              after the row stream; 0 = by launch size
 * SSD_ERR_INVALID_ARG for values outside these sets.
 */
int ssd_cache_set_launch_shape(ssd_cache *cache, int ch, int wpb, int new_rows);

/*
 * The shape the cache's newest attention / step launch took, in the codes of
 * ssd_cache_set_launch_shape: out3 = { ch, wpb, new_rows } (all 0 before the
 * first launch).  Lets a test check which results must be equal bit for bit.
 */
int ssd_cache_last_launch_shape(const ssd_cache *cache, int32_t out3[3]);

/*
 * ssd_dense_decode_attn with the number of row splits given (1..64; 0 = the
 * library's choice, which is what ssd_dense_decode_attn takes).
 */
int ssd_dense_decode_attn_splits(const void *q, const void *K, const void *V, void *out,
                                 int B, int H, int d, int dtype, int n_cap, int n,
                                 float softmax_scale, float *far, float *tot, int mass_stride,
                                 int vis_start, int w, int splits, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Move what a decode launch moves with none of its arithmetic.  n_units units
 * of unit_bytes each (contiguous in buf, a multiple of 512 bytes: two planes
 * of 256-byte rows) are each read once by one wavefront, four units per
 * workgroup; with rows_written = 2 every wavefront then stores one 256-byte row
 * into each plane of its unit -- the least a decode step must write per head
 * (the new token's K and V rows).  Timing it at a launch's shape tells what the
 * memory system allows a kernel of that shape, with and without the writes.
 *   buf  : dev, n_units * unit_bytes bytes, 16-byte aligned; overwritten in part when rows_written = 2
 *   sink : dev, at least 16 bytes (never written in practice)
 */
int ssd_bench_stream(void *buf, size_t unit_bytes, long long n_units, int rows_written,
                     void *sink, void *stream);

/*
 * Copy `bytes` (a multiple of 16) from src to dst with a plain kernel: a launch whose HBM reads and writes are
 * known exactly, for scaling the profiler's byte counters (FETCH_SIZE, WRITE_SIZE) in the run that reads them.
 *   dst, src : dev, 16-byte aligned, not overlapping
 */
int ssd_bench_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SSD_HOOKS_H */
