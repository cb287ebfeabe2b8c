/*
 * libmics -- measurement and test knobs.  Not part of the method (no citation of the paper
 * applies): neither call changes any result, only how the kernels of later calls are
 * launched.  Both are process-wide and may be called at any time; calls that are already
 * enqueued are not affected.  The benchmark, the sweeps and the tests use them; a training
 * loop has no reason to.
 */
#ifndef MICS_TUNING_H
#define MICS_TUNING_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Caps the grid of the streaming kernels at blocks_per_cu workgroups per compute unit (lanes
 * then stride over the data); 0 restores the built-in choice, which covers the data with one
 * pass per lane.  Returns MICS_OK, or MICS_ERR_INVALID_ARG if negative or above 4096.
 */
int mics_set_blocks_per_cu(int blocks_per_cu);

/*
 * The reduce and average kernels leave an accumulator / output of up to `bytes` bytes
 * cacheable and stream a larger one past the caches with non-temporal accesses.  0 restores
 * the built-in policy (224 MiB -- what the 256 MB Infinity Cache of an MI355X absorbs -- and,
 * for reductions over 32 or more buffers, always streamed); 1 makes every call take the
 * streaming kernels and a huge value none, which is how the tests reach both kinds with small
 * buffers.  Returns MICS_OK.
 */
int mics_set_stream_threshold_bytes(size_t bytes);

/*
 * Launch shape of a kernel family for later calls: lanes per workgroup (64, 128, 256 or 512) and
 * the most wavefronts a compute unit may hold at a time (1 .. 32; 32 = as many as fit); 0 for
 * either restores the built-in choice, which depends on the size of the call and on the
 * alignment of its buffers.  Streaming kernels on an MI355X run fastest in single-wavefront
 * workgroups with 8 to 16 wavefronts per compute unit; this knob is how that was measured.
 * Returns MICS_OK or MICS_ERR_INVALID_ARG.
 */
#define MICS_KERNELS_REORDER 0   /* mics_hier_gather_reorder (16-byte aligned geometry)       */
#define MICS_KERNELS_REDUCE  1   /* mics_reduce_scatter_accum, _typed, _coalesced             */
#define MICS_KERNELS_AVERAGE 2   /* mics_replica_average                                      */
#define MICS_KERNELS_ADAM    3   /* mics_adam_shard                                           */
#define MICS_KERNELS_FUSED   4   /* mics_replica_average_adam_shard                           */
int mics_set_launch_shape(int kernel_family, int lanes, int waves_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* MICS_TUNING_H */
