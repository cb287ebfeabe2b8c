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
 * cacheable and stream a larger one past the caches with non-temporal accesses (default
 * 224 MiB: what the 256 MB Infinity Cache of an MI355X absorbs).  0 restores the default;
 * 1 makes every call take the streaming kernels, which is how the tests reach them with
 * small buffers.  Returns MICS_OK.
 */
int mics_set_stream_threshold_bytes(size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* MICS_TUNING_H */
