/*
 * libmics -- the per-GPU data path of MiCS partitioned data parallelism on one
 * AMD MI355X (gfx950), as a plain C ABI.
 *
 * What the library computes is what a rank of a MiCS partition group computes
 * on its own GPU around the collectives; the wire transfers are not part of it
 * and the p ranks of a partition group appear here as p buffers:
 *
 *   mics_hier_gather_reorder   chunk rearrangement of the three-stage
 *                              hierarchical all-gather (paper Section 3.3)
 *   mics_reduce_scatter_accum  reduction arithmetic of the per-micro-step
 *                              reduce-scatter inside the partition group,
 *                              accumulated over micro-steps (Section 3.4)
 *   mics_replica_average       reduction arithmetic of the all-reduce inside
 *                              the replication group at the accumulation
 *                              boundary, plus the scaling to a mean (Section 3.4)
 *   mics_adam_shard            mixed-precision Adam on the rank's shard of the
 *                              model states (Sections 2.1 and 3.2)
 *
 * Notation (paper Section 3.1): k = devices per node, p = devices holding one
 * model replica (partition group size), s = micro-steps.  r = size of a
 * replication group (Section 3.2).  Group rank g sits on node j = g div k with
 * local rank l = g mod k.  S = elements per shard; chunk C_g = shard of rank g;
 * the flat parameter is [C_0, C_1, ..., C_{p-1}] cut to its logical length.
 *
 * Conventions for every entry point
 *   - Data pointers are DEVICE pointers on the current HIP device.  Pointer
 *     tables (`const T* const*`) are HOST arrays of device pointers; they are
 *     read during the call and may be freed or reused as soon as it returns.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     and never synchronises: each call validates its arguments on the host,
 *     enqueues its kernel(s) on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and returns.  Work is ordered by that stream.
 *     No kernel uses scratch memory beyond the caller's buffers.
 *   - State between calls: the thread-local error text, and the three
 *     process-wide measurement knobs of mics_tuning.h (grid cap, launch shape,
 *     cache-hint threshold), which never change a result.  Nothing else.
 *   - Arguments are validated before the first HIP call, so every argument
 *     error is reported without a GPU, and on an argument error nothing is
 *     enqueued.  MICS_ERR_HIP reports the status of the failed launch call
 *     itself (an earlier, unrelated HIP error of the thread is neither reported
 *     nor cleared); every entry point issues a single launch, except the
 *     coalesced ones, which issue one launch per 48 tensors and may have
 *     enqueued earlier launches when a later one fails.
 *   - Return value: MICS_OK or a negative MICS_ERR_*; mics_last_error() gives
 *     the text for the calling thread's most recent failure.
 *   - bf16 values travel as uint16_t bit patterns (upper half of a binary32).
 *   - Pointers must be aligned to their element size; that is all the
 *     element-wise calls (reduce, average, Adam) need for full speed, except
 *     that bf16/fp16 gradient buffers of one call should all start at even or
 *     all at odd element addresses (otherwise up to about 7 % slower).  The reorder
 *     runs at copy speed when every buffer and the shard size are multiples
 *     of 16 bytes and through a re-phasing kernel (about 8 % slower) otherwise.
 *   - Buffers of one call must not overlap unless stated.
 */
#ifndef MICS_H
#define MICS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MICS_OK                 0
#define MICS_ERR_INVALID_ARG   (-1)  /* null pointer, bad count, bad geometry, overlap  */
#define MICS_ERR_ALIGNMENT     (-2)  /* pointer not aligned to its element size          */
#define MICS_ERR_UNSUPPORTED   (-3)  /* e.g. element width other than 2 or 4 bytes       */
#define MICS_ERR_HIP           (-4)  /* the HIP runtime refused the launch               */

#define MICS_MAX_GROUP 128           /* largest p, k, r (the paper's largest group: 128) */

/* Library version: major*10000 + minor*100 + patch. */
int mics_version(void);

/* Text of the calling thread's most recent error ("" if none). Never NULL.
 * The pointer stays valid until the same thread's next failing call. */
const char* mics_last_error(void);

/* Elements per shard for a flat buffer of n elements over p ranks:
 * ceil(n / p) rounded up to a multiple of align_elems (>= 1).  The paper does
 * not say how a tensor that does not divide by p is padded; this library pads
 * the tail with elements the caller keeps at zero.  Returns 0 on bad arguments. */
size_t mics_shard_elems(size_t n, int p, size_t align_elems);

/*
 * Stage 2 of the hierarchical all-gather (Section 3.3), applied to the whole
 * gathered parameter: after stage 1 (inter-node all-gather among the devices
 * of equal local rank) the buffer of local rank l holds the chunks
 * T_l = [C_l, C_{k+l}, ..., C_{(p/k-1)k+l}] in ascending node order; gathering
 * those buffers as they are would yield [T_0, ..., T_{k-1}], which for p = 4,
 * k = 2 is the paper's wrong layout [C0, C2, C1, C3].  This call produces the
 * correct one:
 *     dst_flat[(j*k + l)*S + i] = stage1_bufs[l][j*S + i]
 * for all flat indices below n_valid.  Elements at or beyond n_valid (the
 * padded tail) are not written.
 *
 *   dst_flat     device, n_valid elements of elem_bytes bytes
 *   stage1_bufs  host table of k device pointers, (p/k)*S elements each; one
 *                contiguous gathered buffer W is the case bufs[l] = W + l*(p/k)*S
 *   n_valid      logical length, <= p * shard_elems
 *   shard_elems  S
 *   p, k         1 <= k <= p <= MICS_MAX_GROUP, p divisible by k (Section 3.3)
 *   elem_bytes   2 (bf16/fp16) or 4 (fp32); the data is moved bit-exactly
 * dst_flat must not overlap any source buffer.  k = 1 and k = p are plain
 * concatenations.
 */
int mics_hier_gather_reorder(void* dst_flat, const void* const* stage1_bufs,
                             size_t n_valid, size_t shard_elems, int p, int k,
                             int elem_bytes, void* stream);

/*
 * Hop 1 of the 2-hop gradient synchronisation (Section 3.4): the reduction
 * that the reduce-scatter inside the partition group performs on every
 * micro-step, accumulated across micro-steps into the rank's gradient shard.
 * For x in [elem_offset, elem_offset + count):
 *     partial = (((g_0[x] + g_1[x]) + g_2[x]) + ... + g_{p-1}[x])
 *     acc[x - elem_offset] = (accumulate ? acc[x - elem_offset] : +0) + partial
 * with every gradient widened exactly from bf16 and every addition a separate
 * binary32 round-to-nearest-even operation in exactly this order.
 *
 *   acc          device, count fp32 elements, read (if accumulate) and written
 *   grads_bf16   host table of p device pointers; buffer q is rank q's full
 *                gradient, indexed by the global element index x
 *   elem_offset  first owned element (rank view: g*S; whole group: 0)
 *   count        owned elements (rank view: S; whole group: p*S)
 *   accumulate   0 on the first micro-step of a step, non-zero afterwards
 */
int mics_reduce_scatter_accum(float* acc, const uint16_t* const* grads_bf16,
                              size_t elem_offset, size_t count, int p,
                              int accumulate, void* stream);

/*
 * mics_reduce_scatter_accum for gradients stored in another format.  The paper's runs use
 * "mixed-precision" on V100 GPUs, which have no bf16 (Section 5), and one model in plain
 * float32 (the WideResNet experiment): grad_dtype selects bf16 (as above), IEEE binary16 or
 * binary32 buffers.  Widening to binary32 is exact in all three, the additions and their order
 * are the same.  A loss scale applied to binary16 gradients is undone by folding 1/loss_scale
 * into the `scale` of mics_replica_average.  grads: host table of p device pointers.
 */
#define MICS_DTYPE_BF16 0
#define MICS_DTYPE_F16  1
#define MICS_DTYPE_F32  2
int mics_reduce_scatter_accum_typed(float* acc, const void* const* grads, size_t elem_offset,
                                    size_t count, int p, int accumulate, int grad_dtype,
                                    void* stream);

/*
 * Hop 2 (Section 3.4): the reduction of the all-reduce inside the replication
 * group at the gradient-accumulation boundary, and the single scaling that
 * turns the sums of both hops into the global-batch mean:
 *     out[x] = (((a_0[x] + a_1[x]) + ...) + a_{r-1}[x]) * scale
 * in binary32, replicas in ascending order, one multiply at the end.  The
 * paper does not say where the division by the number of summands happens;
 * here both hops are pure sums and the caller passes scale = 1/(r*p*s)
 * (or 1/r for a plain replica average).
 *
 *   out          device, count fp32; may be the same buffer as acc_copies[0]
 *   acc_copies   host table of r device pointers, count fp32 each
 */
int mics_replica_average(float* out, const float* const* acc_copies,
                         size_t count, int r, float scale, void* stream);

/*
 * Parameter update on the rank's shard: Adam in mixed precision (the paper
 * names the optimizer and its 16 bytes of state per parameter, Section 3.2,
 * not the rule; this is bias-corrected Adam with decoupled weight decay):
 *     m' = beta1*m + (1-beta1)*g          v' = beta2*v + (1-beta2)*(g*g)
 *     w' = w - lr*( (m'/(1-beta1^step)) / (sqrt(v'/(1-beta2^step)) + eps)
 *                   + weight_decay*w )
 *     param_bf16 = round-to-nearest-even(w')
 * computed in binary32 with correctly rounded division and square root and no
 * fused multiply-add; 1-beta^step is evaluated in double on the host and
 * rounded to binary32.
 *
 *   master, exp_avg, exp_avg_sq   device fp32, count each, updated in place
 *   param_bf16                    device, count bf16, written; may be NULL
 *   grad                          device fp32, count, read only
 *   step                          >= 1, the number of this update
 */
int mics_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                    uint16_t* param_bf16, const float* grad, size_t count,
                    float lr, float beta1, float beta2, float eps,
                    float weight_decay, int step, void* stream);

/*
 * mics_replica_average followed by mics_adam_shard in one pass over the shard (Sections 3.4 and
 * 2.1): the averaged gradient
 *     g[x] = (((a_0[x] + a_1[x]) + ...) + a_{r-1}[x]) * scale
 * is formed in registers and consumed by the Adam update at once, so it is never written to or
 * re-read from memory.  Results (master, exp_avg, exp_avg_sq, param_bf16) are bit-identical to
 * the two separate calls; the accumulator copies are only read.  Arguments as in those calls.
 */
int mics_replica_average_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                                    uint16_t* param_bf16, const float* const* acc_copies,
                                    size_t count, int r, float scale, float lr, float beta1,
                                    float beta2, float eps, float weight_decay, int step,
                                    void* stream);

/*
 * mics_adam_shard and mics_replica_average_adam_shard with the 16-bit parameter copy in a
 * chosen format.  The paper trains in "mixed-precision" on V100 GPUs, which have no bf16
 * (Section 5): there the low-precision parameters that the next gather moves are IEEE
 * binary16.  param_dtype = MICS_DTYPE_BF16 (as in the calls above) or MICS_DTYPE_F16:
 * param_out[x] = the new master[x] rounded to nearest even in that format (binary16:
 * subnormals kept, magnitudes of 65520 and above become Inf, NaN stays NaN).
 * MICS_DTYPE_F32 is MICS_ERR_UNSUPPORTED: the master is the binary32 parameter, pass
 * param_out = NULL.  param_out: device, count 2-byte elements, written, may be NULL;
 * everything else as in the calls above, and the fp32 results are the same bit for bit.
 */
int mics_adam_shard_typed(float* master, float* exp_avg, float* exp_avg_sq, void* param_out,
                          int param_dtype, const float* grad, size_t count, float lr,
                          float beta1, float beta2, float eps, float weight_decay, int step,
                          void* stream);
int mics_replica_average_adam_shard_typed(float* master, float* exp_avg, float* exp_avg_sq,
                                          void* param_out, int param_dtype,
                                          const float* const* acc_copies, size_t count, int r,
                                          float scale, float lr, float beta1, float beta2,
                                          float eps, float weight_decay, int step, void* stream);

/*
 * One separately sharded tensor of a coalesced call.  The paper's coalesced collectives
 * (Section 4, "Coalesced communication APIs": all_gather_coalesced, reduce_scatter_coalesced)
 * launch the per-tensor operations of many tensors at once, with no staging copy; the two
 * entry points below are their on-device halves.  Offsets are in elements.
 */
typedef struct mics_segment {
    size_t numel;        /* reorder: logical elements of the tensor; reduce: elements to reduce */
    size_t shard_elems;  /* reorder: S of this tensor (numel <= p*S); reduce: ignored          */
    size_t src_offset;   /* where the tensor's region starts inside every source buffer        */
    size_t dst_offset;   /* where the tensor's region starts inside the destination            */
} mics_segment;

/*
 * mics_hier_gather_reorder for n_segs tensors at once: for every segment t and every flat
 * index x < numel_t, with g = x div S_t, i = x mod S_t, j = g div k, l = g mod k,
 *     dst_flat[dst_offset_t + x] = stage1_bufs[l][src_offset_t + j*S_t + i].
 * Tensor t occupies (p/k)*S_t elements from src_offset_t in every stage-1 buffer and numel_t
 * elements from dst_offset_t in dst_flat; the destination regions of different tensors must not
 * overlap (checked: MICS_ERR_INVALID_ARG).  segs is a HOST array.  Tensors whose addresses and
 * shard sizes are multiples of 16 bytes share one launch per 48 of them, all other tensors
 * another launch per 48: a layer of 16 tensors is moved by at most two launches.
 */
int mics_hier_gather_reorder_coalesced(void* dst_flat, const void* const* stage1_bufs,
                                       const mics_segment* segs, int n_segs, int p, int k,
                                       int elem_bytes, void* stream);

/*
 * mics_reduce_scatter_accum for n_segs tensors at once: for every segment t and i < numel_t
 *     acc[dst_offset_t + i] = (accumulate ? acc[dst_offset_t + i] : +0)
 *                             + (((g_0[src_offset_t + i] + g_1[...]) + ...) + g_{p-1}[...]),
 * same arithmetic and order as mics_reduce_scatter_accum.  For rank g of a partition group
 * whose gradient buffers hold tensor t at offset o_t (p*S_t elements) and whose shard buffer
 * holds it at offset a_t: numel = S_t, src_offset = o_t + g*S_t, dst_offset = a_t.
 * The accumulator regions of different tensors must not overlap (checked).  One launch per
 * 48 tensors, whatever their alignment.
 */
int mics_reduce_scatter_accum_coalesced(float* acc, const uint16_t* const* grads_bf16,
                                        const mics_segment* segs, int n_segs, int p,
                                        int accumulate, void* stream);

/*
 * mics_reduce_scatter_accum_coalesced for gradient buffers stored as bf16, IEEE binary16 or
 * binary32 (grad_dtype = MICS_DTYPE_*, as in mics_reduce_scatter_accum_typed): the paper's own
 * runs put binary16 gradients through its coalesced reduce-scatter (Sections 4 and 5).
 * grads: host table of p device pointers; offsets and sizes in elements of that format.
 */
int mics_reduce_scatter_accum_coalesced_typed(float* acc, const void* const* grads,
                                              const mics_segment* segs, int n_segs, int p,
                                              int accumulate, int grad_dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MICS_H */
