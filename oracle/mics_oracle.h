/*
 * CPU oracle for the per-GPU data path of MiCS partitioned data parallelism.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, scalar reference that the
 * tests, the smoke check and the bench's cpu_baseline leg compare the HIP
 * library against.  It shares no code with the HIP library and the product
 * path never calls it.
 *
 * Notation (paper Section 3.1): p = devices holding one model replica
 * (partition group size), k = devices per node, s = micro-steps; the
 * replication group (Section 3.2) has r members.  Ours: N logical elements in
 * the flat buffer, S elements per shard, chunk C_g = shard of group rank g,
 * node j = g div k, local rank l = g mod k.
 *
 * Every function returns 0 on success and a negative value on bad arguments.
 * Loops are split over threads in static contiguous element ranges (see
 * orc_set_threads); the arithmetic on each element does not depend on the
 * thread count.
 *
 * Pins (tests/test_oracle_*.py): all functions below are pinned; none is
 * "parity unpinned".
 */
#ifndef MICS_ORACLE_H
#define MICS_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of threads later calls use (>= 1).  Returns the value now in force. */
int orc_set_threads(int n);

/* bfloat16 <-> float32.  Widening is exact (bf16 is the top 16 bits of an
 * IEEE-754 binary32).  Narrowing rounds to nearest, ties to even, on the
 * binary32 bit pattern; NaN stays a quiet NaN, +-Inf is preserved. */
float    orc_bf16_widen(uint16_t b);
uint16_t orc_bf16_narrow(float f);
void     orc_bf16_narrow_array(uint16_t* out, const float* in, size_t n);
void     orc_bf16_widen_array(float* out, const uint16_t* in, size_t n);

/* ---- hierarchical all-gather, Section 3.3 -------------------------------- */

/* Stage 1 (inter-node all-gather among the devices with local rank l on the
 * p/k nodes): T_l = [C_l, C_{k+l}, ..., C_{(p/k-1)k+l}], chunks in ascending
 * node order.  shards: p host pointers, S elements each.  T_l: (p/k)*S. */
int orc_stage1_gather(void* T_l, const void* const* shards, size_t S,
                      int p, int k, int l, int elem_bytes);

/* What an intra-node all-gather launched directly on the stage-1 outputs
 * yields (the layout the paper calls wrong): W = [T_0, T_1, ..., T_{k-1}].
 * T: k host pointers of (p/k)*S elements.  W: p*S elements. */
int orc_naive_intra_gather(void* W, const void* const* T, size_t S,
                           int p, int k, int elem_bytes);

/* The correct final layout by definition: [C_0, C_1, ..., C_{p-1}], cut to
 * the first n_valid flat elements.  F: n_valid elements. */
int orc_concat_shards(void* F, const void* const* shards, size_t n_valid,
                      size_t S, int p, int elem_bytes);

/* Stages 2+3 seen from the stage-1 outputs: flat element x of the result is
 * element i = x mod S of chunk g = x div S, which stage 1 left in T_{g mod k}
 * at chunk slot g div k.  Writes flat indices < n_valid only. */
int orc_hier_gather_reorder(void* F, const void* const* T, size_t n_valid,
                            size_t S, int p, int k, int elem_bytes);

/* ---- 2-hop gradient synchronisation, Section 3.4 ------------------------- */

/* Hop 1 arithmetic (reduce-scatter inside the partition group, every
 * micro-step, accumulated over micro-steps as in gradient accumulation):
 * for x in [elem_offset, elem_offset+count):
 *   partial = (((g_0[x] + g_1[x]) + g_2[x]) + ... + g_{p-1}[x])   in binary32
 *   acc[x-elem_offset] = (accumulate ? acc[x-elem_offset] : +0) + partial
 * grads: p host pointers to bf16 buffers indexed by the global x. */
int orc_reduce_scatter_accum(float* acc, const uint16_t* const* grads,
                             size_t elem_offset, size_t count, int p,
                             int accumulate);

/* The same reduction for gradients stored as bf16, IEEE binary16 or binary32 (the paper trains
 * in mixed precision on V100, which has no bf16, and one model in plain float32, Section 5).
 * Widening to binary32 is exact for all three; a loss scale, if any, is undone by the scale
 * of orc_replica_average. */
#define ORC_DTYPE_BF16 0
#define ORC_DTYPE_F16  1
#define ORC_DTYPE_F32  2
int orc_reduce_scatter_accum_typed(float* acc, const void* const* grads,
                                   size_t elem_offset, size_t count, int p,
                                   int accumulate, int dtype);
float orc_f16_widen(uint16_t h);
void  orc_f16_widen_array(float* out, const uint16_t* in, size_t n);
/* binary32 -> binary16, round to nearest even, overflow to Inf, subnormals kept: the parameter
 * format of mixed-precision training on devices without bf16. */
uint16_t orc_f16_narrow(float f);
void     orc_f16_narrow_array(uint16_t* out, const float* in, size_t n);

/* Same sum carried in binary64 (every bf16 value and every partial is exact
 * or nearly so): the yardstick that bounds the binary32 error. */
int orc_reduce_scatter_accum_f64(double* acc, const uint16_t* const* grads,
                                 size_t elem_offset, size_t count, int p,
                                 int accumulate);

/* Hop 2 arithmetic (all-reduce inside the replication group at the
 * accumulation boundary) plus the one scaling that turns sums into a mean:
 *   out[x] = (((a_0[x] + a_1[x]) + ...) + a_{r-1}[x]) * scale     in binary32
 * out may alias copies[0]. */
int orc_replica_average(float* out, const float* const* copies, size_t count,
                        int r, float scale);

/* ---- mixed-precision Adam on the shard (Sections 2.1, 3.2) --------------- */

/* Bias-corrected Adam with decoupled weight decay, evaluated in binary64 from
 * the binary32 inputs, each result rounded once to binary32; param_bf16 (may
 * be NULL) = RNE(binary32 master).  step >= 1.
 *   m' = b1*m + (1-b1)*g          v' = b2*v + (1-b2)*g*g
 *   mhat = m'/(1-b1^step)         vhat = v'/(1-b2^step)
 *   w' = w - lr*( mhat/(sqrt(vhat)+eps) + wd*w )                              */
int orc_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                   uint16_t* param_bf16, const float* grad, size_t count,
                   float lr, float beta1, float beta2, float eps,
                   float weight_decay, int step);

/* The same algebra carried out step by step in binary32 (no fused
 * multiply-add), bias corrections computed in binary64 and rounded to
 * binary32 first: the formulation a single-precision kernel uses. */
int orc_adam_shard_f32(float* master, float* exp_avg, float* exp_avg_sq,
                       uint16_t* param_bf16, const float* grad, size_t count,
                       float lr, float beta1, float beta2, float eps,
                       float weight_decay, int step);

#ifdef __cplusplus
}
#endif
#endif /* MICS_ORACLE_H */
