// Internal interface between the host-side argument checks (api.cpp) and the
// kernel launchers (kernels.hip).  Not installed; the public ABI is include/mics.h.
#pragma once

#include <cstddef>
#include <cstdint>

namespace mics {

constexpr int kMaxGroup = 128;

// Table of device pointers handed to a kernel by value (kernel-argument
// segment), so no device-side table has to be allocated or copied.
struct PtrTable {
    const void* ptr[kMaxGroup];
};

// Launchers: arguments are already validated.  Each returns 0 or the hipError_t
// of the failed launch call (as int) and enqueues on `stream` without waiting.
// Every launcher issues exactly one kernel launch, the coalesced ones one per
// kMaxSegPerLaunch segments.

// vec16: every source, the destination and the shard size are multiples of 16
// bytes -> direct 128-bit copy; otherwise the kernel that re-phases through a lane shift.
int launch_reorder(void* dst, const PtrTable& src, size_t n_valid_bytes,
                   size_t shard_bytes, int p, int k, bool vec16, void* stream);

// grads.ptr[q] already points at element elem_offset of rank q's buffer (aligned to its
// element size; the accumulator to 4 bytes).  kind: 0 bf16, 1 IEEE binary16, 2 binary32.
int launch_reduce_scatter_accum(float* acc, const PtrTable& grads, size_t count,
                                int p, bool accumulate, int kind, void* stream);

int launch_replica_average(float* out, const PtrTable& copies, size_t count,
                           int r, float scale, void* stream);

struct AdamScalars {
    float lr, beta1, beta2, eps, weight_decay;
    float one_minus_beta1, one_minus_beta2;
    float bias_corr1, bias_corr2;  // 1 - beta^step, double on the host, rounded
};

// param_bf16: the 16-bit copy of the new master (NULL = none), bf16 or, with param_f16, binary16.
int launch_adam(float* master, float* exp_avg, float* exp_avg_sq,
                uint16_t* param_bf16, bool param_f16, const float* grad, size_t count,
                const AdamScalars& hp, void* stream);

// Replica average and Adam in one pass (the averaged gradient stays in registers).
int launch_avg_adam(float* master, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16, bool param_f16,
                    const PtrTable& copies, int r, float scale, size_t count, const AdamScalars& hp,
                    void* stream);

// Segment records travel in the kernel-argument segment: at most this many per launch.
constexpr int kMaxSegPerLaunch = 48;

// One separately sharded tensor of a coalesced call (mirrors mics_segment; elements).
struct Segment {
    size_t numel, shard_elems, src_offset, dst_offset;
};

// vec16: every segment satisfies the 16-byte conditions of the vector kernel (bases, shard
// size and both offsets); otherwise the segments go through the lane-shift kernel, which
// takes any element-aligned geometry.
int launch_reorder_coalesced(void* dst, const PtrTable& src, const Segment* segs, int n, int p,
                             int k, int elem_bytes, bool vec16, void* stream);
// numel = elements to reduce; any element-aligned geometry.  kind: 0 bf16, 1 binary16, 2 binary32.
int launch_reduce_coalesced(float* acc, const PtrTable& grads, const Segment* segs, int n, int p,
                            bool accumulate, int kind, void* stream);

// Kernel families whose launch shape can be set (mics_tuning.h).
enum { kFamReorder = 0, kFamReduce = 1, kFamAverage = 2, kFamAdam = 3, kFamFused = 4, kFamilies = 5 };

// 0 = built-in choice.
void set_blocks_per_cu(int n);
void set_stream_threshold_bytes(size_t n);
void set_launch_shape(int family, int lanes, int waves_per_cu);

const char* hip_error_text(int err);

}  // namespace mics
