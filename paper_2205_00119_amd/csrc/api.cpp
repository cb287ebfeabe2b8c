// C ABI of libmics: host-side argument validation and dispatch.
// Every check here runs before the first HIP call, so argument errors are
// reported identically on a machine without a GPU.
#include "../../include/mics.h"
#include "../../include/mics_tuning.h"
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <utility>
#include <vector>

namespace {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

inline uintptr_t addr(const void* p) { return reinterpret_cast<uintptr_t>(p); }
inline bool aligned(const void* p, size_t a) { return (addr(p) & (a - 1)) == 0; }

// [a, a+an) and [b, b+bn) share at least one byte
inline bool overlaps(const void* a, size_t an, const void* b, size_t bn)
{
    return an && bn && addr(a) < addr(b) + bn && addr(b) < addr(a) + an;
}

// True if two of the destination regions [dst_offset, dst_offset + numel) of the segments share an
// element.  *bad_a / *bad_b receive the indices of one offending pair.  Returns -1 if the host
// is out of memory for the sort.
int regions_overlap(const mics_segment* segs, int n, int* bad_a, int* bad_b)
{
    try {
        std::vector<std::pair<size_t, int>> order;
        order.reserve((size_t)n);
        for (int t = 0; t < n; ++t)
            if (segs[t].numel) order.emplace_back(segs[t].dst_offset, t);
        std::sort(order.begin(), order.end());
        for (size_t i = 1; i < order.size(); ++i) {
            const mics_segment& prev = segs[order[i - 1].second];
            if (prev.dst_offset + prev.numel > order[i].first) {
                *bad_a = order[i - 1].second;
                *bad_b = order[i].second;
                return 1;
            }
        }
        return 0;
    } catch (const std::bad_alloc&) {
        return -1;
    }
}

int hip_fail(const char* what, int err)
{
    return fail(MICS_ERR_HIP, "%s: HIP error %d (%s)", what, err, mics::hip_error_text(err));
}

mics::AdamScalars adam_scalars(float lr, float beta1, float beta2, float eps, float weight_decay,
                               int step)
{
    mics::AdamScalars hp;
    hp.lr = lr; hp.beta1 = beta1; hp.beta2 = beta2; hp.eps = eps; hp.weight_decay = weight_decay;
    hp.one_minus_beta1 = 1.0f - beta1;
    hp.one_minus_beta2 = 1.0f - beta2;
    hp.bias_corr1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    hp.bias_corr2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    return hp;
}

}  // namespace

extern "C" {

int mics_version(void) { return 300; }   // 0.3.0

const char* mics_last_error(void) { return g_error; }

size_t mics_shard_elems(size_t n, int p, size_t align_elems)
{
    if (p < 1 || align_elems < 1) return 0;
    size_t per = n / (size_t)p + (n % (size_t)p ? 1 : 0);
    size_t rem = per % align_elems;
    return rem ? per + (align_elems - rem) : per;
}

int mics_set_blocks_per_cu(int blocks_per_cu)
{
    if (blocks_per_cu < 0 || blocks_per_cu > 4096)
        return fail(MICS_ERR_INVALID_ARG, "mics_set_blocks_per_cu: %d not in [0, 4096]", blocks_per_cu);
    mics::set_blocks_per_cu(blocks_per_cu);
    return MICS_OK;
}

int mics_set_stream_threshold_bytes(size_t bytes)
{
    mics::set_stream_threshold_bytes(bytes);
    return MICS_OK;
}

int mics_set_launch_shape(int kernel_family, int lanes, int waves_per_cu)
{
    const char* fn = "mics_set_launch_shape";
    if (kernel_family < 0 || kernel_family >= mics::kFamilies)
        return fail(MICS_ERR_INVALID_ARG, "%s: kernel_family = %d not in [0, %d]", fn, kernel_family,
                    mics::kFamilies - 1);
    if (lanes != 0 && lanes != 64 && lanes != 128 && lanes != 256 && lanes != 512)
        return fail(MICS_ERR_INVALID_ARG, "%s: lanes = %d is not 0, 64, 128, 256 or 512", fn, lanes);
    if (waves_per_cu < 0 || waves_per_cu > 32)
        return fail(MICS_ERR_INVALID_ARG, "%s: waves_per_cu = %d not in [0, 32]", fn, waves_per_cu);
    mics::set_launch_shape(kernel_family, lanes, waves_per_cu);
    return MICS_OK;
}

int mics_hier_gather_reorder(void* dst_flat, const void* const* stage1_bufs,
                             size_t n_valid, size_t shard_elems, int p, int k,
                             int elem_bytes, void* stream)
{
    const char* fn = "mics_hier_gather_reorder";
    if (elem_bytes != 2 && elem_bytes != 4)
        return fail(MICS_ERR_UNSUPPORTED, "%s: elem_bytes = %d, must be 2 or 4", fn, elem_bytes);
    if (p < 1 || p > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d not in [1, %d]", fn, p, MICS_MAX_GROUP);
    if (k < 1 || k > p)
        return fail(MICS_ERR_INVALID_ARG, "%s: k = %d not in [1, p = %d]", fn, k, p);
    if (p % k != 0)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d is not divisible by k = %d", fn, p, k);
    const size_t eb = (size_t)elem_bytes;
    if (shard_elems > SIZE_MAX / eb / (size_t)p)
        return fail(MICS_ERR_INVALID_ARG, "%s: p * shard_elems * elem_bytes overflows", fn);
    if (n_valid > (size_t)p * shard_elems)
        return fail(MICS_ERR_INVALID_ARG, "%s: n_valid = %zu exceeds p * shard_elems = %zu", fn,
                    n_valid, (size_t)p * shard_elems);
    if (!stage1_bufs) return fail(MICS_ERR_INVALID_ARG, "%s: stage1_bufs is NULL", fn);
    if (n_valid == 0) return MICS_OK;
    if (!dst_flat) return fail(MICS_ERR_INVALID_ARG, "%s: dst_flat is NULL", fn);
    if (!aligned(dst_flat, eb))
        return fail(MICS_ERR_ALIGNMENT, "%s: dst_flat not aligned to %d bytes", fn, elem_bytes);

    const size_t shard_bytes = shard_elems * eb;
    const size_t src_bytes = (size_t)(p / k) * shard_bytes;
    const size_t dst_bytes = n_valid * eb;
    mics::PtrTable tab{};
    bool vec16 = aligned(dst_flat, 16) && shard_bytes % 16 == 0;
    for (int l = 0; l < k; ++l) {
        const void* s = stage1_bufs[l];
        if (!s) return fail(MICS_ERR_INVALID_ARG, "%s: stage1_bufs[%d] is NULL", fn, l);
        if (!aligned(s, eb))
            return fail(MICS_ERR_ALIGNMENT, "%s: stage1_bufs[%d] not aligned to %d bytes", fn, l,
                        elem_bytes);
        if (overlaps(dst_flat, dst_bytes, s, src_bytes))
            return fail(MICS_ERR_INVALID_ARG, "%s: dst_flat overlaps stage1_bufs[%d]", fn, l);
        vec16 = vec16 && aligned(s, 16);
        tab.ptr[l] = s;
    }
    int err = mics::launch_reorder(dst_flat, tab, dst_bytes, shard_bytes, p, k, vec16, stream);
    return err ? hip_fail(fn, err) : MICS_OK;
}

}  // extern "C"

namespace {

// fn / table: the entry point's and its table argument's names, for the error texts.
int reduce_scatter_accum(const char* fn, const char* table, float* acc, const void* const* grads,
                         size_t elem_offset, size_t count, int p, int accumulate, int grad_dtype,
                         void* stream)
{
    if (grad_dtype != MICS_DTYPE_BF16 && grad_dtype != MICS_DTYPE_F16 && grad_dtype != MICS_DTYPE_F32)
        return fail(MICS_ERR_UNSUPPORTED, "%s: grad_dtype = %d is not bf16, f16 or f32", fn, grad_dtype);
    const size_t gb = grad_dtype == MICS_DTYPE_F32 ? 4 : 2;
    if (p < 1 || p > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d not in [1, %d]", fn, p, MICS_MAX_GROUP);
    if (!grads) return fail(MICS_ERR_INVALID_ARG, "%s: %s is NULL", fn, table);
    if (elem_offset > SIZE_MAX / 4 - count || count > SIZE_MAX / 4)
        return fail(MICS_ERR_INVALID_ARG, "%s: elem_offset + count overflows", fn);
    if (count == 0) return MICS_OK;
    if (!acc) return fail(MICS_ERR_INVALID_ARG, "%s: acc is NULL", fn);
    if (!aligned(acc, 4)) return fail(MICS_ERR_ALIGNMENT, "%s: acc not aligned to 4 bytes", fn);

    mics::PtrTable tab{};
    for (int q = 0; q < p; ++q) {
        const void* g = grads[q];
        if (!g) return fail(MICS_ERR_INVALID_ARG, "%s: %s[%d] is NULL", fn, table, q);
        if (!aligned(g, gb))
            return fail(MICS_ERR_ALIGNMENT, "%s: %s[%d] not aligned to %zu bytes", fn, table, q, gb);
        const char* first = (const char*)g + elem_offset * gb;
        if (overlaps(acc, count * 4, first, count * gb))
            return fail(MICS_ERR_INVALID_ARG, "%s: acc overlaps %s[%d]", fn, table, q);
        tab.ptr[q] = first;
    }
    const int kind = grad_dtype == MICS_DTYPE_BF16 ? 0 : grad_dtype == MICS_DTYPE_F16 ? 1 : 2;
    int err = mics::launch_reduce_scatter_accum(acc, tab, count, p, accumulate != 0, kind, stream);
    return err ? hip_fail(fn, err) : MICS_OK;
}

}  // namespace

extern "C" {

int mics_reduce_scatter_accum_typed(float* acc, const void* const* grads, size_t elem_offset,
                                    size_t count, int p, int accumulate, int grad_dtype,
                                    void* stream)
{
    return reduce_scatter_accum("mics_reduce_scatter_accum_typed", "grads", acc, grads, elem_offset, count, p,
                                accumulate, grad_dtype, stream);
}

int mics_reduce_scatter_accum(float* acc, const uint16_t* const* grads_bf16,
                              size_t elem_offset, size_t count, int p,
                              int accumulate, void* stream)
{
    return reduce_scatter_accum("mics_reduce_scatter_accum", "grads_bf16", acc,
                                (const void* const*)grads_bf16, elem_offset, count, p, accumulate,
                                MICS_DTYPE_BF16, stream);
}

int mics_replica_average(float* out, const float* const* acc_copies,
                         size_t count, int r, float scale, void* stream)
{
    const char* fn = "mics_replica_average";
    if (r < 1 || r > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: r = %d not in [1, %d]", fn, r, MICS_MAX_GROUP);
    if (!acc_copies) return fail(MICS_ERR_INVALID_ARG, "%s: acc_copies is NULL", fn);
    if (count > SIZE_MAX / 4) return fail(MICS_ERR_INVALID_ARG, "%s: count overflows", fn);
    if (count == 0) return MICS_OK;
    if (!out) return fail(MICS_ERR_INVALID_ARG, "%s: out is NULL", fn);
    if (!aligned(out, 4)) return fail(MICS_ERR_ALIGNMENT, "%s: out not aligned to 4 bytes", fn);

    mics::PtrTable tab{};
    for (int c = 0; c < r; ++c) {
        const float* a = acc_copies[c];
        if (!a) return fail(MICS_ERR_INVALID_ARG, "%s: acc_copies[%d] is NULL", fn, c);
        if (!aligned(a, 4))
            return fail(MICS_ERR_ALIGNMENT, "%s: acc_copies[%d] not aligned to 4 bytes", fn, c);
        // the result may replace the first copy exactly (in-place all-reduce), nothing else
        bool same_as_first = (c == 0 && a == out);
        if (!same_as_first && overlaps(out, count * 4, a, count * 4))
            return fail(MICS_ERR_INVALID_ARG, "%s: out overlaps acc_copies[%d]", fn, c);
        tab.ptr[c] = a;
    }
    int err = mics::launch_replica_average(out, tab, count, r, scale, stream);
    return err ? hip_fail(fn, err) : MICS_OK;
}

}  // extern "C"

namespace {

// `pname` = what the entry point calls its 16-bit parameter output; f16 = binary16, else bf16.
int adam_shard(const char* fn, const char* pname, float* master, float* exp_avg, float* exp_avg_sq,
               uint16_t* param_bf16, bool f16, const float* grad, size_t count, float lr, float beta1,
               float beta2, float eps, float weight_decay, int step, void* stream)
{
    if (step < 1) return fail(MICS_ERR_INVALID_ARG, "%s: step = %d, must be >= 1", fn, step);
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))
        return fail(MICS_ERR_INVALID_ARG, "%s: beta1 = %g, beta2 = %g must lie in [0, 1)", fn,
                    (double)beta1, (double)beta2);
    if (count > SIZE_MAX / 4) return fail(MICS_ERR_INVALID_ARG, "%s: count overflows", fn);
    if (count == 0) return MICS_OK;
    if (!master || !exp_avg || !exp_avg_sq || !grad)
        return fail(MICS_ERR_INVALID_ARG, "%s: master, exp_avg, exp_avg_sq and grad must be non-NULL",
                    fn);
    const void* f32[4] = {master, exp_avg, exp_avg_sq, grad};
    const char* name[4] = {"master", "exp_avg", "exp_avg_sq", "grad"};
    for (int a = 0; a < 4; ++a) {
        if (!aligned(f32[a], 4))
            return fail(MICS_ERR_ALIGNMENT, "%s: %s not aligned to 4 bytes", fn, name[a]);
        for (int b = a + 1; b < 4; ++b)
            if (overlaps(f32[a], count * 4, f32[b], count * 4))
                return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps %s", fn, name[a], name[b]);
        if (param_bf16 && overlaps(f32[a], count * 4, param_bf16, count * 2))
            return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps %s", fn, pname, name[a]);
    }
    if (param_bf16 && !aligned(param_bf16, 2))
        return fail(MICS_ERR_ALIGNMENT, "%s: %s not aligned to 2 bytes", fn, pname);

    const mics::AdamScalars hp = adam_scalars(lr, beta1, beta2, eps, weight_decay, step);
    int err = mics::launch_adam(master, exp_avg, exp_avg_sq, param_bf16, f16, grad, count, hp, stream);
    return err ? hip_fail(fn, err) : MICS_OK;
}

// The 16-bit parameter formats of the typed Adam entry points.
int param_format(const char* fn, int param_dtype, bool* f16)
{
    if (param_dtype == MICS_DTYPE_F32)
        return fail(MICS_ERR_UNSUPPORTED, "%s: param_dtype = MICS_DTYPE_F32: the master is the binary32 parameter; "
                    "pass param_out = NULL", fn);
    if (param_dtype != MICS_DTYPE_BF16 && param_dtype != MICS_DTYPE_F16)
        return fail(MICS_ERR_INVALID_ARG, "%s: param_dtype = %d is not MICS_DTYPE_BF16 or MICS_DTYPE_F16", fn,
                    param_dtype);
    *f16 = param_dtype == MICS_DTYPE_F16;
    return MICS_OK;
}

}  // namespace

extern "C" {

int mics_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                    uint16_t* param_bf16, const float* grad, size_t count,
                    float lr, float beta1, float beta2, float eps,
                    float weight_decay, int step, void* stream)
{
    return adam_shard("mics_adam_shard", "param_bf16", master, exp_avg, exp_avg_sq, param_bf16, false, grad, count,
                      lr, beta1, beta2, eps, weight_decay, step, stream);
}

int mics_adam_shard_typed(float* master, float* exp_avg, float* exp_avg_sq, void* param_out,
                          int param_dtype, const float* grad, size_t count, float lr, float beta1,
                          float beta2, float eps, float weight_decay, int step, void* stream)
{
    const char* fn = "mics_adam_shard_typed";
    bool f16 = false;
    if (int rc = param_format(fn, param_dtype, &f16)) return rc;
    return adam_shard(fn, "param_out", master, exp_avg, exp_avg_sq, (uint16_t*)param_out, f16, grad, count, lr,
                      beta1, beta2, eps, weight_decay, step, stream);
}

int mics_hier_gather_reorder_coalesced(void* dst_flat, const void* const* stage1_bufs,
                                       const mics_segment* segs, int n_segs, int p, int k,
                                       int elem_bytes, void* stream)
{
    const char* fn = "mics_hier_gather_reorder_coalesced";
    if (elem_bytes != 2 && elem_bytes != 4)
        return fail(MICS_ERR_UNSUPPORTED, "%s: elem_bytes = %d, must be 2 or 4", fn, elem_bytes);
    if (p < 1 || p > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d not in [1, %d]", fn, p, MICS_MAX_GROUP);
    if (k < 1 || k > p)
        return fail(MICS_ERR_INVALID_ARG, "%s: k = %d not in [1, p = %d]", fn, k, p);
    if (p % k != 0)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d is not divisible by k = %d", fn, p, k);
    if (n_segs < 0) return fail(MICS_ERR_INVALID_ARG, "%s: n_segs = %d is negative", fn, n_segs);
    if (n_segs == 0) return MICS_OK;
    if (!segs) return fail(MICS_ERR_INVALID_ARG, "%s: segs is NULL", fn);
    if (!stage1_bufs) return fail(MICS_ERR_INVALID_ARG, "%s: stage1_bufs is NULL", fn);
    if (!dst_flat) return fail(MICS_ERR_INVALID_ARG, "%s: dst_flat is NULL", fn);
    const size_t eb = (size_t)elem_bytes;
    if (!aligned(dst_flat, eb))
        return fail(MICS_ERR_ALIGNMENT, "%s: dst_flat not aligned to %d bytes", fn, elem_bytes);
    const size_t limit = SIZE_MAX / 8 / (size_t)p;   // keeps every byte offset below SIZE_MAX / 2
    size_t dst_lo = SIZE_MAX, dst_hi = 0, src_lo = SIZE_MAX, src_hi = 0, total = 0;
    for (int t = 0; t < n_segs; ++t) {
        const mics_segment& sg = segs[t];
        if (sg.shard_elems > limit || sg.src_offset > limit || sg.dst_offset > limit)
            return fail(MICS_ERR_INVALID_ARG, "%s: segment %d: sizes or offsets overflow", fn, t);
        if (sg.numel > (size_t)p * sg.shard_elems)
            return fail(MICS_ERR_INVALID_ARG, "%s: segment %d: numel = %zu exceeds p * shard_elems = %zu",
                        fn, t, sg.numel, (size_t)p * sg.shard_elems);
        if (sg.numel == 0) continue;
        total += sg.numel;
        if (sg.dst_offset < dst_lo) dst_lo = sg.dst_offset;
        if (sg.dst_offset + sg.numel > dst_hi) dst_hi = sg.dst_offset + sg.numel;
        if (sg.src_offset < src_lo) src_lo = sg.src_offset;
        const size_t src_end = sg.src_offset + (size_t)(p / k) * sg.shard_elems;
        if (src_end > src_hi) src_hi = src_end;
    }
    mics::PtrTable tab{};
    bool bases16 = aligned(dst_flat, 16);
    for (int l = 0; l < k; ++l) {
        const void* s = stage1_bufs[l];
        if (!s) return fail(MICS_ERR_INVALID_ARG, "%s: stage1_bufs[%d] is NULL", fn, l);
        if (!aligned(s, eb))
            return fail(MICS_ERR_ALIGNMENT, "%s: stage1_bufs[%d] not aligned to %d bytes", fn, l,
                        elem_bytes);
        if (total && overlaps((const char*)dst_flat + dst_lo * eb, (dst_hi - dst_lo) * eb,
                              (const char*)s + src_lo * eb, (src_hi - src_lo) * eb))
            return fail(MICS_ERR_INVALID_ARG, "%s: dst_flat overlaps stage1_bufs[%d]", fn, l);
        bases16 = bases16 && aligned(s, 16);
        tab.ptr[l] = s;
    }
    if (total == 0) return MICS_OK;
    int bad_a = 0, bad_b = 0;
    if (int ov = regions_overlap(segs, n_segs, &bad_a, &bad_b))
        return ov < 0 ? fail(MICS_ERR_INVALID_ARG, "%s: out of host memory while checking %d segments", fn, n_segs)
                      : fail(MICS_ERR_INVALID_ARG, "%s: the destination regions of segments %d and %d overlap",
                             fn, bad_a, bad_b);

    // Tensors whose bases, shard size and offsets are 16-byte clean go to the vector kernel, all
    // others to the kernel for any alignment: one launch per kMaxSegPerLaunch tensors of either kind.
    mics::Segment clean[mics::kMaxSegPerLaunch], other[mics::kMaxSegPerLaunch];
    int nc = 0, no = 0;
    for (int t = 0; t <= n_segs; ++t) {
        const bool last = (t == n_segs);
        if (!last && segs[t].numel) {
            const mics_segment& sg = segs[t];
            const bool vec16 = bases16 && (sg.shard_elems * eb) % 16 == 0 && (sg.src_offset * eb) % 16 == 0 &&
                               (sg.dst_offset * eb) % 16 == 0;
            mics::Segment& slot = vec16 ? clean[nc++] : other[no++];
            slot.numel = sg.numel; slot.shard_elems = sg.shard_elems;
            slot.src_offset = sg.src_offset; slot.dst_offset = sg.dst_offset;
        }
        if (nc == mics::kMaxSegPerLaunch || (last && nc)) {
            int err = mics::launch_reorder_coalesced(dst_flat, tab, clean, nc, p, k, elem_bytes, true, stream);
            if (err) return hip_fail(fn, err);
            nc = 0;
        }
        if (no == mics::kMaxSegPerLaunch || (last && no)) {
            int err = mics::launch_reorder_coalesced(dst_flat, tab, other, no, p, k, elem_bytes, false, stream);
            if (err) return hip_fail(fn, err);
            no = 0;
        }
    }
    return MICS_OK;
}

}  // extern "C"

namespace {

// `table` = what the entry point calls its pointer table; kind: 0 bf16, 1 binary16, 2 binary32.
int reduce_scatter_accum_coalesced(const char* fn, const char* table, float* acc, const void* const* grads,
                                   const mics_segment* segs, int n_segs, int p, int accumulate, int kind,
                                   void* stream)
{
    const size_t gb = kind == 2 ? 4 : 2;
    if (p < 1 || p > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: p = %d not in [1, %d]", fn, p, MICS_MAX_GROUP);
    if (n_segs < 0) return fail(MICS_ERR_INVALID_ARG, "%s: n_segs = %d is negative", fn, n_segs);
    if (n_segs == 0) return MICS_OK;
    if (!segs) return fail(MICS_ERR_INVALID_ARG, "%s: segs is NULL", fn);
    if (!grads) return fail(MICS_ERR_INVALID_ARG, "%s: %s is NULL", fn, table);
    if (!acc) return fail(MICS_ERR_INVALID_ARG, "%s: acc is NULL", fn);
    if (!aligned(acc, 4)) return fail(MICS_ERR_ALIGNMENT, "%s: acc not aligned to 4 bytes", fn);
    const size_t limit = SIZE_MAX / 16;
    size_t dst_lo = SIZE_MAX, dst_hi = 0, src_lo = SIZE_MAX, src_hi = 0, total = 0;
    for (int t = 0; t < n_segs; ++t) {
        const mics_segment& sg = segs[t];
        if (sg.numel > limit || sg.src_offset > limit || sg.dst_offset > limit)
            return fail(MICS_ERR_INVALID_ARG, "%s: segment %d: sizes or offsets overflow", fn, t);
        if (sg.numel == 0) continue;
        total += sg.numel;
        if (sg.dst_offset < dst_lo) dst_lo = sg.dst_offset;
        if (sg.dst_offset + sg.numel > dst_hi) dst_hi = sg.dst_offset + sg.numel;
        if (sg.src_offset < src_lo) src_lo = sg.src_offset;
        if (sg.src_offset + sg.numel > src_hi) src_hi = sg.src_offset + sg.numel;
    }
    mics::PtrTable tab{};
    for (int q = 0; q < p; ++q) {
        const char* g = (const char*)grads[q];
        if (!g) return fail(MICS_ERR_INVALID_ARG, "%s: %s[%d] is NULL", fn, table, q);
        if (!aligned(g, gb))
            return fail(MICS_ERR_ALIGNMENT, "%s: %s[%d] not aligned to %zu bytes", fn, table, q, gb);
        if (total && overlaps(acc + dst_lo, (dst_hi - dst_lo) * 4, g + src_lo * gb, (src_hi - src_lo) * gb))
            return fail(MICS_ERR_INVALID_ARG, "%s: acc overlaps %s[%d]", fn, table, q);
        tab.ptr[q] = g;
    }
    if (total == 0) return MICS_OK;
    int bad_a = 0, bad_b = 0;
    if (int ov = regions_overlap(segs, n_segs, &bad_a, &bad_b))
        return ov < 0 ? fail(MICS_ERR_INVALID_ARG, "%s: out of host memory while checking %d segments", fn, n_segs)
                      : fail(MICS_ERR_INVALID_ARG, "%s: the accumulator regions of segments %d and %d overlap",
                             fn, bad_a, bad_b);

    // every tensor, whatever its alignment, shares the launch of its batch
    mics::Segment batch[mics::kMaxSegPerLaunch];
    int nb = 0;
    for (int t = 0; t <= n_segs; ++t) {
        const bool last = (t == n_segs);
        if (!last && segs[t].numel) {
            const mics_segment& sg = segs[t];
            batch[nb].numel = sg.numel; batch[nb].shard_elems = 0;
            batch[nb].src_offset = sg.src_offset; batch[nb].dst_offset = sg.dst_offset;
            ++nb;
        }
        if (nb == mics::kMaxSegPerLaunch || (last && nb)) {
            int err = mics::launch_reduce_coalesced(acc, tab, batch, nb, p, accumulate != 0, kind, stream);
            if (err) return hip_fail(fn, err);
            nb = 0;
        }
    }
    return MICS_OK;
}

}  // namespace

extern "C" {

int mics_reduce_scatter_accum_coalesced(float* acc, const uint16_t* const* grads_bf16,
                                        const mics_segment* segs, int n_segs, int p,
                                        int accumulate, void* stream)
{
    return reduce_scatter_accum_coalesced("mics_reduce_scatter_accum_coalesced", "grads_bf16", acc,
                                          (const void* const*)grads_bf16, segs, n_segs, p, accumulate, 0, stream);
}

int mics_reduce_scatter_accum_coalesced_typed(float* acc, const void* const* grads,
                                              const mics_segment* segs, int n_segs, int p,
                                              int accumulate, int grad_dtype, void* stream)
{
    const char* fn = "mics_reduce_scatter_accum_coalesced_typed";
    if (grad_dtype != MICS_DTYPE_BF16 && grad_dtype != MICS_DTYPE_F16 && grad_dtype != MICS_DTYPE_F32)
        return fail(MICS_ERR_UNSUPPORTED, "%s: grad_dtype = %d is not bf16, f16 or f32", fn, grad_dtype);
    return reduce_scatter_accum_coalesced(fn, "grads", acc, grads, segs, n_segs, p, accumulate, grad_dtype, stream);
}

}  // extern "C"

namespace {

int replica_average_adam_shard(const char* fn, const char* pname, float* master, float* exp_avg,
                               float* exp_avg_sq, uint16_t* param_bf16, bool f16,
                               const float* const* acc_copies, size_t count, int r, float scale, float lr,
                               float beta1, float beta2, float eps, float weight_decay, int step, void* stream)
{
    if (step < 1) return fail(MICS_ERR_INVALID_ARG, "%s: step = %d, must be >= 1", fn, step);
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))
        return fail(MICS_ERR_INVALID_ARG, "%s: beta1 = %g, beta2 = %g must lie in [0, 1)", fn,
                    (double)beta1, (double)beta2);
    if (r < 1 || r > MICS_MAX_GROUP)
        return fail(MICS_ERR_INVALID_ARG, "%s: r = %d not in [1, %d]", fn, r, MICS_MAX_GROUP);
    if (!acc_copies) return fail(MICS_ERR_INVALID_ARG, "%s: acc_copies is NULL", fn);
    if (count > SIZE_MAX / 4) return fail(MICS_ERR_INVALID_ARG, "%s: count overflows", fn);
    if (count == 0) return MICS_OK;
    if (!master || !exp_avg || !exp_avg_sq)
        return fail(MICS_ERR_INVALID_ARG, "%s: master, exp_avg and exp_avg_sq must be non-NULL", fn);
    const void* st[3] = {master, exp_avg, exp_avg_sq};
    const char* name[3] = {"master", "exp_avg", "exp_avg_sq"};
    for (int a = 0; a < 3; ++a) {
        if (!aligned(st[a], 4))
            return fail(MICS_ERR_ALIGNMENT, "%s: %s not aligned to 4 bytes", fn, name[a]);
        for (int b = a + 1; b < 3; ++b)
            if (overlaps(st[a], count * 4, st[b], count * 4))
                return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps %s", fn, name[a], name[b]);
        if (param_bf16 && overlaps(st[a], count * 4, param_bf16, count * 2))
            return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps %s", fn, pname, name[a]);
    }
    if (param_bf16 && !aligned(param_bf16, 2))
        return fail(MICS_ERR_ALIGNMENT, "%s: %s not aligned to 2 bytes", fn, pname);
    mics::PtrTable tab{};
    for (int c = 0; c < r; ++c) {
        const float* a = acc_copies[c];
        if (!a) return fail(MICS_ERR_INVALID_ARG, "%s: acc_copies[%d] is NULL", fn, c);
        if (!aligned(a, 4))
            return fail(MICS_ERR_ALIGNMENT, "%s: acc_copies[%d] not aligned to 4 bytes", fn, c);
        for (int b = 0; b < 3; ++b)
            if (overlaps(st[b], count * 4, a, count * 4))
                return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps acc_copies[%d]", fn, name[b], c);
        if (param_bf16 && overlaps(param_bf16, count * 2, a, count * 4))
            return fail(MICS_ERR_INVALID_ARG, "%s: %s overlaps acc_copies[%d]", fn, pname, c);
        tab.ptr[c] = a;
    }
    const mics::AdamScalars hp = adam_scalars(lr, beta1, beta2, eps, weight_decay, step);
    int err = mics::launch_avg_adam(master, exp_avg, exp_avg_sq, param_bf16, f16, tab, r, scale, count, hp,
                                    stream);
    return err ? hip_fail(fn, err) : MICS_OK;
}

}  // namespace

extern "C" {

int mics_replica_average_adam_shard(float* master, float* exp_avg, float* exp_avg_sq,
                                    uint16_t* param_bf16, const float* const* acc_copies,
                                    size_t count, int r, float scale, float lr, float beta1,
                                    float beta2, float eps, float weight_decay, int step,
                                    void* stream)
{
    return replica_average_adam_shard("mics_replica_average_adam_shard", "param_bf16", master, exp_avg, exp_avg_sq,
                                      param_bf16, false, acc_copies, count, r, scale, lr, beta1, beta2, eps,
                                      weight_decay, step, stream);
}

int mics_replica_average_adam_shard_typed(float* master, float* exp_avg, float* exp_avg_sq,
                                          void* param_out, int param_dtype,
                                          const float* const* acc_copies, size_t count, int r,
                                          float scale, float lr, float beta1, float beta2, float eps,
                                          float weight_decay, int step, void* stream)
{
    const char* fn = "mics_replica_average_adam_shard_typed";
    bool f16 = false;
    if (int rc = param_format(fn, param_dtype, &f16)) return rc;
    return replica_average_adam_shard(fn, "param_out", master, exp_avg, exp_avg_sq, (uint16_t*)param_out, f16,
                                      acc_copies, count, r, scale, lr, beta1, beta2, eps, weight_decay, step,
                                      stream);
}

}  // extern "C"
