/* Device twin of the synthetic input generator -- see synth_common.h.
 * Build: hipcc --offload-arch=gfx950 -O3 -shared -fPIC */
#include <hip/hip_runtime.h>
#include <stddef.h>
#include "synth_common.h"

template <typename E>
__global__ __launch_bounds__(256) void synth_fill_kernel(
    E* __restrict__ out, uint64_t x0, size_t n, uint64_t key,
    const E* __restrict__ table, const E* __restrict__ outlier_table,
    uint32_t outlier_threshold)
{
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t h = synth_word(key, x0 + i);
        const E* t = synth_aux(h) < outlier_threshold ? outlier_table : table;
        out[i] = t[synth_slot(h)];
    }
}

/* Device pointers: out, table, outlier_table (may be NULL).  Enqueues on
 * `stream` and returns without waiting.  Returns 0, -1 on bad arguments,
 * -2 when the launch failed. */
extern "C" int synth_fill_device(void* out, uint64_t x0, size_t n, uint64_t key,
                                 const void* table, const void* outlier_table,
                                 uint32_t outlier_threshold, int elem_bytes,
                                 void* stream)
{
    if ((elem_bytes != 2 && elem_bytes != 4) || (n && (!out || !table))) return -1;
    if (n == 0) return 0;
    if (!outlier_table) outlier_threshold = 0;
    size_t want = (n + 255) / 256;
    unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
    hipStream_t st = (hipStream_t)stream;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(synth_fill_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                           (uint16_t*)out, x0, n, key, (const uint16_t*)table,
                           (const uint16_t*)outlier_table, outlier_threshold);
    else
        hipLaunchKernelGGL(synth_fill_kernel<uint32_t>, dim3(blocks), dim3(256), 0, st,
                           (uint32_t*)out, x0, n, key, (const uint32_t*)table,
                           (const uint32_t*)outlier_table, outlier_threshold);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}
