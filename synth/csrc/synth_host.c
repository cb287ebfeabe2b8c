/* Host twin of the synthetic input generator -- see synth_common.h.
 * Build: gcc -O2 -std=c11 -fopenmp -shared -fPIC */
#include "synth_common.h"
#include <stddef.h>

/* out[i] = table[slot(x0+i)] (or outlier_table[...] when the auxiliary word is
 * below outlier_threshold), i in [0, n).  elem_bytes is 2 or 4.  Returns 0, or
 * -1 on bad arguments. */
int synth_fill_host(void* out, uint64_t x0, size_t n, uint64_t key,
                    const void* table, const void* outlier_table,
                    uint32_t outlier_threshold, int elem_bytes, int threads)
{
    if ((elem_bytes != 2 && elem_bytes != 4) || (n && (!out || !table))) return -1;
    if (threads < 1) threads = 1;
    if (!outlier_table) outlier_threshold = 0;
    if (elem_bytes == 2) {
        uint16_t* o = (uint16_t*)out;
        const uint16_t* t0 = (const uint16_t*)table;
        const uint16_t* t1 = (const uint16_t*)outlier_table;
#pragma omp parallel for schedule(static) num_threads(threads)
        for (size_t i = 0; i < n; ++i) {
            uint64_t h = synth_word(key, x0 + i);
            o[i] = (synth_aux(h) < outlier_threshold ? t1 : t0)[synth_slot(h)];
        }
    } else {
        uint32_t* o = (uint32_t*)out;
        const uint32_t* t0 = (const uint32_t*)table;
        const uint32_t* t1 = (const uint32_t*)outlier_table;
#pragma omp parallel for schedule(static) num_threads(threads)
        for (size_t i = 0; i < n; ++i) {
            uint64_t h = synth_word(key, x0 + i);
            o[i] = (synth_aux(h) < outlier_threshold ? t1 : t0)[synth_slot(h)];
        }
    }
    return 0;
}
