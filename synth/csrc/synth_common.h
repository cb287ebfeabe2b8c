/*
 * Seeded, index-addressable synthetic input generator (host and device twins).
 *
 * Holds none of the method's arithmetic: a value is a table entry chosen by an
 * integer hash of (stream key, element index).  The tables (65,536 quantised
 * normal values, already in the element's storage format) are built by the
 * Python side.  Because only integer operations happen here, the host twin
 * (synth_host.c) and the device twin (synth_dev.hip) produce identical bytes.
 */
#ifndef SYNTH_COMMON_H
#define SYNTH_COMMON_H
#include <stdint.h>

#if defined(__HIPCC__)
#define SYNTH_FN static __host__ __device__ inline
#else
#define SYNTH_FN static inline
#endif

/* 64-bit finaliser (Stafford variant 13, as used by splitmix64; public domain). */
SYNTH_FN uint64_t synth_mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* Hash word of element x in the stream `key`. */
SYNTH_FN uint64_t synth_word(uint64_t key, uint64_t x)
{
    return synth_mix64(key + (x + 1) * 0x9E3779B97F4A7C15ull);
}

/* Table slot (top 16 bits) and the independent 32-bit word that decides
 * whether the element is drawn from the outlier table. */
SYNTH_FN uint32_t synth_slot(uint64_t h) { return (uint32_t)(h >> 48); }
SYNTH_FN uint32_t synth_aux(uint64_t h) { return (uint32_t)(h >> 16); }

#endif
