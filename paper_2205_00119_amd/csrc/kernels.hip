// gfx950 kernels of libmics and their launchers.
//
// All four steps stream every byte once and do at most a few operations per
// element, so they are bound by HBM bandwidth, not by the matrix or vector
// units.  The kernels therefore aim at: 128-bit global loads and stores that
// cover contiguous memory per wavefront instruction, all of a lane's loads in
// flight before the first use, no re-reads, and grids with one pass per lane:
// workgroups are dispatched in index order, so the lanes in flight cover a
// compact window of every buffer that advances through memory (measured on
// MI355X: a lane that owns several vectors a grid stride apart, or a small
// persistent grid, loses 5-30 % of the bandwidth, stores most of all).
//
// Alignment.  gfx950 executes a 128-bit global access at any address.  Measured on MI355X
// (p = 16 reduce, 50 M and 200 M elements): accesses that are only 4-byte aligned run at the
// speed of 16-byte aligned ones; 2-byte aligned ones lose about 20 %.  So the element-wise
// kernels use 128-bit accesses on under-aligned vector types everywhere, a lane that would
// cross the end of a buffer works element by element inside the same kernel (no tail
// launches), and only the bf16/fp16 gradient pointers are rounded down to 4 bytes first.
//
// Arithmetic rules (they make the results reproducible bit for bit):
//   - no fused multiply-add (-ffp-contract=off and the pragma below),
//   - sums in the order the header states,
//   - correctly rounded fp32 division and square root,
//   - fp32 denormals are kept.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "internal.h"

#pragma clang fp contract(off)

namespace mics {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// The same vectors at the alignment of their elements (see "Alignment" above).
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));
typedef uint32_t u32_a2 __attribute__((aligned(2)));
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));
typedef f32x2 f32x2_a4 __attribute__((aligned(4)));

// Launch shape and cache hints per kernel family; the defaults are the measured best on
// MI355X for the h = 8192, p = 16 shard shapes.  *_BLOCK = workgroup size, *_BPC = cap on
// workgroups per compute unit (the grid covers the data with one pass per lane unless the
// cap is reached; lanes stride over the rest), *_NTL / *_NTS = non-temporal loads / stores.
#ifndef MICS_REORDER_BLOCK
#define MICS_REORDER_BLOCK 64
#endif
#ifndef MICS_REORDER_BPC
#define MICS_REORDER_BPC 4096
#endif
#ifndef MICS_REORDER_NTL
#define MICS_REORDER_NTL 1
#endif
#ifndef MICS_REORDER_NTS
#define MICS_REORDER_NTS 1
#endif
#ifndef MICS_RSA_BLOCK
#define MICS_RSA_BLOCK 64
#endif
#ifndef MICS_RSA_UNALIGNED_BLOCK
#define MICS_RSA_UNALIGNED_BLOCK 512     // accumulator or gradients off 16 bytes: 6070 against 5740 with 64
#endif
#ifndef MICS_RSA_WAVES
#define MICS_RSA_WAVES 10
#endif
#ifndef MICS_RSA_WAVES_STREAMED
#define MICS_RSA_WAVES_STREAMED 4
#endif
#ifndef MICS_RSA_STREAM_FROM_P
#define MICS_RSA_STREAM_FROM_P 32
#endif
#ifndef MICS_RSA_BPC
#define MICS_RSA_BPC 4096
#endif
#ifndef MICS_RSA_NTL
#define MICS_RSA_NTL 1
#endif
#ifndef MICS_RSA_BATCH
#define MICS_RSA_BATCH 16
#endif
#ifndef MICS_AVG_BLOCK
#define MICS_AVG_BLOCK 64
#endif
#ifndef MICS_AVG_WAVES
#define MICS_AVG_WAVES 12
#endif
#ifndef MICS_AVG_WAVES_STREAMED
#define MICS_AVG_WAVES_STREAMED 10
#endif
#ifndef MICS_AVG_BPC
#define MICS_AVG_BPC 4096
#endif
#ifndef MICS_AVG_NTL
#define MICS_AVG_NTL 1
#endif
#ifndef MICS_ADAM_BLOCK
#define MICS_ADAM_BLOCK 64
#endif
#ifndef MICS_ADAM_WAVES
#define MICS_ADAM_WAVES 12
#endif
#ifndef MICS_ADAM_WAVES_STREAMED
#define MICS_ADAM_WAVES_STREAMED 9
#endif
#ifndef MICS_FUSED_BLOCK
#define MICS_FUSED_BLOCK 64
#endif
#ifndef MICS_FUSED_WAVES
#define MICS_FUSED_WAVES 6
#endif
#ifndef MICS_FUSED_WAVES_STREAMED
#define MICS_FUSED_WAVES_STREAMED 5
#endif
#ifndef MICS_FUSED_COPIES_FIRST
#define MICS_FUSED_COPIES_FIRST 1
#endif
#ifndef MICS_FUSED_NTL_COPIES
#define MICS_FUSED_NTL_COPIES MICS_ADAM_NTL
#endif
#ifndef MICS_ADAM_BPC
#define MICS_ADAM_BPC 4096
#endif
#ifndef MICS_ADAM_NTL
#define MICS_ADAM_NTL 1
#endif
#ifndef MICS_ADAM_NTS
#define MICS_ADAM_NTS 1
#endif
// Small messages on large groups (see rsa_kernel): workgroup size of the one-dword-per-lane
// variant, the loads it keeps in flight, and the largest call (p * count buffer elements)
// and smallest group it is used for.  Measured per launch, 1 MB .. 256 MB of gradient per rank:
// for p = 64 / 128 the variant wins up to 64 MB (1 MB: 7.0 / 11.9 us against 9.5 / 17.6 us for
// the 128-bit kernel in single-wavefront workgroups, 12.5 / 20.6 us before either existed) and
// loses from 128 MB on; for p <= 32 the 128-bit kernel is as fast or faster at every size.
#ifndef MICS_NARROW_BLOCK
#define MICS_NARROW_BLOCK 64
#endif
#ifndef MICS_NARROW_BATCH
#define MICS_NARROW_BATCH 64
#endif
#ifndef MICS_NARROW_MAX_ELEMS
#define MICS_NARROW_MAX_ELEMS (34u << 20)
#endif
#ifndef MICS_NARROW_MIN_P
#define MICS_NARROW_MIN_P 40
#endif

constexpr int kMaxBlock = 512;           // most lanes per workgroup of the element-wise kernels
constexpr int kNarrowBlock = MICS_NARROW_BLOCK;
constexpr bool kReorderNtl = MICS_REORDER_NTL, kReorderNts = MICS_REORDER_NTS;
constexpr bool kRsaNtl = MICS_RSA_NTL;   // gradient loads; the accumulator's hint is chosen per launch
constexpr bool kAvgNtl = MICS_AVG_NTL;   // input loads; the output's hint is chosen per launch
constexpr bool kAdamNtl = MICS_ADAM_NTL, kAdamNts = MICS_ADAM_NTS;

// Compile-time sized pointer table for the unrolled kernels (keeps the
// kernel-argument segment small); the launcher copies out of PtrTable.
template <int N>
struct SmallTable {
    const void* ptr[N];
};

// Load / store through a pointer whose pointee type carries the alignment (macros, not function
// templates: a template parameter would drop the typedef's alignment and promise 16 bytes).
// NT selects the non-temporal form; it is a compile-time constant wherever these are used.
#define MICS_LD(NT, ptr) ((NT) ? __builtin_nontemporal_load(ptr) : *(ptr))
#define MICS_ST(NT, ptr, val) \
    do { if (NT) __builtin_nontemporal_store((val), (ptr)); else *(ptr) = (val); } while (0)

// N consecutive floats at a 4-byte aligned address, as one access.
template <int N, bool NT>
__device__ __forceinline__ void ld_f32(float (&a)[N], const float* p)
{
    static_assert(N == 1 || N == 2 || N == 4 || N == 8, "");
    if constexpr (N == 1) {
        a[0] = MICS_LD(NT, p);
    } else if constexpr (N == 2) {
        const f32x2 t = MICS_LD(NT, (const f32x2_a4*)p);
        a[0] = t.x; a[1] = t.y;
    } else {
        #pragma unroll
        for (int h = 0; h < N / 4; ++h) {
            const f32x4 t = MICS_LD(NT, (const f32x4_a4*)p + h);
            a[4 * h] = t.x; a[4 * h + 1] = t.y; a[4 * h + 2] = t.z; a[4 * h + 3] = t.w;
        }
    }
}

template <int N, bool NT>
__device__ __forceinline__ void st_f32(float* p, const float (&a)[N])
{
    if constexpr (N == 1) {
        MICS_ST(NT, p, a[0]);
    } else if constexpr (N == 2) {
        const f32x2 t = {a[0], a[1]};
        MICS_ST(NT, (f32x2_a4*)p, t);
    } else {
        #pragma unroll
        for (int h = 0; h < N / 4; ++h) {
            const f32x4 t = {a[4 * h], a[4 * h + 1], a[4 * h + 2], a[4 * h + 3]};
            MICS_ST(NT, (f32x4_a4*)p + h, t);
        }
    }
}

// fp32 -> bf16, round to nearest even, two at a time (gfx950 converts a pair
// in one instruction).  Low half = a, high half = b.
__device__ __forceinline__ uint32_t bf16_pack(float a, float b)
{
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ uint16_t bf16_single(float a)
{
    __bf16 h = (__bf16)a;
    return __builtin_bit_cast(uint16_t, h);
}

// fp32 -> IEEE binary16, round to nearest even, subnormals kept, overflow to Inf.
__device__ __forceinline__ uint16_t f16_single(float a)
{
    _Float16 h = (_Float16)a;
    return __builtin_bit_cast(uint16_t, h);
}

// Low-precision copy of the parameters that the Adam kernels write next to the fp32 master.
enum { kParamNone = 0, kParamBf16 = 1, kParamF16 = 2 };

template <int OUT>
__device__ __forceinline__ uint32_t param_pack(float a, float b)
{
    if constexpr (OUT == kParamBf16) return bf16_pack(a, b);
    else return (uint32_t)f16_single(a) | ((uint32_t)f16_single(b) << 16);
}
template <int OUT>
__device__ __forceinline__ uint16_t param_single(float a)
{
    if constexpr (OUT == kParamBf16) return bf16_single(a);
    else return f16_single(a);
}

// ---------------------------------------------------------------------------
// Step 1: chunk rearrangement of the hierarchical all-gather (Section 3.3).
// Chunk g of the result comes from slot g div k of the stage-1 buffer of local
// rank g mod k.  blockIdx.y = g, blockIdx.x strides over the chunk.
// ---------------------------------------------------------------------------

// All addresses and the shard size are multiples of 16 bytes: a remapped copy.
__global__ __launch_bounds__(kMaxBlock) void reorder_vec_kernel(
    u32x4* __restrict__ dst, PtrTable src, size_t shard_vecs, size_t n_valid_bytes, int k)
{
    const size_t g = blockIdx.y;
    const size_t chunk_begin = g * shard_vecs * 16;
    if (chunk_begin >= n_valid_bytes) return;
    size_t valid = n_valid_bytes - chunk_begin;
    if (valid > shard_vecs * 16) valid = shard_vecs * 16;
    const size_t nfull = valid / 16;
    const size_t j = g / (size_t)k, l = g % (size_t)k;
    const u32x4* __restrict__ s = (const u32x4*)src.ptr[l] + j * shard_vecs;
    u32x4* __restrict__ d = dst + g * shard_vecs;

    // One vector per lane and pass.  Workgroups are dispatched in blockIdx order, so the lanes
    // in flight cover one compact, advancing window of the source and of the destination; a
    // lane that strides far ahead (several loads a grid stride apart) measurably lowers the
    // achieved bandwidth, for loads and even more for stores.
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nfull; i += stride)
        MICS_ST(kReorderNts, d + i, MICS_LD(kReorderNtl, s + i));

    // ragged end of the logical buffer: fewer than 16 valid bytes remain
    const size_t tail_halves = (valid - nfull * 16) / 2;
    if (blockIdx.x == 0 && threadIdx.x < tail_halves) {
        const uint16_t* sh = (const uint16_t*)(s + nfull);
        uint16_t* dh = (uint16_t*)(d + nfull);
        dh[threadIdx.x] = sh[threadIdx.x];
    }
}

// Coalesced form (many separately sharded tensors in one launch, all 16-byte aligned):
// blockIdx.y = chunk g, blockIdx.x = tile x - tile_begin[t] of tensor t's chunk.  A tile is
// MICS_SEG_U runs of blockDim.x vectors: the table look-up in every wavefront's prologue has to
// be paid for by two vectors per lane (one: -15 %), more spreads the window (four: -3 %).
// Measured on the h = 8192 layer with two vectors per lane (GB/s): 64 lanes 6375, 128: 6340,
// 256: 6200, 512: 5950.  A small chunk (a bias of h/p elements) costs one workgroup.
#ifndef MICS_SEG_BLOCK
#define MICS_SEG_BLOCK 64
#endif
constexpr int kSegLanes = MICS_SEG_BLOCK;
#ifndef MICS_SEG_U
#define MICS_SEG_U 2
#endif
constexpr int kMaxSeg = kMaxSegPerLaunch;

// Index of the segment whose tile range holds workgroup x (x < 2^31 - 1): tile_begin is
// ascending, unused entries hold kNoTile.  Counting instead of walking keeps the table reads
// independent of one another (a few wide scalar loads), which matters for workgroups that move
// only a few KiB.  The count is written as integer arithmetic on the sign bit so that it stays
// on the scalar unit: as a sum of comparisons it was compiled into some 300 vector
// instructions per wavefront (-18 % on a layer of 16 unaligned tensors).  Counting only the
// entries in use would need the entry count first, and that dependent load costs more than
// the additions it saves (h = 8192 layer: 6.25 against 6.45 TB/s).
constexpr unsigned kNoTile = 0x7FFFFFFFu;
__device__ __forceinline__ int segment_of(const unsigned (&tile_begin)[kMaxSeg + 1], unsigned x)
{
    unsigned t = 0;
    #pragma unroll
    for (int i = 1; i < kMaxSeg; ++i) t += (tile_begin[i] - 1u - x) >> 31;      // 1 iff tile_begin[i] <= x
    return (int)t;
}
struct ReorderSeg {
    unsigned long long shard_vecs, valid_bytes, src_vec, dst_vec;
};
struct ReorderSegTable {
    int n;
    unsigned tile_begin[kMaxSeg + 1];
    ReorderSeg seg[kMaxSeg];
};

__global__ __launch_bounds__(kMaxBlock) void reorder_seg_kernel(
    u32x4* __restrict__ dst, PtrTable src, ReorderSegTable tab, int k)
{
    const unsigned x = blockIdx.x;
    const int t = segment_of(tab.tile_begin, x);
    const size_t shard_vecs = tab.seg[t].shard_vecs, valid_bytes = tab.seg[t].valid_bytes;
    const size_t g = blockIdx.y;
    const size_t chunk_begin = g * shard_vecs * 16;
    if (chunk_begin >= valid_bytes) return;
    size_t valid = valid_bytes - chunk_begin;
    if (valid > shard_vecs * 16) valid = shard_vecs * 16;
    const size_t nfull = valid / 16;
    const size_t j = g / (size_t)k, l = g % (size_t)k;
    const u32x4* __restrict__ s = (const u32x4*)src.ptr[l] + tab.seg[t].src_vec + j * shard_vecs;
    u32x4* __restrict__ d = dst + tab.seg[t].dst_vec + g * shard_vecs;
    const size_t tile_vecs = (size_t)blockDim.x * MICS_SEG_U;
    const size_t tile0 = (size_t)(x - tab.tile_begin[t]) * tile_vecs;
    u32x4 v[MICS_SEG_U];
    #pragma unroll
    for (int u = 0; u < MICS_SEG_U; ++u) {
        const size_t i = tile0 + (size_t)u * blockDim.x + threadIdx.x;
        if (i < nfull) v[u] = MICS_LD(kReorderNtl, s + i);
    }
    #pragma unroll
    for (int u = 0; u < MICS_SEG_U; ++u) {
        const size_t i = tile0 + (size_t)u * blockDim.x + threadIdx.x;
        if (i < nfull) MICS_ST(kReorderNts, d + i, v[u]);
    }
    // ragged end of the tensor: the tile that holds vector index nfull moves the last bytes
    const size_t tail_halves = (valid - nfull * 16) / 2;
    if (tail_halves && nfull / tile_vecs == x - tab.tile_begin[t] && threadIdx.x < tail_halves) {
        const uint16_t* sh = (const uint16_t*)(s + nfull);
        uint16_t* dh = (uint16_t*)(d + nfull);
        dh[threadIdx.x] = sh[threadIdx.x];
    }
}

// General case: source and destination of a chunk sit at different offsets
// within their 16-byte lines (odd shard sizes, sub-buffers that start anywhere
// on an element boundary).  Like reorder_seg_kernel the kernel serves many
// tensors per launch: workgroup x moves tile x - tile_begin[t] of chunk
// blockIdx.y of tensor t.
struct ByteSeg {
    unsigned long long shard_bytes, valid_bytes, src_byte, dst_byte;
};
// Where workgroup x works: many tensors (table in the kernel arguments) ...
struct ByteSegTable {
    int n;
    unsigned tile_begin[kMaxSeg + 1];
    ByteSeg seg[kMaxSeg];
    __device__ __forceinline__ const ByteSeg& locate(unsigned x, size_t* tile) const
    {
        const int t = segment_of(tile_begin, x);
        *tile = x - tile_begin[t];
        return seg[t];
    }
};
// ... or a single tensor: no table, no look-up (4 % faster than a table of one entry).
struct OneTensor {
    ByteSeg seg;
    __device__ __forceinline__ const ByteSeg& locate(unsigned x, size_t* tile) const
    {
        *tile = x;
        return seg;
    }
};

// Destination vectors are written aligned.  gfx950 executes a 128-bit load at any 4-byte
// aligned address at full speed, so a chunk whose source is a multiple of 4 bytes off its
// destination's 16-byte grid is a plain copy with under-aligned loads.  Otherwise (2 bytes off, odd shard sizes of
// 2-byte elements) a lane loads the 16 bytes from 2 bytes before its source -- 4-byte aligned --
// and takes the last 2 bytes it needs from the next lane's first dword through a lane shift;
// only the last lane of a wavefront (or of the chunk) loads those 2 bytes itself.  The phase
// is the same for every vector of a chunk, so the branches are workgroup-uniform.  Partial
// vectors at the two ends of a chunk go in 2-byte units on lanes 0 .. 15 of the chunk's first
// workgroup.  Global memory is touched only inside the chunk.  (An earlier form staged every
// tile in LDS and rebuilt the vectors from two LDS reads: 5.2 TB/s on the layer with odd shards
// where this one reaches 5.8, and 4.6 against 5.0 with 16 tensors per launch.)
#ifndef MICS_SHIFT_U
#define MICS_SHIFT_U 2
#endif
#ifndef MICS_SHIFT_BLOCK
#define MICS_SHIFT_BLOCK 256     // 64 lanes: 5.40 TB/s, 128 .. 512: 5.76 .. 5.84
#endif
#ifndef MICS_SHIFT_NTL
#define MICS_SHIFT_NTL 1
#endif
template <typename Where>
__global__ __launch_bounds__(kMaxBlock) void reorder_shift_kernel(
    unsigned char* __restrict__ dst, PtrTable src, Where where, int k)
{
    size_t tile;
    const ByteSeg& sg = where.locate(blockIdx.x, &tile);
    const size_t shard_bytes = sg.shard_bytes, n_valid_bytes = sg.valid_bytes;
    const size_t g = blockIdx.y;
    const size_t chunk_begin = g * shard_bytes;
    if (chunk_begin >= n_valid_bytes) return;
    size_t valid = n_valid_bytes - chunk_begin;
    if (valid > shard_bytes) valid = shard_bytes;
    const size_t j = g / (size_t)k, l = g % (size_t)k;

    const uintptr_t d_lo = (uintptr_t)dst + sg.dst_byte + chunk_begin;      // chunk in dst
    const uintptr_t d_hi = d_lo + valid;
    const uintptr_t s_chunk = (uintptr_t)src.ptr[l] + sg.src_byte + j * shard_bytes;
    const uintptr_t a_lo = (d_lo + 15) & ~(uintptr_t)15;                    // first full dst vector
    const size_t nfull = a_lo + 16 <= d_hi ? ((d_hi & ~(uintptr_t)15) - a_lo) / 16 : 0;

    if (tile == 0 && threadIdx.x < 16) {
        const uintptr_t head_end = a_lo < d_hi ? a_lo : d_hi;
        const uintptr_t b = threadIdx.x < 8 ? d_lo + 2 * threadIdx.x
                                            : a_lo + nfull * 16 + 2 * (threadIdx.x - 8);
        const bool on = threadIdx.x < 8 ? b < head_end : (b >= head_end && b < d_hi);
        if (on) *(uint16_t*)b = *(const uint16_t*)(s_chunk + (b - d_lo));
    }
    const size_t i0 = tile * ((size_t)blockDim.x * MICS_SHIFT_U);
    if (i0 >= nfull) return;                                                // workgroup-uniform
    const uintptr_t s_lo = s_chunk + (a_lo - d_lo);                         // source of full vector 0
    const bool odd = (s_lo & 2) != 0;                                       // chunk-uniform

    #pragma unroll
    for (int u = 0; u < MICS_SHIFT_U; ++u) {
        const size_t i = i0 + (size_t)u * blockDim.x + threadIdx.x;
        const bool has = i < nfull;
        const uintptr_t s = s_lo + 16 * i;
        u32x4 out = {0, 0, 0, 0};
        if (!odd) {
            if (has) out = MICS_LD(MICS_SHIFT_NTL, (const u32x4_a4*)s);
        } else {
            // vector 0 of a chunk whose destination starts on a 16-byte line has nothing in
            // front of it inside the chunk: that one lane loads from its 2-byte aligned source
            const bool direct = s - 2 < s_chunk;
            u32x4 w = {0, 0, 0, 0};
            if (has) {
                if (direct) w = MICS_LD(MICS_SHIFT_NTL, (const u32x4_a2*)s);
                else w = MICS_LD(MICS_SHIFT_NTL, (const u32x4_a4*)(s - 2));
            }
            uint32_t next = (uint32_t)__shfl_down((int)w.x, 1);             // every lane takes part
            if (has && ((threadIdx.x & 63u) == 63u || i + 1 >= nfull)) next = *(const uint16_t*)(s + 14);
            if (direct) {
                out = w;
            } else {
                out.x = (w.x >> 16) | (w.y << 16);
                out.y = (w.y >> 16) | (w.z << 16);
                out.z = (w.z >> 16) | (w.w << 16);
                out.w = (w.w >> 16) | (next << 16);
            }
        }
        if (has) MICS_ST(kReorderNts, (u32x4*)(a_lo + 16 * i), out);
    }
}

// ---------------------------------------------------------------------------
// Step 2a: reduction of the partition-group reduce-scatter, accumulated over
// micro-steps (Section 3.4).
//
// Gradient formats (KIND): 0 = bf16, 1 = IEEE binary16 (what mixed precision means on GPUs
// without bf16), 2 = binary32 (plain float32 training).  Widening to binary32 is exact.
//
// One kernel for every alignment.  The kernel works in a "virtual" element index space in
// which element e of every (rounded-down) gradient pointer sits at a 4-byte aligned address
// whenever e is a multiple of the lane's element count; the call's elements are the virtual
// range [lead, lead + count), lead = 0 or 1 (1 when the bf16/fp16 pointers had to be rounded
// down by one element).  A lane owns the virtual elements [EPL*i, EPL*i + EPL): one load per
// rank buffer, one load and one store of the accumulator (which is then 4-byte aligned at
// worst).  A lane whose elements are not all inside the range -- at most the first and the
// last one -- adds its elements one by one.
//
// VEC = dwords per load: 4 for bandwidth (8 bf16/fp16 or 4 fp32 elements per lane); 1 for
// small messages on large groups, where the time is the launch plus the serial chain of
// load round trips of one lane: one dword per buffer and lane spreads a 1 MB message over
// 32 compute units instead of 1 and lets a lane keep 64 loads in flight, so p = 128 needs
// two round trips.
// ---------------------------------------------------------------------------

template <int KIND> struct GradFormat {
    static constexpr int kElemBytes = KIND == 2 ? 4 : 2;
    static constexpr int kPerDword = KIND == 2 ? 1 : 2;
};

template <int KIND>
__device__ __forceinline__ void widen_dword(float* out, uint32_t w)
{
    if constexpr (KIND == 0) {          // the bf16 bits are the upper half of the fp32 bits
        out[0] = __uint_as_float(w << 16);
        out[1] = __uint_as_float(w & 0xFFFF0000u);
    } else if constexpr (KIND == 1) {
        out[0] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu));
        out[1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    } else {
        out[0] = __uint_as_float(w);
    }
}

template <int KIND>
__device__ __forceinline__ float widen_one(const void* buf, size_t x)
{
    if constexpr (KIND == 0) return __uint_as_float((uint32_t)((const uint16_t*)buf)[x] << 16);
    else if constexpr (KIND == 1) return (float)((const _Float16*)buf)[x];
    else return ((const float*)buf)[x];
}

template <int KIND, int VEC> struct GradVec;      // the registers of one load
template <int KIND> struct GradVec<KIND, 4> {
    u32x4 v;
    __device__ __forceinline__ void load(const void* base, size_t elem)
    {
        const char* a = (const char*)base + elem * GradFormat<KIND>::kElemBytes;
        if constexpr (KIND == 2) v = MICS_LD(kRsaNtl, (const u32x4_a4*)a);
        else v = MICS_LD(kRsaNtl, (const u32x4_a2*)a);
    }
    __device__ __forceinline__ uint32_t dword(int d) const { return v[d]; }
};
template <int KIND> struct GradVec<KIND, 1> {
    uint32_t v;
    __device__ __forceinline__ void load(const void* base, size_t elem)
    {
        const char* a = (const char*)base + elem * GradFormat<KIND>::kElemBytes;
        if constexpr (KIND == 2) v = MICS_LD(kRsaNtl, (const uint32_t*)a);
        else v = MICS_LD(kRsaNtl, (const u32_a2*)a);
    }
    __device__ __forceinline__ uint32_t dword(int) const { return v; }
};

template <int KIND, int VEC, bool FIRST>
__device__ __forceinline__ void rsa_add(float* s, const GradVec<KIND, VEC>& v)
{
    constexpr int PD = GradFormat<KIND>::kPerDword;
    #pragma unroll
    for (int d = 0; d < VEC; ++d) {
        float w[PD];
        widen_dword<KIND>(w, v.dword(d));
        #pragma unroll
        for (int e = 0; e < PD; ++e) {
            if constexpr (FIRST) s[PD * d + e] = w[e];
            else s[PD * d + e] = s[PD * d + e] + w[e];
        }
    }
}

// s = ((g_0 + g_1) + ...) + g_{p-1} for the lane's elements starting at virtual element `elem`.
// P > 0: p = P at compile time; P == 0: any p.  The loads go out in batches of BATCH, every
// batch entirely in flight before its first addition (P <= BATCH: all of them at once; a
// batch of 32 128-bit loads would leave room for 3 wavefronts per SIMD only).
template <int KIND, int VEC, int P, int BATCH, typename Tab>
__device__ __forceinline__ void rsa_partial(float* s, const Tab& g, int p, size_t elem)
{
    if constexpr (P > 0) {
        #pragma unroll
        for (int q0 = 0; q0 < P; q0 += BATCH) {
            GradVec<KIND, VEC> v[BATCH];
            #pragma unroll
            for (int b = 0; b < BATCH; ++b)
                if (q0 + b < P) v[b].load(g.ptr[q0 + b], elem);
            #pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                if (q0 + b < P) {
                    if (q0 + b == 0) rsa_add<KIND, VEC, true>(s, v[b]);
                    else rsa_add<KIND, VEC, false>(s, v[b]);
                }
            }
        }
    } else {
        {
            GradVec<KIND, VEC> first;
            first.load(g.ptr[0], elem);
            rsa_add<KIND, VEC, true>(s, first);
        }
        for (int q0 = 1; q0 < p; q0 += BATCH) {
            GradVec<KIND, VEC> v[BATCH];
            #pragma unroll
            for (int b = 0; b < BATCH; ++b)
                if (q0 + b < p) v[b].load(g.ptr[q0 + b], elem);
            #pragma unroll
            for (int b = 0; b < BATCH; ++b)
                if (q0 + b < p) rsa_add<KIND, VEC, false>(s, v[b]);
        }
    }
}

// a[0 .. EPL) = (ACCUM ? acc_e[0 .. EPL) : +0) + partial sum at virtual element `elem`.
// SA ("stream the accumulator"): non-temporal accumulator loads and stores.  An accumulator
// that fits the 256 MB Infinity Cache is best left cacheable -- its stores are absorbed there
// and the next micro-step finds it again (plain/plain 6.3 TB/s, NT/NT 6.1 at S = 50 M) -- while
// a larger one is best streamed past the caches (NT/NT 5.8 TB/s, plain/plain 5.4, and the
// mixed NT-load/plain-store 5.1 at S = 200 M); the launcher picks by size.
template <int KIND, int VEC, int P, int BATCH, bool ACCUM, bool SA, typename Tab>
__device__ __forceinline__ void rsa_sum(float (&a)[VEC * GradFormat<KIND>::kPerDword], const float* acc_e,
                                        const Tab& g, int p, size_t elem)
{
    constexpr int EPL = VEC * GradFormat<KIND>::kPerDword;
    #pragma unroll
    for (int e = 0; e < EPL; ++e) a[e] = 0.0f;
    if (ACCUM) ld_f32<EPL, SA>(a, acc_e);          // issued before the gradient loads are consumed
    float s[EPL];
    rsa_partial<KIND, VEC, P, BATCH>(s, g, p, elem);
    #pragma unroll
    for (int e = 0; e < EPL; ++e) a[e] = a[e] + s[e];
}

// One element, the p loads in flight 16 at a time (a lane that waited for each of 128 loads in
// turn would hold up a small call for tens of microseconds).
template <int KIND, bool ACCUM, typename Tab>
__device__ __forceinline__ void rsa_element(float* acc_e, const Tab& g, int p, size_t elem)
{
    constexpr int B = 16;
    float partial = widen_one<KIND>(g.ptr[0], elem);
    for (int q0 = 1; q0 < p; q0 += B) {
        float w[B];
        #pragma unroll
        for (int b = 0; b < B; ++b)
            if (q0 + b < p) w[b] = widen_one<KIND>(g.ptr[q0 + b], elem);
        #pragma unroll
        for (int b = 0; b < B; ++b)
            if (q0 + b < p) partial = partial + w[b];
    }
    *acc_e = (ACCUM ? *acc_e : 0.0f) + partial;
}

// The lane's virtual elements [v0, v0 + EPL) of a call (or segment) whose elements are the
// virtual range [lead, end): `acc` is the accumulator address of virtual element `lead`, and
// virtual element e sits at element src0 + e of every rank buffer.  Consecutive lanes of a
// wavefront hold consecutive v0, and every lane of the wavefront gets here (lanes past `end`
// find nothing to do).  A lane whose elements are not all inside the range does nothing:
// those elements -- fewer than EPL at either end -- are rsa_edges' work.
//
// Streamed accumulators of 8-element lanes are stored through LDS: a lane's two 128-bit
// stores are 32 bytes apart, so each store instruction of the wavefront would fill every
// other 16 bytes of its cache lines, and with non-temporal stores about one line in ten left
// the L2 between the two halves (WRITE_SIZE 1.10 x the accumulator's bytes at 800 M elements).
// Passing the results through 2 KiB of LDS per wavefront lets every store instruction cover
// one contiguous KiB.  Only wavefronts whose 64 lanes all hold full vectors take this path.
template <int KIND, int VEC, int P, int BATCH, bool ACCUM, bool SA, typename Tab>
__device__ __forceinline__ void rsa_lane(float* acc, const Tab& g, int p, size_t src0, size_t v0,
                                         size_t lead, size_t end)
{
    constexpr int EPL = VEC * GradFormat<KIND>::kPerDword;
    const bool full = v0 >= lead && v0 + EPL <= end;
    if constexpr (SA && EPL == 8) {
        if (__builtin_amdgcn_ballot_w64(full) == ~0ull) {       // wavefront-uniform
            extern __shared__ f32x4 stage[];                     // blockDim.x * 2 vectors (launcher)
            const unsigned lane = threadIdx.x & 63u;
            f32x4* mine = stage + (threadIdx.x - lane) * 2;      // this wavefront's 128 vectors
            float* acc_e = acc + (v0 - lead);
            float a[EPL];
            rsa_sum<KIND, VEC, P, BATCH, ACCUM, SA>(a, acc_e, g, p, src0 + v0);
            mine[2 * lane] = f32x4{a[0], a[1], a[2], a[3]};
            mine[2 * lane + 1] = f32x4{a[4], a[5], a[6], a[7]};
            // LDS operations of one wavefront complete in order: no barrier between these
            const f32x4 r0 = mine[lane], r1 = mine[64 + lane];
            f32x4_a4* wave_base = (f32x4_a4*)(acc_e - 8 * lane);
            MICS_ST(true, wave_base + lane, r0);
            MICS_ST(true, wave_base + 64 + lane, r1);
            return;
        }
    }
    if (full) {
        float* acc_e = acc + (v0 - lead);
        float a[EPL];
        rsa_sum<KIND, VEC, P, BATCH, ACCUM, SA>(a, acc_e, g, p, src0 + v0);
        st_f32<EPL, SA>(acc_e, a);
    }
}

// The elements that no lane holds as a full vector: virtual [lead, head) with head = lead
// rounded up to EPL (or `end`), and [tail, end) with tail = `end` rounded down to EPL (or
// head).  One element per lane, lanes 0 .. 2*EPL-1 of the calling workgroup.
template <int KIND, int EPL, bool ACCUM, typename Tab>
__device__ __forceinline__ void rsa_edges(float* acc, const Tab& g, int p, size_t src0, size_t lead, size_t end)
{
    if (threadIdx.x >= 2 * EPL) return;
    size_t head = (lead + EPL - 1) / EPL * EPL;
    if (head > end) head = end;
    size_t tail = end / EPL * EPL;
    if (tail < head) tail = head;
    const size_t e = threadIdx.x < EPL ? lead + threadIdx.x : tail + (threadIdx.x - EPL);
    const size_t stop = threadIdx.x < EPL ? head : end;
    if (e < stop) rsa_element<KIND, ACCUM>(acc + (e - lead), g, p, src0 + e);
}

// Workgroups of blockDim.x lanes (64 .. 512 for VEC = 4: the launcher takes small ones for
// calls that would otherwise occupy a fraction of the compute units), plus one more workgroup
// for the edge elements, so that their load chains run beside the vector work.
template <int KIND, int VEC, int P, bool ACCUM, bool SA, typename Tab>
__global__ __launch_bounds__(VEC == 4 ? kMaxBlock : kNarrowBlock) void rsa_kernel(
    float* __restrict__ acc, Tab g, int p, unsigned lead, size_t count)
{
    constexpr int BATCH = VEC == 4 ? MICS_RSA_BATCH : MICS_NARROW_BATCH;
    constexpr int EPL = VEC * GradFormat<KIND>::kPerDword;
    const size_t end = (size_t)lead + count;
    const size_t nlanes = (end + EPL - 1) / EPL;
    const size_t block = blockDim.x;
    // the last workgroup of the grid does nothing but the edge elements
    if (blockIdx.x == gridDim.x - 1) {
        rsa_edges<KIND, EPL, ACCUM>(acc, g, p, 0, lead, end);
        return;
    }
    const size_t stride = (size_t)(gridDim.x - 1) * block;
    for (size_t base = (size_t)blockIdx.x * block; base < nlanes; base += stride)   // workgroup-uniform
        rsa_lane<KIND, VEC, P, BATCH, ACCUM, SA>(acc, g, p, 0, (base + threadIdx.x) * EPL, lead, end);
}

// Small messages on groups of more than 64: the one-dword-per-lane form with the buffers split
// over the two wavefronts of a workgroup, so that all p <= 128 loads of an element pair are in
// flight at once (a wavefront can wait for 64 loads at most).  Wavefront 1 passes its dwords
// through LDS; wavefront 0 adds everything in rank order.  One round trip to memory instead
// of two: a 1 MB message at p = 128 takes 7.7 us instead of 12.2, 32 MB 9.1 instead of 12.8;
// at 64 MB (33 M buffer elements per call) the two forms are even.
#ifndef MICS_SPLIT_MIN_P
#define MICS_SPLIT_MIN_P 65
#endif
#ifndef MICS_SPLIT_MAX_ELEMS
#define MICS_SPLIT_MAX_ELEMS (20u << 20)     // buffer elements per call (p * count) up to which it wins
#endif
template <int KIND, bool ACCUM>
__global__ __launch_bounds__(128) void rsa_split_kernel(
    float* __restrict__ acc, PtrTable g, int p, unsigned lead, size_t count)
{
    constexpr int PD = GradFormat<KIND>::kPerDword;
    __shared__ uint32_t passed[64 * 64];                       // [buffer - 64][lane]
    const size_t end = (size_t)lead + count;
    if (blockIdx.x == gridDim.x - 1) {                         // the edge elements, as in rsa_kernel
        rsa_edges<KIND, PD, ACCUM>(acc, g, p, 0, lead, end);
        return;
    }
    const unsigned lane = threadIdx.x & 63u;
    const int half = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const size_t v0 = ((size_t)blockIdx.x * 64 + lane) * PD;
    const bool full = v0 >= lead && v0 + PD <= end;
    const int q_lo = half * 64, q_n = (p - q_lo < 64 ? p - q_lo : 64);      // this wavefront's buffers
    GradVec<KIND, 1> v[64];
    if (full) {
        #pragma unroll
        for (int b = 0; b < 64; ++b)
            if (b < q_n) v[b].load(g.ptr[q_lo + b], v0);
    }
    float s[PD];
    if (half == 1) {
        if (full) {
            #pragma unroll
            for (int b = 0; b < 64; ++b)
                if (b < q_n) passed[b * 64 + lane] = v[b].dword(0);
        }
    } else if (full) {
        rsa_add<KIND, 1, true>(s, v[0]);
        #pragma unroll
        for (int b = 1; b < 64; ++b) rsa_add<KIND, 1, false>(s, v[b]);       // p > 64: all 64 are there
    }
    __syncthreads();
    if (half == 0 && full) {
        float a[PD];
        float* acc_e = acc + (v0 - lead);
        #pragma unroll
        for (int e = 0; e < PD; ++e) a[e] = 0.0f;
        if (ACCUM) ld_f32<PD, false>(a, acc_e);
        for (int q = 64; q < p; ++q) {
            GradVec<KIND, 1> w;
            w.v = passed[(q - 64) * 64 + lane];
            rsa_add<KIND, 1, false>(s, w);
        }
        #pragma unroll
        for (int e = 0; e < PD; ++e) a[e] = a[e] + s[e];
        st_f32<PD, false>(acc_e, a);
    }
}

// Coalesced form (many separately sharded tensors in one launch): workgroup x works on
// tile x - tile_begin[t] of segment t.  Every segment has its own virtual index space as in
// rsa_kernel: src0 = position of its virtual element 0 in the rank buffers (for 2-byte
// gradients a multiple of 2 elements from the 4-byte aligned base), [lead, end) = its elements,
// dst = accumulator index of virtual element `lead`.
struct ReduceSeg {
    unsigned long long end, src0, dst;
    unsigned lead, pad;
};
struct ReduceSegTable {
    int n;
    unsigned tile_begin[kMaxSeg + 1];
    ReduceSeg seg[kMaxSeg];
};

template <int KIND, int P, bool ACCUM, bool SA, typename Tab>
__global__ __launch_bounds__(kMaxBlock) void rsa_seg_kernel(
    float* __restrict__ acc, Tab g, int p, ReduceSegTable tab)
{
    constexpr int EPL = 4 * GradFormat<KIND>::kPerDword;
    const unsigned x = blockIdx.x;
    const int t = segment_of(tab.tile_begin, x);
    const size_t end = tab.seg[t].end, lead = tab.seg[t].lead;
    const size_t v0 = ((size_t)(x - tab.tile_begin[t]) * blockDim.x + threadIdx.x) * EPL;
    if (x == tab.tile_begin[t]) rsa_edges<KIND, EPL, ACCUM>(acc + tab.seg[t].dst, g, p, tab.seg[t].src0, lead, end);
    rsa_lane<KIND, 4, P, MICS_RSA_BATCH, ACCUM, SA>(acc + tab.seg[t].dst, g, p, tab.seg[t].src0, v0, lead, end);
}

// ---------------------------------------------------------------------------
// Step 2b: reduction of the replication-group all-reduce at the accumulation
// boundary and the scaling to a mean (Section 3.4).  One lane owns 4 elements
// per copy and pass (the last count mod 4 elements go one per lane).  `out` may be copies[0]: a lane
// reads its elements of every copy before it writes them, and no other lane touches them.
// ---------------------------------------------------------------------------

// s = ((a_0 + a_1) + ...) + a_{r-1} for the 4 elements from x.  R > 0: r = R at compile time,
// all loads in flight at once; R == 0: any r in batches of 16 loads.
template <int R, bool NT, typename Tab>
__device__ __forceinline__ f32x4 avg_sum4(const Tab& a, int r, size_t x)
{
    if constexpr (R > 0) {
        f32x4 v[R];
        #pragma unroll
        for (int c = 0; c < R; ++c) v[c] = MICS_LD(NT, (const f32x4_a4*)((const float*)a.ptr[c] + x));
        f32x4 sum = v[0];
        #pragma unroll
        for (int c = 1; c < R; ++c) sum = sum + v[c];
        return sum;
    } else {
        constexpr int B = 16;
        f32x4 sum = MICS_LD(NT, (const f32x4_a4*)((const float*)a.ptr[0] + x));
        for (int c0 = 1; c0 < r; c0 += B) {
            f32x4 v[B];
            #pragma unroll
            for (int b = 0; b < B; ++b)
                if (c0 + b < r) v[b] = MICS_LD(NT, (const f32x4_a4*)((const float*)a.ptr[c0 + b] + x));
            #pragma unroll
            for (int b = 0; b < B; ++b)
                if (c0 + b < r) sum = sum + v[b];
        }
        return sum;
    }
}

// One element, the r loads in flight 16 at a time.
template <typename Tab>
__device__ __forceinline__ float avg_sum1(const Tab& a, int r, size_t x)
{
    constexpr int B = 16;
    float sum = ((const float*)a.ptr[0])[x];
    for (int c0 = 1; c0 < r; c0 += B) {
        float w[B];
        #pragma unroll
        for (int b = 0; b < B; ++b)
            if (c0 + b < r) w[b] = ((const float*)a.ptr[c0 + b])[x];
        #pragma unroll
        for (int b = 0; b < B; ++b)
            if (c0 + b < r) sum = sum + w[b];
    }
    return sum;
}

// SO ("stream the output"): non-temporal stores for results too large for the Infinity Cache,
// as for the accumulator of the reduce kernels.
template <int R, bool SO, typename Tab>
__global__ __launch_bounds__(kMaxBlock) void avg_kernel(
    float* out, Tab a, int r, float scale, size_t count)
{
    const size_t nlanes = (count + 3) / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nlanes; i += stride) {
        const size_t x = 4 * i;
        if (x + 4 <= count) {
            const f32x4 sum = avg_sum4<R, kAvgNtl>(a, r, x);
            MICS_ST(SO, (f32x4_a4*)(out + x), sum * scale);
        }
    }
    // the last count mod 4 elements: one per lane
    const size_t e = count / 4 * 4 + threadIdx.x;
    if (blockIdx.x == 0 && e < count) out[e] = avg_sum1(a, r, e) * scale;
}

// ---------------------------------------------------------------------------
// Step 3: mixed-precision Adam on the shard (Sections 2.1, 3.2).  One fp32
// operation per line; the order is part of the contract.
// ---------------------------------------------------------------------------

__device__ __forceinline__ void adam_element(float& w, float& m, float& v, float g,
                                             const AdamScalars& hp)
{
    const float t1 = hp.beta1 * m;
    const float t2 = hp.one_minus_beta1 * g;
    const float m_new = t1 + t2;
    const float gg = g * g;
    const float t3 = hp.beta2 * v;
    const float t4 = hp.one_minus_beta2 * gg;
    const float v_new = t3 + t4;
    const float m_hat = m_new / hp.bias_corr1;        // correctly rounded (build flag)
    const float v_hat = v_new / hp.bias_corr2;
    const float root = __builtin_sqrtf(v_hat);       // correctly rounded (build flag)
    const float denom = root + hp.eps;
    const float ratio = m_hat / denom;
    const float decay = hp.weight_decay * w;
    const float update = ratio + decay;
    const float delta = hp.lr * update;
    w = w - delta;
    m = m_new;
    v = v_new;
}

// The update of 4 consecutive elements from x given their gradient, states in place.
template <int OUT>
__device__ __forceinline__ void adam_update4(float* master, float* exp_avg, float* exp_avg_sq,
                                             uint16_t* param_bf16, size_t x, f32x4 g, f32x4 w, f32x4 m,
                                             f32x4 v, const AdamScalars& hp)
{
    #pragma unroll
    for (int e = 0; e < 4; ++e) {
        float we = w[e], me = m[e], ve = v[e];
        adam_element(we, me, ve, g[e], hp);
        w[e] = we; m[e] = me; v[e] = ve;
    }
    MICS_ST(kAdamNts, (f32x4_a4*)(master + x), w);
    MICS_ST(kAdamNts, (f32x4_a4*)(exp_avg + x), m);
    MICS_ST(kAdamNts, (f32x4_a4*)(exp_avg_sq + x), v);
    if constexpr (OUT != kParamNone) {
        u32x2 b = {param_pack<OUT>(w.x, w.y), param_pack<OUT>(w.z, w.w)};
        MICS_ST(kAdamNts, (u32x2_a2*)(param_bf16 + x), b);
    }
}

template <int OUT>
__device__ __forceinline__ void adam_update1(float* master, float* exp_avg, float* exp_avg_sq,
                                             uint16_t* param_bf16, size_t x, float g, const AdamScalars& hp)
{
    float w = master[x], m = exp_avg[x], v = exp_avg_sq[x];
    adam_element(w, m, v, g, hp);
    master[x] = w; exp_avg[x] = m; exp_avg_sq[x] = v;
    if constexpr (OUT != kParamNone) param_bf16[x] = param_single<OUT>(w);
}

// One lane owns 4 consecutive elements per pass, so that every load and store instruction of
// a wavefront covers one contiguous kilobyte (stores that leave gaps between lanes reach
// memory as partial lines and cost extra traffic).  Four 128-bit loads are in flight before
// the first use; the 16-bit parameters (bf16 or binary16, OUT) leave as one 64-bit store.  That
// output may sit anywhere on an element boundary -- for instance inside the stage-1 buffer of
// the next parameter gather, at T_l + j*S.
template <int OUT>
__global__ __launch_bounds__(kMaxBlock) void adam_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, const float* __restrict__ grad, size_t count, AdamScalars hp)
{
    const size_t nlanes = (count + 3) / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nlanes; i += stride) {
        const size_t x = 4 * i;
        if (x + 4 <= count) {
            const f32x4 g = MICS_LD(kAdamNtl, (const f32x4_a4*)(grad + x));
            const f32x4 w = MICS_LD(kAdamNtl, (const f32x4_a4*)(master + x));
            const f32x4 m = MICS_LD(kAdamNtl, (const f32x4_a4*)(exp_avg + x));
            const f32x4 v = MICS_LD(kAdamNtl, (const f32x4_a4*)(exp_avg_sq + x));
            adam_update4<OUT>(master, exp_avg, exp_avg_sq, param_bf16, x, g, w, m, v, hp);
        } else {
            for (size_t e = x; e < count; ++e)
                adam_update1<OUT>(master, exp_avg, exp_avg_sq, param_bf16, e, grad[e], hp);
        }
    }
}

// Replica average fused into the Adam step: the averaged gradient of a lane's 4 elements is
// formed in registers from the r accumulator copies (same additions, same order, same multiply
// as avg_kernel) and goes straight into adam_element, so it is neither written nor re-read:
// 4r + 12 bytes read and 14 written per element instead of (4r + 4) + 30.  R > 0: r = R at
// compile time; R == 0: any r in batches of 16 loads.
template <int R, int OUT, typename Tab>
__global__ __launch_bounds__(kMaxBlock) void avg_adam_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, Tab a, int r, float scale, size_t count, AdamScalars hp)
{
    const size_t nlanes = (count + 3) / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nlanes; i += stride) {
        const size_t x = 4 * i;
        if (x + 4 <= count) {
#if MICS_FUSED_COPIES_FIRST
            const f32x4 sum = avg_sum4<R, MICS_FUSED_NTL_COPIES>(a, r, x);
#endif
            const f32x4 w = MICS_LD(kAdamNtl, (const f32x4_a4*)(master + x));
            const f32x4 m = MICS_LD(kAdamNtl, (const f32x4_a4*)(exp_avg + x));
            const f32x4 v = MICS_LD(kAdamNtl, (const f32x4_a4*)(exp_avg_sq + x));
#if !MICS_FUSED_COPIES_FIRST
            const f32x4 sum = avg_sum4<R, MICS_FUSED_NTL_COPIES>(a, r, x);
#endif
            adam_update4<OUT>(master, exp_avg, exp_avg_sq, param_bf16, x, sum * scale, w, m, v, hp);
        }
    }
    // the last count mod 4 elements: one per lane
    const size_t e = count / 4 * 4 + threadIdx.x;
    if (blockIdx.x == 0 && e < count)
        adam_update1<OUT>(master, exp_avg, exp_avg_sq, param_bf16, e, avg_sum1(a, r, e) * scale, hp);
}

// ---------------------------------------------------------------------------
// Launch helpers
// ---------------------------------------------------------------------------

std::atomic<int> g_blocks_per_cu{0};
// Built-in policy: accumulators (reduce) and outputs (replica average) of up to 224 MiB -- what
// the 256 MB Infinity Cache absorbs -- are left cacheable, larger ones are streamed (see
// rsa_sum); the accumulator of a reduction over 32 or more buffers is always streamed.  There
// it is at most 8 of 72 bytes per element, so a cache hit saves little, while the orderly write
// path of the streaming kernels is worth more (p = 32, 9.8 M elements, the same accumulator on
// consecutive calls: 5.76 TB/s cacheable, 6.02 streamed; fp32 gradients 6.18 / 6.51; p = 16,
// 12.6 M elements: 6.38 / 6.12).  An explicit threshold (0 = none) replaces the policy.
constexpr size_t kDefaultStreamBytes = 224u << 20;
constexpr int kStreamFromGroup = MICS_RSA_STREAM_FROM_P;
std::atomic<size_t> g_stream_bytes{0};

inline bool stream_acc(size_t elements, int p = 0)
{
    const size_t t = g_stream_bytes.load();
    if (t) return elements * 4 > t;
    return elements * 4 > kDefaultStreamBytes || p >= kStreamFromGroup;
}

int compute_units(int* out)
{
    static std::atomic<int> cached[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev < 64 && cached[dev].load() > 0) { *out = cached[dev].load(); return 0; }
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    if (n < 1) n = 1;
    if (dev >= 0 && dev < 64) cached[dev].store(n);
    *out = n;
    return 0;
}

// Workgroups of `block` lanes for `items` lane-sized work items: enough to cover them, at
// most `bpc` per compute unit (the kernels stride over the rest).
int grid_for(size_t items, int block, int bpc, unsigned* blocks)
{
    int cus = 0;
    if (int e = compute_units(&cus)) return e;
    const int forced = g_blocks_per_cu.load();
    if (forced > 0) bpc = forced;
    size_t want = (items + (size_t)block - 1) / (size_t)block;
    const size_t cap = (size_t)cus * (size_t)bpc;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    *blocks = (unsigned)want;
    return 0;
}

template <typename T> struct same_type { typedef T type; };

// Launches `kernel` with `lds` bytes of dynamic LDS and returns the launch call's own status:
// the caller's HIP error state (an earlier, unrelated error of the thread) is neither reported
// nor cleared here.
template <typename... KArgs>
int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
           typename same_type<KArgs>::type... args)
{
    void* ptrs[] = {(void*)&args...};
    return (int)hipLaunchKernel((const void*)kernel, grid, block, ptrs, lds, st);
}

// Launch shape of a kernel family: lanes per workgroup and the most wavefronts a compute unit
// may hold at a time (0 = whatever fits).
//
// Measured on MI355X (same buffers, one process; GB/s of algorithmic bytes): these streaming
// kernels run fastest in single-wavefront workgroups -- a finished wavefront's slot is refilled
// at once instead of when the last of a workgroup's 8 wavefronts has finished -- and with fewer
// wavefronts per compute unit than fit, i.e. with fewer but longer request streams at the memory
// controllers.  lanes x wavefronts per compute unit (32 = no cap), at 50 M elements (outputs
// fit the Infinity Cache) / 200 M elements (they do not):
//   reorder (3.2 GB)  256x32 6335         64x32 6580          64x16 5990           64x8 3860
//   reduce p = 16     512x32 6190 / 5790  64x32 6295 / 6050   64x10 6365 / 5985    64x4 6150 / 6150
//   average r = 8     512x32 5935 / 5570  64x32 6325 / 6185   64x12 6370 / 6365    64x8 6140 / 6170
//   Adam              128x32 6040 / 5715  64x32 5965 / 5830   64x12 6530 / 6305    64x10 6385 / 6510
//   average + Adam    128x32 5845 / 5560  64x32 5910 / 5865   64x8  6235 / 6155    64x6 6395 / 6370
// The cap is enforced with otherwise unused dynamic LDS: a workgroup that asks for 1/n of a
// compute unit's LDS shares the unit with at most n - 1 others.
struct Shape {
    int lanes, waves_per_cu;
};
constexpr Shape kDefaultShape[kFamilies][2] = {
    /* reorder */ {{MICS_REORDER_BLOCK, 0}, {MICS_REORDER_BLOCK, 0}},
    /* reduce  */ {{MICS_RSA_BLOCK, MICS_RSA_WAVES}, {MICS_RSA_BLOCK, MICS_RSA_WAVES_STREAMED}},
    /* average */ {{MICS_AVG_BLOCK, MICS_AVG_WAVES}, {MICS_AVG_BLOCK, MICS_AVG_WAVES_STREAMED}},
    /* Adam    */ {{MICS_ADAM_BLOCK, MICS_ADAM_WAVES}, {MICS_ADAM_BLOCK, MICS_ADAM_WAVES_STREAMED}},
    /* fused   */ {{MICS_FUSED_BLOCK, MICS_FUSED_WAVES}, {MICS_FUSED_BLOCK, MICS_FUSED_WAVES_STREAMED}},
};
std::atomic<int> g_lanes[kFamilies], g_waves[kFamilies];       // 0 = built-in choice

// The tuned shapes pay from a certain amount of traffic per call on; below it a call is over
// before the capped pipeline has filled, and full-size uncapped workgroups are faster (measured
// per launch, buffers rotated so that nothing is cache-resident: reduce p = 16 at 320 MB 57 us
// against 61 us, at 640 MB 108 against 103; average r = 8 at 72 MB 14.3 against 15.9, at 576 MB
// 100 against 94; fused at 116 MB 22.4 against 24.8, at 464 MB 89 against 75; reorder at 32 MB
// 7.7 against 8.7, at 64 MB 13.1 against 12.0; Adam: no difference below 100 MB).
constexpr size_t kTunedFromBytes[kFamilies] = {48u << 20, 448u << 20, 256u << 20, 0, 200u << 20};
constexpr Shape kSmallCallShape = {512, 0};

// `traffic` = algorithmic bytes of the call; `streams` = buffers a lane reads in this call,
// `tuned_streams` = the number the built-in cap was measured with: a lane with fewer loads in
// flight needs proportionally more wavefronts beside it (a lane with more keeps the cap).
Shape shape_of(int family, bool streamed, size_t traffic, int streams = 1, int tuned_streams = 1,
               int default_lanes = 0)
{
    Shape sh = kDefaultShape[family][streamed ? 1 : 0];
    if (default_lanes) sh.lanes = default_lanes;
    if (sh.waves_per_cu > 0 && streams < tuned_streams)
        sh.waves_per_cu = (sh.waves_per_cu * tuned_streams + streams - 1) / streams;
    if (traffic < kTunedFromBytes[family]) sh = kSmallCallShape;
    if (const int l = g_lanes[family].load()) sh.lanes = l;
    if (const int w = g_waves[family].load()) sh.waves_per_cu = w;
    if (sh.waves_per_cu >= 32) sh.waves_per_cu = 0;
    return sh;
}

// Dynamic LDS that keeps the wavefronts of `sh` on a compute unit at or below its cap, at least
// `needed` bytes (what the kernel itself uses).  Without an opt-in a workgroup gets at most
// 64 KiB, so the cap cannot go below 3 workgroups per compute unit.
size_t lds_for(const Shape& sh, size_t needed = 0)
{
    constexpr size_t kLdsPerCu = 160u << 10, kMaxDynamic = 64u << 10;
    const int waves_per_wg = sh.lanes / 64;
    if (sh.waves_per_cu <= 0 || sh.waves_per_cu / waves_per_wg >= 32) return needed;
    size_t wgs = (size_t)sh.waves_per_cu / (size_t)waves_per_wg;
    if (wgs < 1) wgs = 1;
    size_t bytes = (kLdsPerCu / wgs) & ~(size_t)255;
    if (bytes > kMaxDynamic) bytes = kMaxDynamic;
    return bytes > needed ? bytes : needed;
}

// Calls f(std::bool_constant<a>, std::bool_constant<b>) for two runtime flags.
template <typename F>
int dispatch2(bool a, bool b, F&& f)
{
    if (a) return b ? f(std::true_type{}, std::true_type{}) : f(std::true_type{}, std::false_type{});
    return b ? f(std::false_type{}, std::true_type{}) : f(std::false_type{}, std::false_type{});
}

template <int N>
SmallTable<N> small(const PtrTable& t)
{
    SmallTable<N> s;
    for (int i = 0; i < N; ++i) s.ptr[i] = t.ptr[i];
    return s;
}

// Calls f(std::integral_constant<int, P>) with P = p if p has an unrolled kernel, else P = 0.
template <typename F>
int dispatch_group(int p, F&& f)
{
    switch (p) {
        case 1: return f(std::integral_constant<int, 1>{});
        case 2: return f(std::integral_constant<int, 2>{});
        case 4: return f(std::integral_constant<int, 4>{});
        case 8: return f(std::integral_constant<int, 8>{});
        case 16: return f(std::integral_constant<int, 16>{});
        case 32: return f(std::integral_constant<int, 32>{});
        default: return f(std::integral_constant<int, 0>{});
    }
}

}  // namespace

void set_blocks_per_cu(int n) { g_blocks_per_cu.store(n); }

void set_stream_threshold_bytes(size_t n) { g_stream_bytes.store(n); }

void set_launch_shape(int family, int lanes, int waves_per_cu)
{
    g_lanes[family].store(lanes);
    g_waves[family].store(waves_per_cu);
}

const char* hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

int launch_reorder(void* dst, const PtrTable& src, size_t n_valid_bytes, size_t shard_bytes, int p,
                   int k, bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (vec16) {
        // spread the block budget over the p chunks
        unsigned total = 0;
        const Shape sh = shape_of(kFamReorder, true, 2 * n_valid_bytes);
        if (int e = grid_for(shard_bytes / 16 * (size_t)p, sh.lanes, MICS_REORDER_BPC, &total)) return e;
        unsigned bx = (total + (unsigned)p - 1) / (unsigned)p;
        return launch(reorder_vec_kernel, dim3(bx, (unsigned)p), dim3(sh.lanes), lds_for(sh), st, (u32x4*)dst, src,
                      shard_bytes / 16, n_valid_bytes, k);
    }
    const Segment one = {n_valid_bytes, shard_bytes, 0, 0};
    return launch_reorder_coalesced(dst, src, &one, 1, p, k, 1, false, stream);
}

namespace {

template <int KIND, int VEC, int P, bool ACCUM, bool SA>
int rsa_launch(float* acc, const PtrTable& g, int p, unsigned lead, size_t count, unsigned blocks,
               const Shape& sh, hipStream_t st)
{
    // the streamed-accumulator kernels pass their results through 32 bytes of LDS per lane
    const size_t lds = lds_for(sh, SA && VEC == 4 && KIND != 2 ? (size_t)sh.lanes * 32 : 0);
    if constexpr (P > 0)
        return launch(rsa_kernel<KIND, VEC, P, ACCUM, SA, SmallTable<P>>, dim3(blocks + 1), dim3(sh.lanes), lds, st,
                      acc, small<P>(g), p, lead, count);
    else
        return launch(rsa_kernel<KIND, VEC, 0, ACCUM, SA, PtrTable>, dim3(blocks + 1), dim3(sh.lanes), lds, st, acc,
                      g, p, lead, count);
}

template <int KIND>
int rsa_launch_kind(float* acc, const PtrTable& g, int p, unsigned lead, size_t count, bool accumulate,
                    hipStream_t st)
{
    constexpr size_t PD = GradFormat<KIND>::kPerDword;
    unsigned blocks = 0;
    // small message on a group of more than 64: one dword per lane and buffer, the buffers split
    // over two wavefronts
    if (p >= MICS_SPLIT_MIN_P && count <= (size_t)MICS_SPLIT_MAX_ELEMS / (size_t)p) {
        const size_t nlanes = (lead + count + PD - 1) / PD;
        if (int e = grid_for(nlanes, 64, MICS_RSA_BPC, &blocks)) return e;
        if (blocks == (nlanes + 63) / 64)                      // one pass per lane (the kernel has no stride loop)
            return accumulate ? launch(rsa_split_kernel<KIND, true>, dim3(blocks + 1), dim3(128), 0, st, acc, g, p, lead, count)
                              : launch(rsa_split_kernel<KIND, false>, dim3(blocks + 1), dim3(128), 0, st, acc, g, p, lead, count);
    }
    // small message on a large group: one dword per lane and buffer
    if (p >= MICS_NARROW_MIN_P && count <= (size_t)MICS_NARROW_MAX_ELEMS / (size_t)p) {
        const Shape narrow = {kNarrowBlock, 0};
        const size_t nlanes = (lead + count + PD - 1) / PD;
        if (int e = grid_for(nlanes, kNarrowBlock, MICS_RSA_BPC, &blocks)) return e;
        return accumulate ? rsa_launch<KIND, 1, 0, true, false>(acc, g, p, lead, count, blocks, narrow, st)
                          : rsa_launch<KIND, 1, 0, false, false>(acc, g, p, lead, count, blocks, narrow, st);
    }
    const size_t nlanes = (lead + count + 4 * PD - 1) / (4 * PD);
    const bool streamed = stream_acc(count, p);
    const size_t traffic = count * ((size_t)GradFormat<KIND>::kElemBytes * (size_t)p + 8);
    Shape sh = shape_of(kFamReduce, streamed, traffic, p + 2, 18);
    // Single-wavefront workgroups are the fastest when every access is 16-byte aligned; with the
    // accumulator or the gradients off that alignment full-size workgroups are (6070 against
    // 5740 GB/s at 50 M elements).  A call too small to give every compute unit half a
    // full-size workgroup runs in single wavefronts in any case, uncapped (a unit moves about
    // 100 GB/s on its own: 0.5 M elements at p = 16 take 5.3 us instead of 6.2).
    int cus = 0;
    if (int e = compute_units(&cus)) return e;
    bool aligned16 = lead == 0 && ((uintptr_t)acc & 15) == 0;
    for (int q = 0; q < p && aligned16; ++q) aligned16 = ((uintptr_t)g.ptr[q] & 15) == 0;
    if (g_lanes[kFamReduce].load() == 0) {
        if (nlanes * 2 <= (size_t)kMaxBlock * (size_t)cus) sh = Shape{64, 0};
        else if (!aligned16) sh = Shape{MICS_RSA_UNALIGNED_BLOCK, 0};
    }
    // binary16 gradients cost a conversion per element: the arithmetic then needs every wavefront
    // that fits (p = 16, 50 M elements: 6430 GB/s uncapped, 4450 with 10 wavefronts per unit)
    if (KIND == 1 && g_waves[kFamReduce].load() == 0) sh.waves_per_cu = 0;
    if (int e = grid_for(nlanes, sh.lanes, MICS_RSA_BPC, &blocks)) return e;
    return dispatch2(accumulate, streamed, [&](auto A, auto SA) {
        if constexpr (KIND == 0) {
            return dispatch_group(p, [&](auto P) {
                return rsa_launch<KIND, 4, P.value, A.value, SA.value>(acc, g, p, lead, count, blocks, sh, st);
            });
        } else {
            switch (p) {
                case 8: return rsa_launch<KIND, 4, 8, A.value, SA.value>(acc, g, p, lead, count, blocks, sh, st);
                case 16: return rsa_launch<KIND, 4, 16, A.value, SA.value>(acc, g, p, lead, count, blocks, sh, st);
                default: return rsa_launch<KIND, 4, 0, A.value, SA.value>(acc, g, p, lead, count, blocks, sh, st);
            }
        }
    });
}

// Rounds 2-byte element pointers down to 4 bytes when all of them sit at the same position
// inside their dword (rank g's slices of separately allocated buffers do: they all start g*S
// elements in); returns how many elements they moved back (the kernels' `lead`, 0 or 1).  With
// mixed positions the pointers stay and the odd ones are read with 2-byte aligned 128-bit loads
// (about 20 % slower).  Rounding further down, to 16 bytes, was measured too: no gain at
// p = 16 and a 5 % loss at p = 32, the accumulator then being addressed further off its own
// alignment.
unsigned align_gradient_pointers(PtrTable& g, int p, int elem_bytes)
{
    if (elem_bytes != 2) return 0;
    const uintptr_t odd = (uintptr_t)g.ptr[0] & 2;
    for (int q = 1; q < p; ++q)
        if (((uintptr_t)g.ptr[q] & 2) != odd) return 0;
    if (!odd) return 0;
    for (int q = 0; q < p; ++q) g.ptr[q] = (const char*)g.ptr[q] - 2;
    return 1;
}

}  // namespace

int launch_reduce_scatter_accum(float* acc, const PtrTable& grads, size_t count, int p, bool accumulate,
                                int kind, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    PtrTable g = grads;
    const unsigned lead = align_gradient_pointers(g, p, kind == 2 ? 4 : 2);
    switch (kind) {
        case 0: return rsa_launch_kind<0>(acc, g, p, lead, count, accumulate, st);
        case 1: return rsa_launch_kind<1>(acc, g, p, lead, count, accumulate, st);
        default: return rsa_launch_kind<2>(acc, g, p, lead, count, accumulate, st);
    }
}

int launch_replica_average(float* out, const PtrTable& a, size_t count, int r, float scale, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned blocks = 0;
    const bool streamed = stream_acc(count);
    const Shape sh = shape_of(kFamAverage, streamed, count * (4 * (size_t)r + 4), r + 1, 9);
    const size_t lds = lds_for(sh);
    if (int e = grid_for((count + 3) / 4, sh.lanes, MICS_AVG_BPC, &blocks)) return e;
    const dim3 gr(blocks), bl(sh.lanes);
    return dispatch2(streamed, false, [&](auto SO, auto) {
        switch (r) {
            case 1: return launch(avg_kernel<1, SO.value, SmallTable<1>>, gr, bl, lds, st, out, small<1>(a), r, scale, count);
            case 2: return launch(avg_kernel<2, SO.value, SmallTable<2>>, gr, bl, lds, st, out, small<2>(a), r, scale, count);
            case 4: return launch(avg_kernel<4, SO.value, SmallTable<4>>, gr, bl, lds, st, out, small<4>(a), r, scale, count);
            case 8: return launch(avg_kernel<8, SO.value, SmallTable<8>>, gr, bl, lds, st, out, small<8>(a), r, scale, count);
            default: return launch(avg_kernel<0, SO.value, PtrTable>, gr, bl, lds, st, out, a, r, scale, count);
        }
    });
}

namespace {
// Calls f(std::integral_constant<int, OUT>) for the parameter output of a call.
template <typename F>
int dispatch_param(const void* param_out, bool f16, F&& f)
{
    if (!param_out) return f(std::integral_constant<int, kParamNone>{});
    if (f16) return f(std::integral_constant<int, kParamF16>{});
    return f(std::integral_constant<int, kParamBf16>{});
}
}  // namespace

int launch_adam(float* master, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16, bool param_f16,
                const float* grad, size_t count, const AdamScalars& hp, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned blocks = 0;
    const Shape sh = shape_of(kFamAdam, stream_acc(count), count * 30);
    if (int e = grid_for((count + 3) / 4, sh.lanes, MICS_ADAM_BPC, &blocks)) return e;
    return dispatch_param(param_bf16, param_f16, [&](auto OUT) {
        return launch(adam_kernel<OUT.value>, dim3(blocks), dim3(sh.lanes), lds_for(sh), st, master, exp_avg,
                      exp_avg_sq, param_bf16, grad, count, hp);
    });
}

int launch_reorder_coalesced(void* dst, const PtrTable& src, const Segment* segs, int n, int p, int k,
                             int elem_bytes, bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t eb = (size_t)elem_bytes;
    for (int first = 0; first < n; first += kMaxSeg) {
        const int nt = n - first < kMaxSeg ? n - first : kMaxSeg;
        size_t tiles = 0;
        if (vec16) {
            size_t moved = 0;
            for (int t = 0; t < nt; ++t) moved += 2 * segs[first + t].numel * eb;
            const Shape sh = shape_of(kFamReorder, true, moved, 1, 1, kSegLanes);
            const size_t tile_vecs = (size_t)sh.lanes * MICS_SEG_U;
            ReorderSegTable tab;
            tab.n = nt;
            for (int t = 0; t < nt; ++t) {
                const Segment& sg = segs[first + t];
                tab.tile_begin[t] = (unsigned)tiles;
                tab.seg[t].shard_vecs = sg.shard_elems * eb / 16;
                tab.seg[t].valid_bytes = sg.numel * eb;
                tab.seg[t].src_vec = sg.src_offset * eb / 16;
                tab.seg[t].dst_vec = sg.dst_offset * eb / 16;
                tiles += (tab.seg[t].shard_vecs + tile_vecs - 1) / tile_vecs;
                if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
            }
            for (int t = nt; t <= kMaxSeg; ++t) tab.tile_begin[t] = kNoTile;
            if (tiles == 0) continue;
            if (int e = launch(reorder_seg_kernel, dim3((unsigned)tiles, (unsigned)p), dim3(sh.lanes), lds_for(sh), st,
                               (u32x4*)dst, src, tab, k))
                return e;
        } else {
            size_t moved = 0;
            for (int t = 0; t < nt; ++t) moved += 2 * segs[first + t].numel * eb;
            const Shape sh = shape_of(kFamReorder, true, moved, 1, 1, MICS_SHIFT_BLOCK);
            const size_t tile_bytes = (size_t)sh.lanes * MICS_SHIFT_U * 16;
            // tiles of full destination vectors; at least one per tensor, for the chunk ends
            auto tiles_of = [&](const ByteSeg& sg) {
                const size_t t = (sg.shard_bytes + tile_bytes - 1) / tile_bytes;
                return sg.valid_bytes ? (t ? t : 1) : 0;
            };
            if (nt == 1) {
                const Segment& sg = segs[first];
                OneTensor one;
                one.seg.shard_bytes = sg.shard_elems * eb;
                one.seg.valid_bytes = sg.numel * eb;
                one.seg.src_byte = sg.src_offset * eb;
                one.seg.dst_byte = sg.dst_offset * eb;
                tiles = tiles_of(one.seg);
                if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
                if (tiles == 0) continue;
                if (int e = launch(reorder_shift_kernel<OneTensor>, dim3((unsigned)tiles, (unsigned)p), dim3(sh.lanes),
                                   lds_for(sh), st, (unsigned char*)dst, src, one, k))
                    return e;
                continue;
            }
            ByteSegTable tab;
            tab.n = nt;
            for (int t = 0; t < nt; ++t) {
                const Segment& sg = segs[first + t];
                tab.tile_begin[t] = (unsigned)tiles;
                tab.seg[t].shard_bytes = sg.shard_elems * eb;
                tab.seg[t].valid_bytes = sg.numel * eb;
                tab.seg[t].src_byte = sg.src_offset * eb;
                tab.seg[t].dst_byte = sg.dst_offset * eb;
                tiles += tiles_of(tab.seg[t]);
                if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
            }
            for (int t = nt; t <= kMaxSeg; ++t) tab.tile_begin[t] = kNoTile;
            if (tiles == 0) continue;
            if (int e = launch(reorder_shift_kernel<ByteSegTable>, dim3((unsigned)tiles, (unsigned)p), dim3(sh.lanes),
                               lds_for(sh), st, (unsigned char*)dst, src, tab, k))
                return e;
        }
    }
    return 0;
}

namespace {

template <int KIND>
int reduce_coalesced_kind(float* acc, PtrTable g, const Segment* segs, int n, int p, bool accumulate,
                          hipStream_t st)
{
    constexpr size_t GB = GradFormat<KIND>::kElemBytes, EPL = 4 * GradFormat<KIND>::kPerDword;
    const size_t base_lead = align_gradient_pointers(g, p, (int)GB);
    for (int first = 0; first < n; first += kMaxSeg) {
        ReduceSegTable tab;
        tab.n = n - first < kMaxSeg ? n - first : kMaxSeg;
        size_t elements = 0;
        for (int t = 0; t < tab.n; ++t) elements += segs[first + t].numel;
        const bool streamed = stream_acc(elements, p);
        // as in rsa_launch_kind: single-wavefront workgroups if every access is 16-byte aligned
        // (h = 8192 layer: 6460 against 6220 GB/s), full-size ones otherwise; binary16 uncapped
        Shape sh = shape_of(kFamReduce, streamed, elements * (GB * (size_t)p + 8), p + 2, 18);
        bool aligned16 = base_lead == 0 && ((uintptr_t)acc & 15) == 0;
        for (int q = 0; q < p && aligned16; ++q) aligned16 = ((uintptr_t)g.ptr[q] & 15) == 0;
        for (int t = 0; t < tab.n && aligned16; ++t)
            aligned16 = segs[first + t].src_offset % (16 / GB) == 0 && segs[first + t].dst_offset % 4 == 0;
        if (!aligned16 && g_lanes[kFamReduce].load() == 0) sh = Shape{MICS_RSA_UNALIGNED_BLOCK, 0};
        if (KIND == 1 && g_waves[kFamReduce].load() == 0) sh.waves_per_cu = 0;
        const size_t tile_elems = (size_t)sh.lanes * EPL;
        size_t tiles = 0;
        for (int t = 0; t < tab.n; ++t) {
            const Segment& sg = segs[first + t];
            // position of the segment's first element in the (for 2-byte gradients rounded-down)
            // buffers; its virtual element 0 is the 4-byte aligned position at or below it
            const size_t src = sg.src_offset + base_lead;
            const unsigned lead = GB == 2 ? (unsigned)(src & 1) : 0u;
            tab.tile_begin[t] = (unsigned)tiles;
            tab.seg[t].lead = lead;
            tab.seg[t].pad = 0;
            tab.seg[t].end = lead + sg.numel;
            tab.seg[t].src0 = src - lead;
            tab.seg[t].dst = sg.dst_offset;
            if (sg.numel) tiles += (lead + sg.numel + tile_elems - 1) / tile_elems;
            else tab.seg[t].end = 0;
            if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
        }
        for (int t = tab.n; t <= kMaxSeg; ++t) tab.tile_begin[t] = kNoTile;
        if (tiles == 0) continue;
        const int err = dispatch2(accumulate, streamed, [&](auto A, auto SA) {
            // the streamed-accumulator kernels pass their results through 32 bytes of LDS per lane
            const size_t lds = lds_for(sh, SA.value && EPL == 8 ? (size_t)sh.lanes * 32 : 0);
            const dim3 gr((unsigned)tiles), bl(sh.lanes);
            if constexpr (KIND == 0) {
                return dispatch_group(p, [&](auto P) {
                    if constexpr (P.value > 0)
                        return launch(rsa_seg_kernel<KIND, P.value, A.value, SA.value, SmallTable<P.value>>, gr, bl,
                                      lds, st, acc, small<P.value>(g), p, tab);
                    else
                        return launch(rsa_seg_kernel<KIND, 0, A.value, SA.value, PtrTable>, gr, bl, lds, st, acc, g,
                                      p, tab);
                });
            } else {
                switch (p) {
                    case 8: return launch(rsa_seg_kernel<KIND, 8, A.value, SA.value, SmallTable<8>>, gr, bl, lds, st, acc, small<8>(g), p, tab);
                    case 16: return launch(rsa_seg_kernel<KIND, 16, A.value, SA.value, SmallTable<16>>, gr, bl, lds, st, acc, small<16>(g), p, tab);
                    default: return launch(rsa_seg_kernel<KIND, 0, A.value, SA.value, PtrTable>, gr, bl, lds, st, acc, g, p, tab);
                }
            }
        });
        if (err) return err;
    }
    return 0;
}

}  // namespace

int launch_reduce_coalesced(float* acc, const PtrTable& grads, const Segment* segs, int n, int p,
                            bool accumulate, int kind, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    switch (kind) {
        case 0: return reduce_coalesced_kind<0>(acc, grads, segs, n, p, accumulate, st);
        case 1: return reduce_coalesced_kind<1>(acc, grads, segs, n, p, accumulate, st);
        default: return reduce_coalesced_kind<2>(acc, grads, segs, n, p, accumulate, st);
    }
}

int launch_avg_adam(float* master, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16, bool param_f16,
                    const PtrTable& copies, int r, float scale, size_t count, const AdamScalars& hp,
                    void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned blocks = 0;
    const Shape sh = shape_of(kFamFused, stream_acc(count), count * (4 * (size_t)r + 26), r + 3, 11);
    const size_t lds = lds_for(sh);
    if (int e = grid_for((count + 3) / 4, sh.lanes, MICS_ADAM_BPC, &blocks)) return e;
    return dispatch_param(param_bf16, param_f16, [&](auto BF) {
        const dim3 gr(blocks), bl(sh.lanes);
        switch (r) {
            case 1: return launch(avg_adam_kernel<1, BF.value, SmallTable<1>>, gr, bl, lds, st, master, exp_avg, exp_avg_sq, param_bf16, small<1>(copies), r, scale, count, hp);
            case 2: return launch(avg_adam_kernel<2, BF.value, SmallTable<2>>, gr, bl, lds, st, master, exp_avg, exp_avg_sq, param_bf16, small<2>(copies), r, scale, count, hp);
            case 4: return launch(avg_adam_kernel<4, BF.value, SmallTable<4>>, gr, bl, lds, st, master, exp_avg, exp_avg_sq, param_bf16, small<4>(copies), r, scale, count, hp);
            case 8: return launch(avg_adam_kernel<8, BF.value, SmallTable<8>>, gr, bl, lds, st, master, exp_avg, exp_avg_sq, param_bf16, small<8>(copies), r, scale, count, hp);
            default: return launch(avg_adam_kernel<0, BF.value, PtrTable>, gr, bl, lds, st, master, exp_avg, exp_avg_sq, param_bf16, copies, r, scale, count, hp);
        }
    });
}

}  // namespace mics
