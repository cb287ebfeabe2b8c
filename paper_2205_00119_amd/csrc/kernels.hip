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

// Launch shape and cache hints per kernel family; the defaults are the measured best on
// MI355X for the h = 8192, p = 16 shard shapes.  *_BLOCK = workgroup size, *_BPC = cap on
// workgroups per compute unit (the grid covers the data with one pass per lane unless the
// cap is reached; lanes stride over the rest), *_NTL / *_NTS = non-temporal loads / stores.
#ifndef MICS_REORDER_BLOCK
#define MICS_REORDER_BLOCK 256
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
#define MICS_RSA_BLOCK 512
#endif
#ifndef MICS_RSA_BPC
#define MICS_RSA_BPC 4096
#endif
#ifndef MICS_RSA_NTL
#define MICS_RSA_NTL 1
#endif
#ifndef MICS_AVG_BLOCK
#define MICS_AVG_BLOCK 512
#endif
#ifndef MICS_AVG_BPC
#define MICS_AVG_BPC 4096
#endif
#ifndef MICS_AVG_NTL
#define MICS_AVG_NTL 1
#endif
#ifndef MICS_ADAM_BLOCK
#define MICS_ADAM_BLOCK 256
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

constexpr int kBlock = 256;              // element-wise (tail / unaligned) kernels, LDS reorder
constexpr int kReorderBlock = MICS_REORDER_BLOCK;
constexpr int kRsaBlock = MICS_RSA_BLOCK;
constexpr int kAvgBlock = MICS_AVG_BLOCK;
constexpr int kAdamBlock = MICS_ADAM_BLOCK;
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

template <bool NT, typename V>
__device__ __forceinline__ V ld(const V* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename V>
__device__ __forceinline__ void st(V* p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// bf16 -> fp32 is exact: the bf16 bits are the upper half of the fp32 bits.
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_one(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

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

// ---------------------------------------------------------------------------
// Step 1: chunk rearrangement of the hierarchical all-gather (Section 3.3).
// Chunk g of the result comes from slot g div k of the stage-1 buffer of local
// rank g mod k.  blockIdx.y = g, blockIdx.x strides over the chunk.
// ---------------------------------------------------------------------------

// All addresses and the shard size are multiples of 16 bytes: a remapped copy.
__global__ __launch_bounds__(kReorderBlock) void reorder_vec_kernel(
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
    const size_t stride = (size_t)gridDim.x * kReorderBlock;
    for (size_t i = (size_t)blockIdx.x * kReorderBlock + threadIdx.x; i < nfull; i += stride)
        st<kReorderNts>(d + i, ld<kReorderNtl>(s + i));

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
// MICS_SEG_U runs of kSegBlock vectors.  Measured on the h = 8192 layer (GB/s): 256 lanes x 1:
// 5200, x 2: 6100, x 4: 5900; 512 x 1: 4600; 1024 x 1: 3600 -- the table look-up in every
// wavefront's prologue has to be paid for by two vectors per lane, more spreads the window.
// A small chunk (a bias of h/p elements) costs one workgroup.
#ifndef MICS_SEG_BLOCK
#define MICS_SEG_BLOCK 256
#endif
#ifndef MICS_SEG_U
#define MICS_SEG_U 2
#endif
constexpr int kMaxSeg = kMaxSegPerLaunch;
constexpr int kSegBlock = MICS_SEG_BLOCK;
constexpr int kSegTileVecs = kSegBlock * MICS_SEG_U;

// Index of the segment whose tile range holds workgroup x: tile_begin is ascending, unused
// entries hold 0xFFFFFFFF.  Counting instead of walking keeps the table reads independent of
// one another (a few wide scalar loads), which matters for workgroups that move only 4 KiB.
__device__ __forceinline__ int segment_of(const unsigned (&tile_begin)[kMaxSeg + 1], unsigned x)
{
    int t = 0;
    #pragma unroll
    for (int i = 1; i < kMaxSeg; ++i) t += tile_begin[i] <= x ? 1 : 0;
    return t;
}
struct ReorderSeg {
    unsigned long long shard_vecs, valid_bytes, src_vec, dst_vec;
};
struct ReorderSegTable {
    int n;
    unsigned tile_begin[kMaxSeg + 1];
    ReorderSeg seg[kMaxSeg];
};

__global__ __launch_bounds__(kSegBlock) void reorder_seg_kernel(
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
    const size_t tile0 = (size_t)(x - tab.tile_begin[t]) * kSegTileVecs;
    u32x4 v[MICS_SEG_U];
    #pragma unroll
    for (int u = 0; u < MICS_SEG_U; ++u) {
        const size_t i = tile0 + (size_t)u * kSegBlock + threadIdx.x;
        if (i < nfull) v[u] = ld<kReorderNtl>(s + i);
    }
    #pragma unroll
    for (int u = 0; u < MICS_SEG_U; ++u) {
        const size_t i = tile0 + (size_t)u * kSegBlock + threadIdx.x;
        if (i < nfull) st<kReorderNts>(d + i, v[u]);
    }
    // ragged end of the tensor: the tile that holds vector index nfull moves the last bytes
    const size_t tail_halves = (valid - nfull * 16) / 2;
    if (tail_halves && nfull / kSegTileVecs == x - tab.tile_begin[t] && threadIdx.x < tail_halves) {
        const uint16_t* sh = (const uint16_t*)(s + nfull);
        uint16_t* dh = (uint16_t*)(d + nfull);
        dh[threadIdx.x] = sh[threadIdx.x];
    }
}

// General case: source and destination of a chunk sit at different offsets
// within their 16-byte lines (odd shard sizes, sub-buffers that start anywhere
// on an element boundary).  A workgroup stages the source bytes of one
// destination tile in LDS with aligned 128-bit loads, then every lane rebuilds
// its aligned 128-bit destination vector from two LDS vectors shifted by the
// (workgroup-uniform) phase.  The partial vectors at the two ends of a chunk
// are moved in 2-byte units.  Global memory is touched only inside the chunk.
constexpr int kStageVecsPerThread = 4;
constexpr int kTileVecs = kBlock * kStageVecsPerThread;   // destination vectors per tile
constexpr int kTileBytes = kTileVecs * 16;

__global__ __launch_bounds__(kBlock) void reorder_lds_kernel(
    unsigned char* __restrict__ dst, PtrTable src, size_t shard_bytes, size_t n_valid_bytes, int k)
{
    __shared__ u32x4 stage[kTileVecs + 2];
    const size_t g = blockIdx.y;
    const size_t chunk_begin = g * shard_bytes;
    if (chunk_begin >= n_valid_bytes) return;
    size_t valid = n_valid_bytes - chunk_begin;
    if (valid > shard_bytes) valid = shard_bytes;
    const size_t j = g / (size_t)k, l = g % (size_t)k;

    const uintptr_t d_lo = (uintptr_t)dst + chunk_begin;              // chunk in dst
    const uintptr_t d_hi = d_lo + valid;
    const uintptr_t s_chunk = (uintptr_t)src.ptr[l] + j * shard_bytes;  // chunk in src
    const uintptr_t grid0 = d_lo & ~(uintptr_t)15;                     // 16-byte grid of dst
    const size_t ntiles = (d_hi - grid0 + kTileBytes - 1) / kTileBytes;
    const unsigned phase = (unsigned)((s_chunk - d_lo) & 15);           // even, uniform
    const unsigned dshift = phase >> 2, half = (phase >> 1) & 1;
    const uint16_t* stage_h = (const uint16_t*)stage;

    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const uintptr_t tile0 = grid0 + tile * kTileBytes;
        const uintptr_t t_lo = tile0 > d_lo ? tile0 : d_lo;
        const uintptr_t t_hi = tile0 + kTileBytes < d_hi ? tile0 + kTileBytes : d_hi;
        const uintptr_t s_lo = s_chunk + (t_lo - d_lo), s_hi = s_chunk + (t_hi - d_lo);
        const uintptr_t sa = s_lo & ~(uintptr_t)15;
        const unsigned nsv = (unsigned)(((s_hi + 15) & ~(uintptr_t)15) - sa) / 16;   // <= kTileVecs+1

        for (unsigned v = threadIdx.x; v < nsv; v += kBlock) {
            const uintptr_t a = sa + (uintptr_t)v * 16;
            if (a >= s_lo && a + 16 <= s_hi) {
                stage[v] = *(const u32x4*)a;
            } else {
                uint16_t* row = (uint16_t*)&stage[v];
                for (unsigned h = 0; h < 8; ++h) {
                    const uintptr_t b = a + 2 * h;
                    if (b >= s_lo && b < s_hi) row[h] = *(const uint16_t*)b;
                }
            }
        }
        __syncthreads();

        for (unsigned vv = threadIdx.x; vv < kTileVecs; vv += kBlock) {
            const uintptr_t a = tile0 + (uintptr_t)vv * 16;      // aligned dst address
            if (a + 16 <= t_lo || a >= t_hi) continue;
            // byte offset of this vector's source bytes inside the staged range
            const long o = (long)(a - d_lo) + (long)(s_chunk - sa);   // a may lie below d_lo
            if (a >= t_lo && a + 16 <= t_hi) {
                const unsigned o16 = (unsigned)o >> 4;
                const u32x4 lo = stage[o16], hi = stage[o16 + 1];
                // shift the 8 staged dwords down by `dshift` dwords (uniform), then by
                // half a dword if the phase is an odd number of 2-byte units
                uint32_t w0 = lo.x, w1 = lo.y, w2 = lo.z, w3 = lo.w;
                uint32_t w4 = hi.x, w5 = hi.y, w6 = hi.z, w7 = hi.w;
                if (dshift & 1) { w0 = w1; w1 = w2; w2 = w3; w3 = w4; w4 = w5; w5 = w6; w6 = w7; }
                if (dshift & 2) { w0 = w2; w1 = w3; w2 = w4; w3 = w5; w4 = w6; }
                u32x4 out = {w0, w1, w2, w3};
                if (half) {
                    out.x = (w0 >> 16) | (w1 << 16);
                    out.y = (w1 >> 16) | (w2 << 16);
                    out.z = (w2 >> 16) | (w3 << 16);
                    out.w = (w3 >> 16) | (w4 << 16);
                }
                *(u32x4*)a = out;
            } else {
                for (unsigned h = 0; h < 8; ++h) {
                    const uintptr_t b = a + 2 * h;
                    if (b >= t_lo && b < t_hi) *(uint16_t*)b = stage_h[(o + 2 * (long)h) >> 1];
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Step 2a: reduction of the partition-group reduce-scatter, accumulated over
// micro-steps (Section 3.4).  One lane owns 8 consecutive elements: one
// 128-bit load per rank buffer, all issued before the first addition.
// ---------------------------------------------------------------------------

template <bool ACCUM>
__device__ __forceinline__ float rsa_element(const PtrTable& g, int p, size_t x, float before)
{
    float partial = bf16_one(((const uint16_t*)g.ptr[0])[x]);
    for (int q = 1; q < p; ++q) partial = partial + bf16_one(((const uint16_t*)g.ptr[q])[x]);
    return (ACCUM ? before : 0.0f) + partial;
}

// Partial sum over the p rank buffers of the 8 consecutive elements that start at element
// `elem` (a multiple of 8 from 16-byte aligned bases), ranks in ascending order.  P > 0:
// p = P known at compile time, all P loads issued before the first addition; P == 0: any p,
// consumed in batches of 32 loads (a lane's additions are a serial chain, so the number of
// load round trips per lane, p/32, is what a small message on a large group waits for: batches
// of 8 put the floor of a p = 128 call at 25 us).
template <int P, typename Tab>
__device__ __forceinline__ void rsa_partial8(float (&s)[8], const Tab& g, int p, size_t elem)
{
    if constexpr (P > 0) {
        u32x4 v[P];
        #pragma unroll
        for (int q = 0; q < P; ++q)
            v[q] = ld<kRsaNtl>((const u32x4*)((const uint16_t*)g.ptr[q] + elem));
        #pragma unroll
        for (int e = 0; e < 4; ++e) { s[2 * e] = bf16_lo(v[0][e]); s[2 * e + 1] = bf16_hi(v[0][e]); }
        #pragma unroll
        for (int q = 1; q < P; ++q) {
            #pragma unroll
            for (int e = 0; e < 4; ++e) {
                s[2 * e] = s[2 * e] + bf16_lo(v[q][e]);
                s[2 * e + 1] = s[2 * e + 1] + bf16_hi(v[q][e]);
            }
        }
    } else {
        constexpr int B = 32;
        {
            u32x4 first = ld<kRsaNtl>((const u32x4*)((const uint16_t*)g.ptr[0] + elem));
            #pragma unroll
            for (int e = 0; e < 4; ++e) { s[2 * e] = bf16_lo(first[e]); s[2 * e + 1] = bf16_hi(first[e]); }
        }
        for (int q0 = 1; q0 < p; q0 += B) {
            u32x4 v[B];
            #pragma unroll
            for (int b = 0; b < B; ++b)
                if (q0 + b < p) v[b] = ld<kRsaNtl>((const u32x4*)((const uint16_t*)g.ptr[q0 + b] + elem));
            #pragma unroll
            for (int b = 0; b < B; ++b) {
                if (q0 + b < p) {
                    #pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        s[2 * e] = s[2 * e] + bf16_lo(v[b][e]);
                        s[2 * e + 1] = s[2 * e + 1] + bf16_hi(v[b][e]);
                    }
                }
            }
        }
    }
}

// acc8 (16-byte aligned, 8 floats) = (ACCUM ? acc8 : +0) + partial sum at `elem`.
// SA ("stream the accumulator"): non-temporal accumulator loads and stores.  An accumulator
// that fits the 256 MB Infinity Cache is best left cacheable -- its stores are absorbed there
// and the next micro-step finds it again (plain/plain 6.3 TB/s, NT/NT 6.1 at S = 50 M) -- while
// a larger one is best streamed past the caches (NT/NT 5.8 TB/s, plain/plain 5.4, and the
// mixed NT-load/plain-store 5.1 at S = 200 M); the launcher picks by size.
template <int P, bool ACCUM, bool SA, typename Tab>
__device__ __forceinline__ void rsa_update8(float* __restrict__ acc8, const Tab& g, int p, size_t elem)
{
    f32x4 a0 = {0.0f, 0.0f, 0.0f, 0.0f}, a1 = a0;
    if (ACCUM) {   // issued before the gradient loads are consumed
        a0 = ld<SA>((const f32x4*)acc8);
        a1 = ld<SA>((const f32x4*)acc8 + 1);
    }
    float s[8];
    rsa_partial8<P>(s, g, p, elem);
    f32x4 o0 = {a0.x + s[0], a0.y + s[1], a0.z + s[2], a0.w + s[3]};
    f32x4 o1 = {a1.x + s[4], a1.y + s[5], a1.z + s[6], a1.w + s[7]};
    st<SA>((f32x4*)acc8, o0);
    st<SA>((f32x4*)acc8 + 1, o1);
}

template <int P, bool ACCUM, bool SA>
__global__ __launch_bounds__(kRsaBlock) void rsa_vec_kernel(
    float* __restrict__ acc, SmallTable<P> g, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * kRsaBlock;
    for (size_t i = (size_t)blockIdx.x * kRsaBlock + threadIdx.x; i < nvec; i += stride)
        rsa_update8<P, ACCUM, SA>(acc + 8 * i, g, P, 8 * i);
}

// Any p.
template <bool ACCUM, bool SA>
__global__ __launch_bounds__(kRsaBlock) void rsa_vec_anyp_kernel(
    float* __restrict__ acc, PtrTable g, int p, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * kRsaBlock;
    for (size_t i = (size_t)blockIdx.x * kRsaBlock + threadIdx.x; i < nvec; i += stride)
        rsa_update8<0, ACCUM, SA>(acc + 8 * i, g, p, 8 * i);
}

// Rank buffers that all start at the same non-zero offset `phase` (even, 2..14 bytes) inside
// their 16-byte lines -- what an odd shard size gives: rank g's slice of every buffer starts
// at g*S elements -- while the accumulator is aligned.  A lane rebuilds its 8 elements of each
// buffer from the two aligned vectors that hold them (funnel shift by the uniform phase); the
// second load of a lane is the first load of its neighbour, so memory traffic does not grow.
// g.ptr[q] is the buffer address rounded DOWN to 16 bytes; vectors [v_begin, v_end) are done
// here, and the launcher keeps v_begin >= 1 and v_end <= nvec - 1 so that both aligned loads
// stay inside the caller's buffers (the first and last 8 elements go the element-wise way).
__device__ __forceinline__ u32x4 funnel16(u32x4 lo, u32x4 hi, unsigned phase)
{
    uint32_t w0 = lo.x, w1 = lo.y, w2 = lo.z, w3 = lo.w, w4 = hi.x, w5 = hi.y, w6 = hi.z, w7 = hi.w;
    if (phase & 4) { w0 = w1; w1 = w2; w2 = w3; w3 = w4; w4 = w5; w5 = w6; w6 = w7; }
    if (phase & 8) { w0 = w2; w1 = w3; w2 = w4; w3 = w5; w4 = w6; }
    u32x4 out = {w0, w1, w2, w3};
    if (phase & 2) {
        out.x = (w0 >> 16) | (w1 << 16);
        out.y = (w1 >> 16) | (w2 << 16);
        out.z = (w2 >> 16) | (w3 << 16);
        out.w = (w3 >> 16) | (w4 << 16);
    }
    return out;
}

template <int P, bool ACCUM, bool SA, typename Tab>
__global__ __launch_bounds__(kRsaBlock) void rsa_shift_kernel(
    float* __restrict__ acc, Tab g, int p, unsigned phase, size_t v_begin, size_t v_end)
{
    const size_t stride = (size_t)gridDim.x * kRsaBlock;
    for (size_t i = v_begin + (size_t)blockIdx.x * kRsaBlock + threadIdx.x; i < v_end; i += stride) {
        f32x4 a0 = {0.0f, 0.0f, 0.0f, 0.0f}, a1 = a0;
        if (ACCUM) {
            a0 = ld<SA>((const f32x4*)acc + 2 * i);
            a1 = ld<SA>((const f32x4*)acc + 2 * i + 1);
        }
        float s[8];
        constexpr int B = P > 0 ? P : 16;
        for (int q0 = 0; q0 < p; q0 += B) {
            u32x4 lo[B], hi[B];
            #pragma unroll
            for (int b = 0; b < B; ++b) {
                if (q0 + b < p) {
                    lo[b] = ((const u32x4*)g.ptr[q0 + b])[i];
                    hi[b] = ((const u32x4*)g.ptr[q0 + b])[i + 1];
                }
            }
            #pragma unroll
            for (int b = 0; b < B; ++b) {
                if (q0 + b < p) {
                    const u32x4 v = funnel16(lo[b], hi[b], phase);
                    if (q0 + b == 0) {
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) { s[2 * e] = bf16_lo(v[e]); s[2 * e + 1] = bf16_hi(v[e]); }
                    } else {
                        #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            s[2 * e] = s[2 * e] + bf16_lo(v[e]);
                            s[2 * e + 1] = s[2 * e + 1] + bf16_hi(v[e]);
                        }
                    }
                }
            }
        }
        f32x4 o0 = {a0.x + s[0], a0.y + s[1], a0.z + s[2], a0.w + s[3]};
        f32x4 o1 = {a1.x + s[4], a1.y + s[5], a1.z + s[6], a1.w + s[7]};
        st<SA>((f32x4*)acc + 2 * i, o0);
        st<SA>((f32x4*)acc + 2 * i + 1, o1);
    }
}

// Coalesced form (many separately sharded tensors in one launch): workgroup x works on tile
// x - tile_begin[t] of segment t; a lane owns 8 consecutive elements of the segment, the last
// lane of a segment finishes a ragged end element by element.
struct ReduceSeg {
    unsigned long long count, src_off, dst_off;   // elements
};
struct ReduceSegTable {
    int n;
    unsigned tile_begin[kMaxSeg + 1];
    ReduceSeg seg[kMaxSeg];
};

template <int P, bool ACCUM, bool SA, typename Tab>
__global__ __launch_bounds__(kRsaBlock) void rsa_seg_kernel(
    float* __restrict__ acc, Tab g, int p, ReduceSegTable tab)
{
    const unsigned x = blockIdx.x;
    const int t = segment_of(tab.tile_begin, x);
    const size_t count = tab.seg[t].count, src = tab.seg[t].src_off, dst = tab.seg[t].dst_off;
    const size_t e0 = ((size_t)(x - tab.tile_begin[t]) * kRsaBlock + threadIdx.x) * 8;
    if (e0 >= count) return;
    if (e0 + 8 <= count) {
        rsa_update8<P, ACCUM, SA>(acc + dst + e0, g, p, src + e0);
    } else {
        for (size_t e = e0; e < count; ++e) {
            float partial = bf16_one(((const uint16_t*)g.ptr[0])[src + e]);
            for (int q = 1; q < p; ++q) partial = partial + bf16_one(((const uint16_t*)g.ptr[q])[src + e]);
            acc[dst + e] = (ACCUM ? acc[dst + e] : 0.0f) + partial;
        }
    }
}

// Gradients stored as IEEE binary16 (KIND 1: what mixed precision means on GPUs without bf16)
// or binary32 (KIND 2: plain float32 training).  Same reduction, same order; widening is exact.
// A lane owns one 128-bit vector per rank buffer: 8 binary16 or 4 binary32 elements.

template <int KIND>
__device__ __forceinline__ void widen_vec(float (&out)[8], u32x4 v)
{
    if constexpr (KIND == 1) {
        #pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t pair = v[e];
            out[2 * e] = (float)__builtin_bit_cast(_Float16, (uint16_t)(pair & 0xFFFFu));
            out[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(pair >> 16));
        }
    } else {
        #pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = __uint_as_float(v[e]);
    }
}

template <int KIND>
__device__ __forceinline__ float widen_one(const void* buf, size_t x)
{
    if constexpr (KIND == 1) return (float)((const _Float16*)buf)[x];
    else return ((const float*)buf)[x];
}

template <int KIND, int P, bool ACCUM, bool SA, typename Tab>
__global__ __launch_bounds__(kRsaBlock) void rsa_typed_vec_kernel(
    float* __restrict__ acc, Tab g, int p, size_t nvec)
{
    constexpr int EPV = KIND == 1 ? 8 : 4;     // elements per 128-bit vector
    const size_t stride = (size_t)gridDim.x * kRsaBlock;
    for (size_t i = (size_t)blockIdx.x * kRsaBlock + threadIdx.x; i < nvec; i += stride) {
        float a[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        if (ACCUM) {
            #pragma unroll
            for (int h = 0; h < EPV / 4; ++h) {
                const f32x4 t = ld<SA>((const f32x4*)acc + (EPV / 4) * i + h);
                a[4 * h] = t.x; a[4 * h + 1] = t.y; a[4 * h + 2] = t.z; a[4 * h + 3] = t.w;
            }
        }
        float s[8], w[8];
        if constexpr (P > 0) {
            u32x4 v[P];
            #pragma unroll
            for (int q = 0; q < P; ++q) v[q] = ld<kRsaNtl>((const u32x4*)g.ptr[q] + i);
            widen_vec<KIND>(s, v[0]);
            #pragma unroll
            for (int q = 1; q < P; ++q) {
                widen_vec<KIND>(w, v[q]);
                #pragma unroll
                for (int e = 0; e < EPV; ++e) s[e] = s[e] + w[e];
            }
        } else {
            constexpr int B = 32;
            widen_vec<KIND>(s, ld<kRsaNtl>((const u32x4*)g.ptr[0] + i));
            for (int q0 = 1; q0 < p; q0 += B) {
                u32x4 v[B];
                #pragma unroll
                for (int b = 0; b < B; ++b)
                    if (q0 + b < p) v[b] = ld<kRsaNtl>((const u32x4*)g.ptr[q0 + b] + i);
                #pragma unroll
                for (int b = 0; b < B; ++b) {
                    if (q0 + b < p) {
                        widen_vec<KIND>(w, v[b]);
                        #pragma unroll
                        for (int e = 0; e < EPV; ++e) s[e] = s[e] + w[e];
                    }
                }
            }
        }
        #pragma unroll
        for (int h = 0; h < EPV / 4; ++h) {
            const f32x4 o = {a[4 * h] + s[4 * h], a[4 * h + 1] + s[4 * h + 1], a[4 * h + 2] + s[4 * h + 2],
                             a[4 * h + 3] + s[4 * h + 3]};
            st<SA>((f32x4*)acc + (EPV / 4) * i + h, o);
        }
    }
}

template <int KIND, bool ACCUM>
__global__ __launch_bounds__(kBlock) void rsa_typed_scalar_kernel(
    float* __restrict__ acc, PtrTable g, int p, size_t first, size_t count)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t x = first + (size_t)blockIdx.x * kBlock + threadIdx.x; x < count; x += stride) {
        float partial = widen_one<KIND>(g.ptr[0], x);
        for (int q = 1; q < p; ++q) partial = partial + widen_one<KIND>(g.ptr[q], x);
        acc[x] = (ACCUM ? acc[x] : 0.0f) + partial;
    }
}

// One element per lane: the tail of the vector kernels (elements [first, count))
// and the whole range when some buffer is not 16-byte aligned.
template <bool ACCUM>
__global__ __launch_bounds__(kBlock) void rsa_scalar_kernel(
    float* __restrict__ acc, PtrTable g, int p, size_t first, size_t count)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t x = first + (size_t)blockIdx.x * kBlock + threadIdx.x; x < count; x += stride)
        acc[x] = rsa_element<ACCUM>(g, p, x, ACCUM ? acc[x] : 0.0f);
}

// ---------------------------------------------------------------------------
// Step 2b: reduction of the replication-group all-reduce at the accumulation
// boundary and the scaling to a mean (Section 3.4).  One lane owns 4 elements
// per copy and pass.  `out` may be copies[0]: a lane reads its elements of every copy
// before it writes them, and no other lane touches them.
// ---------------------------------------------------------------------------

// SO ("stream the output"): non-temporal stores for results too large for the Infinity Cache,
// as for the accumulator of the reduce kernels.
template <int R, bool SO>
__global__ __launch_bounds__(kAvgBlock) void avg_vec_kernel(
    float* out, SmallTable<R> a, float scale, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * kAvgBlock;
    for (size_t i = (size_t)blockIdx.x * kAvgBlock + threadIdx.x; i < nvec; i += stride) {
        f32x4 v[R];
        #pragma unroll
        for (int c = 0; c < R; ++c) v[c] = ld<kAvgNtl>((const f32x4*)a.ptr[c] + i);
        f32x4 sv = v[0];
        #pragma unroll
        for (int c = 1; c < R; ++c) sv = sv + v[c];
        st<SO>((f32x4*)out + i, sv * scale);
    }
}

template <bool SO>
__global__ __launch_bounds__(kAvgBlock) void avg_vec_anyr_kernel(
    float* out, PtrTable a, int r, float scale, size_t nvec)
{
    constexpr int B = 8;
    const size_t stride = (size_t)gridDim.x * kAvgBlock;
    for (size_t i = (size_t)blockIdx.x * kAvgBlock + threadIdx.x; i < nvec; i += stride) {
        f32x4 sum = ld<kAvgNtl>((const f32x4*)a.ptr[0] + i);
        for (int c0 = 1; c0 < r; c0 += B) {
            f32x4 v[B];
            #pragma unroll
            for (int b = 0; b < B; ++b)
                if (c0 + b < r) v[b] = ld<kAvgNtl>((const f32x4*)a.ptr[c0 + b] + i);
            #pragma unroll
            for (int b = 0; b < B; ++b)
                if (c0 + b < r) sum = sum + v[b];
        }
        st<SO>((f32x4*)out + i, sum * scale);
    }
}

__global__ __launch_bounds__(kBlock) void avg_scalar_kernel(
    float* out, PtrTable a, int r, float scale, size_t first, size_t count)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t x = first + (size_t)blockIdx.x * kBlock + threadIdx.x; x < count; x += stride) {
        float sum = ((const float*)a.ptr[0])[x];
        for (int c = 1; c < r; ++c) sum = sum + ((const float*)a.ptr[c])[x];
        out[x] = sum * scale;
    }
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

// One lane owns 4 consecutive elements per pass, so that every load and store instruction of
// a wavefront covers one contiguous kilobyte (stores that leave gaps between lanes reach
// memory as partial lines and cost extra traffic).  Four 128-bit loads are in flight before
// the first use; the bf16 parameters leave as one 64-bit store.
template <bool BF16>
__global__ __launch_bounds__(kAdamBlock) void adam_vec_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, const float* __restrict__ grad, size_t nvec, AdamScalars hp)
{
    const size_t stride = (size_t)gridDim.x * kAdamBlock;
    for (size_t i = (size_t)blockIdx.x * kAdamBlock + threadIdx.x; i < nvec; i += stride) {
        f32x4 g = ld<kAdamNtl>((const f32x4*)grad + i);
        f32x4 w = ld<kAdamNtl>((const f32x4*)master + i);
        f32x4 m = ld<kAdamNtl>((const f32x4*)exp_avg + i);
        f32x4 v = ld<kAdamNtl>((const f32x4*)exp_avg_sq + i);
        #pragma unroll
        for (int e = 0; e < 4; ++e) {
            float we = w[e], me = m[e], ve = v[e];
            adam_element(we, me, ve, g[e], hp);
            w[e] = we; m[e] = me; v[e] = ve;
        }
        st<kAdamNts>((f32x4*)master + i, w);
        st<kAdamNts>((f32x4*)exp_avg + i, m);
        st<kAdamNts>((f32x4*)exp_avg_sq + i, v);
        if (BF16) {
            u32x2 b = {bf16_pack(w.x, w.y), bf16_pack(w.z, w.w)};
            st<kAdamNts>((u32x2*)param_bf16 + i, b);
        }
    }
}

// Replica average fused into the Adam step: the averaged gradient of a lane's 4 elements is
// formed in registers from the r accumulator copies (same additions, same order, same multiply
// as avg_vec_kernel) and goes straight into adam_element, so it is neither written nor re-read:
// 4r + 12 bytes read and 14 written per element instead of (4r + 4) + 30.  R > 0: r = R at
// compile time; R == 0: any r in batches of 8 loads.
template <int R, bool BF16, typename Tab>
__global__ __launch_bounds__(kAdamBlock) void avg_adam_vec_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, Tab a, int r, float scale, size_t nvec, AdamScalars hp)
{
    const size_t stride = (size_t)gridDim.x * kAdamBlock;
    for (size_t i = (size_t)blockIdx.x * kAdamBlock + threadIdx.x; i < nvec; i += stride) {
        f32x4 w = ld<kAdamNtl>((const f32x4*)master + i);
        f32x4 m = ld<kAdamNtl>((const f32x4*)exp_avg + i);
        f32x4 v = ld<kAdamNtl>((const f32x4*)exp_avg_sq + i);
        f32x4 sum;
        if constexpr (R > 0) {
            f32x4 c[R];
            #pragma unroll
            for (int q = 0; q < R; ++q) c[q] = ld<kAdamNtl>((const f32x4*)a.ptr[q] + i);
            sum = c[0];
            #pragma unroll
            for (int q = 1; q < R; ++q) sum = sum + c[q];
        } else {
            constexpr int B = 8;
            sum = ld<kAdamNtl>((const f32x4*)a.ptr[0] + i);
            for (int q0 = 1; q0 < r; q0 += B) {
                f32x4 c[B];
                #pragma unroll
                for (int b = 0; b < B; ++b)
                    if (q0 + b < r) c[b] = ld<kAdamNtl>((const f32x4*)a.ptr[q0 + b] + i);
                #pragma unroll
                for (int b = 0; b < B; ++b)
                    if (q0 + b < r) sum = sum + c[b];
            }
        }
        const f32x4 g = sum * scale;
        #pragma unroll
        for (int e = 0; e < 4; ++e) {
            float we = w[e], me = m[e], ve = v[e];
            adam_element(we, me, ve, g[e], hp);
            w[e] = we; m[e] = me; v[e] = ve;
        }
        st<kAdamNts>((f32x4*)master + i, w);
        st<kAdamNts>((f32x4*)exp_avg + i, m);
        st<kAdamNts>((f32x4*)exp_avg_sq + i, v);
        if (BF16) {
            u32x2 b = {bf16_pack(w.x, w.y), bf16_pack(w.z, w.w)};
            st<kAdamNts>((u32x2*)param_bf16 + i, b);
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void avg_adam_scalar_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, PtrTable a, int r, float scale, size_t first, size_t count,
    AdamScalars hp)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t x = first + (size_t)blockIdx.x * kBlock + threadIdx.x; x < count; x += stride) {
        float sum = ((const float*)a.ptr[0])[x];
        for (int c = 1; c < r; ++c) sum = sum + ((const float*)a.ptr[c])[x];
        const float g = sum * scale;
        float w = master[x], m = exp_avg[x], v = exp_avg_sq[x];
        adam_element(w, m, v, g, hp);
        master[x] = w; exp_avg[x] = m; exp_avg_sq[x] = v;
        if (BF16) param_bf16[x] = bf16_single(w);
    }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void adam_scalar_kernel(
    float* __restrict__ master, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
    uint16_t* __restrict__ param_bf16, const float* __restrict__ grad, size_t first, size_t count,
    AdamScalars hp)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t x = first + (size_t)blockIdx.x * kBlock + threadIdx.x; x < count; x += stride) {
        float w = master[x], m = exp_avg[x], v = exp_avg_sq[x];
        adam_element(w, m, v, grad[x], hp);
        master[x] = w; exp_avg[x] = m; exp_avg_sq[x] = v;
        if (BF16) param_bf16[x] = bf16_single(w);
    }
}

// ---------------------------------------------------------------------------
// Launch helpers
// ---------------------------------------------------------------------------

std::atomic<int> g_blocks_per_cu{0};

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

constexpr int kTailBpc = 8;

inline int launch_status()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? 0 : (int)e;
}

// Accumulators up to this size are left cacheable, larger ones are streamed (see rsa_update8).
constexpr size_t kAccCacheableBytes = 224u << 20;
inline bool stream_acc(size_t elements) { return elements * 4 > kAccCacheableBytes; }

// Calls f(std::bool_constant<a>, std::bool_constant<b>) for two runtime flags.
template <typename F>
void dispatch2(bool a, bool b, F&& f)
{
    if (a) { if (b) f(std::true_type{}, std::true_type{}); else f(std::true_type{}, std::false_type{}); }
    else   { if (b) f(std::false_type{}, std::true_type{}); else f(std::false_type{}, std::false_type{}); }
}

template <int N>
SmallTable<N> small(const PtrTable& t)
{
    SmallTable<N> s;
    for (int i = 0; i < N; ++i) s.ptr[i] = t.ptr[i];
    return s;
}

template <int P>
void rsa_launch_fixed(float* acc, const PtrTable& g, size_t nvec, bool accumulate, unsigned blocks,
                      hipStream_t st)
{
    dispatch2(accumulate, stream_acc(nvec * 8), [&](auto A, auto SA) {
        hipLaunchKernelGGL((rsa_vec_kernel<P, A.value, SA.value>), dim3(blocks), dim3(kRsaBlock), 0, st, acc,
                           small<P>(g), nvec);
    });
}

template <int R>
void avg_launch_fixed(float* out, const PtrTable& a, float scale, size_t nvec, unsigned blocks,
                      hipStream_t st)
{
    dispatch2(stream_acc(nvec * 4), false, [&](auto SO, auto) {
        hipLaunchKernelGGL((avg_vec_kernel<R, SO.value>), dim3(blocks), dim3(kAvgBlock), 0, st, out,
                           small<R>(a), scale, nvec);
    });
}

}  // namespace

void set_blocks_per_cu(int n) { g_blocks_per_cu.store(n); }

const char* hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

int launch_reorder(void* dst, const PtrTable& src, size_t n_valid_bytes, size_t shard_bytes, int p,
                   int k, bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned total = 0;
    if (vec16) {
        // spread the block budget over the p chunks
        if (int e = grid_for(shard_bytes / 16 * (size_t)p, kReorderBlock, MICS_REORDER_BPC, &total)) return e;
        unsigned bx = (total + (unsigned)p - 1) / (unsigned)p;
        hipLaunchKernelGGL(reorder_vec_kernel, dim3(bx, (unsigned)p), dim3(kReorderBlock), 0, st,
                           (u32x4*)dst, src, shard_bytes / 16, n_valid_bytes, k);
    } else {
        size_t tiles = (shard_bytes + 15 + kTileBytes - 1) / kTileBytes + 1;
        if (int e = grid_for(tiles * (size_t)p * kBlock, kBlock, MICS_REORDER_BPC, &total)) return e;
        unsigned bx = (total + (unsigned)p - 1) / (unsigned)p;
        if (bx > tiles) bx = (unsigned)tiles;
        hipLaunchKernelGGL(reorder_lds_kernel, dim3(bx, (unsigned)p), dim3(kBlock), 0, st,
                           (unsigned char*)dst, src, shard_bytes, n_valid_bytes, k);
    }
    return launch_status();
}

namespace {
void rsa_scalar_launch(float* acc, const PtrTable& g, int p, size_t first, size_t end, bool accumulate,
                       unsigned blocks, hipStream_t st)
{
    if (accumulate)
        hipLaunchKernelGGL(rsa_scalar_kernel<true>, dim3(blocks), dim3(kBlock), 0, st, acc, g, p, first, end);
    else
        hipLaunchKernelGGL(rsa_scalar_kernel<false>, dim3(blocks), dim3(kBlock), 0, st, acc, g, p, first, end);
}
}  // namespace

// grad_phase: 0 = every buffer 16-byte aligned (with an aligned accumulator); 2..14 = every
// gradient buffer starts that many bytes into a 16-byte line (accumulator aligned); -1 = no
// common alignment: element-wise kernel.
int launch_reduce_scatter_accum(float* acc, const PtrTable& g, size_t count, int p, bool accumulate,
                                int grad_phase, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    unsigned blocks = 0;
    const size_t nvec_all = count / 8;
    if (grad_phase > 0 && nvec_all >= 3) {
        // middle vectors through the shift kernel, first and last 8 (+ tail) elements one by one
        PtrTable down{};
        for (int q = 0; q < p; ++q) down.ptr[q] = (const char*)g.ptr[q] - grad_phase;
        const size_t v_begin = 1, v_end = nvec_all - 1;
        if (int e = grid_for(v_end - v_begin, kRsaBlock, MICS_RSA_BPC, &blocks)) return e;
        dispatch2(accumulate, stream_acc(count), [&](auto A, auto SA) {
            if (p == 16)
                hipLaunchKernelGGL((rsa_shift_kernel<16, A.value, SA.value, SmallTable<16>>), dim3(blocks),
                                   dim3(kRsaBlock), 0, st, acc, small<16>(down), p, (unsigned)grad_phase,
                                   v_begin, v_end);
            else
                hipLaunchKernelGGL((rsa_shift_kernel<0, A.value, SA.value, PtrTable>), dim3(blocks),
                                   dim3(kRsaBlock), 0, st, acc, down, p, (unsigned)grad_phase, v_begin, v_end);
        });
        if (int e = launch_status()) return e;
        if (int e = grid_for(8, kBlock, kTailBpc, &blocks)) return e;
        rsa_scalar_launch(acc, g, p, 0, 8, accumulate, blocks, st);
        if (int e = launch_status()) return e;
        if (int e = grid_for(count - v_end * 8, kBlock, kTailBpc, &blocks)) return e;
        rsa_scalar_launch(acc, g, p, v_end * 8, count, accumulate, blocks, st);
        return launch_status();
    }
    const size_t nvec = grad_phase == 0 ? nvec_all : 0;
    if (nvec) {
        if (int e = grid_for(nvec, kRsaBlock, MICS_RSA_BPC, &blocks)) return e;
        switch (p) {
            case 1: rsa_launch_fixed<1>(acc, g, nvec, accumulate, blocks, st); break;
            case 2: rsa_launch_fixed<2>(acc, g, nvec, accumulate, blocks, st); break;
            case 4: rsa_launch_fixed<4>(acc, g, nvec, accumulate, blocks, st); break;
            case 8: rsa_launch_fixed<8>(acc, g, nvec, accumulate, blocks, st); break;
            case 16: rsa_launch_fixed<16>(acc, g, nvec, accumulate, blocks, st); break;
            case 32: rsa_launch_fixed<32>(acc, g, nvec, accumulate, blocks, st); break;
            default:
                dispatch2(accumulate, stream_acc(count), [&](auto A, auto SA) {
                    hipLaunchKernelGGL((rsa_vec_anyp_kernel<A.value, SA.value>), dim3(blocks),
                                       dim3(kRsaBlock), 0, st, acc, g, p, nvec);
                });
        }
        if (int e = launch_status()) return e;
    }
    const size_t first = nvec * 8;
    if (first < count) {
        if (int e = grid_for(count - first, kBlock, kTailBpc, &blocks)) return e;
        rsa_scalar_launch(acc, g, p, first, count, accumulate, blocks, st);
        if (int e = launch_status()) return e;
    }
    return 0;
}

int launch_replica_average(float* out, const PtrTable& a, size_t count, int r, float scale,
                           bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t nvec = vec16 ? count / 4 : 0;
    unsigned blocks = 0;
    if (nvec) {
        if (int e = grid_for(nvec, kAvgBlock, MICS_AVG_BPC, &blocks)) return e;
        switch (r) {
            case 1: avg_launch_fixed<1>(out, a, scale, nvec, blocks, st); break;
            case 2: avg_launch_fixed<2>(out, a, scale, nvec, blocks, st); break;
            case 4: avg_launch_fixed<4>(out, a, scale, nvec, blocks, st); break;
            case 8: avg_launch_fixed<8>(out, a, scale, nvec, blocks, st); break;
            default:
                dispatch2(stream_acc(count), false, [&](auto SO, auto) {
                    hipLaunchKernelGGL(avg_vec_anyr_kernel<SO.value>, dim3(blocks), dim3(kAvgBlock), 0, st,
                                       out, a, r, scale, nvec);
                });
        }
        if (int e = launch_status()) return e;
    }
    const size_t first = nvec * 4;
    if (first < count) {
        if (int e = grid_for(count - first, kBlock, kTailBpc, &blocks)) return e;
        hipLaunchKernelGGL(avg_scalar_kernel, dim3(blocks), dim3(kBlock), 0, st, out, a, r, scale,
                           first, count);
        if (int e = launch_status()) return e;
    }
    return 0;
}

int launch_adam(float* master, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16,
                const float* grad, size_t count, const AdamScalars& hp, bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t nvec = vec16 ? count / 4 : 0;
    unsigned blocks = 0;
    if (nvec) {
        if (int e = grid_for(nvec, kAdamBlock, MICS_ADAM_BPC, &blocks)) return e;
        if (param_bf16)
            hipLaunchKernelGGL(adam_vec_kernel<true>, dim3(blocks), dim3(kAdamBlock), 0, st, master,
                               exp_avg, exp_avg_sq, param_bf16, grad, nvec, hp);
        else
            hipLaunchKernelGGL(adam_vec_kernel<false>, dim3(blocks), dim3(kAdamBlock), 0, st,
                               master, exp_avg, exp_avg_sq, param_bf16, grad, nvec, hp);
        if (int e = launch_status()) return e;
    }
    const size_t first = nvec * 4;
    if (first < count) {
        if (int e = grid_for(count - first, kBlock, kTailBpc, &blocks)) return e;
        if (param_bf16)
            hipLaunchKernelGGL(adam_scalar_kernel<true>, dim3(blocks), dim3(kBlock), 0, st, master,
                               exp_avg, exp_avg_sq, param_bf16, grad, first, count, hp);
        else
            hipLaunchKernelGGL(adam_scalar_kernel<false>, dim3(blocks), dim3(kBlock), 0, st, master,
                               exp_avg, exp_avg_sq, param_bf16, grad, first, count, hp);
        if (int e = launch_status()) return e;
    }
    return 0;
}

int launch_reorder_coalesced(void* dst, const PtrTable& src, const Segment* segs, int n, int p, int k,
                             int elem_bytes, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t eb = (size_t)elem_bytes;
    for (int first = 0; first < n; first += kMaxSeg) {
        ReorderSegTable tab;
        tab.n = n - first < kMaxSeg ? n - first : kMaxSeg;
        size_t tiles = 0;
        for (int t = 0; t < tab.n; ++t) {
            const Segment& sg = segs[first + t];
            tab.tile_begin[t] = (unsigned)tiles;
            tab.seg[t].shard_vecs = sg.shard_elems * eb / 16;
            tab.seg[t].valid_bytes = sg.numel * eb;
            tab.seg[t].src_vec = sg.src_offset * eb / 16;
            tab.seg[t].dst_vec = sg.dst_offset * eb / 16;
            tiles += (tab.seg[t].shard_vecs + kSegTileVecs - 1) / kSegTileVecs;
            if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
        }
        for (int t = tab.n; t <= kMaxSeg; ++t) tab.tile_begin[t] = 0xFFFFFFFFu;
        if (tiles == 0) continue;
        hipLaunchKernelGGL(reorder_seg_kernel, dim3((unsigned)tiles, (unsigned)p), dim3(kSegBlock),
                           0, st, (u32x4*)dst, src, tab, k);
        if (int e = launch_status()) return e;
    }
    return 0;
}

namespace {
template <int P>
void rsa_seg_launch(float* acc, const PtrTable& g, int p, const ReduceSegTable& tab, unsigned tiles,
                    bool accumulate, bool sa, hipStream_t st)
{
    dispatch2(accumulate, sa, [&](auto A, auto SA) {
        if constexpr (P > 0)
            hipLaunchKernelGGL((rsa_seg_kernel<P, A.value, SA.value, SmallTable<P>>), dim3(tiles),
                               dim3(kRsaBlock), 0, st, acc, small<P>(g), p, tab);
        else
            hipLaunchKernelGGL((rsa_seg_kernel<0, A.value, SA.value, PtrTable>), dim3(tiles), dim3(kRsaBlock),
                               0, st, acc, g, p, tab);
    });
}
}  // namespace

int launch_reduce_coalesced(float* acc, const PtrTable& g, const Segment* segs, int n, int p,
                            bool accumulate, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    constexpr size_t kTileElems = (size_t)kRsaBlock * 8;
    for (int first = 0; first < n; first += kMaxSeg) {
        ReduceSegTable tab;
        tab.n = n - first < kMaxSeg ? n - first : kMaxSeg;
        size_t tiles = 0, elements = 0;
        for (int t = 0; t < tab.n; ++t) {
            const Segment& sg = segs[first + t];
            elements += sg.numel;
            tab.tile_begin[t] = (unsigned)tiles;
            tab.seg[t].count = sg.numel;
            tab.seg[t].src_off = sg.src_offset;
            tab.seg[t].dst_off = sg.dst_offset;
            tiles += (sg.numel + kTileElems - 1) / kTileElems;
            if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
        }
        for (int t = tab.n; t <= kMaxSeg; ++t) tab.tile_begin[t] = 0xFFFFFFFFu;
        if (tiles == 0) continue;
        switch (p) {
            case 1: rsa_seg_launch<1>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            case 2: rsa_seg_launch<2>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            case 4: rsa_seg_launch<4>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            case 8: rsa_seg_launch<8>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            case 16: rsa_seg_launch<16>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            case 32: rsa_seg_launch<32>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st); break;
            default: rsa_seg_launch<0>(acc, g, p, tab, (unsigned)tiles, accumulate, stream_acc(elements), st);
        }
        if (int e = launch_status()) return e;
    }
    return 0;
}

namespace {
template <int R, bool BF16>
void avg_adam_launch(float* w, float* m, float* v, uint16_t* pb, const PtrTable& a, int r, float scale,
                     size_t nvec, const AdamScalars& hp, unsigned blocks, hipStream_t st)
{
    if constexpr (R > 0)
        hipLaunchKernelGGL((avg_adam_vec_kernel<R, BF16, SmallTable<R>>), dim3(blocks), dim3(kAdamBlock), 0,
                           st, w, m, v, pb, small<R>(a), r, scale, nvec, hp);
    else
        hipLaunchKernelGGL((avg_adam_vec_kernel<0, BF16, PtrTable>), dim3(blocks), dim3(kAdamBlock), 0, st,
                           w, m, v, pb, a, r, scale, nvec, hp);
}

template <bool BF16>
void avg_adam_dispatch(float* w, float* m, float* v, uint16_t* pb, const PtrTable& a, int r, float scale,
                       size_t nvec, const AdamScalars& hp, unsigned blocks, hipStream_t st)
{
    switch (r) {
        case 1: avg_adam_launch<1, BF16>(w, m, v, pb, a, r, scale, nvec, hp, blocks, st); break;
        case 2: avg_adam_launch<2, BF16>(w, m, v, pb, a, r, scale, nvec, hp, blocks, st); break;
        case 4: avg_adam_launch<4, BF16>(w, m, v, pb, a, r, scale, nvec, hp, blocks, st); break;
        case 8: avg_adam_launch<8, BF16>(w, m, v, pb, a, r, scale, nvec, hp, blocks, st); break;
        default: avg_adam_launch<0, BF16>(w, m, v, pb, a, r, scale, nvec, hp, blocks, st);
    }
}
}  // namespace

int launch_avg_adam(float* master, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16,
                    const PtrTable& copies, int r, float scale, size_t count, const AdamScalars& hp,
                    bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const size_t nvec = vec16 ? count / 4 : 0;
    unsigned blocks = 0;
    if (nvec) {
        if (int e = grid_for(nvec, kAdamBlock, MICS_ADAM_BPC, &blocks)) return e;
        if (param_bf16)
            avg_adam_dispatch<true>(master, exp_avg, exp_avg_sq, param_bf16, copies, r, scale, nvec, hp,
                                    blocks, st);
        else
            avg_adam_dispatch<false>(master, exp_avg, exp_avg_sq, param_bf16, copies, r, scale, nvec, hp,
                                     blocks, st);
        if (int e = launch_status()) return e;
    }
    const size_t first = nvec * 4;
    if (first < count) {
        if (int e = grid_for(count - first, kBlock, kTailBpc, &blocks)) return e;
        if (param_bf16)
            hipLaunchKernelGGL(avg_adam_scalar_kernel<true>, dim3(blocks), dim3(kBlock), 0, st, master,
                               exp_avg, exp_avg_sq, param_bf16, copies, r, scale, first, count, hp);
        else
            hipLaunchKernelGGL(avg_adam_scalar_kernel<false>, dim3(blocks), dim3(kBlock), 0, st, master,
                               exp_avg, exp_avg_sq, param_bf16, copies, r, scale, first, count, hp);
        if (int e = launch_status()) return e;
    }
    return 0;
}

namespace {
template <int KIND, int P, bool ACCUM>
void rsa_typed_launch(float* acc, const PtrTable& g, int p, size_t nvec, bool sa, unsigned blocks,
                      hipStream_t st)
{
    dispatch2(sa, false, [&](auto SA, auto) {
        if constexpr (P > 0)
            hipLaunchKernelGGL((rsa_typed_vec_kernel<KIND, P, ACCUM, SA.value, SmallTable<P>>), dim3(blocks),
                               dim3(kRsaBlock), 0, st, acc, small<P>(g), p, nvec);
        else
            hipLaunchKernelGGL((rsa_typed_vec_kernel<KIND, 0, ACCUM, SA.value, PtrTable>), dim3(blocks),
                               dim3(kRsaBlock), 0, st, acc, g, p, nvec);
    });
}

template <int KIND, bool ACCUM>
int rsa_typed_all(float* acc, const PtrTable& g, size_t count, int p, bool vec16, hipStream_t st)
{
    constexpr size_t EPV = KIND == 1 ? 8 : 4;
    const size_t nvec = vec16 ? count / EPV : 0;
    unsigned blocks = 0;
    if (nvec) {
        if (int e = grid_for(nvec, kRsaBlock, MICS_RSA_BPC, &blocks)) return e;
        switch (p) {
            case 8: rsa_typed_launch<KIND, 8, ACCUM>(acc, g, p, nvec, stream_acc(count), blocks, st); break;
            case 16: rsa_typed_launch<KIND, 16, ACCUM>(acc, g, p, nvec, stream_acc(count), blocks, st); break;
            default: rsa_typed_launch<KIND, 0, ACCUM>(acc, g, p, nvec, stream_acc(count), blocks, st);
        }
        if (int e = launch_status()) return e;
    }
    const size_t first = nvec * EPV;
    if (first < count) {
        if (int e = grid_for(count - first, kBlock, kTailBpc, &blocks)) return e;
        hipLaunchKernelGGL((rsa_typed_scalar_kernel<KIND, ACCUM>), dim3(blocks), dim3(kBlock), 0, st, acc, g,
                           p, first, count);
        if (int e = launch_status()) return e;
    }
    return 0;
}
}  // namespace

int launch_reduce_scatter_accum_typed(float* acc, const PtrTable& g, size_t count, int p,
                                      bool accumulate, int kind, bool vec16, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (kind == 1)
        return accumulate ? rsa_typed_all<1, true>(acc, g, count, p, vec16, st)
                          : rsa_typed_all<1, false>(acc, g, count, p, vec16, st);
    return accumulate ? rsa_typed_all<2, true>(acc, g, count, p, vec16, st)
                      : rsa_typed_all<2, false>(acc, g, count, p, vec16, st);
}

}  // namespace mics
