// One small training step of a rank through the C ABI of libmics, from a plain host program:
// hipMalloc'd buffers, a stream of its own, no Python and no PyTorch.  The inputs are chosen
// so that every result has a closed form the program can check by itself (exact integer sums,
// a power-of-two average, Adam's first step on a constant gradient, Sections 3.3, 3.4, 2.1).
// Exit status 0 = every check passed.
//
// Build (done by paper_2205_00119_amd/build.py):
//   hipcc --offload-arch=gfx950 -O2 step_from_c.cpp -I../../include -L.. -lmics -Wl,-rpath,'$ORIGIN/..'
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "mics.h"

#define HIP_OK(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                   \
            return 2;                                                                         \
        }                                                                                     \
    } while (0)
#define MICS_OK_OR_FAIL(call)                                                                 \
    do {                                                                                      \
        if ((call) != MICS_OK) {                                                              \
            std::fprintf(stderr, "%s: %s\n", #call, mics_last_error());                       \
            return 3;                                                                         \
        }                                                                                     \
    } while (0)

static uint16_t bf16_of_small_int(int v)       // exact for |v| < 256
{
    float f = (float)v;
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static float widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

int main()
{
    const int p = 4, k = 2, r = 2, s = 2;
    const size_t S = mics_shard_elems(4 * 4100 - 5, p, 8);      // 4104
    const size_t n_pad = S * p, n_valid = n_pad - 5;
    const int g_rank = 3;                                       // the rank whose shard is updated
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));

    // ---- step 1: stage-1 buffers T_l = [C_l, C_{k+l}], element (g, i) tagged with its flat index
    std::vector<uint16_t> h_T[k];
    uint16_t* d_T[k];
    for (int l = 0; l < k; ++l) {
        h_T[l].resize((size_t)(p / k) * S);
        for (int j = 0; j < p / k; ++j)
            for (size_t i = 0; i < S; ++i) h_T[l][(size_t)j * S + i] = (uint16_t)(((size_t)(j * k + l) * S + i) * 7u);
        HIP_OK(hipMalloc((void**)&d_T[l], h_T[l].size() * 2));
        HIP_OK(hipMemcpy(d_T[l], h_T[l].data(), h_T[l].size() * 2, hipMemcpyHostToDevice));
    }
    uint16_t* d_F;
    HIP_OK(hipMalloc((void**)&d_F, n_pad * 2));
    HIP_OK(hipMemset(d_F, 0xEE, n_pad * 2));
    const void* tab_T[k] = {d_T[0], d_T[1]};
    MICS_OK_OR_FAIL(mics_hier_gather_reorder(d_F, tab_T, n_valid, S, p, k, 2, st));
    std::vector<uint16_t> h_F(n_pad);
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipMemcpy(h_F.data(), d_F, n_pad * 2, hipMemcpyDeviceToHost));
    for (size_t x = 0; x < n_pad; ++x) {
        const uint16_t want = x < n_valid ? (uint16_t)(x * 7u) : (uint16_t)0xEEEE;
        if (h_F[x] != want) { std::fprintf(stderr, "reorder: element %zu\n", x); return 1; }
    }
    std::puts("ok gather-reorder");

    // ---- step 2a: p rank buffers of small integers, s micro-steps into the shard of rank g_rank
    uint16_t* d_g[p];
    std::vector<uint16_t> h_g(n_pad);
    for (int q = 0; q < p; ++q) {
        for (size_t x = 0; x < n_pad; ++x) h_g[x] = bf16_of_small_int((int)((x + 3 * q) % 7) - 3);
        HIP_OK(hipMalloc((void**)&d_g[q], n_pad * 2));
        HIP_OK(hipMemcpy(d_g[q], h_g.data(), n_pad * 2, hipMemcpyHostToDevice));
    }
    float* d_acc;
    HIP_OK(hipMalloc((void**)&d_acc, S * 4));
    const uint16_t* tab_g[p] = {d_g[0], d_g[1], d_g[2], d_g[3]};
    for (int t = 0; t < s; ++t)
        MICS_OK_OR_FAIL(mics_reduce_scatter_accum(d_acc, tab_g, (size_t)g_rank * S, S, p, t > 0, st));
    std::vector<float> h_acc(S);
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipMemcpy(h_acc.data(), d_acc, S * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < S; ++i) {
        const size_t x = (size_t)g_rank * S + i;
        int sum = 0;
        for (int q = 0; q < p; ++q) sum += (int)((x + 3 * q) % 7) - 3;
        if (h_acc[i] != (float)(s * sum)) { std::fprintf(stderr, "reduce: element %zu\n", i); return 1; }
    }
    std::puts("ok reduce-scatter-accumulate");

    // ---- step 2b: the other replica's copy is 8 - acc, so the sum is 8 and the mean (scale 1/8) is 1
    std::vector<float> h_other(S);
    for (size_t i = 0; i < S; ++i) h_other[i] = 8.0f - h_acc[i];
    float *d_other, *d_avg;
    HIP_OK(hipMalloc((void**)&d_other, S * 4));
    HIP_OK(hipMalloc((void**)&d_avg, S * 4));
    HIP_OK(hipMemcpy(d_other, h_other.data(), S * 4, hipMemcpyHostToDevice));
    const float* tab_a[r] = {d_acc, d_other};
    MICS_OK_OR_FAIL(mics_replica_average(d_avg, tab_a, S, r, 0.125f, st));

    // ---- step 3: Adam's first step on the constant gradient 1: w' = w - lr / (1 + eps)
    const float lr = 1e-3f, eps = 1e-8f;
    std::vector<float> h_w(S), zero(S, 0.0f);
    for (size_t i = 0; i < S; ++i) h_w[i] = 0.02f * (float)((int)(i % 201) - 100) / 100.0f;
    float *d_w, *d_m, *d_v;
    uint16_t* d_pb;
    HIP_OK(hipMalloc((void**)&d_w, S * 4));
    HIP_OK(hipMalloc((void**)&d_m, S * 4));
    HIP_OK(hipMalloc((void**)&d_v, S * 4));
    HIP_OK(hipMalloc((void**)&d_pb, S * 2));
    HIP_OK(hipMemcpy(d_w, h_w.data(), S * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_m, zero.data(), S * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_v, zero.data(), S * 4, hipMemcpyHostToDevice));
    MICS_OK_OR_FAIL(mics_adam_shard(d_w, d_m, d_v, d_pb, d_avg, S, lr, 0.9f, 0.999f, eps, 0.0f, 1, st));
    std::vector<float> h_avg(S), h_w2(S);
    std::vector<uint16_t> h_pb(S);
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipMemcpy(h_avg.data(), d_avg, S * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_w2.data(), d_w, S * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_pb.data(), d_pb, S * 2, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < S; ++i) {
        if (h_avg[i] != 1.0f) { std::fprintf(stderr, "average: element %zu = %g\n", i, h_avg[i]); return 1; }
        const double want = (double)h_w[i] - (double)lr / (1.0 + (double)eps);
        const double scale = std::fmax(std::fabs(want), std::fabs((double)h_w[i]));
        if (std::fabs((double)h_w2[i] - want) > 1e-6 * scale) { std::fprintf(stderr, "Adam: element %zu\n", i); return 1; }
        // the bf16 copy is the nearest bf16 value: within half a unit of its last place (2^-8 relative)
        if (std::fabs((double)widen_bf16(h_pb[i]) - (double)h_w2[i]) > std::ldexp(std::fabs((double)h_w2[i]), -8)) {
            std::fprintf(stderr, "bf16 parameter: element %zu\n", i);
            return 1;
        }
    }
    std::puts("ok replica-average");
    std::puts("ok adam-shard");

    // an argument error comes back as a code and a text, and enqueues nothing
    if (mics_hier_gather_reorder(d_F, tab_T, n_valid, S, p, 3, 2, st) != MICS_ERR_INVALID_ARG) return 1;
    std::printf("ok error path: %s\n", mics_last_error());
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipStreamDestroy(st));
    std::printf("libmics %d: all checks passed\n", mics_version());
    return 0;
}
