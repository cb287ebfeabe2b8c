// Exercises every entry point's host-side path (accepting and rejecting) with fake device addresses.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mics.h"
#include "mics_tuning.h"

namespace mics { extern int g_launches; }

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "%s:%d: %s [%s]\n", __FILE__, __LINE__, #cond, mics_last_error()); std::exit(1); } } while (0)

int main()
{
    auto fake = [](size_t i) { return reinterpret_cast<void*>(0x7F0000000000ull + (i << 28)); };
    std::vector<const void*> tab(MICS_MAX_GROUP);
    for (int i = 0; i < MICS_MAX_GROUP; ++i) tab[i] = fake(i + 8);
    void* A = fake(1);

    // accepted calls reach a launcher exactly once, whatever the alignment
    int before = mics::g_launches;
    CHECK(mics_hier_gather_reorder(A, tab.data(), 4 * 1000 - 3, 1000, 4, 2, 2, nullptr) == MICS_OK);
    CHECK(mics_hier_gather_reorder(A, tab.data(), 128 * 8, 8, 128, 8, 4, nullptr) == MICS_OK);
    CHECK(mics_reduce_scatter_accum((float*)A, (const uint16_t* const*)tab.data(), 1000, 999, 16, 1, nullptr) == MICS_OK);
    CHECK(mics_reduce_scatter_accum_typed((float*)A, tab.data(), 8, 4096, 128, 0, MICS_DTYPE_F32, nullptr) == MICS_OK);
    CHECK(mics_replica_average((float*)A, (const float* const*)tab.data(), 12345, 8, 0.5f, nullptr) == MICS_OK);
    tab[0] = A;   // in place on the first copy
    CHECK(mics_replica_average((float*)A, (const float* const*)tab.data(), 12345, 8, 0.5f, nullptr) == MICS_OK);
    tab[0] = fake(8);
    CHECK(mics_adam_shard((float*)fake(1), (float*)fake(2), (float*)fake(3), (uint16_t*)fake(4), (const float*)fake(5),
                          777, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 3, nullptr) == MICS_OK);
    CHECK(mics_adam_shard((float*)fake(1), (float*)fake(2), (float*)fake(3), nullptr, (const float*)fake(5),
                          777, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, nullptr) == MICS_OK);
    CHECK(mics_replica_average_adam_shard((float*)fake(1), (float*)fake(2), (float*)fake(3), (uint16_t*)fake(4),
                                          (const float* const*)tab.data(), 777, 128, 0.25f, 1e-4f, 0.9f, 0.999f,
                                          1e-8f, 0.0f, 1, nullptr) == MICS_OK);
    CHECK(mics::g_launches == before + 9);
    before = mics::g_launches;
    CHECK(mics_adam_shard_typed((float*)fake(1), (float*)fake(2), (float*)fake(3), fake(4), MICS_DTYPE_F16,
                                (const float*)fake(5), 777, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 3, nullptr) == MICS_OK);
    CHECK(mics_replica_average_adam_shard_typed((float*)fake(1), (float*)fake(2), (float*)fake(3), fake(4),
                                                MICS_DTYPE_F16, (const float* const*)tab.data(), 777, 128, 0.25f,
                                                1e-4f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, nullptr) == MICS_OK);
    CHECK(mics_adam_shard_typed((float*)fake(1), (float*)fake(2), (float*)fake(3), fake(4), MICS_DTYPE_F32,
                                (const float*)fake(5), 777, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 3, nullptr)
          == MICS_ERR_UNSUPPORTED);
    CHECK(mics::g_launches == before + 2);
    // misaligned buffers and odd counts still cost one launch
    before = mics::g_launches;
    for (int i = 0; i < 16; ++i) tab[i] = (const char*)fake(i + 8) + 2 * (i % 2) + 6;
    CHECK(mics_reduce_scatter_accum((float*)((char*)A + 4), (const uint16_t* const*)tab.data(), 1001, 999, 16, 1, nullptr) == MICS_OK);
    for (int i = 0; i < 16; ++i) tab[i] = (const char*)fake(i + 8) + 4 * (i % 3);
    CHECK(mics_replica_average((float*)((char*)A + 8), (const float* const*)tab.data(), 12345, 8, 0.5f, nullptr) == MICS_OK);
    CHECK(mics_adam_shard((float*)((char*)fake(1) + 4), (float*)fake(2), (float*)((char*)fake(3) + 12), (uint16_t*)((char*)fake(4) + 2),
                          (const float*)fake(5), 777, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 3, nullptr) == MICS_OK);
    CHECK(mics_hier_gather_reorder((char*)A + 2, tab.data(), 4 * 1001 - 3, 1001, 4, 2, 2, nullptr) == MICS_OK);
    CHECK(mics::g_launches == before + 4);
    for (int i = 0; i < MICS_MAX_GROUP; ++i) tab[i] = fake(i + 8);

    // coalesced calls: one launch per 48 tensors of a kind
    std::vector<mics_segment> segs;
    size_t s_off = 0, d_off = 0;
    for (int t = 0; t < 131; ++t) {        // more than one launch's worth, some not 16-byte clean
        size_t S = 8 + (t % 5), n = 4 * S - (t % 3);
        segs.push_back({n, S, s_off, d_off});
        s_off += 2 * S; d_off += n;
    }
    before = mics::g_launches;
    CHECK(mics_hier_gather_reorder_coalesced(A, tab.data(), segs.data(), (int)segs.size(), 4, 2, 2, nullptr) == MICS_OK);
    CHECK(mics::g_launches - before >= 3 && mics::g_launches - before <= 4);   // 131 tensors of two kinds
    for (auto& sg : segs) sg.shard_elems = 0;
    before = mics::g_launches;
    CHECK(mics_reduce_scatter_accum_coalesced((float*)A, (const uint16_t* const*)tab.data(), segs.data(),
                                              (int)segs.size(), 16, 1, nullptr) == MICS_OK);
    CHECK(mics::g_launches == before + 3);
    // a transformer layer's 16 tensors sharded with odd sizes (nothing 16-byte clean): at most
    // two launches for the gather, one for the reduction
    {
        const size_t h = 130;              // hidden size; tensor sizes as in a transformer layer
        const size_t numels[16] = {3 * h * h, 3 * h, h * h, h, h, h, 4 * h * h, 4 * h, 4 * h * h, h, h, h, h + 1, 7, h, 3};
        std::vector<mics_segment> layer;
        size_t so = 1, dn = 3;
        for (size_t n : numels) {
            size_t S = n / 8 + 1;          // p = 8 shards, align 1
            layer.push_back({n, S, so, dn});
            so += S; dn += n;
        }
        before = mics::g_launches;
        CHECK(mics_hier_gather_reorder_coalesced(A, tab.data(), layer.data(), 16, 8, 8, 2, nullptr) == MICS_OK);
        CHECK(mics::g_launches - before >= 1 && mics::g_launches - before <= 2);
        std::vector<mics_segment> red;
        size_t go = 5, ao = 1;
        for (auto& sg : layer) { red.push_back({sg.shard_elems, 0, go + 3 * sg.shard_elems, ao}); go += 8 * sg.shard_elems; ao += sg.shard_elems; }
        before = mics::g_launches;
        CHECK(mics_reduce_scatter_accum_coalesced((float*)A, (const uint16_t* const*)tab.data(), red.data(), 16, 8, 0, nullptr) == MICS_OK);
        CHECK(mics_reduce_scatter_accum_coalesced_typed((float*)A, (const void* const*)tab.data(), red.data(), 16, 8, 1, MICS_DTYPE_F32, nullptr) == MICS_OK);
        CHECK(mics::g_launches == before + 2);
    }

    // rejected calls never reach a launcher
    before = mics::g_launches;
    CHECK(mics_hier_gather_reorder(A, tab.data(), 10, 10, 4, 3, 2, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(std::strstr(mics_last_error(), "not divisible") != nullptr);
    CHECK(mics_hier_gather_reorder(A, tab.data(), 41, 10, 4, 2, 2, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_hier_gather_reorder(A, tab.data(), 10, 10, 4, 2, 3, nullptr) == MICS_ERR_UNSUPPORTED);
    CHECK(mics_hier_gather_reorder((char*)A + 1, tab.data(), 10, 10, 4, 2, 2, nullptr) == MICS_ERR_ALIGNMENT);
    CHECK(mics_hier_gather_reorder(A, tab.data(), 10, (size_t)-1 / 2, 4, 2, 2, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_reduce_scatter_accum((float*)A, (const uint16_t* const*)tab.data(), (size_t)-1, 2, 4, 0, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_reduce_scatter_accum((float*)A, nullptr, 0, 2, 4, 0, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_reduce_scatter_accum_typed((float*)A, tab.data(), 0, 2, 4, 0, 9, nullptr) == MICS_ERR_UNSUPPORTED);
    CHECK(mics_replica_average((float*)A, (const float* const*)tab.data(), 8, 129, 1.0f, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_adam_shard((float*)fake(1), (float*)fake(2), (float*)fake(3), nullptr, (const float*)fake(5), 8,
                          1e-4f, 1.5f, 0.999f, 1e-8f, 0.0f, 1, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_adam_shard((float*)fake(1), (float*)fake(1), (float*)fake(3), nullptr, (const float*)fake(5), 8,
                          1e-4f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, nullptr) == MICS_ERR_INVALID_ARG);
    mics_segment bad = {100, 10, 0, 0};
    CHECK(mics_hier_gather_reorder_coalesced(A, tab.data(), &bad, 1, 4, 2, 2, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_reduce_scatter_accum_coalesced((float*)A, (const uint16_t* const*)tab.data(), nullptr, 3, 4, 0, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(mics_set_blocks_per_cu(-3) == MICS_ERR_INVALID_ARG);
    CHECK(mics_reduce_scatter_accum_typed((float*)A, nullptr, 0, 2, 4, 0, MICS_DTYPE_F16, nullptr) == MICS_ERR_INVALID_ARG);
    CHECK(std::strstr(mics_last_error(), "mics_reduce_scatter_accum_typed: grads is NULL") != nullptr);
    {   // destination regions of two tensors overlap
        mics_segment two[2] = {{40, 10, 0, 0}, {40, 10, 40, 39}};
        CHECK(mics_hier_gather_reorder_coalesced(A, tab.data(), two, 2, 4, 2, 2, nullptr) == MICS_ERR_INVALID_ARG);
        CHECK(std::strstr(mics_last_error(), "segments 0 and 1 overlap") != nullptr);
        mics_segment red[2] = {{40, 0, 0, 8}, {16, 0, 100, 0}};
        CHECK(mics_reduce_scatter_accum_coalesced((float*)A, (const uint16_t* const*)tab.data(), red, 2, 4, 0, nullptr) == MICS_ERR_INVALID_ARG);
        CHECK(std::strstr(mics_last_error(), "overlap") != nullptr);
    }
    CHECK(mics::g_launches == before);

    // nothing to do is fine and launches nothing
    CHECK(mics_reduce_scatter_accum(nullptr, (const uint16_t* const*)tab.data(), 0, 0, 4, 0, nullptr) == MICS_OK);
    CHECK(mics_adam_shard(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, nullptr) == MICS_OK);
    CHECK(mics::g_launches == before);
    CHECK(mics_set_stream_threshold_bytes(1) == MICS_OK && mics_set_stream_threshold_bytes(0) == MICS_OK);
    CHECK(mics_set_launch_shape(MICS_KERNELS_REDUCE, 128, 8) == MICS_OK && mics_set_launch_shape(MICS_KERNELS_REDUCE, 0, 0) == MICS_OK);
    CHECK(mics_set_launch_shape(7, 64, 8) == MICS_ERR_INVALID_ARG && mics_set_launch_shape(0, 100, 8) == MICS_ERR_INVALID_ARG);
    CHECK(mics_shard_elems(805412864, 16, 8) == 50338304);
    std::puts("host checks ok");
    return 0;
}
