"""Pins for the oracle's coalesced variants: the paper's coalesced collectives (Section 4) launch
many per-tensor operations at once without changing what each computes, so the result must equal
the per-tensor result, which is rebuilt here by plain list manipulation."""
import numpy as np


def test_layer_tensor_inventory_adds_up(gen):
    for h in (2560, 4096, 5120, 8192):
        t = gen.layer_tensors(h)
        assert len(t) == 16 and sum(n for _, n in t) == 12 * h * h + 13 * h
        assert sum(1 for name, _ in t if name.endswith(".bias")) == 8


def test_coalesced_reorder_equals_per_tensor_concatenation(orc, gen):
    p, k = 6, 3
    numels = [37, 6, 120, 1, 55]          # not divisible by p: every tensor has its own ragged tail
    lay = gen.coalesced_layout(numels, p, k, align=1)
    nodes = p // k
    # shards per tensor: element i of tensor t, rank g is tagged
    shards = [[(1_000_000 * (t + 1) + 1000 * g + np.arange(lay.S[t])).astype(np.uint32) for g in range(p)]
              for t in range(len(numels))]
    # coalesced stage-1 buffer of local rank l: for each tensor the chunks of ranks l, k+l, ...
    T = [np.concatenate([np.concatenate([shards[t][j * k + l] for j in range(nodes)])
                         for t in range(len(numels))]) for l in range(k)]
    assert T[0].size == lay.stage1_off[-1]
    out = np.full(lay.flat_off[-1], 0xDEADBEEF, dtype=np.uint32)
    orc.hier_gather_reorder_coalesced(T, lay.reorder_segments(), p, out)
    want = np.concatenate([np.concatenate(shards[t])[:numels[t]] for t in range(len(numels))])
    assert np.array_equal(out, want)
    # a single tensor is the plain call
    one = gen.coalesced_layout([numels[2]], p, k, align=1)
    T2 = [orc.stage1_gather(shards[2], k, l) for l in range(k)]
    out2 = np.zeros(numels[2], np.uint32)
    orc.hier_gather_reorder_coalesced(T2, one.reorder_segments(), p, out2)
    assert np.array_equal(out2, orc.hier_gather_reorder(T2, numels[2], lay.S[2], p))


def test_coalesced_reduce_equals_per_tensor_integer_sums(orc, gen):
    p, k = 4, 2
    numels = [100, 8, 33, 64]
    lay = gen.coalesced_layout(numels, p, k, align=8)
    table = gen.small_int_table(-8, 8, "bf16")
    total = lay.grad_off[-1]
    for g in (0, 3):
        acc = np.full(lay.shard_off[-1], np.nan, np.float32)
        want = np.zeros(lay.shard_off[-1], np.int64)
        for t_step in range(3):
            grads = [gen.fill_host(gen.stream_key(41, gen.ROLE_GRAD, 0, t_step, q), 0, total, table)
                     for q in range(p)]
            orc.reduce_scatter_accum_coalesced(acc, grads, lay.reduce_segments(g), t_step > 0)
            wide = [(gq.astype(np.uint32) << 16).view(np.float32).astype(np.int64) for gq in grads]
            for t in range(len(numels)):
                lo = lay.grad_off[t] + g * lay.S[t]
                want[lay.shard_off[t]:lay.shard_off[t] + lay.S[t]] += sum(w[lo:lo + lay.S[t]] for w in wide)
        assert np.array_equal(acc.astype(np.int64), want)


def test_typed_coalesced_reduce_equals_per_tensor_integer_sums_in_every_format(orc, gen):
    p, k = 4, 2
    numels = [100, 8, 33, 64]
    lay = gen.coalesced_layout(numels, p, k, align=1)
    table = gen.small_int_table(-8, 8, "f32")
    total = lay.grad_off[-1]
    g = 2
    f32 = [gen.fill_host(gen.stream_key(42, gen.ROLE_GRAD, 0, 0, q), 0, total, table) for q in range(p)]
    want = np.zeros(lay.shard_off[-1], np.int64)
    for t in range(len(numels)):
        lo = lay.grad_off[t] + g * lay.S[t]
        want[lay.shard_off[t]:lay.shard_off[t] + lay.S[t]] = 1 + sum(w[lo:lo + lay.S[t]].astype(np.int64) for w in f32)
    variants = {orc.DTYPE_F32: f32, orc.DTYPE_F16: [x.astype(np.float16).view(np.uint16) for x in f32],
                orc.DTYPE_BF16: [orc.bf16_narrow(x) for x in f32]}
    for dtype, grads in variants.items():
        acc = np.ones(lay.shard_off[-1], np.float32)
        orc.reduce_scatter_accum_coalesced_typed(acc, grads, lay.reduce_segments(g), True, dtype)
        assert np.array_equal(acc.astype(np.int64), want), dtype
