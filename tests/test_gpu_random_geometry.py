"""Seeded random geometries through every entry point: group sizes, counts, offsets and alignments
drawn at random (with weight on the awkward ones: odd sizes, chunks shorter than a vector, counts
next to tile boundaries), each call compared with the oracle to the bars of test_gpu_parity.py
and checked for writes outside its output.  The draws are fixed by the seeds below."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

mics = pytest.importorskip("paper_2205_00119_amd")
from gpu_util import Guarded, upload  # noqa: E402

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
GROUPS = [1, 2, 3, 4, 5, 7, 8, 12, 16, 20, 32, 37, 48, 64, 100, 128]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    yield
    torch.cuda.synchronize()


def awkward_count(rng, hi):
    """A count in [1, hi]: small, next to a power of two or a multiple of 512, or anything."""
    kind = rng.integers(0, 4)
    if kind == 0:
        return int(rng.integers(1, 40))
    if kind == 1:
        return int(min(hi, max(1, (1 << int(rng.integers(3, 17))) + int(rng.integers(-9, 10)))))
    if kind == 2:
        return int(min(hi, max(1, 512 * int(rng.integers(1, 60)) + int(rng.integers(-9, 10)))))
    return int(rng.integers(1, hi + 1))


def tagged(gen, seed, n, dtype):
    tab = gen.normal_table(1.0, "bf16") if dtype == np.uint16 else gen.normal_table(1.0, "f32").view(np.uint32)
    return gen.fill_host(gen.stream_key(seed, gen.ROLE_PARAM), 0, n, tab)


@pytest.mark.parametrize("seed", range(24))
def test_random_gather_reorder(orc, gen, seed):
    rng = np.random.default_rng(9000 + seed)
    p = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 64, 128]))
    k = int(rng.choice([d for d in range(1, p + 1) if p % d == 0]))
    eb = int(rng.choice([2, 4]))
    S = awkward_count(rng, 30000 if p <= 16 else 3000)
    n_valid = p * S - int(rng.integers(0, min(2 * S, p * S)))
    sskew, dskew = int(rng.integers(0, 8)), int(rng.integers(0, 8))
    dtype = np.uint16 if eb == 2 else np.uint32
    shards = [tagged(gen, 9100 + g, S, dtype) for g in range(p)]
    T = [orc.stage1_gather(shards, k, l) for l in range(k)]
    # every stage-1 buffer at its own offset
    T_dev = [Guarded(t.size, dtype, skew=(sskew + 3 * l) % 8, fill=t) for l, t in enumerate(T)]
    dst = Guarded(p * S, dtype, skew=dskew)
    before = dst.numpy().copy()
    mics.mics_hier_gather_reorder(dst.t, [t.t for t in T_dev], n_valid, S, p, k, eb)
    torch.cuda.synchronize()
    got = dst.numpy()
    assert np.array_equal(got[:n_valid], orc.concat_shards(shards, n_valid)), (p, k, S, eb, n_valid, sskew, dskew)
    assert np.array_equal(got[n_valid:], before[n_valid:])
    assert dst.guards_intact() and all(t.guards_intact() for t in T_dev)


@pytest.mark.parametrize("seed", range(36))
def test_random_reduce_scatter_accum(orc, gen, seed):
    rng = np.random.default_rng(9300 + seed)
    name = ["bf16", "f16", "f32"][seed % 3]
    dtype = {"bf16": mics.MICS_DTYPE_BF16, "f16": mics.MICS_DTYPE_F16, "f32": mics.MICS_DTYPE_F32}[name]
    code = {"bf16": orc.DTYPE_BF16, "f16": orc.DTYPE_F16, "f32": orc.DTYPE_F32}[name]
    tab = (gen.normal_table(1e-3, "bf16") if name == "bf16" else
           gen.normal_table(3e-5, "f32").astype(np.float16).view(np.uint16) if name == "f16" else
           gen.normal_table(1e-3, "f32"))
    np_dt = np.float32 if name == "f32" else np.uint16
    p = int(rng.choice(GROUPS))
    count = awkward_count(rng, 60000 if p <= 32 else 9000)
    off = int(rng.integers(0, 18))
    mixed = bool(rng.integers(0, 4) == 0)                       # buffers at unrelated offsets
    skews = [int(rng.integers(0, 8)) if mixed else off % 8 for _ in range(p)]
    acc = Guarded(count, np.float32, skew=int(rng.integers(0, 4)))
    ref = np.full(count, np.nan, np.float32)
    mics.mics_set_stream_threshold_bytes(int(rng.choice([0, 1, 1 << 40])))
    try:
        for t in range(2):
            host = [gen.fill_host(gen.stream_key(9400 + seed, gen.ROLE_GRAD, 0, t, q), 0, off + count + 5, tab)
                    for q in range(p)]
            dev = [Guarded(h.size, np_dt, skew=skews[q], fill=h) for q, h in enumerate(host)]
            mics.mics_reduce_scatter_accum_typed(acc.t, [d.t for d in dev], off, count, t > 0, dtype)
            torch.cuda.synchronize()
            orc.reduce_scatter_accum_typed(ref, host, off, t > 0, code)
            assert all(d.guards_intact() and np.array_equal(d.numpy(), h) for d, h in zip(dev, host))
    finally:
        mics.mics_set_stream_threshold_bytes(0)
    assert np.array_equal(acc.numpy().view(np.uint32), ref.view(np.uint32)), (name, p, count, off, skews)
    assert acc.guards_intact()


@pytest.mark.parametrize("seed", range(16))
def test_random_coalesced_layers(orc, gen, seed):
    rng = np.random.default_rng(9600 + seed)
    p = int(rng.choice([2, 3, 4, 8, 16, 32]))
    k = int(rng.choice([d for d in range(1, p + 1) if p % d == 0]))
    align = int(rng.choice([1, 8]))
    n_t = int(rng.choice([1, 2, 5, 16, 49, 70]))
    numels = [awkward_count(rng, 20000 if n_t <= 16 else 3000) for _ in range(n_t)]
    lay = gen.coalesced_layout(numels, p, k, align=align, flat_align=8 if align == 8 else 1)
    nodes = p // k
    # gather
    shards = [[tagged(gen, 9700 + 131 * t + g, lay.S[t], np.uint16) for g in range(p)] for t in range(n_t)]
    T = [np.concatenate([np.concatenate([shards[t][j * k + l] for j in range(nodes)]) for t in range(n_t)])
         for l in range(k)]
    T_dev = [Guarded(t.size, np.uint16, fill=t) for t in T]
    dst = Guarded(lay.flat_off[-1], np.uint16)
    want = dst.numpy().copy()
    mics.mics_hier_gather_reorder_coalesced(dst.t, [t.t for t in T_dev], lay.reorder_segments(), p, k, 2)
    torch.cuda.synchronize()
    orc.hier_gather_reorder_coalesced(T, lay.reorder_segments(), p, want)
    assert np.array_equal(dst.numpy(), want), (p, k, align, numels)
    assert dst.guards_intact() and all(t.guards_intact() for t in T_dev)
    # reduce, in the format the seed picks
    name = ["bf16", "f16", "f32"][seed % 3]
    dtype = {"bf16": mics.MICS_DTYPE_BF16, "f16": mics.MICS_DTYPE_F16, "f32": mics.MICS_DTYPE_F32}[name]
    code = {"bf16": orc.DTYPE_BF16, "f16": orc.DTYPE_F16, "f32": orc.DTYPE_F32}[name]
    tab = (gen.normal_table(1e-3, "bf16") if name == "bf16" else
           gen.normal_table(3e-5, "f32").astype(np.float16).view(np.uint16) if name == "f16" else
           gen.normal_table(1e-3, "f32"))
    np_dt = np.float32 if name == "f32" else np.uint16
    rank = int(rng.integers(0, p))
    segs = lay.reduce_segments(rank)
    acc = Guarded(lay.shard_off[-1], np.float32)
    ref = np.full(lay.shard_off[-1], np.nan, np.float32)
    for t in range(2):
        host = [gen.fill_host(gen.stream_key(9800 + seed, gen.ROLE_GRAD, 0, t, q), 0, lay.grad_off[-1], tab)
                for q in range(p)]
        dev = [Guarded(h.size, np_dt, skew=int(rng.integers(0, 2)) * 2, fill=h) for h in host]
        mics.mics_reduce_scatter_accum_coalesced_typed(acc.t, [d.t for d in dev], segs, t > 0, dtype)
        torch.cuda.synchronize()
        orc.reduce_scatter_accum_coalesced_typed(ref, host, segs, t > 0, code)
    assert np.array_equal(acc.numpy().view(np.uint32), ref.view(np.uint32)), (name, p, k, align, numels, rank)
    assert acc.guards_intact()


@pytest.mark.parametrize("seed", range(16))
def test_random_average_and_adam(orc, gen, seed):
    rng = np.random.default_rng(9900 + seed)
    r = int(rng.choice([1, 2, 3, 4, 8, 9, 20, 64, 128]))
    count = awkward_count(rng, 50000 if r <= 20 else 6000)
    skew = int(rng.integers(0, 4))
    scale = float(np.float32(1.0 / (r * 24)))
    atab = gen.normal_table(3e-3, "f32")
    copies = [gen.fill_host(gen.stream_key(9950 + seed, gen.ROLE_ACC, c), 0, count, atab) for c in range(r)]
    dev = [Guarded(count, np.float32, skew=(skew + c) % 4, fill=h) for c, h in enumerate(copies)]
    in_place = bool(rng.integers(0, 2))
    out = dev[0] if in_place else Guarded(count, np.float32, skew=skew)
    avg_ref = orc.replica_average(copies, scale)
    # the fused step reads the copies before the separate average may overwrite the first one
    kind = [None, "bf16", "f16"][seed % 3]
    w0 = gen.fill_host(gen.stream_key(9950 + seed, gen.ROLE_MASTER), 0, count, gen.normal_table(0.02, "f32"))
    st = [Guarded(count, np.float32, skew=skew, fill=x) for x in (w0, np.zeros(count, np.float32), np.zeros(count, np.float32))]
    po = Guarded(count, np.uint16, skew=int(rng.integers(0, 8))) if kind else None
    code = mics.MICS_DTYPE_F16 if kind == "f16" else mics.MICS_DTYPE_BF16
    mics.mics_replica_average_adam_shard_typed(st[0].t, st[1].t, st[2].t, po.t if po else None, code,
                                               [d.t for d in dev], count, scale, step=3, **HP)
    mics.mics_replica_average(out.t, [d.t for d in dev], count, scale)
    torch.cuda.synchronize()
    assert np.array_equal(out.numpy().view(np.uint32), avg_ref.view(np.uint32)), (r, count, skew, in_place)
    for c in range(1, r):
        assert np.array_equal(dev[c].numpy(), copies[c])
    wr, mr, vr = w0.copy(), np.zeros(count, np.float32), np.zeros(count, np.float32)
    pr = orc.adam_shard(wr, mr, vr, avg_ref, step=3, f32=True, want_bf16=kind is not None,
                        param_dtype=kind or "bf16", **HP)
    assert np.array_equal(st[0].numpy().view(np.uint32), wr.view(np.uint32)), (r, count, skew, kind)
    assert np.array_equal(st[1].numpy().view(np.uint32), mr.view(np.uint32))
    assert np.array_equal(st[2].numpy().view(np.uint32), vr.view(np.uint32))
    if kind:
        assert np.array_equal(po.numpy(), pr) and po.guards_intact()
    # the separate Adam call on the averaged gradient gives the same state
    st2 = [Guarded(count, np.float32, skew=skew, fill=x) for x in (w0, np.zeros(count, np.float32), np.zeros(count, np.float32))]
    g = Guarded(count, np.float32, skew=skew, fill=avg_ref)
    mics.mics_adam_shard_typed(st2[0].t, st2[1].t, st2[2].t, None, mics.MICS_DTYPE_BF16, g.t, count, step=3, **HP)
    torch.cuda.synchronize()
    assert np.array_equal(st2[0].numpy().view(np.uint32), wr.view(np.uint32))
    assert all(x.guards_intact() for x in dev + st + st2 + [out, g])
