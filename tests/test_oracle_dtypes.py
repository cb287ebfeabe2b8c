"""Pins for the oracle's gradient-dtype variants: binary16 widening and the typed reduction."""
import numpy as np


def test_binary16_widening_is_exact_for_every_pattern(orc):
    bits = np.arange(1 << 16, dtype=np.uint16)
    ours = orc.f16_widen(bits)
    lib = bits.view(np.float16).astype(np.float32)          # the library's conversion
    nan = np.isnan(lib)
    assert np.array_equal(ours[~nan].view(np.uint32), lib[~nan].view(np.uint32))
    assert np.all(np.isnan(ours[nan]))
    assert ours[0x0001] == np.float32(2.0 ** -24) and ours[0x03FF] == np.float32(1023 * 2.0 ** -24)
    assert ours[0x3C00] == 1.0 and ours[0x7BFF] == 65504.0 and np.isinf(ours[0x7C00])
    assert ours.view(np.uint32)[0x8000] == 0x80000000


def test_typed_reduction_matches_the_bf16_one_and_plain_float_arithmetic(orc, gen):
    p, n, off = 5, 4000, 17
    tab = gen.normal_table(1e-2, "bf16")
    bf = [gen.fill_host(gen.stream_key(51, gen.ROLE_GRAD, 0, 0, q), 0, n + off, tab) for q in range(p)]
    a = orc.reduce_scatter_accum(np.zeros(n, np.float32), bf, off, False)
    b = orc.reduce_scatter_accum_typed(np.full(n, np.nan, np.float32), bf, off, False, orc.DTYPE_BF16)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # float32 and binary16 gradients: ranks ascending, one binary32 addition at a time
    f32 = [orc.bf16_widen(g) * np.float32(3.0) for g in bf]
    f16 = [g.astype(np.float16) for g in f32]
    for grads, dtype, wide in ((f32, orc.DTYPE_F32, f32),
                               ([g.view(np.uint16) for g in f16], orc.DTYPE_F16,
                                [g.astype(np.float32) for g in f16])):
        acc = np.full(n, 0.25, np.float32)
        orc.reduce_scatter_accum_typed(acc, grads, off, True, dtype)
        partial = wide[0][off:off + n].copy()
        for q in range(1, p):
            partial = partial + wide[q][off:off + n]
        want = np.full(n, 0.25, np.float32) + partial
        assert np.array_equal(acc.view(np.uint32), want.view(np.uint32))


def test_typed_reduction_of_integers_is_exact_in_every_dtype(orc, gen):
    p, n = 16, 999
    tab = gen.small_int_table(-8, 8, "f32")
    f32 = [gen.fill_host(gen.stream_key(52, gen.ROLE_GRAD, 0, 0, q), 0, n, tab) for q in range(p)]
    want = sum(g.astype(np.int64) for g in f32)
    variants = {
        orc.DTYPE_F32: f32,
        orc.DTYPE_F16: [g.astype(np.float16).view(np.uint16) for g in f32],
        orc.DTYPE_BF16: [orc.bf16_narrow(g) for g in f32],
    }
    for dtype, grads in variants.items():
        acc = orc.reduce_scatter_accum_typed(np.zeros(n, np.float32), grads, 0, False, dtype)
        assert np.array_equal(acc.astype(np.int64), want)
