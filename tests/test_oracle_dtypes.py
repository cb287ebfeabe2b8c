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


# ---- binary16 narrowing (the parameter format of fp16 mixed precision) ---------------------------

def _lib_f16(x):
    """The library's float32 -> float16 conversion (numpy), as bit patterns."""
    with np.errstate(over="ignore"):
        return np.asarray(x, np.float32).astype(np.float16).view(np.uint16)


def test_binary16_narrowing_round_trips_every_binary16_value(orc):
    bits = np.arange(1 << 16, dtype=np.uint16)
    wide = bits.view(np.float16).astype(np.float32)
    back = orc.f16_narrow(wide)
    nan = np.isnan(wide)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all((back[nan] & 0x7C00) == 0x7C00) and np.all((back[nan] & 0x03FF) != 0)   # still NaN


def test_binary16_narrowing_agrees_with_the_library_on_random_patterns_and_ties(orc):
    rng = np.random.default_rng(77)
    pats = rng.integers(0, 1 << 32, size=4_000_000, dtype=np.uint64).astype(np.uint32)
    # more weight on the exponents binary16 can hold (2^-26 .. 2^17) than a uniform draw gives
    dense = (rng.integers(127 - 26, 127 + 18, size=4_000_000, dtype=np.uint64).astype(np.uint32) << 23) \
        | rng.integers(0, 1 << 23, size=4_000_000, dtype=np.uint64).astype(np.uint32) \
        | (rng.integers(0, 2, size=4_000_000, dtype=np.uint64).astype(np.uint32) << 31)
    # every midpoint between neighbouring binary16 values (exact in binary32), and its two
    # binary32 neighbours: ties go to the even pattern, anything off the tie to the nearer one
    h = np.arange(0x7C00, dtype=np.uint16)                  # all non-negative finite values
    lo = h.view(np.float16).astype(np.float64)
    hi = np.where(h == 0x7BFF, 65536.0, (h + 1).astype(np.uint16).view(np.float16).astype(np.float64))
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    ties = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf))])
    ties = np.concatenate([ties, -ties])
    for x in (pats.view(np.float32), dense.view(np.float32), ties):
        ours, lib = orc.f16_narrow(x), _lib_f16(x)
        nan = np.isnan(x)
        assert np.array_equal(ours[~nan], lib[~nan])
        assert np.all((ours[nan] & 0x7C00) == 0x7C00) and np.all((ours[nan] & 0x03FF) != 0)
    # ties by definition: 1 + 2^-11 lies between 0x3C00 (even) and 0x3C01; 1 + 3*2^-11 between 0x3C01 and 0x3C02
    assert orc.f16_narrow(np.float32([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11])).tolist() == [0x3C00, 0x3C02]


def test_binary16_narrowing_at_the_ends_of_the_range(orc):
    x = np.float32([65504.0, 65519.996, 65520.0, 1e10, np.inf, -65520.0,
                    2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -23), 2.0 ** -26, 1e-45, 0.0, -0.0,
                    2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -11), 1023.5 * 2.0 ** -24])
    want = [0x7BFF, 0x7BFF, 0x7C00, 0x7C00, 0x7C00, 0xFC00,
            0x0001, 0x0000, 0x0001, 0x0000, 0x0000, 0x0000, 0x8000,
            0x0400, 0x0400, 0x0400]
    assert orc.f16_narrow(x).tolist() == want


def test_adam_can_hand_back_binary16_parameters(orc, gen):
    n = 5000
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    w0 = gen.fill_host(gen.stream_key(61, gen.ROLE_MASTER), 0, n, gen.normal_table(0.02, "f32"))
    g = gen.fill_host(gen.stream_key(61, gen.ROLE_ACC), 0, n, gen.normal_table(1e-3, "f32"))
    for f32 in (False, True):
        wa, ma, va = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        wb, mb, vb = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
        pa = orc.adam_shard(wa, ma, va, g, step=1, f32=f32, **hp)
        pb = orc.adam_shard(wb, mb, vb, g, step=1, f32=f32, param_dtype="f16", **hp)
        assert np.array_equal(wa.view(np.uint32), wb.view(np.uint32))      # the update itself is the same
        assert np.array_equal(pa, orc.bf16_narrow(wa))
        assert np.array_equal(pb, _lib_f16(wb))                            # parameter = RNE(new master)
