"""Pins for the oracle's bfloat16 conversions (its definition: the top 16 bits of an
IEEE-754 binary32, narrowing by round-to-nearest-even on the bit pattern)."""
import numpy as np
import torch


def test_widen_is_the_upper_half_of_binary32(orc):
    bits = np.arange(1 << 16, dtype=np.uint16)
    w = orc.bf16_widen(bits)
    assert np.array_equal(w.view(np.uint32), bits.astype(np.uint32) << 16)


def test_every_bf16_value_survives_widen_then_narrow(orc):
    bits = np.arange(1 << 16, dtype=np.uint16)
    back = orc.bf16_narrow(orc.bf16_widen(bits))
    exp, frac = (bits >> 7) & 0xFF, bits & 0x7F
    is_nan = (exp == 0xFF) & (frac != 0)
    assert np.array_equal(back[~is_nan], bits[~is_nan])
    # NaNs stay NaNs of the same sign
    assert np.all(((back[is_nan] >> 7) & 0xFF) == 0xFF) and np.all((back[is_nan] & 0x7F) != 0)
    assert np.array_equal(back[is_nan] & 0x8000, bits[is_nan] & 0x8000)


def test_ties_go_to_the_even_neighbour(orc):
    def narrow_bits(u32):
        return int(orc.bf16_narrow(np.array([u32], dtype=np.uint32).view(np.float32))[0])
    assert narrow_bits(0x3F808000) == 0x3F80      # halfway 0x3F80/0x3F81 -> even 0x3F80
    assert narrow_bits(0x3F818000) == 0x3F82      # halfway 0x3F81/0x3F82 -> even 0x3F82
    assert narrow_bits(0x3F808001) == 0x3F81      # just above the tie rounds up
    assert narrow_bits(0x3F817FFF) == 0x3F81      # just below the tie rounds down
    assert narrow_bits(0xBF808000) == 0xBF80      # sign-symmetric
    assert narrow_bits(0x7F7FFFFF) == 0x7F80      # largest binary32 overflows to +Inf
    assert narrow_bits(0x7F800000) == 0x7F80      # Inf preserved
    assert narrow_bits(0xFF800000) == 0xFF80
    assert narrow_bits(0x00000001) == 0x0000      # tiny denormal rounds to zero
    assert narrow_bits(0x00008000) == 0x0000      # tie between 0 and the smallest denormal: even
    assert narrow_bits(0x00018000) == 0x0002
    assert narrow_bits(0x80000000) == 0x8000      # -0 keeps its sign
    nan = narrow_bits(0x7F800001)                 # NaN whose payload sits in the dropped bits
    assert (nan >> 7) & 0xFF == 0xFF and nan & 0x7F != 0


def test_narrow_agrees_with_the_library_conversion(orc):
    rng = np.random.default_rng(7)
    u = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    f = u.view(np.float32)
    finite_or_inf = ~np.isnan(f)
    ours = orc.bf16_narrow(f)
    lib = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours[finite_or_inf], lib[finite_or_inf])
    # NaN payloads are not unique; both must be NaN
    assert np.all(np.isnan(orc.bf16_widen(ours[~finite_or_inf])))
