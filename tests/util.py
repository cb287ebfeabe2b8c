"""Error measures shared by the tests (no method arithmetic)."""
import numpy as np


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in bf16 steps between bit patterns; +0 and -0 coincide."""
    def ordered(u):
        u = np.asarray(u, dtype=np.uint16).astype(np.int32)
        mag = u & 0x7FFF
        return np.where(u & 0x8000, -mag, mag)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def reduction_rel_err(got, want, abs_sum):
    """|got - want| / sum|terms|: the error of a sum relative to the magnitude of what was summed
    (the quantity the classical summation bound |s_hat - s| <= (n-1) u sum|x_i| controls).  The
    plain relative error |got - want| / |want| has no bound when the terms cancel -- and among
    5e7 sums of zero-mean gradients some cancel almost completely -- so it is not used."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.asarray(abs_sum, dtype=np.float64)
    denom = np.where(denom == 0, 1.0, denom)
    return np.abs(got - want) / denom


def adam_rel_err(got_w, want_w, old_w):
    """|got - want| / max(|w'|, |w|, |w' - w|): safe where the new weight lands near zero."""
    got = np.asarray(got_w, dtype=np.float64)
    want = np.asarray(want_w, dtype=np.float64)
    old = np.asarray(old_w, dtype=np.float64)
    denom = np.maximum(np.maximum(np.abs(want), np.abs(old)), np.abs(want - old))
    denom = np.where(denom == 0, 1.0, denom)
    return np.abs(got - want) / denom


def state_rel_err(got, want, floor):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.maximum(np.abs(want), floor)
    return np.abs(got - want) / denom
