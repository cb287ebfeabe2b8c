"""Pins for the oracle's 2-hop gradient synchronisation arithmetic (paper Section 3.4):
hop 1 = reduce-scatter in the partition group on every micro-step, accumulated;
hop 2 = all-reduce in the replication group at the accumulation boundary."""
import numpy as np
import pytest

from util import reduction_rel_err


def bf16_of(values):
    """bf16 bit patterns of values that are exactly representable (checked)."""
    f = np.asarray(values, dtype=np.float32)
    u = f.view(np.uint32)
    assert np.all(u & 0xFFFF == 0), "value not representable in bf16"
    return (u >> 16).astype(np.uint16)


def widen(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def test_single_rank_group_just_widens(orc, gen):
    g = gen.fill_host(gen.stream_key(1, gen.ROLE_GRAD), 0, 1000, gen.normal_table(1e-2, "bf16"))
    acc = np.full(1000, np.nan, dtype=np.float32)          # overwrite must ignore old contents
    orc.reduce_scatter_accum(acc, [g], 0, accumulate=False)
    assert np.array_equal(acc, widen(g))


@pytest.mark.parametrize("p,s", [(2, 1), (4, 3), (16, 5), (7, 2)])
def test_integer_gradients_sum_exactly(orc, gen, p, s):
    n = 777
    table = gen.small_int_table(-8, 8, "bf16")
    acc = np.zeros(n, dtype=np.float32)
    total = np.zeros(n, dtype=np.int64)
    for t in range(s):
        grads = [gen.fill_host(gen.stream_key(3, gen.ROLE_GRAD, 0, t, q), 0, n, table) for q in range(p)]
        total += sum(widen(g).astype(np.int64) for g in grads)
        orc.reduce_scatter_accum(acc, grads, 0, accumulate=(t > 0))
    assert np.array_equal(acc.astype(np.int64), total)
    assert np.abs(total).max() > 8          # the data really exercised multi-term sums


def test_rank_view_is_a_slice_of_the_group_view(orc, gen):
    p, S = 4, 50
    table = gen.normal_table(1e-2, "bf16")
    grads = [gen.fill_host(gen.stream_key(5, gen.ROLE_GRAD, 0, 0, q), 0, p * S, table) for q in range(p)]
    whole = orc.reduce_scatter_accum(np.zeros(p * S, np.float32), grads, 0, accumulate=False)
    for g in range(p):
        mine = orc.reduce_scatter_accum(np.zeros(S, np.float32), grads, g * S, accumulate=False)
        assert np.array_equal(mine, whole[g * S:(g + 1) * S])


def test_summation_order_is_ascending_rank_then_one_add_into_acc(orc):
    one, tiny = 1.0, 2.0 ** -24          # 1 + 2^-24 is a tie that rounds back to 1 in binary32
    # ((1 + t) + t) = 1  but  ((t + t) + 1) = 1 + 2^-23
    acc = orc.reduce_scatter_accum(np.zeros(1, np.float32),
                                   [bf16_of([one]), bf16_of([tiny]), bf16_of([tiny])], 0, False)
    assert acc[0] == np.float32(1.0)
    acc = orc.reduce_scatter_accum(np.zeros(1, np.float32),
                                   [bf16_of([tiny]), bf16_of([tiny]), bf16_of([one])], 0, False)
    assert acc[0] == np.float32(1.0 + 2.0 ** -23)
    # the ranks' partial sum is formed first and added to the accumulator once
    acc = orc.reduce_scatter_accum(np.ones(1, np.float32), [bf16_of([tiny]), bf16_of([tiny])], 0, True)
    assert acc[0] == np.float32(1.0 + 2.0 ** -23)


def test_first_micro_step_adds_into_positive_zero(orc):
    neg_zero = np.array([0x8000], dtype=np.uint16)
    acc = orc.reduce_scatter_accum(np.full(1, 5.0, np.float32), [neg_zero, neg_zero], 0, False)
    assert acc.view(np.uint32)[0] == 0          # (+0) + (-0) = +0


def test_binary32_sum_stays_within_the_a_priori_bound_of_the_binary64_sum(orc, gen):
    p, s, n = 16, 12, 20000
    table = gen.normal_table(1e-4, "bf16")
    acc32 = np.zeros(n, np.float32)
    acc64 = np.zeros(n, np.float64)
    ref = np.zeros(n, np.float64)
    abs_sum = np.zeros(n, np.float64)
    for t in range(s):
        grads = [gen.fill_host(gen.stream_key(9, gen.ROLE_GRAD, 0, t, q), 0, n, table) for q in range(p)]
        orc.reduce_scatter_accum(acc32, grads, 0, accumulate=(t > 0))
        orc.reduce_scatter_accum(acc64, grads, 0, accumulate=(t > 0), f64=True)
        stack = np.stack([widen(g).astype(np.float64) for g in grads])
        ref += stack.sum(axis=0)
        abs_sum += np.abs(stack).sum(axis=0)
    assert np.allclose(acc64, ref, rtol=0, atol=1e-15 * abs_sum.max())
    assert np.all(np.abs(acc32 - acc64) <= (p * s) * 2.0 ** -24 * abs_sum)
    assert reduction_rel_err(acc32, acc64, abs_sum).max() < 1e-5


def test_replica_average_is_exact_for_power_of_two_scale_and_integers(orc, gen):
    r, n = 4, 333
    table = gen.small_int_table(-100, 100, "f32")
    copies = [gen.fill_host(gen.stream_key(11, gen.ROLE_ACC, c), 0, n, table) for c in range(r)]
    out = orc.replica_average(copies, 1.0 / 64)
    want = sum(c.astype(np.int64) for c in copies) / 64.0
    assert np.array_equal(out.astype(np.float64), want)


def test_replica_average_order_scale_and_aliasing(orc):
    one, tiny = np.float32(1.0), np.float32(2.0 ** -24)
    a = [np.array([v], np.float32) for v in (one, tiny, tiny)]
    assert orc.replica_average(a, 1.0)[0] == np.float32(1.0)
    assert orc.replica_average(a[::-1], 1.0)[0] == np.float32(1.0 + 2.0 ** -23)
    # scale applied once, after the sum, as a binary32 multiply
    third = np.float32(1.0 / 3.0)
    b = [np.array([v], np.float32) for v in (0.1, 0.2, 0.7)]
    s = np.float32(np.float32(np.float32(0.1) + np.float32(0.2)) + np.float32(0.7))
    assert orc.replica_average(b, third)[0] == np.float32(s * third)
    # the result may overwrite the first copy (in-place all-reduce)
    first = b[0].copy()
    orc.replica_average([first, b[1], b[2]], third, out=first)
    assert first[0] == np.float32(s * third)


def test_two_hop_result_is_the_global_mean_of_all_micro_batch_gradients(orc, gen):
    # The paper's alternative schedule (all-reduce over every device at every micro-step, then
    # keep the owned part) synchronises the same gradient; both equal the plain mean over all
    # r*p*s per-device micro-batch gradients.
    p, r, s, S = 4, 3, 5, 64
    n = p * S
    table = gen.normal_table(1e-3, "bf16")
    g = {(c, t, q): gen.fill_host(gen.stream_key(13, gen.ROLE_GRAD, c, t, q), 0, n, table)
         for c in range(r) for t in range(s) for q in range(p)}
    stack = np.stack([widen(v).astype(np.float64) for v in g.values()])
    mean = stack.mean(axis=0)
    abs_sum = np.abs(stack).sum(axis=0)
    scale = np.float32(1.0 / (r * p * s))
    for rank in range(p):
        copies = []
        for c in range(r):
            acc = np.zeros(S, np.float32)
            for t in range(s):
                orc.reduce_scatter_accum(acc, [g[(c, t, q)] for q in range(p)], rank * S, t > 0)
            copies.append(acc)
        two_hop = orc.replica_average(copies, scale)
        # alternative schedule: one running all-reduce over all r*p devices per micro-step
        alt = np.zeros(S, np.float32)
        for t in range(s):
            every = [g[(c, t, q)] for c in range(r) for q in range(p)]
            orc.reduce_scatter_accum(alt, every, rank * S, t > 0)
        alt = orc.replica_average([alt], scale)
        sl = slice(rank * S, (rank + 1) * S)
        scaled_abs = abs_sum[sl] / (r * p * s)
        assert reduction_rel_err(two_hop, mean[sl], scaled_abs).max() < 1e-5
        assert reduction_rel_err(alt, mean[sl], scaled_abs).max() < 1e-5
        assert reduction_rel_err(two_hop, alt, scaled_abs).max() < 1e-5
