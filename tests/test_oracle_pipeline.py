"""Whole-path invariants of the oracle: sharding commutes with the element-wise steps, and
gathering the updated shards reproduces the full updated parameter (Sections 3.2-3.4)."""
import numpy as np

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def test_update_per_shard_then_hierarchical_gather_equals_update_of_the_whole(orc, gen):
    p, k, r, s, S = 6, 3, 2, 3, 40
    n = p * S - 5                       # ragged: the last shard owns fewer valid elements
    n_pad = p * S
    gtab = gen.normal_table(1e-2, "bf16")
    master = gen.fill_host(gen.stream_key(31, gen.ROLE_MASTER), 0, n_pad, gen.normal_table(0.02, "f32"))
    master[n:] = 0.0                    # padding is zeros
    grads = {(c, t, q): gen.fill_host(gen.stream_key(31, gen.ROLE_GRAD, c, t, q), 0, n_pad, gtab)
             for c in range(r) for t in range(s) for q in range(p)}
    scale = np.float32(1.0 / (r * p * s))

    # group view: every step over the whole padded buffer at once
    copies = []
    for c in range(r):
        acc = np.empty(n_pad, np.float32)
        for t in range(s):
            orc.reduce_scatter_accum(acc, [grads[(c, t, q)] for q in range(p)], 0, t > 0)
        copies.append(acc)
    avg = orc.replica_average(copies, scale)
    w_full, m_full, v_full = master.copy(), np.zeros(n_pad, np.float32), np.zeros(n_pad, np.float32)
    bf_full = orc.adam_shard(w_full, m_full, v_full, avg, step=1, **HP)

    # rank view: each rank works on its own shard only
    shards_bf = []
    for g in range(p):
        sl = slice(g * S, (g + 1) * S)
        rc = []
        for c in range(r):
            acc = np.empty(S, np.float32)
            for t in range(s):
                orc.reduce_scatter_accum(acc, [grads[(c, t, q)] for q in range(p)], g * S, t > 0)
            rc.append(acc)
        a = orc.replica_average(rc, scale)
        w, m, v = master[sl].copy(), np.zeros(S, np.float32), np.zeros(S, np.float32)
        shards_bf.append(orc.adam_shard(w, m, v, a, step=1, **HP))
        assert np.array_equal(w, w_full[sl]) and np.array_equal(m, m_full[sl])

    # next iteration's gather: stage 1 across nodes, then the reorder
    T = [orc.stage1_gather(shards_bf, k, l) for l in range(k)]
    flat = orc.hier_gather_reorder(T, n, S, p)
    assert np.array_equal(flat, bf_full[:n])
    assert not np.array_equal(orc.naive_intra_gather(T, p)[:n], bf_full[:n])   # the fix matters
