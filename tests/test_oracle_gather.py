"""Pins for the oracle's hierarchical all-gather functions (paper Section 3.3)."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            out.setdefault(key.strip(), []).append(val.strip())
    return out


def tagged_shards(p, S, dtype):
    # element i of chunk C_g carries the tag g*1e6 + i (or a 16-bit fold of it)
    if dtype == np.uint32:
        return [(g * 1_000_000 + np.arange(S)).astype(np.uint32) for g in range(p)]
    return [((g * 4099 + np.arange(S) * 7 + 1) % 65521).astype(np.uint16) for g in range(p)]


def test_paper_worked_example_p4_k2(orc):
    gold = read_golden("hier_gather_p4_k2.txt")
    p, k = int(gold["p"][0]), int(gold["k"][0])
    S = 3
    shards = tagged_shards(p, S, np.uint32)
    name_of = {f"C{g}": shards[g] for g in range(p)}

    def layout(names):
        return np.concatenate([name_of[n] for n in names.split()])

    T = [orc.stage1_gather(shards, k, l) for l in range(k)]
    assert np.array_equal(T[0], layout(gold["stage1_local_rank_0"][0]))
    assert np.array_equal(orc.naive_intra_gather(T, p), layout(gold["wrong_layout"][0]))
    want = layout(gold["correct_layout"][0])
    assert np.array_equal(orc.hier_gather_reorder(T, p * S, S, p), want)
    assert np.array_equal(orc.concat_shards(shards, p * S), want)
    assert p // k == int(gold["intra_node_all_gathers"][0])
    assert len(T[0]) // S == p // k   # each stage-1 buffer holds one chunk per node


def test_traffic_reduction_figures_fix_the_geometry():
    gold = read_golden("traffic_reduction.txt")
    k = int(gold["k"][0])
    for row in gold["p"]:
        p_txt, _, pct = row.partition("reduction_percent:")
        p = int(p_txt)
        assert p % k == 0
        reduction = 100.0 * (1.0 - (p - k) / (p - 1))
        # the paper prints these to one decimal, truncated or rounded
        assert abs(reduction - float(pct)) < 0.1


@pytest.mark.parametrize("dtype", [np.uint16, np.uint32])
def test_brute_force_all_small_geometries(orc, dtype):
    for p in range(1, 13):
        for k in [d for d in range(1, p + 1) if p % d == 0]:
            for S in (1, 2, 3, 5, 8):
                shards = tagged_shards(p, S, dtype)
                # stage 1 by plain list manipulation: channel l gathers ranks l, k+l, 2k+l, ...
                T_py = [np.concatenate([shards[g] for g in range(l, p, k)]) for l in range(k)]
                T = [orc.stage1_gather(shards, k, l) for l in range(k)]
                for a, b in zip(T, T_py):
                    assert np.array_equal(a, b), (p, k, S)
                assert np.array_equal(orc.naive_intra_gather(T, p), np.concatenate(T_py))
                full = np.concatenate(shards)
                for n_valid in {p * S, p * S - 1, max(p * S - S - 1, 0), 1, 0}:
                    got = orc.hier_gather_reorder(T, n_valid, S, p)
                    assert np.array_equal(got, full[:n_valid]), (p, k, S, n_valid)
                    assert np.array_equal(orc.concat_shards(shards, n_valid), full[:n_valid])


def test_single_node_and_one_device_per_node_are_plain_concatenation(orc):
    p, S = 6, 5
    shards = tagged_shards(p, S, np.uint32)
    full = np.concatenate(shards)
    for k in (1, p):
        T = [orc.stage1_gather(shards, k, l) for l in range(k)]
        assert np.array_equal(orc.naive_intra_gather(T, p), full)      # nothing to fix
        assert np.array_equal(orc.hier_gather_reorder(T, p * S, S, p), full)


def test_reordering_twice_with_swapped_grid_is_identity(orc):
    # the reorder transposes the k x (p/k) chunk matrix; transposing back restores it
    p, k, S = 12, 4, 3
    shards = tagged_shards(p, S, np.uint32)
    T = [orc.stage1_gather(shards, k, l) for l in range(k)]
    W = orc.naive_intra_gather(T, p)
    F = orc.hier_gather_reorder(T, p * S, S, p)
    k2 = p // k
    T2 = [F[b * k * S:(b + 1) * k * S].copy() for b in range(k2)]
    assert np.array_equal(orc.hier_gather_reorder(T2, p * S, S, p), W)


def test_only_valid_elements_are_written_and_bad_geometry_is_refused(orc):
    p, k, S = 4, 2, 4
    shards = tagged_shards(p, S, np.uint16)
    T = [orc.stage1_gather(shards, k, l) for l in range(k)]
    assert orc.hier_gather_reorder(T, 0, S, p).size == 0
    with pytest.raises(ValueError):
        orc.hier_gather_reorder(T, p * S + 1, S, p)
    with pytest.raises(ValueError):
        orc.stage1_gather(tagged_shards(6, S, np.uint16), 4, 0)     # 6 not divisible by 4
