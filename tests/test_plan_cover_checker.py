"""CPU: the checker of the GEMM work lists (plan_cover.check_cover) accepts lists written out plainly from the
rows' keep patterns and rejects every planted mistake: a missing item, an item listed twice, an item that
stops short, a K range with a gap, a partition missing from a mask, two pieces writing the same output."""
import numpy as np
import pytest

from plan_cover import check_cover

BM, P, F, D, E = 256, 2, 512, 512, 3   # Fp = 256: two neuron tiles of 128 and 8 K stages per partition; two column tiles


def plain_plan(seed=0):
    """Row tiles of 256, one item per (tile, partition the tile keeps, neuron tile) and per (tile, column tile)."""
    rng = np.random.default_rng(seed)
    nrows = np.array([300, 0, 513])
    row0 = np.array([0, 512, 512])  # tile-aligned starts
    cap = 512 + 768
    bits = np.zeros(cap, np.uint8)
    items1, items2 = [], []
    for e in range(E):
        n, r0 = int(nrows[e]), int(row0[e])
        # rows sorted by keep pattern: both partitions first, then partition 0 only
        both = int(n * 0.6)
        bits[r0:r0 + both] = 3
        bits[r0 + both:r0 + n] = 1
        for i in range((n + BM - 1) // BM):
            a, cnt = i * BM, min(BM, n - i * BM)
            tb = int(np.bitwise_or.reduce(bits[r0 + a:r0 + a + cnt]))
            for p in range(P):
                if not (tb >> p) & 1:
                    continue
                last = int(np.flatnonzero((bits[r0 + a:r0 + a + cnt] >> p) & 1).max()) + 1
                for jt in range(2):
                    items1.append([r0 + a, last, e, p, jt, cnt, 0, 0])
            for jd in range(2):
                items2.append([r0 + a, cnt, e, jd, tb, 0, 8, 0])
    it1, it2 = np.array(items1, np.int32), np.array(items2, np.int32)
    return {"tile_rows": BM, "shared_rows": 0, "row_bits": bits, "expert_row0": row0, "expert_nrows": nrows,
            "counters": np.array([len(it1), len(it2), 0, 1, 0]), "items1": it1, "items2": it2}


def check(plan):
    plan = dict(plan)
    plan["counters"] = np.array([len(plan["items1"]), len(plan["items2"]), 0, 1, 0])
    check_cover(plan, name="hand-made", T=1000, D=D, F=F, P=P, E_res=E)


def test_plain_lists_pass():
    check(plain_plan())


def test_split_k_ranges_and_halves_pass():
    plan = plain_plan()
    it2 = plan["items2"].tolist()
    first = it2.pop(0)  # one item as three K ranges, the extra two into partial-output tiles
    it2 += [first[:5] + [0, 3, 0], first[:5] + [3, 2, 1], first[:5] + [5, 3, 2]]
    plan["items2"] = np.array(it2, np.int32)
    it1 = plan["items1"].tolist()
    k = next(i for i, v in enumerate(it1) if v[1] <= 128)  # an item of at most 128 rows as two halves of 64 neurons
    v = it1.pop(k)
    it1 += [v[:6] + [1, 0], v[:6] + [2, 0]]
    plan["items1"] = np.array(it1, np.int32)
    check(plan)


def mutate1(f):
    plan = plain_plan()
    it = plan["items1"].tolist()
    f(it)
    plan["items1"] = np.array(it, np.int32)
    return plan


def mutate2(f):
    plan = plain_plan()
    it = plan["items2"].tolist()
    f(it)
    plan["items2"] = np.array(it, np.int32)
    return plan


MISTAKES = {
    "gemm1_item_missing": lambda: mutate1(lambda it: it.pop(3)),
    "gemm1_item_twice": lambda: mutate1(lambda it: it.append(list(it[5]))),
    "gemm1_item_stops_short": lambda: mutate1(lambda it: it[0].__setitem__(1, it[0][1] - 1)),
    # a tile only some of whose rows keep the partition: the second GEMM reads all of its rows of H, so the rest must be zero-filled
    "gemm1_rows_not_filled": lambda: mutate1(lambda it: next(v for v in it if v[1] < v[5]).__setitem__(5, next(v for v in it if v[1] < v[5])[1])),
    "gemm1_second_half_missing": lambda: mutate1(lambda it: it.__setitem__(slice(len(it) - 1, len(it)), [it[-1][:6] + [1, 0]])),
    "gemm2_item_missing": lambda: mutate2(lambda it: it.pop(1)),
    "gemm2_item_twice": lambda: mutate2(lambda it: it.append(list(it[2]))),
    "gemm2_k_range_gap": lambda: mutate2(lambda it: it.__setitem__(slice(0, 1), [it[0][:5] + [0, 3, 0], it[0][:5] + [4, 4, 1]])),
    "gemm2_k_range_overlap": lambda: mutate2(lambda it: it.__setitem__(slice(0, 1), [it[0][:5] + [0, 5, 0], it[0][:5] + [4, 4, 1]])),
    "gemm2_partition_missing": lambda: mutate2(lambda it: it[0].__setitem__(4, 1)),
    "gemm2_two_writers": lambda: mutate2(lambda it: it.__setitem__(slice(0, 1), [it[0][:5] + [0, 4, 0], it[0][:5] + [4, 4, 0]])),
    "gemm2_pool_tile_twice": lambda: mutate2(lambda it: it.__setitem__(slice(0, 2), [it[0][:5] + [0, 4, 0], it[0][:5] + [4, 4, 1], it[1][:5] + [0, 4, 0], it[1][:5] + [4, 4, 1]])),
}


@pytest.mark.parametrize("name", list(MISTAKES))
def test_planted_mistakes_are_caught(name):
    with pytest.raises(AssertionError):
        check(MISTAKES[name]())
