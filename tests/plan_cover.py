"""Checks that the work lists of the two grouped GEMMs cover every kept unit exactly once (used by the GPU
test on the plan kernel's lists, and by a CPU test on hand-made lists with planted mistakes).

plan: dict of numpy arrays / ints as DualSparseLayer.plan() returns them (row_bits, expert_row0, expert_nrows,
tile_rows, shared_rows, counters, items1, items2).  Raises AssertionError on the first violation.
"""
import numpy as np


def check_cover(plan, *, name, T, D, F, P, E_res, n_shared=0, F_sh=0):
    BM = int(plan["tile_rows"])
    assert BM == 256
    Fp = F // P
    F_sh = n_shared * F_sh
    bits = plan["row_bits"].astype(np.int64)
    sh_rows = int(plan["shared_rows"])
    # experts in the order of the lists' expert field: resident experts 0..E_res-1, then the shared pseudo-expert
    experts = [(e, int(plan["expert_row0"][e]), int(plan["expert_nrows"][e]), P, Fp) for e in range(E_res)]
    if n_shared:
        experts.append((E_res, 0, T, 1, F_sh))
        assert sh_rows >= T
    it1 = plan["items1"].astype(np.int64)
    it2 = plan["items2"].astype(np.int64)
    assert len(it1) == plan["counters"][0] and len(it2) == plan["counters"][1]
    ND2 = (D + 255) // 256

    pool_tiles = it2[it2[:, 7] > 0, 7]
    assert len(np.unique(pool_tiles)) == len(pool_tiles) and (len(pool_tiles) == 0 or pool_tiles.max() <= 768)

    for e, r0, n, nparts, fp in experts:
        nt1 = (fp + 127) // 128
        ksp = fp // 32
        rows_bits = bits[r0:r0 + n] if e < E_res else np.ones(n, np.int64)
        assert n == 0 or np.all(rows_bits != 0)  # only pairs that keep something have a row
        mine1 = it1[it1[:, 2] == e]
        mine2 = it2[it2[:, 2] == e]
        if n == 0:
            assert len(mine1) == 0 and len(mine2) == 0
            continue
        # ---- second GEMM: groups (first row, rows, column tile)
        reads = np.zeros((nparts, n), bool)  # rows of H (per partition) that some item of the second GEMM reads
        for jd in range(ND2):
            cover = np.zeros(n, np.int64)
            col = mine2[mine2[:, 3] == jd]
            for key in {(int(a), int(b)) for a, b in col[:, :2]}:
                grp = col[(col[:, 0] == key[0]) & (col[:, 1] == key[1])]
                a, cnt = key[0] - r0, key[1]
                assert 0 <= a and a + cnt <= n and 1 <= cnt <= 320, (name, e, key)
                cover[a:a + cnt] += 1
                kmask = int(grp[0, 4])
                assert np.all(grp[:, 4] == kmask) and 0 < kmask < (1 << nparts)
                need = int(np.bitwise_or.reduce(rows_bits[a:a + cnt])) & ((1 << nparts) - 1)
                assert need & ~kmask == 0, (name, e, key, need, kmask)  # it sums over every partition one of its rows keeps
                order = np.argsort(grp[:, 5])
                lo = 0
                for g in grp[order]:
                    assert g[5] == lo and g[6] >= 1, (name, e, key, grp)  # K ranges without gap or overlap
                    lo += g[6]
                assert lo == ksp, (name, e, key, lo, ksp)
                assert np.sum(grp[:, 7] == 0) == 1  # one piece writes the rows of the per-pair output
                if jd == 0:
                    for p in range(nparts):
                        if (kmask >> p) & 1:
                            reads[p, a:a + cnt] = True
            assert np.all(cover == 1), (name, e, jd, np.flatnonzero(cover != 1)[:8])
        # ---- first GEMM
        for p in range(nparts):
            keeps = ((rows_bits >> p) & 1).astype(bool)
            for jt in range(nt1):
                sel = mine1[(mine1[:, 3] == p) & (mine1[:, 4] == jt)]
                live = fp - jt * 128
                mult = {0: np.zeros(n, np.int64), 1: np.zeros(n, np.int64), 2: np.zeros(n, np.int64)}
                fill = {0: np.zeros(n, np.int64), 1: np.zeros(n, np.int64), 2: np.zeros(n, np.int64)}
                for row0, nrows, _, _, _, nfill, half, _ in sel:
                    a = row0 - r0
                    assert 0 <= a and 1 <= nrows <= nfill <= 320 and a + nfill <= ((n + BM - 1) // BM) * BM, (name, e, p, jt, row0, nrows, nfill)
                    assert half in (0, 1, 2) and (half == 0 or nrows <= 128)
                    mult[int(half)][a:min(a + nrows, n)] += 1
                    fill[int(half)][a:min(a + nfill, n)] += 1
                second_half_exists = live > 64
                halves = mult[1] + mult[2]
                assert np.all((mult[0] > 0) + (halves > 0) <= 1)  # whole items and halves never overlap
                m = mult[0] + mult[1]  # a whole item, or the first half
                assert np.all(m[keeps] == 1) and np.all(m <= 1), (name, e, p, jt)
                if second_half_exists:
                    assert np.array_equal(mult[2], mult[1]) and np.array_equal(fill[2], fill[1]), (name, e, p, jt)  # where there is a first half there is a second
                else:
                    assert not mult[2].any()
                f = fill[0] + fill[1]
                assert np.all(f <= 1) and np.all(f[reads[p]] == 1), (name, e, p, jt, np.flatnonzero(reads[p] & (f != 1))[:8])
        # no item for a partition or neuron tile that does not exist
        assert np.all((mine1[:, 3] < nparts) & (mine1[:, 4] < nt1))
