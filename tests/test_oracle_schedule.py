"""Pins of the schedule oracle (Algorithm 1 restatement + validator); no GPU needed."""
import os

import numpy as np
import pytest

import tf_inputs as ti
from oracle import schedule as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_tile_size_rule_golden():
    with open(os.path.join(GOLDEN, "tile_size_rule.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 5
    for n, ct, p, t in rows:
        assert so.tile_size_rule(int(n), int(ct), int(p)) == int(t)


def as_general(res, n):
    """(tiles, wf1 units) of an algorithm1() result in the validator's general form."""
    tiles = [(np.arange(i0, i1), rows) for (i0, i1, rows) in res["tiles"]]
    return tiles, [res["wf1_rows"]]


@pytest.mark.parametrize("seed", range(6))
def test_step1_against_set_brute_force(seed):
    n = 37
    A = ti.random_pattern_csr(n, n, 0.08, np.float64, seed, sort_cols=False, duplicates=True,
                              empty_row_prob=0.2)
    for t in (1, 4, 7, 16, 37, 50):
        res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
        assert res["t"] == t
        for (i0, i1, rows) in res["tiles"]:
            assert list(rows) == so.fused_in_range_bruteforce(A.rowptr, A.colidx, i0, i1)
        tiles, units = as_general(res, n)
        so.validate(A.rowptr, A.colidx, tiles, units, res["spill"])
        # spill set by brute force
        wf1 = set(int(j) for j in res["wf1_rows"])
        need = set()
        for j in wf1:
            need |= set(int(c) for c in A.colidx[A.rowptr[j]:A.rowptr[j + 1]])
        assert set(np.nonzero(res["spill"])[0]) == need


def count_fused(res):
    return sum(len(r) for (_, _, r) in res["tiles"])


def test_banded_closed_form_counts():
    n, h = 4096, 8
    A = ti.banded(n, h, np.float64, 1)
    expect = {16: 16, 32: 2064, 256: 3856}
    for t in (16, 32, 64, 128, 256, 512, 2048):
        res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
        assert count_fused(res) == so.banded_fused_count(n, t, h)
        if t in expect:
            assert count_fused(res) == expect[t]
        if t >= 4 * h:
            assert int(res["spill"].sum()) == (n // t - 1) * 4 * h
    assert int(so.algorithm1(A.rowptr, A.colidx, 256, 1)["spill"].sum()) == 480


def test_laplacian_closed_form_counts():
    g = 32                                    # half-bandwidth 32, n = 1024
    A = ti.laplacian_2d(g, np.float32)
    for t in (32, 64, 128, 256, 512):
        res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
        assert count_fused(res) == so.banded_fused_count(g * g, t, g)
    g = 8                                     # 3D: half-bandwidth g*g = 64, n = 512
    A = ti.laplacian_3d(g, np.float64)
    for t in (64, 128, 256):
        res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
        assert count_fused(res) == so.banded_fused_count(g ** 3, t, g * g)
    assert count_fused(so.algorithm1(A.rowptr, A.colidx, 64, 1)) == 0


def test_special_cases():
    n = 100
    eye = ti.Csr(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                 np.ones(n))
    res = so.algorithm1(eye.rowptr, eye.colidx, ct_size=7, p=1)
    assert count_fused(res) == n and not res["spill"].any() and res["wf1_rows"].size == 0
    A = ti.random_pattern_csr(n, n, 0.1, np.float64, 3)
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=n, p=1)        # one tile holds everything
    assert len(res["tiles"]) == 1 and count_fused(res) == n
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=2048, p=1)     # t > n
    assert count_fused(res) == n
    # a row with an entry at distance >= t can never be fused
    t = 10
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
    fused = np.zeros(n, bool)
    for (_, _, r) in res["tiles"]:
        fused[r] = True
    for j in range(n):
        cols = A.colidx[A.rowptr[j]:A.rowptr[j + 1]]
        if cols.size and np.abs(cols - j).max() >= t:
            assert not fused[j]


def test_step2_splitting():
    n, h = 1024, 4
    A = ti.banded(n, h, np.float64, 2)
    cost = lambda i0, i1: (i1 - i0) * 100 + 50
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=512, p=1, cost=cost, fast_mem=100 * 128 + 50)
    sizes = [i1 - i0 for (i0, i1, _) in res["tiles"]]
    assert sizes == [128] * 8                      # 512 -> 256 -> 128
    assert [len(r) for (_, _, r) in res["coarse"]] == [512 - h, 512 - h]
    assert count_fused(res) == so.banded_fused_count(n, 128, h)
    tiles, units = as_general(res, n)
    out = so.validate(A.rowptr, A.colidx, tiles, units, res["spill"],
                      tile_cost=lambda rows: rows * 100 + 50, fast_mem=100 * 128 + 50)
    assert out["n_fused_rows"] == count_fused(res) and out["superfluous_spill"] == 0
    # odd sizes: the left half gets the floor
    res = so.algorithm1(A.rowptr[:78], A.colidx[:A.rowptr[77]].clip(max=76), ct_size=77, p=1,
                        cost=lambda a, b: b - a, fast_mem=20)
    assert [i1 - i0 for (i0, i1, _) in res["tiles"]] == [19, 19, 19, 20]


def test_validator_catches_planted_mistakes():
    n = 60
    A = ti.banded(n, 2, np.float64, 9)
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=20, p=1)
    tiles, units = as_general(res, n)
    so.validate(A.rowptr, A.colidx, tiles, units, res["spill"])

    def expect(code, tiles_, units_, spill_):
        with pytest.raises(so.ScheduleError, match=code):
            so.validate(A.rowptr, A.colidx, tiles_, units_, spill_)

    # V1: a first-operation row produced twice / never
    t2 = [(np.append(tiles[0][0], 25), tiles[0][1])] + tiles[1:]
    expect("V1", t2, units, res["spill"])
    t2 = [(tiles[0][0][:-1], tiles[0][1])] + tiles[1:]
    expect("V1", t2, units, res["spill"])
    # V2: a second-operation row dropped / run twice
    expect("V2", tiles, [units[0][1:]], res["spill"])
    expect("V2", tiles, [np.append(units[0], tiles[0][1][0])], res["spill"])
    # V3: a boundary row forced into the tile
    j = int(units[0][0])
    t2 = [(tiles[0][0], np.append(tiles[0][1], j))] + tiles[1:]
    expect("V3", t2, [units[0][1:]], res["spill"])
    # V4: a needed spill bit cleared
    s2 = res["spill"].copy()
    s2[np.nonzero(s2)[0][0]] = False
    expect("V4", tiles, units, s2)
    # V7: a fusable row left in the second wavefront
    j = int(tiles[1][1][3])
    t2 = [tiles[0], (tiles[1][0], tiles[1][1][tiles[1][1] != j])] + tiles[2:]
    s2 = so.spill_set(A.rowptr, A.colidx, np.append(units[0], j))
    expect("V7", t2, [np.append(units[0], j)], s2)
    # V5 is a count, not an error
    s2 = np.ones(n, bool)
    assert so.validate(A.rowptr, A.colidx, tiles, units, s2)["superfluous_spill"] > 0
    # V6: a tile larger than the fast memory.  Tiles have 20 rows; with a cost of 10 per row a
    # budget of 200 holds them exactly, one less does not, and a tile that grew by merging two
    # (still a valid schedule otherwise) breaks a budget that held the original ones
    cost = lambda rows: 10 * rows
    so.validate(A.rowptr, A.colidx, tiles, units, res["spill"], tile_cost=cost, fast_mem=200)
    with pytest.raises(so.ScheduleError, match="V6"):
        so.validate(A.rowptr, A.colidx, tiles, units, res["spill"], tile_cost=cost, fast_mem=199)
    merged = so.algorithm1(A.rowptr, A.colidx, ct_size=40, p=1)
    mt, mu = as_general(merged, n)
    so.validate(A.rowptr, A.colidx, mt, mu, merged["spill"], tile_cost=cost, fast_mem=400)
    with pytest.raises(so.ScheduleError, match="V6"):
        so.validate(A.rowptr, A.colidx, mt, mu, merged["spill"], tile_cost=cost, fast_mem=200)
    # the check needs both the cost and the budget: without either nothing is tested
    so.validate(A.rowptr, A.colidx, mt, mu, merged["spill"], tile_cost=cost)


def test_validator_with_unread_rows_skipped():
    """A pattern whose columns 3 and 7 are read by no row: their first-operation rows may be
    missing from the tiles when the option says so, a row that is read may not."""
    n = 10
    cols = [[0, 1], [1], [2, 4], [4], [4, 5], [5], [6], [6, 8], [8, 9], [9]]
    rowptr = np.cumsum([0] + [len(c) for c in cols])
    colidx = np.concatenate(cols)
    res = so.algorithm1(rowptr, colidx, ct_size=5, p=1)
    tiles, units = as_general(res, n)
    so.validate(rowptr, colidx, tiles, units, res["spill"])
    drop = lambda first, r: first[first != r]
    skipped = [(drop(tiles[0][0], 3), tiles[0][1]), (drop(tiles[1][0], 7), tiles[1][1])]
    with pytest.raises(so.ScheduleError, match="V1"):
        so.validate(rowptr, colidx, skipped, units, res["spill"], check_maximal=False)
    so.validate(rowptr, colidx, skipped, units, res["spill"], check_maximal=False,
                unread_may_be_skipped=True)
    # row 4 is read: it has to stay
    bad = [(drop(tiles[0][0], 4), tiles[0][1]), tiles[1]]
    with pytest.raises(so.ScheduleError, match="V1"):
        so.validate(rowptr, colidx, bad, units, res["spill"], check_maximal=False,
                    unread_may_be_skipped=True)
    # an unread row may still not be produced twice
    twice = [(np.append(tiles[0][0], 7), tiles[0][1]), tiles[1]]
    with pytest.raises(so.ScheduleError, match="V1"):
        so.validate(rowptr, colidx, twice, units, res["spill"], check_maximal=False,
                    unread_may_be_skipped=True)


def test_fused_ratio_forms():
    n, h, t = 512, 4, 64
    A = ti.banded(n, h, np.float64, 4)
    res = so.algorithm1(A.rowptr, A.colidx, ct_size=t, p=1)
    fused = np.concatenate([r for (_, _, r) in res["tiles"]])
    fr = so.fused_ratios(A.rowptr, fused.size, fused)
    assert fr["rows"] == fused.size / n
    assert fr["eq3"] == fused.size / (2 * n) <= 0.5            # Eq. 3: denominator |I| + |J|
    lens = np.diff(A.rowptr)
    assert abs(fr["nnz"] - lens[fused].sum() / A.nnz) < 1e-15


def test_full_size_config_patterns():
    """Fused-row counts on the real config-2 and config-4 patterns (closed forms)."""
    A = ti.laplacian_2d(512, np.float32)
    for t, want in ((1024, 1024), (2048, 132096), (4096, 197632)):
        assert count_fused(so.algorithm1(A.rowptr, A.colidx, t, 1)) == want
    A = ti.laplacian_3d(64, np.float64)
    for t, want in ((4096, 0), (8192, 8192), (16384, 139264)):
        assert count_fused(so.algorithm1(A.rowptr, A.colidx, t, 1)) == want
