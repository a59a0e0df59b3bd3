"""Helpers shared by the test modules (harness only: no arithmetic of the method)."""
import numpy as np

from oracle import schedule as so


def tiles_of(s):
    """(first, second) row arrays per first-wavefront tile of a schedule view dict."""
    fp, sp = s["tile_first_ptr"], s["tile_second_ptr"]
    return [(s["first_rows"][fp[v]:fp[v + 1]], s["second_rows"][sp[v]:sp[v + 1]])
            for v in range(len(fp) - 1)]


def units_of(s):
    up = s["wf1_unit_ptr"]
    return [s["wf1_rows"][up[u]:up[u + 1]] for u in range(len(up) - 1)]


def footprint(s, rows):
    g = s["lds_row_granule"]
    return s["lds_fixed_bytes"] + -(-rows // g) * g * s["lds_bytes_per_row"]


def check_schedule(A, s, ct_size, p):
    """Bit-exact comparison of a plan's schedule with the oracle's Algorithm 1 for the same
    tile-size inputs and the same fast-memory cost, plus the implementation-free validator."""
    ref = so.algorithm1(A.rowptr, A.colidx, ct_size=ct_size, p=p,
                        cost=lambda i0, i1: footprint(s, i1 - i0), fast_mem=s["fast_mem_bytes"])
    assert s["t"] == ref["t"]
    assert s["n_coarse_tiles"] == len(ref["coarse"])
    tiles = tiles_of(s)
    assert len(tiles) == len(ref["tiles"])
    for (first, second), (i0, i1, rows) in zip(tiles, ref["tiles"]):
        assert first.size == i1 - i0 and (first.size == 0 or (first[0] == i0 and first[-1] == i1 - 1))
        assert np.array_equal(first, np.arange(i0, i1))
        assert np.array_equal(np.sort(second), rows)     # the order inside a tile is free
    assert np.array_equal(np.sort(s["wf1_rows"]), ref["wf1_rows"])
    assert np.array_equal(s["spill"].astype(bool), ref["spill"])
    out = so.validate(A.rowptr, A.colidx, tiles, units_of(s), s["spill"].astype(bool),
                      tile_cost=lambda rows: footprint(s, rows), fast_mem=s["fast_mem_bytes"])
    assert out["superfluous_spill"] == 0
    assert out["n_fused_rows"] == s["n_fused_rows"]
    assert out["n_wf1_rows"] == s["n_wf1_rows"]
    assert out["n_spill"] == s["n_spill_rows"]
    fr = so.fused_ratios(A.rowptr, out["n_fused_rows"], out["fused_rows"])
    assert abs(fr["eq3"] - s["fused_ratio_eq3"]) < 1e-15
    assert abs(fr["rows"] - s["fused_ratio_rows"]) < 1e-15
    assert abs(fr["nnz"] - s["fused_ratio_nnz"]) < 1e-15
    lens = np.diff(A.rowptr.astype(np.int64))
    assert s["fused_nnz"] == int(lens[out["fused_rows"]].sum())
    return ref


def check_schedule_general(A, s):
    """Schedules whose tiles are not ranges of consecutive rows have many valid answers: they are
    checked by the implementation-free validator only (every iteration exactly once, every
    dependence inside its tile or across the barrier, minimal spill set, maximal fusion for the
    tiles chosen, footprint within the fast memory) and by a recount of the reported ratios."""
    tiles = tiles_of(s)
    # (a library-chosen schedule may leave fusable rows to the second wavefront and says how many:
    # maximality is then not a property to check)
    out = so.validate(A.rowptr, A.colidx, tiles, units_of(s), s["spill"].astype(bool),
                      tile_cost=lambda rows: footprint(s, rows), fast_mem=s["fast_mem_bytes"],
                      check_maximal=s["n_demoted_rows"] == 0)
    assert out["superfluous_spill"] == 0
    assert out["n_fused_rows"] == s["n_fused_rows"]
    assert out["n_wf1_rows"] == s["n_wf1_rows"]
    assert out["n_spill"] == s["n_spill_rows"]
    fr = so.fused_ratios(A.rowptr, out["n_fused_rows"], out["fused_rows"])
    assert abs(fr["rows"] - s["fused_ratio_rows"]) < 1e-15
    assert abs(fr["nnz"] - s["fused_ratio_nnz"]) < 1e-15
    for first, _ in tiles:
        assert np.all(np.diff(first) > 0)            # ascending inside a tile
    return out
