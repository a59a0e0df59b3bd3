"""Schedule oracle for tile fusion  --  TEST INFRASTRUCTURE, not part of the product.

Two independent things live here, both integer-only and written from the paper's Section 3.1:

1.  `algorithm1`: the tile fusion scheduler (Algorithm 1) for tiles of consecutive iterations.
    Step 1 forms uniform tiles of `t` consecutive rows and fuses a second-operation row into the
    tile of the same range exactly when every one of its incoming edges (the column indices of
    its row of A) lies inside the tile; all other rows go to the second wavefront.  Step 2
    halves every fused tile whose cost exceeds the fast-memory size until it fits.
    Readings taken where the printed algorithm is ambiguous:
      * the fusion test is  i0 <= col < i1  for *every* stored entry of the row (the printed
        strict "<" on the left would exclude a dependence on the tile's own first row, which
        the prose and the example of Section 3.1.1 include); an empty row is fused;
      * the outer loop advances by t, tile number v = i0 / t, the last tile may be short;
      * t = ctSize when ceil(n / ctSize) >= p, otherwise ceil(n / p);
      * `split` cuts a tile's row range at its midpoint (left half gets floor(rows / 2)) and
        re-tests every row of the tile against the half that contains it; rows that reach
        across the cut move to the second wavefront; recursion stops at a one-row tile;
      * the cost of a tile is supplied by the caller (on the GPU it is the LDS footprint of the
        tile; Eq. 2's value is a diagnostic only and is unpinned);
      * the spill set (first-operation rows whose D1 row some second-wavefront row reads) is
        not in the paper; it follows from the single barrier between the two wavefronts.

2.  `validate`: an implementation-free check of *any* schedule (consecutive tiles or not),
    from the properties the paper states: a wavefront's tiles are independent and need no
    synchronisation (Section 3.1.1), a row is fused only if all its incoming edges are in the
    tile (Algorithm 1), there are exactly two wavefronts with one barrier between them and no
    redundant computation (Section 3.1 "Objective and Constraints", Section 6).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- Algorithm 1

def tile_size_rule(n: int, ct_size: int, p: int) -> int:
    """First line of step 1: t = ctSize if ceil(n/ctSize) >= p else ceil(n/p)."""
    if n <= 0:
        return max(1, ct_size)
    if -(-n // ct_size) >= p:
        return ct_size
    return -(-n // p)


def _row_min_max(rowptr: np.ndarray, colidx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Smallest and largest column index of every row (empty rows: +inf-like / -1)."""
    n = rowptr.size - 1
    lo = np.full(n, np.iinfo(np.int64).max, dtype=np.int64)
    hi = np.full(n, -1, dtype=np.int64)
    lens = np.diff(rowptr.astype(np.int64))
    nz = np.nonzero(lens > 0)[0]
    if nz.size:
        starts = rowptr[nz].astype(np.int64)
        c = colidx.astype(np.int64)
        lo[nz] = np.minimum.reduceat(c, starts)
        hi[nz] = np.maximum.reduceat(c, starts)
    return lo, hi


def fused_in_range(rowptr, colidx, i0: int, i1: int,
                   minmax: Optional[Tuple[np.ndarray, np.ndarray]] = None) -> np.ndarray:
    """Rows j in [i0, i1) whose stored columns all lie in [i0, i1) (empty rows included)."""
    lo, hi = minmax if minmax is not None else _row_min_max(np.asarray(rowptr), np.asarray(colidx))
    j = np.arange(i0, i1, dtype=np.int64)
    ok = (hi[j] < 0) | ((lo[j] >= i0) & (hi[j] < i1))
    return j[ok]


def fused_in_range_bruteforce(rowptr, colidx, i0: int, i1: int) -> List[int]:
    """Same as `fused_in_range`, written with Python sets for tiny inputs."""
    tile = set(range(i0, i1))
    out = []
    for j in range(i0, i1):
        deps = set(int(c) for c in colidx[rowptr[j]:rowptr[j + 1]])
        if deps <= tile:
            out.append(j)
    return out


def algorithm1(rowptr, colidx, ct_size: int, p: int,
               cost: Optional[Callable[[int, int], int]] = None,
               fast_mem: Optional[int] = None) -> Dict:
    """Tile fusion scheduler for consecutive tiles.  Returns
        t            the uniform step-1 tile size
        tiles        list of (i0, i1, fused_rows ndarray) after step 2, ordered by i0
        coarse       the same list after step 1 only
        wf1_rows     sorted ndarray of second-wavefront rows
        spill        bool[n]: first-operation rows read by some second-wavefront row
    """
    rowptr = np.asarray(rowptr)
    colidx = np.asarray(colidx)
    n = rowptr.size - 1
    t = tile_size_rule(n, ct_size, p)
    mm = _row_min_max(rowptr, colidx)
    coarse = []
    for i0 in range(0, n, t):
        i1 = min(n, i0 + t)
        coarse.append((i0, i1, fused_in_range(rowptr, colidx, i0, i1, mm)))

    def split(i0: int, i1: int) -> List[Tuple[int, int, np.ndarray]]:
        if cost is None or fast_mem is None or cost(i0, i1) <= fast_mem or i1 - i0 <= 1:
            return [(i0, i1, fused_in_range(rowptr, colidx, i0, i1, mm))]
        mid = i0 + (i1 - i0) // 2
        return split(i0, mid) + split(mid, i1)

    tiles = []
    for (i0, i1, _) in coarse:
        tiles.extend(split(i0, i1))
    fused = np.zeros(n, dtype=bool)
    for (_, _, rows) in tiles:
        fused[rows] = True
    wf1_rows = np.nonzero(~fused)[0]
    spill = spill_set(rowptr, colidx, wf1_rows)
    return dict(t=t, tiles=tiles, coarse=coarse, wf1_rows=wf1_rows, spill=spill)


def spill_set(rowptr, colidx, wf1_rows) -> np.ndarray:
    """spill[i] is True iff some second-wavefront row has a stored entry in column i."""
    rowptr = np.asarray(rowptr).astype(np.int64)
    n = rowptr.size - 1
    in_wf1 = np.zeros(n, dtype=bool)
    in_wf1[np.asarray(wf1_rows, dtype=np.int64)] = True
    entry_row = np.repeat(np.arange(n), np.diff(rowptr))
    spill = np.zeros(n, dtype=bool)
    spill[np.asarray(colidx)[in_wf1[entry_row]]] = True
    return spill


def fused_ratios(rowptr, n_fused_rows: int, fused_rows: np.ndarray) -> Dict[str, float]:
    """Three forms of the fused ratio: Eq. 3 literally (denominator |I| + |J| = 2n), the share
    of second-operation rows that are fused, and the share of second-operation nonzeros
    (= floating-point work) executed in the first wavefront."""
    rowptr = np.asarray(rowptr).astype(np.int64)
    n = rowptr.size - 1
    nnz = int(rowptr[-1])
    lens = np.diff(rowptr)
    fused_nnz = int(lens[np.asarray(fused_rows, dtype=np.int64)].sum())
    return dict(eq3=(n_fused_rows / (2.0 * n)) if n else 0.0,
                rows=(n_fused_rows / float(n)) if n else 0.0,
                nnz=(fused_nnz / float(nnz)) if nnz else 0.0)


# --------------------------------------------------------------------------- closed forms

def banded_fused_count(n: int, t: int, h: int) -> int:
    """Number of fused rows after step 1 for a matrix whose every row reaches exactly h columns
    to each side (clipped at the matrix edges), when t divides n and n / t >= 2: interior
    tiles lose h rows at each end, the first and last tile only at their inner end."""
    assert n % t == 0 and n // t >= 2
    return (n // t - 2) * max(0, t - 2 * h) + 2 * max(0, t - h)


# --------------------------------------------------------------------------- validator

class ScheduleError(AssertionError):
    pass


def validate(rowptr, colidx, tiles: Sequence[Tuple[np.ndarray, np.ndarray]],
             wf1_units: Sequence[np.ndarray], spill: np.ndarray,
             tile_cost: Optional[Callable[[int], int]] = None,
             fast_mem: Optional[int] = None, check_maximal: bool = True,
             unread_may_be_skipped: bool = False) -> Dict:
    """Checks a schedule given in its most general form.

    tiles      sequence of (first, second): the first-operation rows the tile produces and the
               second-operation rows it consumes them with
    wf1_units  sequence of row arrays of the second wavefront
    spill      bool[n]

    Raises ScheduleError naming the violated property:
      V1  every first-operation row is produced by exactly one first-wavefront tile
          (with unread_may_be_skipped: every row that some row of A reads exactly once, the
          others at most once; V7 then needs check_maximal=False, a skipped row has no tile)
      V2  every second-operation row runs exactly once over both wavefronts
      V3  every incoming edge of a fused row is a first-operation row of the same tile
      V4  every incoming edge of a second-wavefront row is spilled
      V6  every tile's cost is within the fast memory
      V7  (maximality) a second-wavefront row has an incoming edge outside the tile that
          produces its own first-operation row
    and returns counts, including V5 (number of spilled rows no second-wavefront row reads).
    """
    rowptr = np.asarray(rowptr).astype(np.int64)
    colidx = np.asarray(colidx).astype(np.int64)
    n = rowptr.size - 1
    tile_of = np.full(n, -1, dtype=np.int64)
    produced = np.zeros(n, dtype=np.int64)
    for v, (first, _) in enumerate(tiles):
        first = np.asarray(first, dtype=np.int64)
        if first.size and (first.min() < 0 or first.max() >= n):
            raise ScheduleError(f"V1: tile {v} lists a first-operation row outside [0, n)")
        np.add.at(produced, first, 1)
        tile_of[first] = v
    wrong = produced != 1
    if unread_may_be_skipped:
        is_read = np.zeros(n, dtype=bool)
        is_read[colidx] = True
        wrong = np.where(is_read, produced != 1, produced > 1)
    if np.any(wrong):
        bad = int(np.nonzero(wrong)[0][0])
        raise ScheduleError(f"V1: first-operation row {bad} produced {int(produced[bad])} times")

    runs = np.zeros(n, dtype=np.int64)
    fused_tile = np.full(n, -1, dtype=np.int64)
    for v, (_, second) in enumerate(tiles):
        second = np.asarray(second, dtype=np.int64)
        if second.size and (second.min() < 0 or second.max() >= n):
            raise ScheduleError(f"V2: tile {v} lists a second-operation row outside [0, n)")
        np.add.at(runs, second, 1)
        fused_tile[second] = v
    wf1_mask = np.zeros(n, dtype=bool)
    for u, rows in enumerate(wf1_units):
        rows = np.asarray(rows, dtype=np.int64)
        if rows.size and (rows.min() < 0 or rows.max() >= n):
            raise ScheduleError(f"V2: second-wavefront unit {u} lists a row outside [0, n)")
        np.add.at(runs, rows, 1)
        wf1_mask[rows] = True
    if np.any(runs != 1):
        bad = int(np.nonzero(runs != 1)[0][0])
        raise ScheduleError(f"V2: second-operation row {bad} runs {int(runs[bad])} times")

    entry_row = np.repeat(np.arange(n), np.diff(rowptr))
    is_fused_entry = fused_tile[entry_row] >= 0
    bad = is_fused_entry & (tile_of[colidx] != fused_tile[entry_row])
    if np.any(bad):
        q = int(np.nonzero(bad)[0][0])
        raise ScheduleError(f"V3: fused row {int(entry_row[q])} depends on row {int(colidx[q])} "
                            f"of another tile")
    spill = np.asarray(spill, dtype=bool)
    if spill.shape != (n,):
        raise ScheduleError("V4: spill mask has the wrong length")
    bad = wf1_mask[entry_row] & ~spill[colidx]
    if np.any(bad):
        q = int(np.nonzero(bad)[0][0])
        raise ScheduleError(f"V4: second-wavefront row {int(entry_row[q])} reads unspilled row "
                            f"{int(colidx[q])}")
    needed = np.zeros(n, dtype=bool)
    needed[colidx[wf1_mask[entry_row]]] = True
    superfluous = int(np.count_nonzero(spill & ~needed))

    if tile_cost is not None and fast_mem is not None:
        for v, (first, _) in enumerate(tiles):
            if tile_cost(len(first)) > fast_mem:
                raise ScheduleError(f"V6: tile {v} costs {tile_cost(len(first))} > {fast_mem}")

    if check_maximal:
        # a second-wavefront row all of whose edges stay inside its own tile should have been fused
        own = tile_of[entry_row]
        outside = np.zeros(n, dtype=bool)
        outside[entry_row[tile_of[colidx] != own]] = True
        lazy = wf1_mask & ~outside
        if np.any(lazy):
            raise ScheduleError(f"V7: row {int(np.nonzero(lazy)[0][0])} could have been fused")

    n_fused = int(np.count_nonzero(fused_tile >= 0))
    return dict(n_fused_rows=n_fused, n_wf1_rows=int(wf1_mask.sum()),
                n_spill=int(spill.sum()), superfluous_spill=superfluous,
                fused_rows=np.nonzero(fused_tile >= 0)[0])
