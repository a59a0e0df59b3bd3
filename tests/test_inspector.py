"""Host logic of the library: the inspector behind tf_plan_create, checked without a GPU
(TF_FLAG_SCHEDULE_ONLY) against the schedule oracle, bit for bit, and its error paths."""
import numpy as np
import pytest

import paper_2407_00243_amd as tf
import tf_inputs as ti
from util import check_schedule, check_schedule_general, footprint, tiles_of, units_of

SO = tf.TF_FLAG_SCHEDULE_ONLY


def plan_schedule(A, bcol, ccol, sparse, **kw):
    flags = kw.pop("flags", 0) | SO
    with tf.Plan(A, bcol, ccol, sparse, flags=flags, **kw) as pl:
        return pl.schedule()


@pytest.mark.parametrize("seed", range(5))
def test_random_patterns_match_oracle(seed):
    n = 200 + 37 * seed
    A = ti.random_pattern_csr(n, n, 0.02, np.float64, seed, sort_cols=False, duplicates=True,
                              empty_row_prob=0.15)
    # widen the band of some rows so that fused and unfused rows both occur
    for ct, p in ((16, 1), (64, 1), (50, 3), (2048, 7), (2048, 1)):
        s = plan_schedule(A, 8, 8, False, ct_size=ct, p=p)
        check_schedule(A, s, ct, p)
        s = plan_schedule(A, n, 8, True, ct_size=ct, p=p)
        check_schedule(A, s, ct, p)


@pytest.mark.parametrize("cfg,params", [
    (1, dict(ct_size=2048, p=256)), (1, dict(ct_size=2048, p=32)), (1, dict(ct_size=256, p=1)),
    (2, dict(ct_size=2048, p=32)), (2, dict(ct_size=4096, p=1, col_slice=16)),
    (2, dict(ct_size=8192, p=1, col_slice=8)),
    (4, dict(ct_size=2048, p=32)), (4, dict(ct_size=16384, p=1, col_slice=2)),
])
def test_structured_configs_match_oracle(cfg, params):
    prob = ti.config(cfg)
    s = plan_schedule(prob.A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm", **params)
    check_schedule(prob.A, s, params["ct_size"], params["p"])
    assert s["n_slices"] == -(-prob.ccol // s["col_slice"])
    for first, _ in tiles_of(s):
        assert footprint(s, first.size) <= s["fast_mem_bytes"]


@pytest.mark.parametrize("cfg,scale,params", [
    (1, None, dict()), (2, None, dict()), (2, None, dict(col_slice=32)), (4, None, dict()),
    (4, None, dict(col_slice=16)), (3, 13, dict()), (5, 13, dict(ct_size=300)),
])
def test_graph_grown_tiles_are_valid(cfg, scale, params):
    prob = ti.config(cfg, scale_down=scale)
    s = plan_schedule(prob.A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm",
                      flags=tf.TF_FLAG_REORDER, **params)
    check_schedule_general(prob.A, s)
    sizes = np.diff(s["tile_first_ptr"])
    assert np.all(sizes[:-1] == sizes[0]) and sizes[-1] <= sizes[0]    # all tiles full but the last
    assert footprint(s, int(sizes[0])) <= s["fast_mem_bytes"]
    if cfg == 2:
        # consecutive tiles of this size fuse nothing on the 2D grid; graph-grown tiles do
        assert s["fused_ratio_rows"] > 0.8 and s["n_spill_rows"] < 0.3 * prob.n
    if cfg == 4:
        assert s["fused_ratio_rows"] > 0.5


def test_graph_grown_tiles_on_random_patterns():
    for seed in range(4):
        n = 300
        A = ti.random_local_csr(n, 9, 4, 0.2, np.float32, seed)
        for ct in (16, 50, 2048):
            s = plan_schedule(A, 16, 16, False, ct_size=ct, p=1, flags=tf.TF_FLAG_REORDER)
            check_schedule_general(A, s)
            assert np.diff(s["tile_first_ptr"]).max() <= max(16, ct // 16 * 16)


def test_closed_form_counts_through_the_abi():
    A = ti.banded(4096, 8, np.float64, 1)
    for t, want in ((16, 16), (32, 2064), (256, 3856)):
        s = plan_schedule(A, 32, 32, False, ct_size=t, p=1)
        assert s["n_fused_rows"] == want
    s = plan_schedule(A, 32, 32, False, ct_size=256, p=1)
    assert s["n_spill_rows"] == 480
    # Algorithm 1's rule with p = 256 "cores" leaves 16-row tiles and almost nothing to fuse
    s = plan_schedule(A, 32, 32, False, ct_size=2048, p=256)
    assert s["t"] == 16 and s["n_fused_rows"] == 16


@pytest.mark.parametrize("cfg,scale", [(3, 14), (5, 14)])
def test_graph_configs_match_oracle(cfg, scale):
    prob = ti.config(cfg, scale_down=scale)
    s = plan_schedule(prob.A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm", ct_size=2048, p=32)
    check_schedule(prob.A, s, 2048, 32)
    lens = np.diff(prob.A.rowptr)
    # long rows get a unit of their own, placed first, longest first
    units = units_of(s)
    long_rows = [u[0] for u in units if u.size == 1 and lens[u[0]] >= 2048]
    assert all(lens[long_rows[i]] >= lens[long_rows[i + 1]] for i in range(len(long_rows) - 1))
    assert set(np.nonzero(lens >= 2048)[0]) - set(s["second_rows"]) == set(long_rows)


def test_step2_splits_to_the_lds_budget():
    prob = ti.config(2, scale_down=128)           # n = 16384, fp32, 64 -> 64
    s = plan_schedule(prob.A, 64, 64, False, ct_size=4096, p=1, fast_mem_bytes=96 * 1024)
    ref = check_schedule(prob.A, s, 4096, 1)
    sizes = {i1 - i0 for (i0, i1, _) in ref["tiles"]}
    assert sizes == {256}                          # 4096 -> ... -> 256 rows * 272 B + 16 KiB
    assert s["n_coarse_tiles"] == 4 and s["n_tiles"] == 64
    with pytest.raises(tf.TfError) as e:
        plan_schedule(prob.A, 64, 64, False, ct_size=4096, p=1, fast_mem_bytes=96 * 1024,
                      flags=tf.TF_FLAG_NO_SPLIT)
    assert e.value.status_name == "TF_EUNSUPPORTED"


def test_default_column_slice_narrows_until_the_tiles_fit():
    """A default column slice is cCol / k (rounded up to 16 columns) for the smallest k = 1, 2, 4,
    ... whose tiles hold t rows, or 256 rows if t is larger; an explicit slice is taken as given."""
    A = ti.banded(512, 3, np.float64, 5)

    def rows_that_fit(s):
        room = s["fast_mem_bytes"] - s["lds_fixed_bytes"]
        g = s["lds_row_granule"]
        return room // s["lds_bytes_per_row"] // g * g

    # fp64, bCol = 256, cCol = 128: a 128-column C slice is 256 KiB, more than the fast memory
    s = plan_schedule(A, 256, 128, False, ct_size=64, p=1)
    assert s["col_slice"] % 16 == 0 and 16 <= s["col_slice"] < 128
    assert s["n_slices"] == -(-128 // s["col_slice"])
    assert rows_that_fit(s) >= 64 or s["col_slice"] == 16
    check_schedule(A, s, 64, 1)
    with pytest.raises(tf.TfError) as e:
        plan_schedule(A, 256, 128, False, ct_size=64, p=1, col_slice=128)
    assert e.value.status_name == "TF_EUNSUPPORTED"
    # fp64, 128 -> 128: the full-width C slice fits (128 KiB) but leaves tiles of a few rows
    wide = plan_schedule(A, 128, 128, False, ct_size=64, p=1, col_slice=128)
    assert rows_that_fit(wide) < 64
    s = plan_schedule(A, 128, 128, False, ct_size=64, p=1)
    assert s["col_slice"] == 64 and rows_that_fit(s) >= 64
    assert s["n_fused_rows"] > wide["n_fused_rows"]
    # a large t asks for 256 rows, not for t
    s = plan_schedule(A, 128, 128, False, ct_size=2048, p=1)
    assert rows_that_fit(s) >= 256 and s["col_slice"] == 32
    s2 = plan_schedule(A, 128, 128, False, ct_size=2048, p=1, col_slice=2 * s["col_slice"])
    assert rows_that_fit(s2) < 256
    # nothing to narrow when the tiles fit as they are
    s = plan_schedule(ti.config(2, scale_down=64).A, 64, 64, False, ct_size=65536, p=1)
    assert s["col_slice"] == 64 and s["n_slices"] == 1


@pytest.mark.parametrize("width,dtype", [(32, np.float32), (64, np.float32), (32, np.float64),
                                         (128, np.float64)])
def test_graph_grown_tiles_fill_the_workgroups_evenly(width, dtype):
    """One workgroup per compute unit (256 when no device is asked) walks the tiles of its column
    slice: the tile count is brought close below a multiple of the workgroups per slice, so the
    last round is nearly full, by shrinking the tiles by less than half."""
    A = ti.laplacian_2d(512, dtype)
    s = plan_schedule(A, width, width, False, ct_size=65536, p=1, flags=tf.TF_FLAG_REORDER)
    per_slice = 256 // s["n_slices"]
    nt = s["n_tiles"]
    rounds = -(-nt // per_slice)
    assert nt / (rounds * per_slice) >= 0.95
    sizes = np.diff(s["tile_first_ptr"])
    room = (s["fast_mem_bytes"] - s["lds_fixed_bytes"]) // s["lds_bytes_per_row"]
    assert sizes.max() <= room and sizes.max() > room // 2 - s["lds_row_granule"]
    check_schedule_general(A, s)


def test_large_matrix_schedule_built_by_several_threads():
    """A matrix of a quarter of a million rows is classified and packed by several host threads;
    the schedule must be valid, must not depend on how the tiles were dealt out (two builds
    agree, and so does a build by a single thread) and, for consecutive tiles, must equal the
    oracle's Algorithm 1."""
    A = ti.laplacian_2d(512, np.float32)
    s1 = plan_schedule(A, 64, 64, False, ct_size=65536, p=1, flags=tf.TF_FLAG_REORDER)
    s2 = plan_schedule(A, 64, 64, False, ct_size=65536, p=1, flags=tf.TF_FLAG_REORDER)
    for key in ("first_rows", "second_rows", "tile_second_ptr", "wf1_rows", "wf1_unit_ptr", "spill"):
        assert np.array_equal(s1[key], s2[key]), key
    assert s1["fused_nnz"] == s2["fused_nnz"] and s1["eq2_cost_max"] == s2["eq2_cost_max"]
    check_schedule_general(A, s1)
    import os
    os.environ["TF_HOST_THREADS"] = "1"            # read at every plan creation
    try:
        s3 = plan_schedule(A, 64, 64, False, ct_size=65536, p=1, flags=tf.TF_FLAG_REORDER)
    finally:
        del os.environ["TF_HOST_THREADS"]
    for key in ("tile_first_ptr", "first_rows", "second_rows", "tile_second_ptr", "wf1_rows",
                "wf1_unit_ptr", "spill"):
        assert np.array_equal(s1[key], s3[key]), key
    assert s1["fused_nnz"] == s3["fused_nnz"] and s1["second_block_bytes"] == s3["second_block_bytes"]
    B = ti.banded(300000, 3, np.float64, 3)
    s = plan_schedule(B, 16, 16, False, ct_size=512, p=1)
    assert s["n_tiles"] >= 64
    check_schedule(B, s, 512, 1)


def test_schedule_view_reports_the_second_phase_blocks():
    prob = ti.config(2, scale_down=128)
    s = plan_schedule(prob.A, 64, 64, False, ct_size=256, p=1)
    # per fused row: a 4-byte id and, per padded entry slot, a 2-byte position and a 4-byte value
    rows = np.diff(s["tile_second_ptr"]).max()
    assert s["second_block_bytes"] >= rows * (4 + 4 * (2 + 4))
    assert s["second_block_in_lds"] == 1 and s["lds_launch_bytes"] == 0      # schedule only


@pytest.mark.parametrize("reorder", [0, 1])
def test_unread_rows_leave_the_first_lists(reorder):
    """TF_FLAG_SKIP_UNREAD: the first lists are those of the plain plan without the rows that no
    row of A reads (a tile whose rows are all unread keeps its first); second lists, second
    wavefront and spill set do not change."""
    from oracle import schedule as so
    prob = ti.config(5, scale_down=12)            # R-MAT: many vertices without an edge
    A = prob.A
    read = np.zeros(A.n_rows, bool)
    read[A.colidx] = True
    assert 0.2 < read.mean() < 0.9
    base = tf.TF_FLAG_REORDER if reorder else 0
    s0 = plan_schedule(A, 8, 32, True, ct_size=200, p=1, flags=base)
    s1 = plan_schedule(A, 8, 32, True, ct_size=200, p=1, flags=base | tf.TF_FLAG_SKIP_UNREAD)
    assert s0["n_first_rows"] == A.n_rows and s1["n_first_rows"] == s1["first_rows"].size
    for key in ("second_rows", "tile_second_ptr", "wf1_rows", "wf1_unit_ptr", "spill"):
        assert np.array_equal(s0[key], s1[key]), key
    all_unread = 0
    for (f0, _), (f1, _) in zip(tiles_of(s0), tiles_of(s1)):
        keep = f0[read[f0]]
        if keep.size == 0:
            keep = f0[:1]
            all_unread += 1
        assert np.array_equal(f1, keep)
    assert s1["n_first_rows"] == int(read.sum()) + all_unread
    so.validate(A.rowptr, A.colidx, tiles_of(s1), units_of(s1), s1["spill"].astype(bool),
                check_maximal=False, unread_may_be_skipped=True)
    # a matrix with a full diagonal has no unread row: nothing changes
    B = ti.config(3, scale_down=12).A
    t0 = plan_schedule(B, 16, 16, False, ct_size=200, p=1)
    t1 = plan_schedule(B, 16, 16, False, ct_size=200, p=1, flags=tf.TF_FLAG_SKIP_UNREAD)
    assert np.array_equal(t0["first_rows"], t1["first_rows"])


def test_degenerate_inputs():
    empty = ti.Csr(0, 0, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    s = plan_schedule(empty, 4, 4, False)
    assert s["n_tiles"] == 0 and s["n_wf1_units"] == 0 and s["n_fused_rows"] == 0
    n = 10
    no_entries = ti.Csr(n, n, np.zeros(n + 1, np.int32), np.zeros(0, np.int32),
                        np.zeros(0, np.float64))
    s = plan_schedule(no_entries, 4, 4, False, ct_size=4, p=1)
    assert s["n_fused_rows"] == n and s["n_wf1_rows"] == 0 and s["n_spill_rows"] == 0
    one = ti.Csr(1, 1, np.array([0, 1], np.int32), np.array([0], np.int32), np.ones(1, np.float32))
    s = plan_schedule(one, 1, 1, False)
    assert s["n_tiles"] == 1 and s["n_fused_rows"] == 1


def bad(A, **kw):
    with pytest.raises(tf.TfError) as e:
        plan_schedule(A, kw.pop("bcol", 4), kw.pop("ccol", 4), False, **kw)
    return e.value.status_name


def test_error_paths():
    A = ti.banded(32, 2, np.float64, 1)
    assert bad(A, bcol=0) == "TF_EINVAL"
    assert bad(A, ccol=-1) == "TF_EINVAL"
    assert bad(A, ct_size=-1) == "TF_EINVAL"
    assert bad(A, fast_mem_bytes=64) == "TF_EUNSUPPORTED"     # not even one D1 row fits
    assert bad(A, ccol=64, col_slice=5) == "TF_EINVAL"        # not a multiple of 16 bytes
    rp = A.rowptr.copy()
    rp[5], rp[6] = rp[6], rp[5]
    assert bad(A._replace(rowptr=rp)) == "TF_EBADCSR"
    rp = A.rowptr.copy()
    rp[-1] -= 1
    assert bad(A._replace(rowptr=rp)) == "TF_EBADCSR"
    ci = A.colidx.copy()
    ci[3] = 32
    assert bad(A._replace(colidx=ci)) == "TF_EBADCSR"
    ci[3] = -1
    assert bad(A._replace(colidx=ci)) == "TF_EBADCSR"
    assert bad(A._replace(n_cols=33)) == "TF_EINVAL"           # not square
    assert "square" in tf.tf_last_error()
    # the transpose of C is a dense-B variant; it leaves the schedule as it is
    with pytest.raises(tf.TfError) as e:
        tf.Plan(A, 4, 4, True, flags=SO | tf.TF_FLAG_C_TRANSPOSED)
    assert e.value.status_name == "TF_EUNSUPPORTED"
    with tf.Plan(A, 4, 8, False, flags=SO) as p0, \
            tf.Plan(A, 4, 8, False, flags=SO | tf.TF_FLAG_C_TRANSPOSED) as p1:
        s0, s1 = p0.schedule(), p1.schedule()
        assert np.array_equal(s0["first_rows"], s1["first_rows"])
        assert np.array_equal(s0["second_rows"], s1["second_rows"])
    # a schedule-only plan cannot execute
    with tf.Plan(A, 4, 4, False, flags=SO) as pl:
        with pytest.raises(tf.TfError) as e:
            tf.tf_gemm_spmm(pl.handle, 16, 16, 16)
        assert e.value.status_name == "TF_EINVAL"


# ---------------------------------------------------------------- the tiling left to the library

def test_defaults_leave_the_tiling_to_the_library_stencils_and_band():
    """tf_plan_create without tile parameters on the band and stencil configurations at full size:
    the band keeps Algorithm 1's consecutive tiles (p = a quarter of 256 compute units gives t =
    64, three quarters of the rows fuse); the stencils in natural ordering, where consecutive
    tiles that fit the fast memory fuse nothing, get graph-grown tiles.  Fused shares are at least
    those of the hand-picked parameters the benchmark used before the library chose by itself."""
    floor = {1: 0.75, 2: 0.80, 4: 0.54}
    for cfg in (1, 2, 4):
        prob = ti.config(cfg)
        s = plan_schedule(prob.A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm")
        check_schedule_general(prob.A, s)
        assert s["automatic"] == 1 and s["far_rows"] == 0 and s["n_demoted_rows"] == 0
        assert s["grown_tiles"] == (0 if cfg == 1 else 1)
        assert s["fused_ratio_nnz"] >= floor[cfg], (cfg, s["fused_ratio_nnz"])
        assert s["first_wavefront_streams"] == 0 and s["d1_slices"] == 1
        if cfg == 1:
            assert s["t"] == 64
            check_schedule(prob.A, s, 2048, 64)         # Algorithm 1 to the letter, with p = 64
        if cfg == 2:
            assert s["fast_mem_bytes"] == 80 * 1024     # two workgroups per compute unit
    # any explicit tile size or tile count switches the choice off
    prob = ti.config(2)
    s = plan_schedule(prob.A, prob.bcol, prob.ccol, False, ct_size=2048)
    assert s["automatic"] == 0 and s["grown_tiles"] == 0 and s["n_fused_rows"] == 0
    check_schedule(prob.A, s, 2048, 32)


@pytest.mark.parametrize("cfg", [3, 5])
def test_defaults_on_graphs_stream_the_first_wavefront(cfg):
    """The graph configurations at a quarter of their size: only rows with nothing but a diagonal
    entry (config 3) or with no entry at all (config 5) fuse, plus a handful whose few neighbours
    happen to sit in the same tile; those are left to the second wavefront (counted), so that no
    fused row reads the LDS tile and the first wavefront streams.  Config 3's workspace (512-byte
    rows, more than 64 MiB of them, read from all over the matrix) is cut into four slices."""
    prob = ti.config(cfg, scale_down=18)
    A = prob.A
    s = plan_schedule(A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm")
    check_schedule_general(A, s)
    lens = np.diff(A.rowptr.astype(np.int64))
    diag_only = (lens == 1) & (A.colidx[np.minimum(A.rowptr[:-1], A.nnz - 1)] == np.arange(A.n_rows))
    assert s["automatic"] == 1 and s["far_rows"] == 1 and s["grown_tiles"] == 0
    assert s["n_direct_rows"] == int((lens == 0).sum() + diag_only.sum()) == s["n_fused_rows"]
    assert s["first_wavefront_streams"] == 1
    assert 0 < s["n_demoted_rows"] < 100
    assert s["d1_slices"] == (4 if cfg == 3 else 1)
    assert s["d1_rows"] == s["n_spill_rows"] == int(s["spill"].sum())
    # the same matrix with Algorithm 1's parameters given keeps every row that a tile can fuse
    s1 = plan_schedule(A, prob.bcol, prob.ccol, prob.kind == "spmm_spmm", ct_size=2048, p=64)
    assert s1["n_demoted_rows"] == 0 and s1["n_fused_rows"] == s["n_fused_rows"] + s["n_demoted_rows"]
    assert s1["first_wavefront_streams"] == 0
    check_schedule(A, s1, 2048, 64)


def test_csr_validate_checks_a_matrix_on_request():
    """The execution calls take a CSR B as given; tf_csr_validate is the check a caller can run
    first: monotone row pointers from 0 to nnz, columns inside the matrix (host arrays here)."""
    B = ti.random_pattern_csr(50, 30, 0.1, np.float32, 3)
    tf.tf_csr_validate(B)

    def bad(M):
        with pytest.raises(tf.TfError) as e:
            tf.tf_csr_validate(M)
        return e.value.status_name

    rp = B.rowptr.copy()
    rp[0] = 1
    assert bad(B._replace(rowptr=rp)) == "TF_EBADCSR"
    rp = B.rowptr.copy()
    rp[10], rp[11] = rp[11] + 1, rp[10]
    assert bad(B._replace(rowptr=rp)) == "TF_EBADCSR"
    ci = B.colidx.copy()
    ci[5] = 30                                   # one past the last column
    assert bad(B._replace(colidx=ci)) == "TF_EBADCSR"
    ci[5] = -1
    assert bad(B._replace(colidx=ci)) == "TF_EBADCSR"
    assert bad(B._replace(rowptr=B.rowptr[:-1].copy(), n_rows=49)) == "TF_EBADCSR"   # rowptr[n] != nnz
