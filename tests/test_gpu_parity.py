"""Parity of the HIP path with the CPU oracle, through the C ABI.  All tests need a GPU."""
import numpy as np
import pytest

import oracle
import tf_inputs as ti
from util import check_schedule, check_schedule_general, tiles_of, units_of

pytestmark = pytest.mark.gpu


def _case(prob, **params):
    from gpu_util import Case
    return Case(prob, **params)


def _parity(prob, rows=None, fused=True, **params):
    from gpu_util import assert_parity
    c = _case(prob, **params)
    try:
        D = c.run(fused=fused)
        err = assert_parity(prob, D, rows, what=f"{prob.name} {params} fused={fused}")
        return c.plan.schedule(), D, err
    finally:
        c.close()


# ---------------------------------------------------------------- small versions of the configs

SMALL = [
    (1, 1000, dict(ct_size=128, p=1)),                    # ragged: 1000 rows, 7 full tiles + 104
    (1, 4096, dict(ct_size=2048, p=32)),                  # config 1 itself, default rule
    (1, 4096, dict(ct_size=256, p=1, col_slice=16)),      # two column slices
    (2, 96, dict(ct_size=1024, p=1)),                     # n = 9216, half-bandwidth 96
    (2, 96, dict(ct_size=2048, p=1, col_slice=16)),       # sliced, tiles split by step 2
    (3, 12, dict(ct_size=2048, p=32)),                    # graph with hubs and isolated vertices
    (4, 20, dict(ct_size=2048, p=1)),                     # n = 8000
    (4, 20, dict(ct_size=4000, p=1, col_slice=8)),        # sliced so that whole planes fuse
    (5, 12, dict(ct_size=2048, p=32)),
]


@pytest.mark.parametrize("cfg,scale,params", SMALL)
@pytest.mark.parametrize("fused", [True, False])
def test_small_configs(cfg, scale, params, fused):
    prob = ti.config(cfg, scale_down=scale)
    s, D, err = _parity(prob, fused=fused, **params)
    check_schedule(prob.A, s, params["ct_size"], params["p"])
    empty = np.diff(prob.A.rowptr) == 0
    assert np.all(D[empty] == 0)


REORDERED = [
    (1, 1000, dict(ct_size=128)),
    (2, 96, dict()),
    (2, 96, dict(col_slice=32)),
    (3, 12, dict()),
    (4, 20, dict()),
    (4, 20, dict(col_slice=16)),
    (5, 12, dict(ct_size=500)),
]


@pytest.mark.parametrize("cfg,scale,params", REORDERED)
def test_small_configs_graph_grown_tiles(cfg, scale, params):
    import paper_2407_00243_amd as tf
    prob = ti.config(cfg, scale_down=scale)
    s, D, err = _parity(prob, flags=tf.TF_FLAG_REORDER, **params)
    check_schedule_general(prob.A, s)
    empty = np.diff(prob.A.rowptr) == 0
    assert np.all(D[empty] == 0)


# ---------------------------------------------------------------- exact integer inputs

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
@pytest.mark.parametrize("shape", [(300, 32, 32), (257, 20, 12), (130, 7, 5), (64, 1, 1),
                                   (500, 48, 160)])
def test_small_integers_bit_exact(dtype, kind, shape):
    """Entries in {-2..2}: every summation order is exact, so the fused path, the unfused path
    and the oracle must agree bit for bit; any missed, doubled or mis-indexed term shows."""
    n, bcol, ccol = shape
    A = ti.random_local_csr(n, 6, 5, 0.15, dtype, 41, int_values=True)
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 42)
    else:
        B = ti.random_pattern_csr(n, bcol, min(1.0, 4.0 / bcol), dtype, 42, int_values=True,
                                  duplicates=True, sort_cols=False)
    C = ti.dense_small_int(bcol, ccol, dtype, 43)
    prob = ti.Problem("ints", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    import paper_2407_00243_amd as tf
    with tf.Plan(A, bcol, ccol, kind == "spmm_spmm", flags=tf.TF_FLAG_SCHEDULE_ONLY) as pl:
        s0 = pl.schedule()
    small_lds = s0["lds_fixed_bytes"] + 48 * s0["lds_bytes_per_row"]     # forces step 2 to split
    for params in (dict(ct_size=64, p=1), dict(ct_size=150, p=1, fast_mem_bytes=small_lds),
                   dict(ct_size=64, p=1, flags=tf.TF_FLAG_REORDER)):
        c = _case(prob, **params)
        try:
            s = c.plan.schedule()
            assert 0 < s["n_fused_rows"] and (n < 100 or s["n_wf1_rows"] > 0)
            if params.get("flags"):
                check_schedule_general(A, s)
            else:
                check_schedule(A, s, params["ct_size"], params["p"])
            for fused in (True, False):
                D = c.run(fused=fused)
                assert np.array_equal(D.astype(np.float64), D_ref), (params, fused)
        finally:
            c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("bcol", [16, 32, 64, 128, 256])
@pytest.mark.parametrize("ccol", [16, 32, 64, 128])
def test_every_specialised_gemm_shape_bit_exact(dtype, bcol, ccol):
    """The dense-B kernels are instantiated per depth of k (bCol / 16 or / 8 steps) and per number
    of 16-column MFMA blocks, with the C operands in registers or in LDS: one exact case each, on
    tiles of several 16-row blocks with a ragged last one, for the fused and the unfused path."""
    n = 333
    A = ti.random_local_csr(n, 5, 6, 0.1, dtype, 91, int_values=True)
    B = ti.dense_small_int(n, bcol, dtype, 92)
    C = ti.dense_small_int(bcol, ccol, dtype, 93)
    prob = ti.Problem("shapes", "gemm_spmm", np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    c = _case(prob, ct_size=100, p=1)
    try:
        s = c.plan.schedule()
        assert 0 < s["n_fused_rows"] < n
        for fused in (True, False):
            assert np.array_equal(c.run(fused=fused).astype(np.float64), D_ref), fused
    finally:
        c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("bcol,ccol", [(16, 32), (32, 16), (64, 64), (128, 128), (64, 128),
                                       (256, 48), (20, 12), (7, 5), (48, 160)])
def test_transposed_c_bit_exact(dtype, bcol, ccol):
    """D = A (B C^T) with C handed over as cCol x bCol (Section 3.2): the shapes cover the C
    operands in registers, in LDS, the generic k loop and two column slices; non-square shapes
    make a swapped stride read a different element.  Integer entries, so bit-exact."""
    import paper_2407_00243_amd as tf
    n = 333
    A = ti.random_local_csr(n, 5, 6, 0.1, dtype, 51, int_values=True)
    B = ti.dense_small_int(n, bcol, dtype, 52)
    Ct = ti.dense_small_int(ccol, bcol, dtype, 53)
    D_ref, _ = oracle.chain_ct(A, B, Ct)
    # the case tells the two readings of the array apart
    assert not np.array_equal(D_ref, oracle.chain(A, B, Ct.reshape(bcol, ccol))[0])
    prob = ti.Problem("transposed C", "gemm_spmm", np.dtype(dtype), A, B, Ct)
    for flags in (tf.TF_FLAG_C_TRANSPOSED, tf.TF_FLAG_C_TRANSPOSED | tf.TF_FLAG_REORDER):
        c = _case(prob, ct_size=100, p=1, flags=flags)
        try:
            assert 0 < c.plan.schedule()["n_fused_rows"] < n
            for fused in (True, False):
                assert np.array_equal(c.run(fused=fused).astype(np.float64), D_ref), (flags, fused)
        finally:
            c.close()


@pytest.mark.parametrize("cfg,scale,params", [(1, 1000, dict(ct_size=128, p=1)),
                                              (2, 96, dict(ct_size=1024, p=1)),
                                              (3, 12, dict(ct_size=2048, p=32))])
def test_transposed_c_small_configs(cfg, scale, params):
    """The dense-B configurations with C handed over transposed: same result as the oracle's
    chain with C^T, to the floating-point bar."""
    import paper_2407_00243_amd as tf
    from gpu_util import TOL
    prob = ti.config(cfg, scale_down=scale)
    Ct = np.ascontiguousarray(prob.C.T)
    D_ref, W = oracle.chain_ct(prob.A, prob.B, Ct)
    tprob = ti.Problem(prob.name + " Ct", "gemm_spmm", prob.dtype, prob.A, prob.B, Ct)
    c = _case(tprob, flags=tf.TF_FLAG_C_TRANSPOSED, **params)
    try:
        for fused in (True, False):
            D = c.run(fused=fused)
            assert np.all(np.isfinite(D))
            assert oracle.rowwise_rel_err(D, D_ref, W) <= TOL[np.dtype(prob.dtype)], fused
    finally:
        c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
@pytest.mark.parametrize("reorder", [0, 1])
def test_unread_d1_rows_skipped(dtype, kind, reorder):
    """TF_FLAG_SKIP_UNREAD on a graph with many edgeless vertices: D is the oracle's bit for bit
    (integer entries) although about half of the D1 rows are never computed."""
    import paper_2407_00243_amd as tf
    A0 = ti.config(5, scale_down=11).A
    n = A0.n_rows
    rng = np.random.default_rng(5)
    A = ti.Csr(n, n, A0.rowptr, A0.colidx, rng.integers(-2, 3, A0.colidx.size).astype(dtype))
    bcol, ccol = 24, 40
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 61)
    else:
        B = ti.random_pattern_csr(n, bcol, 0.2, dtype, 61, int_values=True)
    C = ti.dense_small_int(bcol, ccol, dtype, 62)
    prob = ti.Problem("unread rows", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    flags = tf.TF_FLAG_SKIP_UNREAD | (tf.TF_FLAG_REORDER if reorder else 0)
    c = _case(prob, ct_size=128, p=1, flags=flags)
    try:
        s = c.plan.schedule()
        assert s["n_first_rows"] < 0.8 * n
        assert np.array_equal(c.run().astype(np.float64), D_ref)
        assert np.array_equal(c.run(fused=False).astype(np.float64), D_ref)
    finally:
        c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
def test_packed_entries_too_large_for_lds_are_read_in_place(dtype, kind):
    """One tile holds a dense 64 x 64 block of A (64 fused rows of 64 entries) while the average
    row has 5 entries: the tile's packed entries exceed what the schedule set aside beside the
    D1 tile, so the kernels read them from device memory instead of staging them in LDS."""
    import paper_2407_00243_amd as tf
    n, bcol, ccol = 1024, 16, 16
    rng = np.random.default_rng(77)
    rows = [np.arange(64) if j < 64 else np.array([j]) for j in range(n)]
    rowptr = np.zeros(n + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum([r.size for r in rows])
    colidx = np.concatenate(rows).astype(np.int32)
    A = ti.Csr(n, n, rowptr, colidx, rng.integers(-2, 3, colidx.size).astype(dtype))
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 78)
    else:
        B = ti.random_pattern_csr(n, bcol, 0.3, dtype, 78, int_values=True)
    C = ti.dense_small_int(bcol, ccol, dtype, 79)
    prob = ti.Problem("dense block", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    for fast_mem, staged in ((24 * 1024, 0), (0, 1)):
        c = _case(prob, ct_size=64, p=1, fast_mem_bytes=fast_mem)
        try:
            s = c.plan.schedule()
            assert s["second_block_in_lds"] == staged
            assert s["second_block_bytes"] >= 64 * 64 * (2 + np.dtype(dtype).itemsize)
            assert s["lds_launch_bytes"] <= 160 * 1024
            assert s["n_fused_rows"] == n
            assert np.array_equal(c.run().astype(np.float64), D_ref)
        finally:
            c.close()


def test_gcn_layers_reuse_one_plan():
    """Two graph-convolution layers H_{l+1} = relu(A_hat (H_l W_l)) with one plan (scheduler-overhead analysis of Section 4:
    the schedule depends on the pattern of A only, so it is built once and amortised over
    layers and epochs).  The second layer's input is the first layer's GPU output, so each layer
    is compared with the oracle on exactly the operands it was given."""
    import torch
    from gpu_util import TOL, dev
    prob = ti.config(3, scale_down=12)
    n, w = prob.n, 32
    A = prob.A
    H0 = ti.dense_normal(n, w, np.float32, 71)
    W = [ti.dense_uniform(w, w, np.float32, 72 + l, bound=float(np.sqrt(6.0 / (2 * w))))
         for l in range(2)]
    c = _case(ti.Problem("gcn layers", "gemm_spmm", np.dtype(np.float32), A, H0, W[0]),
              ct_size=256, p=1)
    try:
        stream = torch.cuda.current_stream().cuda_stream
        H = dev(H0)
        for l in range(2):
            D = torch.full((n, w), float("nan"), dtype=torch.float32, device="cuda")
            c.plan.run(H, dev(W[l]), D, stream)
            torch.cuda.synchronize()
            D_ref, Wn = oracle.chain(A, H.cpu().numpy(), W[l])
            got = D.cpu().numpy()
            assert np.all(np.isfinite(got))
            assert oracle.rowwise_rel_err(got, D_ref, Wn) <= TOL[np.dtype(np.float32)], l
            H = torch.relu(D)
    finally:
        c.close()


@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
def test_execution_calls_can_be_captured_in_a_graph(kind):
    """The execution calls allocate nothing and never synchronise, so a stream capture records
    them (two kernel launches each).  The graph is replayed several times with new operand values
    written into the same buffers and other work of the process in between; every replay must
    equal the eager result for the same operands bit for bit, and the oracle to the parity bar."""
    import torch
    from gpu_util import TOL, dev, dev_csr
    prob = ti.config(1 if kind == "gemm_spmm" else 4, scale_down=1000 if kind == "gemm_spmm" else 16)
    c = _case(prob, ct_size=128, p=1)
    try:
        n, ccol = prob.n, prob.ccol
        Cs = dev(prob.C)
        D = torch.zeros((n, ccol), dtype=c.tdtype, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            c.plan.run(c.B, Cs, D, side.cuda_stream)          # warm-up outside the capture
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            c.plan.run(c.B, Cs, D, torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            Cn = ti.dense_normal(prob.C.shape[0], ccol, prob.dtype, 300 + rep)
            Cs.copy_(dev(Cn))
            D.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = D.cpu().numpy()
            E = torch.full((n, ccol), float("nan"), dtype=c.tdtype, device="cuda")
            c.plan.run(c.B, Cs, E, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert np.array_equal(got, E.cpu().numpy()), rep
            D_ref, Wn = oracle.chain(prob.A, prob.B, Cn)
            assert oracle.rowwise_rel_err(got, D_ref, Wn) <= TOL[np.dtype(prob.dtype)], rep
    finally:
        c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("ccol", [8, 32, 100])
def test_csr_b_rows_of_every_length(dtype, ccol):
    """The CSR-B kernels stage up to 8 entries of a row of B in LDS and gather longer rows from
    device memory: rows of B with 0, 1, ..., 8, 9, ... 40 entries (duplicates, unsorted columns)
    side by side, so that both paths and every padding pattern of the staged slots occur in one
    wave; integer entries, so bit-exact, fused and unfused, consecutive and graph-grown tiles."""
    import paper_2407_00243_amd as tf
    n, bcol = 700, 90
    rng = np.random.default_rng(17)
    A = ti.random_local_csr(n, 6, 5, 0.15, dtype, 18, int_values=True)
    lens = np.concatenate([np.arange(0, 41), rng.integers(0, 12, n - 41)])
    rng.shuffle(lens)
    rowptr = np.zeros(n + 1, np.int32)
    rowptr[1:] = np.cumsum(lens)
    colidx = np.concatenate([rng.integers(0, bcol, l) for l in lens]).astype(np.int32)
    B = ti.Csr(n, bcol, rowptr, colidx, rng.integers(-2, 3, colidx.size).astype(dtype))
    C = ti.dense_small_int(bcol, ccol, dtype, 19)
    prob = ti.Problem("row lengths", "spmm_spmm", np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    for params in (dict(ct_size=96, p=1), dict(ct_size=96, p=1, flags=tf.TF_FLAG_REORDER)):
        c = _case(prob, **params)
        try:
            assert 0 < c.plan.schedule()["n_fused_rows"] < n
            for fused in (True, False):
                assert np.array_equal(c.run(fused=fused).astype(np.float64), D_ref), (params, fused)
        finally:
            c.close()


def test_csr_b_tiles_of_more_rows_than_threads():
    """Narrow fp32 C (4 columns): LDS holds tiles of 1200 rows, more rows than a workgroup has
    threads, so every per-row staging loop of the CSR-B kernel takes more than one trip."""
    import paper_2407_00243_amd as tf
    dtype = np.float32
    n, bcol, ccol = 9000, 50, 4
    A = ti.random_local_csr(n, 4, 3, 0.1, dtype, 31, int_values=True)
    B = ti.random_pattern_csr(n, bcol, 0.08, dtype, 32, int_values=True, empty_row_prob=0.1)
    C = ti.dense_small_int(bcol, ccol, dtype, 33)
    prob = ti.Problem("big tiles", "spmm_spmm", np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    for params in (dict(ct_size=2400, p=1), dict(ct_size=1200, p=1, flags=tf.TF_FLAG_REORDER)):
        c = _case(prob, **params)
        try:
            s = c.plan.schedule()
            assert np.diff(s["tile_first_ptr"]).max() > 1024 and s["n_tiles"] >= 2
            for fused in (True, False):
                assert np.array_equal(c.run(fused=fused).astype(np.float64), D_ref), (params, fused)
        finally:
            c.close()


@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
def test_wavefronts_one_by_one_and_the_workspace(kind):
    """tf_run_wavefront(0) writes exactly the fused rows of D and leaves the spilled D1 rows in
    the plan's workspace; tf_run_wavefront(1) then writes exactly the remaining rows.  Integer
    entries: everything is compared bit for bit with the oracle's D1 = B C and D = A D1."""
    import torch
    import paper_2407_00243_amd as tf
    dtype = np.float64
    n, bcol, ccol = 600, 24, 40
    A = ti.random_local_csr(n, 6, 5, 0.15, dtype, 81, int_values=True)
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 82)
        D1_ref = oracle.gemm(B, ti.dense_small_int(bcol, ccol, dtype, 83))
    else:
        B = ti.random_pattern_csr(n, bcol, 0.2, dtype, 82, int_values=True)
        D1_ref = oracle.spmm(B.rowptr, B.colidx, B.vals, ti.dense_small_int(bcol, ccol, dtype, 83))
    C = ti.dense_small_int(bcol, ccol, dtype, 83)
    prob = ti.Problem("wavefronts", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    c = _case(prob, ct_size=100, p=1)
    try:
        s = c.plan.schedule()
        fused = np.zeros(n, bool)
        fused[s["second_rows"]] = True
        assert 0 < fused.sum() < n and s["n_spill_rows"] > 0
        stream = torch.cuda.current_stream().cuda_stream
        D = torch.full((n, ccol), float("nan"), dtype=torch.float64, device="cuda")
        c.plan.run_wavefront(0, c.B, c.C, D, stream)
        torch.cuda.synchronize()
        got = D.cpu().numpy()
        assert np.array_equal(got[fused], D_ref[fused])
        assert np.all(np.isnan(got[~fused]))
        from gpu_util import read_workspace
        ws = read_workspace(c.plan, s, ccol, np.float64)
        spill = s["spill"].astype(bool)
        slot = s["spill_slot"]
        # one slot per spilled row, in row order, none for the others
        assert ws.shape[0] == max(1, spill.sum()) == s["d1_rows"]
        assert np.array_equal(slot[spill], np.arange(spill.sum())) and np.all(slot[~spill] == -1)
        assert np.array_equal(ws[slot[spill]], D1_ref[spill])
        c.plan.run_wavefront(1, None, c.C, D, stream)
        torch.cuda.synchronize()
        assert np.array_equal(D.cpu().numpy(), D_ref)
    finally:
        c.close()


# ---------------------------------------------------------------- column slices of the workspace

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
@pytest.mark.parametrize("ccol,slices", [(128, 8), (128, 4), (128, 2), (64, 4), (64, 2), (32, 2),
                                         (256, 8), (48, 1)])
def test_gather_slices_bit_exact(dtype, kind, ccol, slices):
    """The D1 workspace cut into column slices, each gathered by its own XCDs: a graph-like matrix
    (rows that reach anywhere, hub rows that are split over many lane groups, rows with only a
    diagonal entry and empty rows, which leave from registers) with small-integer entries, so that
    the fused path, the unfused path and the oracle agree bit for bit; the workspaces hold D1 in
    the sliced layout."""
    from gpu_util import read_workspace
    n, bcol = 900, 32
    A = ti.random_hub_csr(n, dtype, 71)
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 72)
        D1_ref = oracle.gemm(B, ti.dense_small_int(bcol, ccol, dtype, 73))
    else:
        B = ti.random_pattern_csr(n, bcol, 0.2, dtype, 72, int_values=True, empty_row_prob=0.05)
        D1_ref = oracle.spmm(B.rowptr, B.colidx, B.vals, ti.dense_small_int(bcol, ccol, dtype, 73))
    C = ti.dense_small_int(bcol, ccol, dtype, 73)
    prob = ti.Problem("slices", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    if slices > 1 and ccol // slices * np.dtype(dtype).itemsize < 64:
        pytest.skip("slices narrower than 64 bytes are not offered")
    c = _case(prob, ct_size=128, p=1, gather_slices=slices)
    try:
        s = c.plan.schedule()
        check_schedule(A, s, 128, 1)
        assert s["d1_slices"] == slices and s["d1_slice_cols"] * slices == ccol
        assert s["n_direct_rows"] > 0 and s["n_wf1_rows"] > 0
        D = c.run(fused=True)
        assert np.array_equal(D.astype(np.float64), D_ref)
        spill = s["spill"].astype(bool)
        ws = read_workspace(c.plan, s, ccol, dtype)
        assert np.array_equal(ws[s["spill_slot"][spill]].astype(np.float64), D1_ref[spill])
        D = c.run(fused=False)
        assert np.array_equal(D.astype(np.float64), D_ref)
        ws = read_workspace(c.plan, s, ccol, dtype, unfused=True)
        assert np.array_equal(ws.astype(np.float64), D1_ref)
    finally:
        c.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["gemm_spmm", "spmm_spmm"])
@pytest.mark.parametrize("ccol,col_slice,slices", [(128, 64, 4), (128, 32, 2), (128, 64, 8), (64, 32, 4)])
def test_fused_column_slices_with_workspace_slices(dtype, kind, ccol, col_slice, slices):
    """A fused workgroup's column slice and the workspace's column slices are independent cuts of
    the columns: every 16-column block a workgroup produces lands in the workspace slice that holds
    its columns.  Small integers, bit for bit."""
    n, bcol = 700, 16
    if ccol // slices * np.dtype(dtype).itemsize < 64:
        pytest.skip("slices narrower than 64 bytes are not offered")
    A = ti.random_hub_csr(n, dtype, 61, n_hubs=2, hub_len=200)
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 62)
    else:
        B = ti.random_pattern_csr(n, bcol, 0.3, dtype, 62, int_values=True)
    C = ti.dense_small_int(bcol, ccol, dtype, 63)
    prob = ti.Problem("slices2", kind, np.dtype(dtype), A, B, C)
    D_ref, _ = oracle.chain(A, B, C)
    c = _case(prob, ct_size=96, p=1, col_slice=col_slice, gather_slices=slices)
    try:
        s = c.plan.schedule()
        assert s["n_slices"] == ccol // col_slice and s["d1_slices"] == slices
        for fused in (True, False):
            assert np.array_equal(c.run(fused=fused).astype(np.float64), D_ref), fused
    finally:
        c.close()


@pytest.mark.parametrize("cfg,width", [(3, 128), (3, 64), (3, 256), (5, 32), (5, 128)])
@pytest.mark.parametrize("slices", [0, 1, 2, 4, 8])
def test_graph_configs_with_gather_slices(cfg, width, slices):
    """Small versions of the graph configurations for every slice count that fits (0 = the
    inspector's own choice), fused and unfused, against the oracle at the stated tolerance."""
    prob = ti.config(cfg, scale_down=13, width=width)
    if slices > 1 and width // slices * prob.dtype.itemsize < 64:
        pytest.skip("slices narrower than 64 bytes are not offered")
    for fused in (True, False):
        s, D, err = _parity(prob, fused=fused, ct_size=256, p=1, gather_slices=slices)
    assert s["n_direct_rows"] > 0
    empty = np.diff(prob.A.rowptr) == 0
    assert np.all(D[empty] == 0)
    # the same with the unread D1 rows skipped: a dense B then runs the tiled kernels (the dense
    # product works on blocks of sixteen rows and cannot leave single rows out), a CSR B still
    # streams and leaves the rows out one by one
    import paper_2407_00243_amd as tf
    # (tiling left to the library, which leaves the few rows that would read an LDS tile to the
    # second wavefront)
    s2, D2, _ = _parity(prob, fused=True, gather_slices=slices, flags=tf.TF_FLAG_SKIP_UNREAD)
    assert s2["first_wavefront_streams"] == (1 if prob.kind == "spmm_spmm" else 0)
    assert np.all(D2[empty] == 0)
    if cfg == 5:
        assert s2["n_first_rows"] < prob.n
    # and with given tile parameters (tiled kernels, rows leave the tiles' first lists)
    s3, D3, _ = _parity(prob, fused=True, ct_size=256, p=1, gather_slices=slices,
                        flags=tf.TF_FLAG_SKIP_UNREAD)
    assert np.all(D3[empty] == 0)


def test_rows_that_leave_from_registers():
    """Fused rows with a single diagonal entry are the D1 row times that entry, empty rows are
    zeros: both are stored by the lanes that hold the D1 row and are listed as fused rows; a plan
    none of whose fused rows reads the LDS tile keeps no tile (smaller LDS per workgroup)."""
    import paper_2407_00243_amd as tf
    n, bcol, ccol = 500, 16, 32
    rng = np.random.default_rng(5)
    # diagonal entries only, with every third row empty
    keep = np.arange(n) % 3 != 0
    rowptr = np.concatenate([[0], np.cumsum(keep)]).astype(np.int32)
    diag = ti.Csr(n, n, rowptr, np.nonzero(keep)[0].astype(np.int32),
                  rng.integers(-2, 3, size=int(keep.sum())).astype(np.float64))
    for kind in ("gemm_spmm", "spmm_spmm"):
        if kind == "gemm_spmm":
            B = ti.dense_small_int(n, bcol, np.float64, 6)
        else:
            B = ti.random_pattern_csr(n, bcol, 0.3, np.float64, 6, int_values=True)
        C = ti.dense_small_int(bcol, ccol, np.float64, 7)
        prob = ti.Problem("diag", kind, np.dtype(np.float64), diag, B, C)
        D_ref, _ = oracle.chain(diag, B, C)
        c = _case(prob, ct_size=64, p=1)
        try:
            s = c.plan.schedule()
            check_schedule(diag, s, 64, 1)
            assert s["n_fused_rows"] == n == s["n_direct_rows"] and s["n_spill_rows"] == 0
            assert s["first_wavefront_streams"] == 1
            with tf.Plan(ti.banded(n, 2, np.float64, 3), bcol, ccol, kind == "spmm_spmm", ct_size=64,
                         p=1) as other:
                assert s["lds_launch_bytes"] < other.schedule()["lds_launch_bytes"]
            assert np.array_equal(c.run(fused=True), D_ref)
            assert np.array_equal(c.run(fused=False), D_ref)
        finally:
            c.close()


# ---------------------------------------------------------------- invariants on the GPU

def test_identity_a_returns_bc():
    n, bcol, ccol = 777, 64, 64
    eye = ti.Csr(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                 np.ones(n, dtype=np.float64))
    B = ti.dense_normal(n, bcol, np.float64, 51)
    C = ti.dense_normal(bcol, ccol, np.float64, 52)
    prob = ti.Problem("A=I", "gemm_spmm", np.dtype(np.float64), eye, B, C)
    s, D, _ = _parity(prob, ct_size=100, p=1)
    assert s["n_fused_rows"] == n and s["n_spill_rows"] == 0 and s["n_wf1_units"] == 0
    _, D_unf, _ = _parity(prob, fused=False, ct_size=100, p=1)
    assert np.array_equal(D, D_unf)          # same MFMA order for D1, then 1.0 * x


def test_column_slices_do_not_change_the_result():
    """Columns of D are independent and slicing keeps every element's summation order."""
    prob = ti.config(1, scale_down=2048)
    _, D_full, _ = _parity(prob, ct_size=256, p=1)
    for cs in (16, 8):
        _, D_cs, _ = _parity(prob, ct_size=256, p=1, col_slice=cs)
        assert np.array_equal(D_full, D_cs)


def test_plan_is_reusable_and_overwrites():
    prob = ti.config(2, scale_down=64)
    c = _case(prob, ct_size=512, p=1)
    try:
        D1 = c.run(fill=7.0)
        D2 = c.run(fill=float("nan"))
        D3 = c.run(fused=False)
        assert np.array_equal(D1, D2)
        from gpu_util import assert_parity
        assert_parity(prob, D3)
    finally:
        c.close()


def test_plan_from_device_csr():
    from gpu_util import assert_parity, dev, dev_csr
    import paper_2407_00243_amd as tf
    import torch
    prob = ti.config(4, scale_down=12)
    Ad = dev_csr(prob.A)
    with tf.Plan(Ad, prob.bcol, prob.ccol, True, ct_size=300, p=1) as pl:
        C = dev(prob.C)
        D = torch.empty((prob.n, prob.ccol), dtype=torch.float64, device="cuda")
        pl.run(Ad, C, D, torch.cuda.current_stream().cuda_stream)      # B aliases A
        torch.cuda.synchronize()
        assert_parity(prob, D.cpu().numpy())


def test_execution_error_paths():
    import paper_2407_00243_amd as tf
    import torch
    from gpu_util import dev, dev_csr
    prob = ti.config(1, scale_down=256)
    with tf.Plan(prob.A, 32, 32, False) as pl:
        B, C = dev(prob.B), dev(prob.C)
        D = torch.empty((256, 32), dtype=torch.float64, device="cuda")
        with pytest.raises(tf.TfError) as e:
            tf.tf_spmm_spmm(pl.handle, dev_csr(prob.A), C, D)
        assert e.value.status_name == "TF_EMISMATCH"
        with pytest.raises(tf.TfError) as e:
            tf.tf_gemm_spmm(pl.handle, B, C, D.data_ptr() + 8)
        assert e.value.status_name == "TF_EINVAL"
        with pytest.raises(tf.TfError) as e:
            tf.tf_gemm_spmm(pl.handle, None, C, D)
        assert e.value.status_name == "TF_EINVAL"
    with tf.Plan(prob.A, 256, 32, True) as pl:
        A32 = prob.A._replace(vals=prob.A.vals.astype(np.float32))
        with pytest.raises(tf.TfError) as e:
            tf.tf_spmm_spmm(pl.handle, dev_csr(A32), dev(prob.C), D)
        assert e.value.status_name == "TF_EMISMATCH"


# ------------------------------------------------------------------ seeded random shapes

@pytest.mark.parametrize("seed", range(40))
def test_random_shapes_bit_exact(seed):
    """Shapes, precisions, kinds of B, tile sizes, column slices, fast-memory sizes and plan flags
    drawn from a seeded generator (the seed names the case): small integer entries, so the fused
    path and the unfused path must both equal the oracle bit for bit."""
    import paper_2407_00243_amd as tf
    rng = np.random.default_rng(1000 + seed)
    dtype = [np.float32, np.float64][int(rng.integers(2))]
    kind = ["gemm_spmm", "spmm_spmm"][int(rng.integers(2))]
    n = int(rng.choice([1, 2, 15, 16, 17, 63, 255, 256, 257, 700, 1500, 3000]))
    bcol = int(rng.choice([1, 3, 8, 16, 20, 32, 33, 64, 100, 128, 256, 300]))
    ccol = int(rng.choice([1, 2, 5, 8, 16, 24, 32, 40, 64, 96, 128, 130, 200]))
    width = int(rng.choice([1, 3, 8, 40]))
    A = ti.random_local_csr(n, min(width, n), int(rng.integers(1, 9)), float(rng.choice([0.0, 0.1, 0.5])),
                            dtype, 2000 + seed, int_values=True,
                            empty_row_prob=float(rng.choice([0.0, 0.1, 0.6])))
    if kind == "gemm_spmm":
        B = ti.dense_small_int(n, bcol, dtype, 3000 + seed)
    else:
        B = ti.random_pattern_csr(n, bcol, min(1.0, float(rng.choice([1.0, 4.0, 20.0])) / bcol), dtype,
                                  3000 + seed, int_values=True, duplicates=bool(rng.integers(2)),
                                  sort_cols=bool(rng.integers(2)),
                                  empty_row_prob=float(rng.choice([0.0, 0.3])))
    flags = int(rng.choice([0, tf.TF_FLAG_REORDER, tf.TF_FLAG_SKIP_UNREAD,
                            tf.TF_FLAG_REORDER | tf.TF_FLAG_SKIP_UNREAD, tf.TF_FLAG_NO_SPLIT]))
    transposed = kind == "gemm_spmm" and bool(rng.integers(2))
    if transposed:
        flags |= tf.TF_FLAG_C_TRANSPOSED
        C = ti.dense_small_int(ccol, bcol, dtype, 4000 + seed)
        D_ref, _ = oracle.chain_ct(A, B, C)
    else:
        C = ti.dense_small_int(bcol, ccol, dtype, 4000 + seed)
        D_ref, _ = oracle.chain(A, B, C)
    prob = ti.Problem(f"random {seed}", kind, np.dtype(dtype), A, B, C)
    params = dict(ct_size=int(rng.choice([1, 16, 50, 64, 200, 1024, 65536])), p=1, flags=flags)
    if flags & tf.TF_FLAG_NO_SPLIT:
        params["ct_size"] = min(params["ct_size"], 16)     # tiles that fit without being split
    v = 4 if dtype == np.float32 else 2
    slices = [0] + [c for c in (16, 32, 48, 64) if c < ccol and ccol % v == 0]
    params["col_slice"] = int(rng.choice(slices))
    with tf.Plan(A, bcol, ccol, kind == "spmm_spmm", flags=tf.TF_FLAG_SCHEDULE_ONLY,
                 col_slice=params["col_slice"]) as pl:
        s0 = pl.schedule()
    if rng.integers(2) and not flags & tf.TF_FLAG_NO_SPLIT:
        rows = int(rng.choice([16, 48, 200]))              # a fast memory of so many rows
        params["fast_mem_bytes"] = int(s0["lds_fixed_bytes"] + rows * s0["lds_bytes_per_row"])
    print(f"seed {seed}: {kind} {np.dtype(dtype).name} n={n} bCol={bcol} cCol={ccol} "
          f"transposed={transposed} {params}", flush=True)
    c = _case(prob, **params)
    try:
        s = c.plan.schedule()
        if not flags & (tf.TF_FLAG_SKIP_UNREAD | tf.TF_FLAG_NO_SPLIT):
            if flags & tf.TF_FLAG_REORDER:
                check_schedule_general(A, s)
            else:
                check_schedule(A, s, params["ct_size"], 1)
        for fused in (True, False):
            D = c.run(fused=fused)
            assert np.array_equal(D.astype(np.float64), D_ref), (seed, fused)
    finally:
        c.close()


def test_plans_built_by_one_and_by_many_host_threads_agree():
    """A matrix large enough for the inspector's host threads (2^18 entries or more): the plan built
    with TF_HOST_THREADS=1 and the plan built with the default number of threads must produce
    the same D bit for bit (integer entries), fused and unfused, equal to the oracle on sampled
    rows: the packed units and tile blocks are filled in by the threads."""
    import os
    import paper_2407_00243_amd as tf
    A = ti.laplacian_2d(512, np.float32)
    n, bcol, ccol = A.n_rows, 16, 16
    prob = ti.Problem("threads", "gemm_spmm", np.dtype(np.float32), A,
                      ti.dense_small_int(n, bcol, np.float32, 71), ti.dense_small_int(bcol, ccol, np.float32, 72))
    out = []
    for threads in ("1", None):
        if threads:
            os.environ["TF_HOST_THREADS"] = threads
        try:
            c = _case(prob, ct_size=65536, p=1, flags=tf.TF_FLAG_REORDER)
        finally:
            os.environ.pop("TF_HOST_THREADS", None)
        try:
            out.append((c.run(fused=True), c.run(fused=False)))
        finally:
            c.close()
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])
    assert np.array_equal(out[0][0], out[0][1])
    rows = np.random.default_rng(7).choice(n, 400, replace=False)
    D_ref, _ = oracle.chain_rows(prob.A, prob.B, prob.C, rows)
    assert np.array_equal(out[1][0][rows].astype(np.float64), D_ref)


# ---------------------------------------------------------------- the paper's experiment grid

GRID_SCALE = {1: 3000, 2: 96, 3: 13, 4: 20, 5: 13}


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("width", [32, 64, 128])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_experiment_grid_with_default_plans(cfg, width, dtype):
    """Section 4.1 runs every matrix with 32, 64 and 128 columns in single and double precision:
    every configuration at reduced size over that grid, with the plans the library makes when no
    tile parameter is given, fused and unfused, against the oracle."""
    prob = ti.config(cfg, scale_down=GRID_SCALE[cfg], width=width, dtype=dtype)
    for fused in (True, False):
        s, D, err = _parity(prob, fused=fused)
    assert s["automatic"] == 1
    check_schedule_general(prob.A, s)
    empty = np.diff(prob.A.rowptr) == 0
    assert np.all(D[empty] == 0)


# ---------------------------------------------------------------- workspaces of 4 GiB and more

def test_workspace_slices_of_four_gib_and_more():
    """Operand offsets inside a slice of the D1 workspace are formed in 32 bits unless the slice
    spans 4 GiB or more; this case has such slices on both paths: 10.5 million rows with two
    columns anywhere in the matrix (nearly nine rows in ten are read by a row of another tile),
    128 fp32 columns, the workspace kept in one slice.  Rows of D sampled over the whole matrix
    against the oracle; every row must have been written."""
    import torch
    from gpu_util import Case, TOL
    n, bcol, ccol = 10_500_000, 16, 128
    rng = np.random.default_rng(77)
    colidx = rng.integers(0, n, size=2 * n).astype(np.int32)
    A = ti.Csr(n, n, np.arange(0, 2 * n + 1, 2, dtype=np.int32), colidx,
               rng.uniform(-1.0, 1.0, size=2 * n).astype(np.float32))
    prob = ti.Problem("wide", "gemm_spmm", np.dtype(np.float32), A,
                      ti.dense_normal(n, bcol, np.float32, 78), ti.dense_normal(bcol, ccol, np.float32, 79))
    print("wide: plan", flush=True)
    c = Case(prob, ct_size=2048, p=1, gather_slices=1)
    try:
        s = c.plan.schedule()
        assert s["d1_slices"] == 1 and s["d1_rows"] * ccol * 4 >= 1 << 32       # fused workspace
        rows = np.unique(np.concatenate([[0, 1, n - 2, n - 1], rng.integers(0, n, size=400)]))
        D_ref, W = oracle.chain_rows(A, prob.B, prob.C, rows)
        stream = torch.cuda.current_stream().cuda_stream
        idx = torch.from_numpy(rows).cuda()
        for fused in (True, False):
            print(f"wide: fused={fused}", flush=True)
            D = torch.full((n, ccol), float("nan"), dtype=torch.float32, device="cuda")
            (c.plan.run if fused else c.plan.run_unfused)(c.B, c.C, D, stream)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(D).all()), "a row of D was not written"
            err = oracle.rowwise_rel_err(D[idx].cpu().numpy(), D_ref, W)
            assert err <= TOL[np.dtype(np.float32)], (fused, err)
            del D
    finally:
        c.close()


def test_csr_validate_on_device_arrays():
    """tf_csr_validate copies device arrays to the host and applies the same checks."""
    import torch
    import paper_2407_00243_amd as tf
    from gpu_util import dev_csr
    B = ti.random_pattern_csr(200, 64, 0.05, np.float64, 8)
    tf.tf_csr_validate(dev_csr(B))
    ci = B.colidx.copy()
    ci[3] = 64
    with pytest.raises(tf.TfError) as e:
        tf.tf_csr_validate(dev_csr(B._replace(colidx=ci)))
    assert e.value.status_name == "TF_EBADCSR"
