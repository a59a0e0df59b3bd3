"""The entry point that allocates nothing: tf_gemm_spmm_static keeps the D1 rows that cross tiles
in a fixed device array of the library instead of the plan's workspace.  Its output must equal
tf_gemm_spmm's bit for bit (same kernels, same order), on two calls in a row, the second with a
smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

import oracle
import tf_inputs as ti

pytestmark = pytest.mark.gpu


def _run(prob, params, static):
    import torch
    import paper_2407_00243_amd as tf
    from gpu_util import Case
    c = Case(prob, **params)
    try:
        D = torch.full((prob.n, c.ccol), float("nan"), dtype=c.tdtype, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        if static:
            tf.tf_gemm_spmm_static(c.plan.handle, c.B, c.C, D, stream)
        else:
            tf.tf_gemm_spmm(c.plan.handle, c.B, c.C, D, stream)
        torch.cuda.synchronize()
        return D.cpu().numpy(), c.plan.schedule()
    finally:
        c.close()


def test_static_workspace_matches_the_plan_workspace_twice():
    from gpu_util import TOL
    # first call: config 2 at a quarter of its grid edge (n = 16384, fp32, 64 -> 64), graph-grown
    # tiles; second call: a smaller band matrix in fp64 with another width
    import paper_2407_00243_amd as tf
    cases = [(ti.config(2, scale_down=128), dict(flags=tf.TF_FLAG_REORDER)),
             (ti.config(1, scale_down=1500), dict(ct_size=128, p=1))]
    for prob, params in cases:
        D_plan, s = _run(prob, params, static=False)
        D_static, _ = _run(prob, params, static=True)
        assert s["n_spill_rows"] > 0 and s["n_wf1_rows"] > 0
        assert np.all(np.isfinite(D_static))
        assert np.array_equal(D_static, D_plan)
        D_ref, W = oracle.chain(prob.A, prob.B, prob.C, parallel=True)
        assert oracle.rowwise_rel_err(D_static, D_ref, W) <= TOL[np.dtype(prob.dtype)]


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    import paper_2407_00243_amd as tf
    from gpu_util import Case
    # a band of half-bandwidth 40 with tiles of 64 rows: every D1 row crosses tiles, so the
    # workspace is n x 256 fp64 = 2048 n bytes; n = 40000 needs 78 MiB, more than the 64 MiB array
    n, w = 40000, 256
    A = ti.banded(n, 40, np.float64, 3)
    prob = ti.Problem("big", "gemm_spmm", np.dtype(np.float64), A,
                      ti.dense_normal(n, 16, np.float64, 4), ti.dense_normal(16, w, np.float64, 5))
    c = Case(prob, ct_size=64, p=1)
    try:
        s = c.plan.schedule()
        assert s["d1_slices"] * s["d1_rows"] * s["d1_slice_cols"] * 8 > 64 << 20
        D = torch.empty((n, w), dtype=torch.float64, device="cuda")
        with pytest.raises(tf.TfError) as e:
            tf.tf_gemm_spmm_static(c.plan.handle, c.B, c.C, D, None)
        assert e.value.status_name == "TF_EUNSUPPORTED" and "64" in str(e.value)
        tf.tf_gemm_spmm(c.plan.handle, c.B, c.C, D, None)       # the plan's own workspace still serves
        torch.cuda.synchronize()
    finally:
        c.close()
