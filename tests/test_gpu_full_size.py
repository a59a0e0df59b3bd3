"""Parity at the full benchmark sizes, in the launch configuration bench.py times: sampled rows of
D (the oracle computes them one by one), plus properties that hold at any size."""
import numpy as np
import pytest

import tf_inputs as ti
from util import check_schedule, check_schedule_general

pytestmark = pytest.mark.gpu


def sample_rows(prob, rng, count=48):
    lens = np.diff(prob.A.rowptr.astype(np.int64))
    n = prob.n
    picks = [0, 1, n // 2, n - 2, n - 1]
    picks += list(np.argsort(lens)[-3:])                      # the longest rows (hubs)
    empty = np.nonzero(lens == 0)[0]
    picks += list(empty[:3])
    ones = np.nonzero(lens == 1)[0]
    picks += list(ones[:3])
    picks += list(rng.integers(0, n, size=count - len(picks)))
    return np.unique(np.asarray(picks, dtype=np.int64))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size_config(cfg):
    import bench
    import paper_2407_00243_amd as tf
    from gpu_util import Case, assert_parity
    print(f"config {cfg}: generating", flush=True)
    prob = ti.config(cfg)
    params = bench.tile_params(cfg)
    c = Case(prob, **params)
    try:
        s = c.plan.schedule()
        if params.get("flags", 0) & tf.TF_FLAG_REORDER:
            check_schedule_general(prob.A, s)
        else:
            check_schedule(prob.A, s, params["ct_size"], params["p"])
        rows = sample_rows(prob, np.random.default_rng(cfg))
        lens = np.diff(prob.A.rowptr)
        for fused in (True, False):
            print(f"config {cfg}: running fused={fused}", flush=True)
            D = c.run(fused=fused)
            assert np.all(np.isfinite(D)), "a row of D was not written"
            assert np.all(D[lens == 0] == 0)
            err = assert_parity(prob, D, rows, what=f"cfg{cfg} fused={fused}")
            print(f"config {cfg}: fused={fused} row-wise rel err {err:.2e} on {rows.size} rows",
                  flush=True)
            if fused:
                D_fused = D
        # the two executions differ only in summation order
        D64, F64 = D.astype(np.float64), D_fused.astype(np.float64)
        scale = np.abs(F64).max(axis=1) + np.abs(D64).max(axis=1) + 1e-300
        tol = 1e-4 if prob.dtype == np.float32 else 1e-11
        assert (np.abs(F64 - D64).max(axis=1) / scale).max() < tol
    finally:
        c.close()
