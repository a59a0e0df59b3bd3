"""Parity at the full benchmark sizes, in the launch configuration bench.py times: every row of D
of every configuration, fused and unfused, against the oracle's chain over all rows."""
import numpy as np
import pytest

import oracle
import tf_inputs as ti
from util import check_schedule, check_schedule_general

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size_config(cfg):
    import bench
    import paper_2407_00243_amd as tf
    from gpu_util import Case, TOL
    print(f"config {cfg}: generating", flush=True)
    prob = ti.config(cfg)
    params = bench.tile_params(cfg)
    c = Case(prob, **params)
    try:
        s = c.plan.schedule()
        if params.get("flags", 0) & tf.TF_FLAG_REORDER or not params.get("ct_size"):
            check_schedule_general(prob.A, s)
        else:
            check_schedule(prob.A, s, params["ct_size"], params["p"])
        print(f"config {cfg}: oracle over all {prob.n} rows", flush=True)
        D_ref, W = oracle.chain(prob.A, prob.B, prob.C, parallel=True)
        lens = np.diff(prob.A.rowptr)
        tol = TOL[np.dtype(prob.dtype)]
        for fused in (True, False):
            print(f"config {cfg}: running fused={fused}", flush=True)
            D = c.run(fused=fused)
            assert np.all(np.isfinite(D)), "a row of D was not written"
            assert np.all(D[lens == 0] == 0)
            err = oracle.rowwise_rel_err(D, D_ref, W)
            print(f"config {cfg}: fused={fused} row-wise rel err {err:.2e} over all rows", flush=True)
            assert err <= tol, f"cfg{cfg} fused={fused}: {err:.3e} > {tol:.0e}"
    finally:
        c.close()
