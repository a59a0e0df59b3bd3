"""GPU-side harness for the parity tests: upload, run through the C ABI, download."""
import numpy as np
import torch

import oracle
import paper_2407_00243_amd as tf
import tf_inputs as ti

TOL = {np.dtype(np.float32): 1e-5, np.dtype(np.float64): 1e-12}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_csr(M):
    return tf.DeviceCsr(M.n_rows, M.n_cols, dev(M.rowptr), dev(M.colidx), dev(M.vals))


def read_workspace(plan, s, ccol, dtype, unfused=False):
    """Host copy of a plan's D1 workspace as a (rows x cCol) array, slot by slot: the device array
    is d1_slices column slices of d1_slice_cols columns, slice after slice."""
    import ctypes
    rows = s["n"] if unfused else s["d1_rows"]
    n_sl, sw = s["d1_slices"], s["d1_slice_cols"]
    raw = np.empty(n_sl * rows * sw, dtype=dtype)
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    ptr = plan.workspace_unfused() if unfused else plan.workspace()
    assert ptr, "the workspace does not exist"
    assert hip.hipMemcpy(raw.ctypes.data, ptr, raw.nbytes, 2) == 0          # device to host
    out = raw.reshape(n_sl, rows, sw).transpose(1, 0, 2).reshape(rows, n_sl * sw)
    return np.ascontiguousarray(out[:, :ccol])


class Case:
    """One problem resident on the GPU with a plan; `run(fused)` returns D as numpy."""

    def __init__(self, prob, **params):
        self.prob = prob
        self.sparse = prob.kind == "spmm_spmm"
        # with TF_FLAG_C_TRANSPOSED prob.C holds the cCol x bCol array
        self.bcol, self.ccol = prob.C.shape
        if params.get("flags", 0) & tf.TF_FLAG_C_TRANSPOSED:
            self.bcol, self.ccol = self.ccol, self.bcol
        self.plan = tf.Plan(prob.A, self.bcol, self.ccol, self.sparse, **params)
        self.B = dev_csr(prob.B) if self.sparse else dev(prob.B)
        self.C = dev(prob.C)
        self.tdtype = torch.float32 if prob.dtype == np.float32 else torch.float64

    def run(self, fused=True, fill=float("nan")):
        D = torch.full((self.prob.n, self.ccol), fill, dtype=self.tdtype, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        if fused:
            self.plan.run(self.B, self.C, D, stream)
        else:
            self.plan.run_unfused(self.B, self.C, D, stream)
        torch.cuda.synchronize()
        return D.cpu().numpy()

    def close(self):
        self.plan.close()


def assert_parity(prob, D_gpu, rows=None, what=""):
    """Element-by-element comparison with the oracle, row-wise normalised by |A||B||C|."""
    if rows is None:
        D_ref, W = oracle.chain(prob.A, prob.B, prob.C, parallel=True)
        got = D_gpu
    else:
        D_ref, W = oracle.chain_rows(prob.A, prob.B, prob.C, rows)
        got = D_gpu[rows]
    assert np.all(np.isfinite(got)), f"{what}: non-finite output (a row was not written?)"
    err = oracle.rowwise_rel_err(got, D_ref, W)
    tol = TOL[np.dtype(prob.dtype)]
    assert err <= tol, f"{what}: row-wise relative error {err:.3e} > {tol:.0e}"
    return err
