"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import paper_2407_00243_amd as tf
from paper_2407_00243_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tilefusion.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tf_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = ctypes.CDLL(tf.library_path())
    names = declared_symbols()
    assert {"tf_plan_create", "tf_plan_destroy", "tf_plan_schedule", "tf_gemm_spmm",
            "tf_spmm_spmm", "tf_unfused_gemm_spmm", "tf_unfused_spmm_spmm",
            "tf_run_wavefront", "tf_last_error"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names


def test_binding_has_the_same_names():
    for name in declared_symbols():
        assert callable(getattr(tf, name)), name
    assert tf.tf_version() == "0.1"


def test_struct_layouts_match_the_header():
    # sizes follow from the field lists in the header (LP64)
    assert ctypes.sizeof(binding.tf_csr) == 3 * 8 + 3 * 8 + 2 * 4
    assert ctypes.sizeof(binding.tf_tile_params) == 4 + 4 + 8 + 4 + 4 + 4 + 4
    assert ctypes.sizeof(binding.tf_schedule_view) == 2 * 8 + 6 * 4 + 2 * 8 + 4 * 8 + 8 + 3 * 8 + \
        4 * 8 + 3 * 8 + 3 * 8 + 2 * 4 + 2 * 8 + 2 * 8 + 2 * 8 + 8 + 8 + 8 + 2 * 4 + 8 + 2 * 4 + 8 + 2 * 4
