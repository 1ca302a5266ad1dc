"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sparse_topk.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2302_01425_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2302_01425_amd import build
        build.build_library(verbose=False)
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(topk\w*)\s*\(", text)
    return sorted(set(names))


def test_exports_match_header(lib):
    from paper_2302_01425_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_argument_validation_without_gpu(lib):
    from paper_2302_01425_amd import binding as b
    one = ctypes.c_void_p(256)          # never dereferenced: validation happens first
    f = lib.topk_mask_fwd
    assert f(one, -1, 8, 2, 2.0, 1.0, one, None) == -1          # rows < 0
    assert f(one, 4, 0, 0, 2.0, 1.0, one, None) == -1           # n < 1
    assert f(one, 4, 8, 9, 2.0, 1.0, one, None) == -1           # k > n
    assert f(one, 4, 8, -1, 2.0, 1.0, one, None) == -1          # k < 0
    assert f(one, 4, 8, 2, 2.0, 0.0, one, None) == -1           # lambda <= 0
    assert f(one, 4, 8, 2, 2.0, float("inf"), one, None) == -1
    assert f(one, 4, 8, 2, 2.0, float("nan"), one, None) == -1
    assert f(one, 4, 1 << 30, 2, 2.0, 1.0, one, None) == -1     # n too large
    assert f(one, 4, 8, 2, 1.5, 1.0, one, None) == -3           # unsupported p
    assert f(None, 4, 8, 2, 2.0, 1.0, one, None) == -2          # null input
    assert f(one, 4, 8, 2, 2.0, 1.0, None, None) == -2          # null output
    assert f(one, 0, 8, 2, 2.0, 1.0, one, None) == 0            # rows == 0: no-op
    assert lib.topkmag_fwd(one, 4, 8, 2, 1.0, 1.0, one, None) == -3         # p = 1: no pooling step
    assert lib.topk_mask_jvp(one, None, 4, 8, 2, 2.0, 1.0, None, one, None) == -2
    assert lib.topk_mask_jvp(one, one, 4, 8, 2, 2.0, 1.0, None, None, None) == -2
    assert lib.topk_argsort_desc(one, 4, 8, None, None) == -2
    # long rows without a workspace
    assert b.workspace_bytes(b.TOPK_OP_MASK_FWD, 4, 8, 2, 2.0) == 0
    # rows of up to 2048 elements run by value in one wavefront, except top-k in magnitude, p = 4/3
    for op in (b.TOPK_OP_MASK_FWD, b.TOPK_OP_MASK_JVP, b.TOPK_OP_MAG_FWD, b.TOPK_OP_MAG_JVP):
        assert b.workspace_bytes(op, 4, 2048, 2, 2.0) == 0
        assert b.workspace_bytes(op, 4, 2049, 2, 2.0) >= 4 * 4 * 2049 * 4
    assert b.workspace_bytes(b.TOPK_OP_MASK_JVP, 4, 2048, 2, 4.0 / 3.0) == 0
    assert b.workspace_bytes(b.TOPK_OP_MAG_JVP, 4, 2048, 2, 4.0 / 3.0) >= 4 * 4 * 2048 * 4
    assert b.workspace_bytes(b.TOPK_OP_MAG_JVP, 4, 1024, 2, 4.0 / 3.0) == 0
    assert b.workspace_bytes(b.TOPK_OP_MASK_SPARSE, 4, 1024, 2, 2.0) == 0
    assert b.workspace_bytes(b.TOPK_OP_MASK_SPARSE, 4, 1025, 2, 2.0) >= 4 * 4 * 1025 * 4
    assert b.workspace_bytes(b.TOPK_OP_ARGSORT, 4, 1025, 0, 2.0) >= 4 * 4 * 1025 * 4
    need = b.workspace_bytes(b.TOPK_OP_MASK_JVP, 2, 5000, 2, 2.0)
    assert need >= 4 * 2 * 5000 * 4
    lib.topk_set_workspace(None, 0)
    assert f(one, 2, 5000, 2, 2.0, 1.0, one, None) == -4
    assert lib.topk_set_workspace(ctypes.c_void_p(257), 1024) == -1   # misaligned
    assert lib.topk_set_workspace(None, 16) == -1
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(b.strerror(code)) > 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    from paper_2302_01425_amd import binding as b
    with pytest.raises(b.TopkError):
        b.topk_mask_fwd(torch.zeros(2, 8), 2, 2.0, 1.0)


def test_argument_validation_of_the_wider_entry_points(lib):
    from paper_2302_01425_amd import binding as b
    one = ctypes.c_void_p(256)          # never dereferenced: validation happens first
    g = lib.topk_general_fwd
    assert g(one, one, 0, 4, 8, b.TOPK_PHI_IDENTITY, 2.0, 1.0, one, None) != -1     # reaches the launch
    assert g(one, one, 3, 4, 8, 0, 2.0, 1.0, one, None) == -1                       # stride not 0 or n
    assert g(one, one, 0, 4, 200000, 0, 2.0, 1.0, one, None) == -1                  # rows above 131072
    assert g(one, one, 0, 4, 8, 7, 2.0, 1.0, one, None) == -1                       # unknown phi
    assert g(one, one, 0, 4, 8, 0, 1.5, 1.0, one, None) == -3
    assert g(one, None, 0, 4, 8, 0, 2.0, 1.0, one, None) == -2                      # null weights
    assert lib.topk_general_jvp(one, one, 0, None, 4, 8, 0, 2.0, 1.0, None, one, None) == -2
    d = lib.topk_mask_dykstra_fwd
    assert d(one, 4, 2000, 2, 1.0, 10, one, None) == -1                             # rows above 1024
    assert d(one, 4, 8, 2, 1.0, -1, one, None) == -1                                # iterations < 0
    assert d(None, 4, 8, 2, 1.0, 10, one, None) == -2
    assert d(one, 0, 8, 2, 1.0, 10, one, None) == 0
    # the operators on |x| need workspace beyond the rows that one fused kernel handles (3..2048)
    for op in (b.TOPK_OP_SIGNED_MASK, b.TOPK_OP_MASKED_VALUE):
        assert b.workspace_bytes(op, 4, 8, 2, 2.0) == 0
        assert b.workspace_bytes(op, 4, 2000, 2, 2.0) == 0
        assert b.workspace_bytes(op, 4, 2, 1, 2.0) >= 2 * 4 * 2 * 4
        assert b.workspace_bytes(op, 4, 3000, 2, 2.0) >= 2 * 4 * 3000 * 4
        assert b.workspace_bytes(op, 2, 5000, 2, 2.0) > b.workspace_bytes(b.TOPK_OP_MASK_JVP, 2, 5000, 2, 2.0)
    lib.topk_set_workspace(None, 0)
    assert g(one, one, 0, 4, 2000, 0, 2.0, 1.0, one, None) == -4                    # long rows: workspace
    assert b.workspace_bytes(b.TOPK_OP_GENERAL, 4, 2000, 0, 2.0) > 4 * 2001 * 8 * 4
    assert b.workspace_bytes(b.TOPK_OP_GENERAL, 4, 1000, 0, 2.0) == 0
    assert lib.topk_signed_mask_fwd(one, 4, 3000, 2, 2.0, 1.0, one, None) == -4
    assert lib.topk_masked_value_jvp(one, one, 4, 8, 2, 2.0, 1.0, None, one, None) == -2   # out required
    assert lib.topk_signed_mask_fwd(one, 4, 8, 9, 2.0, 1.0, one, None) == -1


def test_product_never_reaches_the_oracle():
    """The library, its binding and the build script import nothing from oracle/ (the oracle is
    test infrastructure), and the oracle imports nothing from the product package."""
    pkg = os.path.join(ROOT, "paper_2302_01425_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle|import_module\([\"']oracle|libtopk_oracle"
                                     r"|topk_oracle\.cpp|#include\s+\"[^\"]*oracle", text, flags=re.M), \
                    os.path.join(dirpath, name)
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".cpp")):
            assert "paper_2302_01425_amd" not in open(os.path.join(ROOT, "oracle", name)).read()


def test_workloads_are_seeded_and_shaped():
    import numpy as np
    from paper_2302_01425_amd.workloads import WORKLOADS
    w = WORKLOADS["moe_router"]
    x1, t1 = w.inputs()
    x2, t2 = w.inputs()
    assert x1.dtype == np.float32 and x1.shape == (16384, 64) and np.array_equal(x1, x2)
    assert np.array_equal(t1, t2) and not np.array_equal(x1, t1)
    # planted exact duplicates: about 5 % of the positions of a row
    dup = np.mean([64 - len(np.unique(r)) for r in x1[:200]])
    assert 2.0 <= dup <= 4.5
    assert (WORKLOADS["magnitude_pruning"].rows, WORKLOADS["magnitude_pruning"].n) == (1, 1 << 24)
    assert WORKLOADS["magnitude_pruning"].k == -(-(1 << 24) // 10)
    assert (WORKLOADS["expert_choice"].rows, WORKLOADS["expert_choice"].n, WORKLOADS["expert_choice"].k) \
        == (64, 32768, 1024)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
