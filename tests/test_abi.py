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
