"""The entry point that allocates nothing (topk_mask_jvp_static): through the C ABI, against
topk_mask_jvp on the same inputs, two calls in a row on the shared static scratch, the second on a
smaller input."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

P2, P43 = 2.0, 4.0 / 3.0


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    from paper_2302_01425_amd import binding as b
    lib = b.load()
    assert torch.cuda.is_available()
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    r = np.random.default_rng(77)
    # rows of 32768 elements (one-workgroup-per-row kernel, scratch in use), then a smaller call that
    # finds the first call's contents in the scratch, then short rows (no scratch at all)
    cases = [(48, 32768, 1024, P2, 0.1), (5, 3000, 200, P43, 0.5), (3, 1500, 1, P2, 0.01),
             (100, 64, 2, P2, 0.5)]
    for rows, n, k, p, lam in cases:
        print(f"case rows={rows} n={n} k={k} p={p:.4f} lam={lam}", flush=True)
        x = torch.from_numpy(r.normal(size=(rows, n)).astype(np.float32)).cuda()
        t = torch.from_numpy(r.normal(size=(rows, n)).astype(np.float32)).cuda()
        ref_out, ref_jvp = b.topk_mask_jvp(x, t, k, p, lam)          # registered workspace
        torch.cuda.synchronize()
        out = torch.full_like(x, 7.0)
        jvp = torch.full_like(x, 7.0)
        rc = lib.topk_mask_jvp_static(_ptr(x), _ptr(t), rows, n, k, p, lam, _ptr(out), _ptr(jvp), sp)
        assert rc == 0, b.strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(jvp, ref_jvp), (rows, n, k, p, lam)
        # JVP only (out = NULL)
        jvp2 = torch.full_like(x, 7.0)
        rc = lib.topk_mask_jvp_static(_ptr(x), _ptr(t), rows, n, k, p, lam, None, _ptr(jvp2), sp)
        assert rc == 0, b.strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(jvp2, ref_jvp)
    # the registered workspace plays no part: the call works with none registered
    b.set_workspace(None)
    x = torch.from_numpy(r.normal(size=(4, 5000)).astype(np.float32)).cuda()
    t = torch.from_numpy(r.normal(size=(4, 5000)).astype(np.float32)).cuda()
    out, jvp = torch.empty_like(x), torch.empty_like(x)
    assert lib.topk_mask_jvp(_ptr(x), _ptr(t), 4, 5000, 50, P2, 0.2, _ptr(out), _ptr(jvp), sp) == -4
    assert lib.topk_mask_jvp_static(_ptr(x), _ptr(t), 4, 5000, 50, P2, 0.2, _ptr(out), _ptr(jvp), sp) == 0
    torch.cuda.synchronize()
    ref_out, ref_jvp = b.topk_mask_jvp(x, t, 50, P2, 0.2)            # registers a workspace again
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out) and torch.equal(jvp, ref_jvp)


def test_static_scratch_limit_is_an_error_and_enqueues_nothing():
    from paper_2302_01425_amd import binding as b
    lib = b.load()
    one = ctypes.c_void_p(256)          # never dereferenced: the shape is refused first
    rows, n = 1, 1 << 24
    assert b.workspace_bytes(b.TOPK_OP_MASK_JVP, rows, n, n // 10, P2) > (64 << 20)
    assert lib.topk_mask_jvp_static(one, one, rows, n, n // 10, P2, 1e-3, one, one, None) == -6
    assert "static" in b.strerror(-6)
    assert lib.topk_mask_jvp_static(one, one, 4, 8, 9, P2, 1.0, one, one, None) == -1
    assert lib.topk_mask_jvp_static(one, None, 4, 8, 2, P2, 1.0, one, one, None) == -2
