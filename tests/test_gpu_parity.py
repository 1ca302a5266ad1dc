"""Parity of the HIP library against the CPU oracle, element by element, through the C ABI.

Bars (BASELINE the benchmark spec): the sorting permutation bit-exact; mask and JVP values within 1e-5
absolute.  float32 cannot represent a value v more finely than 2^-24 |v|, so for outputs of large
magnitude (the JVP scales like 1/lambda) the bar is 1e-5 + 1.2e-7 |v|, i.e. one float32 ulp.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

P2, P43 = 2.0, 4.0 / 3.0


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2302_01425_amd import binding
    binding.load()
    return binding


import contextlib


@contextlib.contextmanager
def long_rows_route(gpu, mode):
    """Run the body with rows above 1024 elements on the named route ("auto", "select", "sort")."""
    code = {"auto": gpu.TOPK_LONG_ROWS_AUTO, "select": gpu.TOPK_LONG_ROWS_SELECT,
            "sort": gpu.TOPK_LONG_ROWS_SORT, "wide": gpu.TOPK_LONG_ROWS_WIDE,
            "indexed": gpu.TOPK_LONG_ROWS_ONE_LAUNCH_INDEXED}[mode]
    gpu.set_route(gpu.TOPK_ROUTE_LONG_ROWS, code)
    try:
        yield
    finally:
        gpu.set_route(gpu.TOPK_ROUTE_LONG_ROWS, gpu.TOPK_LONG_ROWS_AUTO)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def close(got, ref, what):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    tol = 1e-5 + 1.2e-7 * np.abs(ref)
    err = np.abs(got - ref)
    bad = err > tol
    assert not bad.any(), (what, int(bad.sum()), float(err.max()),
                           np.argwhere(bad)[:5].tolist(), got[bad][:5], ref[bad][:5])


def run_case(gpu, oracle, op, x, t, k, p, lam, check_perm=True):
    print(f"case op={op} shape={x.shape} k={k} p={p:.4f} lam={lam}", flush=True)
    ofn = oracle.topk_mask if op == "mask" else oracle.topkmag
    ref = ofn(x, k, p, lam, tangent=t, want_perm=True)
    xd, td = dev(x), dev(t)
    fwd = gpu.topk_mask_fwd if op == "mask" else gpu.topkmag_fwd
    jvpf = gpu.topk_mask_jvp if op == "mask" else gpu.topkmag_jvp
    out1 = host(fwd(xd, k, p, lam))
    out2, jv = jvpf(xd, td, k, p, lam)
    out2, jv = host(out2), host(jv)
    _, jv_only = jvpf(xd, td, k, p, lam, want_out=False)
    jv_only = host(jv_only)
    close(out1, ref["out"], "fwd")
    assert np.array_equal(out1, out2), "fused forward differs from forward"
    assert np.array_equal(jv, jv_only), "JVP-only differs from fused JVP"
    close(jv, ref["jvp"], "jvp")
    # sparsity: exact zeros where the oracle has exact zeros
    assert np.all(out1[ref["out"] == 0.0] == 0.0)
    if check_perm:
        z = np.abs(x) if op == "mag" else x
        perm = host(gpu.topk_argsort_desc(dev(z)))
        assert np.array_equal(perm, ref["perm"]), "sorting permutation differs"
    return out1, jv


# ---- the five workloads at full size ---------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny", "moe_router", "moe_router_smooth", "expert_choice",
                                  "magnitude_pruning", "magnitude_pruning_smooth"])
def test_workload_parity(gpu, oracle, name):
    from paper_2302_01425_amd.workloads import WORKLOADS
    w = WORKLOADS[name]
    x, t = w.inputs()
    out, jv = run_case(gpu, oracle, w.op, x, t, w.k, w.p, w.lam)
    if w.op == "mask":
        assert np.abs(out.astype(np.float64).sum(axis=1) - w.k).max() < 1e-3 * max(1, w.k / 100)


# ---- short rows: every lane-group shape, ragged lengths, ties, both p ----------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 16, 17, 31, 33, 64, 65, 100, 128, 129, 200, 256, 300,
                               512, 777, 1024])
def test_short_rows(gpu, oracle, n):
    r = np.random.default_rng(1000 + n)
    for rows in (1, 7, 133):
        for p in (P2, P43):
            x = r.normal(size=(rows, n)).astype(np.float32)
            if n >= 4:
                x[:, 1] = x[:, 0]                       # ties
                x[rows // 2, :] = np.round(x[rows // 2, :])   # a row of many ties
            t = r.normal(size=(rows, n)).astype(np.float32)
            for k in sorted({0, 1, max(1, n // 10), n // 2, n - 1, n} & set(range(n + 1))):
                lam = float(r.choice([0.05, 0.5, 2.0]))
                run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=(k == 1))
        x = (r.laplace(size=(rows, n)) * 0.1).astype(np.float32)
        x[0, 0] = 0.0
        if n >= 3:
            x[0, 2] = -x[0, 1]
        t = r.normal(size=(rows, n)).astype(np.float32)
        for k in sorted({0, 1, n // 3, n} & set(range(n + 1))):
            run_case(gpu, oracle, "mag", x, t, k, P2, float(r.choice([1e-3, 0.1, 1.0])),
                     check_perm=(k == 1))
            run_case(gpu, oracle, "mag", x, t, k, P43, float(r.choice([0.05, 0.3, 1.0])),
                     check_perm=False)


# ---- long rows: several tiles, ragged tails, several rows -----------------------------------------
@pytest.mark.parametrize("rows,n", [(1, 1025), (3, 3000), (2, 4096), (2, 4097), (5, 10000),
                                    (1, 70001), (130, 2048)])
def test_long_rows(gpu, oracle, rows, n):
    r = np.random.default_rng(7 * n + rows)
    x = r.normal(size=(rows, n)).astype(np.float32)
    x[:, 5] = x[:, 4]
    x[-1, :] = np.round(x[-1, :] * 4) / 4                 # heavy ties in the last row
    t = r.normal(size=(rows, n)).astype(np.float32)
    for p in (P2, P43):
        for k in (1, n // 10, n // 2, n - 1):
            lam = float(r.choice([0.01, 0.1, 1.0]))
            run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=(k == 1 and p == P2))
    for k in (0, n // 10, n):
        run_case(gpu, oracle, "mag", x * np.float32(0.02), t, k, P2, float(r.choice([1e-3, 0.05])),
                 check_perm=(k == 0))
    for k, lam in ((0, 0.1), (n // 10, 0.02), (n // 3, 0.3), (n, 0.1)):
        run_case(gpu, oracle, "mag", x[:2] * np.float32(0.5), t[:2], k, P43, lam, check_perm=False)
    # large lambda: the block spans most of the row (many sweep chunks)
    run_case(gpu, oracle, "mask", x, t, n // 3, P2, 50.0, check_perm=False)
    run_case(gpu, oracle, "mask", x, t, n // 3, P43, 50.0, check_perm=False)


def test_long_rows_kinks_ties_and_full_sort_agreement(gpu, oracle):
    """Long rows whose block boundary falls inside runs of equal values (the position of each tied
    index decides its JVP), and agreement of the candidate-selection path with the full sort."""
    r = np.random.default_rng(5)
    n = 9000
    heads = [([2.0, 2.0, 0.0, -1.0], 2, 0.5), ([3.0, 1.5, 1.0, 0.0], 2, 0.5),
             ([1.0, 1.0, 1.0, 1.0], 2, 1.0), ([2.0] + [1.0] * 8 + [-5.0], 2, 2.0)]
    for head, k, lam in heads:
        x = (-50.0 - r.random(size=(2, n))).astype(np.float32)
        pos = r.permutation(n)[: len(head)]
        x[0, np.sort(pos)] = head                       # in order
        x[1, pos] = head                                # scattered: ties meet in another index order
        t = r.normal(size=(2, n)).astype(np.float32)
        for p in (P2, P43):
            run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=False)
        run_case(gpu, oracle, "mag", x + np.float32(50.0), t, k, P2, lam, check_perm=False)
    # quantised values: every boundary is a tie; both paths must give identical bits
    x = (np.round(r.normal(size=(3, 20000)) * 8) / 8).astype(np.float32)
    t = r.normal(size=x.shape).astype(np.float32)
    xd, td = dev(x), dev(t)
    for op, p, k, lam in [("mask", P2, 500, 0.3), ("mask", P43, 3000, 1.0), ("mag", P2, 7000, 0.2),
                          ("mask", P2, 19999, 100.0), ("mask", P2, 1, 1e-3)]:
        run_case(gpu, oracle, op, x, t, k, p, lam, check_perm=False)
        jvpf = gpu.topk_mask_jvp if op == "mask" else gpu.topkmag_jvp
        o_def, j_def = (host(a) for a in jvpf(xd, td, k, p, lam))
        for mode in ("select", "sort", "wide", "indexed"):
            with long_rows_route(gpu, mode):
                o_alt, j_alt = (host(a) for a in jvpf(xd, td, k, p, lam))
            assert np.array_equal(o_def, o_alt) and np.array_equal(j_def, j_alt), (mode, op, p, k, lam)


@pytest.mark.parametrize("mode", ["auto", "select", "wide"])
def test_degenerate_windows(gpu, oracle, mode):
    """Rows whose candidate window degenerates: constant rows (one key), two values, windows that
    touch +0 / -0, rows of mostly zeros where s_k itself is zero."""
    r = np.random.default_rng(31)
    n = 6000
    t = r.normal(size=(6, n)).astype(np.float32)
    x = np.empty((6, n), dtype=np.float32)
    x[0] = 1.25                                               # constant
    x[1] = np.where(r.random(n) < 0.3, 2.0, -1.0)             # two values
    x[2] = np.where(r.random(n) < 0.5, 0.0, -0.0)             # zeros of both signs only
    x[3] = r.normal(size=n) * (r.random(n) < 0.02)            # sparse: s_k is an exact zero for large k
    x[3, ::7] = -0.0
    x[4] = np.round(r.normal(size=n) * 2) * np.float32(1e-38)   # tiny values around zero (denormals)
    x[5] = -np.abs(r.normal(size=n))                          # all negative
    with long_rows_route(gpu, mode):
        for k in (1, 100, n // 2, n - 1):
            for p, lam in ((P2, 0.5), (P43, 0.5), (P2, 1e-3)):
                run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=False)
            run_case(gpu, oracle, "mag", x, t, k, P2, 0.1, check_perm=False)


@pytest.mark.parametrize("mode", ["select", "sort", "wide"])
def test_long_rows_multi_launch_paths(gpu, oracle, mode):
    """The multi-launch paths (candidate selection + sort of the candidates; full sort), which by
    default only rows above 131072 elements take, on sizes the oracle finishes quickly."""
    r = np.random.default_rng(11)
    with long_rows_route(gpu, mode):
        for rows, n in [(3, 3000), (2, 4097), (1, 70001)]:
            x = r.normal(size=(rows, n)).astype(np.float32)
            x[-1, :] = np.round(x[-1, :] * 4) / 4
            t = r.normal(size=(rows, n)).astype(np.float32)
            for p, k, lam in [(P2, 1, 0.1), (P2, n // 10, 0.01), (P43, n // 2, 1.0), (P2, n - 1, 0.1),
                              (P43, n // 3, 50.0)]:
                run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=False)
            for k in (0, n // 10, n):
                run_case(gpu, oracle, "mag", x * np.float32(0.02), t, k, P2, 0.05, check_perm=False)


def test_rows_above_the_fused_kernel_limit(gpu, oracle):
    r = np.random.default_rng(12)
    n = 200000
    x = r.normal(size=(2, n)).astype(np.float32)
    x[1] = np.round(x[1] * 16) / 16
    t = r.normal(size=(2, n)).astype(np.float32)
    run_case(gpu, oracle, "mask", x, t, n // 20, P2, 0.05, check_perm=False)
    # (lambda chosen so that the p = 4/3 block holds some ten thousand elements: the oracle's
    # cost is quadratic in the block length, see below)
    run_case(gpu, oracle, "mask", x, t, n // 3, P43, 0.1, check_perm=False)
    # one long pooled block with p = 4/3 (more than 50 000 positions; the oracle needs some 15 s)
    ref = oracle.topk_mask(x[:1], n // 3, P43, 0.7, tangent=t[:1])
    assert int(((ref["out"] > 0) & (ref["out"] < 1)).sum()) >= 50000
    o, j = gpu.topk_mask_jvp(dev(x[:1]), dev(t[:1]), n // 3, P43, 0.7)
    close(host(o), ref["out"], "fwd, long p = 4/3 block")
    close(host(j), ref["jvp"], "jvp, long p = 4/3 block")
    run_case(gpu, oracle, "mag", x, t, n // 10, P2, 0.01, check_perm=False)
    run_case(gpu, oracle, "mag", x[:1], t[:1], n // 10, P43, 0.05, check_perm=False)
    # mostly exact zeros of both signs: s_k is a zero, the window starts at the zeros
    z = (r.normal(size=(2, n)) * (r.random((2, n)) < 0.02)).astype(np.float32)
    z[:, ::5] = -0.0
    z[1] = 3.5                                                # and a constant row
    run_case(gpu, oracle, "mag", z, t, n // 10, P2, 0.1, check_perm=False)
    run_case(gpu, oracle, "mask", z, t, n // 10, P2, 0.5, check_perm=False)
    # (p = 4/3 without the constant row: the oracle re-solves the cubic over the whole block at
    # every merge, which is quadratic in the block length)
    run_case(gpu, oracle, "mask", z[:1], t[:1], 100, P43, 0.2, check_perm=False)


@pytest.mark.parametrize("rows,n", [(1, 8193), (3, 12345), (2, 32768), (16, 32768), (40, 20000),
                                    (128, 8200), (129, 8200)])
def test_rows_of_8193_to_32768_elements(gpu, oracle, rows, n):
    """The kernel that keeps a row in the registers of one workgroup of 1024 threads: few and many
    rows, ragged last wavefronts, ties, windows that hold more candidates than LDS takes."""
    r = np.random.default_rng(13 * n + rows)
    x = r.normal(size=(rows, n)).astype(np.float32)
    x[-1, :] = np.round(x[-1, :] * 4) / 4                 # heavy ties in the last row
    x[0, n - 3:] = 9.0                                    # the largest values at the end of the row
    t = r.normal(size=(rows, n)).astype(np.float32)
    for p, k, lam in [(P2, 1, 0.1), (P2, n // 32, 0.1), (P43, n // 10, 0.05), (P2, n - 1, 0.5)]:
        run_case(gpu, oracle, "mask", x, t, k, p, lam, check_perm=False)
    run_case(gpu, oracle, "mag", x * np.float32(0.02), t, n // 10, P2, 1e-2, check_perm=False)
    run_case(gpu, oracle, "mag", x[:2], t[:2], n // 7, P43, 0.05, check_perm=False)
    # a window that holds the whole row (more candidates than one workgroup sorts in LDS)
    run_case(gpu, oracle, "mask", x[:3], t[:3], n // 3, P2, 50.0, check_perm=False)
    c = np.full((2, n), 0.75, dtype=np.float32)           # constant rows
    run_case(gpu, oracle, "mask", c, t[:2] if rows >= 2 else np.vstack([t, t]), n // 2, P2, 0.3,
             check_perm=False)


# ---- the row lengths at which the kernel family changes ---------------------------------------------
@pytest.mark.parametrize("n", [128, 129, 1024, 1025, 8192, 8193, 131072, 131073])
def test_kernel_family_boundaries(gpu, oracle, n):
    r = np.random.default_rng(800 + n)
    x = r.normal(size=(2, n)).astype(np.float32)
    x[1, :] = np.round(x[1, :] * 8) / 8
    t = r.normal(size=(2, n)).astype(np.float32)
    k = max(1, n // 10)
    run_case(gpu, oracle, "mask", x, t, k, P2, 0.3, check_perm=(n <= 8193))
    run_case(gpu, oracle, "mask", x, t, k, P43, 0.05, check_perm=False)
    run_case(gpu, oracle, "mag", x, t, k, P2, 0.1, check_perm=False)
    run_case(gpu, oracle, "mag", x[:1], t[:1], k, P43, 0.02, check_perm=False)


# ---- many rows: grids of 10^4 .. 10^5 workgroups --------------------------------------------------------
@pytest.mark.parametrize("rows,n,k", [(1 << 21, 8, 2), (300000, 300, 30), (30000, 2048, 200)])
def test_many_rows(gpu, oracle, rows, n, k):
    r = np.random.default_rng(1100 + n)
    x = r.normal(size=(rows, n)).astype(np.float32)
    t = r.normal(size=(rows, n)).astype(np.float32)
    run_case(gpu, oracle, "mask", x, t, k, P2, 0.3, check_perm=False)
    run_case(gpu, oracle, "mag", x, t, k, P43, 0.05, check_perm=False)


# ---- arrays that are not 16-byte aligned (no vector loads) -----------------------------------------------
@pytest.mark.parametrize("rows,n", [(9, 64), (5, 128), (3, 400), (2, 1024), (2, 5000), (1, 150000)])
def test_unaligned_arrays(gpu, oracle, rows, n):
    import torch
    r = np.random.default_rng(900 + n)
    x = r.normal(size=(rows, n)).astype(np.float32)
    t = r.normal(size=(rows, n)).astype(np.float32)

    def shifted(a):                     # the same values, 4 bytes past a 16-byte boundary
        flat = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
        flat[1:] = torch.from_numpy(a.reshape(-1)).cuda()
        v = flat[1:].view(a.shape)
        assert v.data_ptr() % 16 == 4 and v.is_contiguous()
        return v

    xd, td = shifted(x), shifted(t)
    k = max(1, n // 7)
    for op, fn, ofn in (("mask", gpu.topk_mask_jvp, oracle.topk_mask), ("mag", gpu.topkmag_jvp, oracle.topkmag)):
        for p, lam in ((P2, 0.4), (P43, 0.05)):
            out_buf = shifted(np.zeros_like(x))
            jvp_buf = shifted(np.zeros_like(x))
            ref = ofn(x, k, p, lam, tangent=t)
            out, jv = fn(xd, td, k, p, lam, out=out_buf, jvp_out=jvp_buf)
            close(host(out), ref["out"], op + " fwd, unaligned")
            close(host(jv), ref["jvp"], op + " jvp, unaligned")
    for name, ofn in (("topk_signed_mask", oracle.topk_signed_mask), ("topk_masked_value", oracle.topk_masked_value)):
        ref = ofn(x, k, P2, 0.4, tangent=t)
        out, jv = getattr(gpu, name + "_jvp")(xd, td, k, P2, 0.4, out=shifted(np.zeros_like(x)),
                                              jvp_out=shifted(np.zeros_like(x)))
        close(host(out), ref["out"], name + " fwd, unaligned")
        close(host(jv), ref["jvp"], name + " jvp, unaligned")
    perm = host(gpu.topk_argsort_desc(xd))
    assert np.array_equal(perm, oracle.argsort_desc(x))


# ---- finite but extreme inputs: huge and tiny magnitudes, denormals, both signs of zero -----------------
@pytest.mark.parametrize("n", [64, 100, 1000, 5000, 200000])
def test_extreme_finite_values(gpu, oracle, n):
    r = np.random.default_rng(700 + n)
    rows = 3 if n <= 5000 else 1
    # magnitudes up to 1e12: beyond about 2^52 lambda the oracle's float64 subtraction s - v of a
    # top-k singleton (v = s - lambda) returns 0 instead of lambda, while the library writes the
    # exact 1 there
    expo = r.integers(-40, 12, size=(rows, n)).astype(np.float64)
    x = (r.normal(size=(rows, n)) * 10.0 ** expo).astype(np.float32)      # includes denormals and zeros
    x[:, ::7] = 0.0
    x[:, 1::7] = -0.0
    x[0, :8] = [3e12, -3e12, 1e-45, -1e-45, 1.0, -1.0, 1e10, 1e-30]
    t = r.normal(size=(rows, n)).astype(np.float32)
    for k in (1, max(2, n // 10), n - 1):
        for p in (P2, P43):
            # lambda is large against most magnitudes: a long pooled block for the middle k; the
            # oracle's p = 4/3 pooling is quadratic in the block length, so on the long row p = 4/3
            # runs only for k = 1 (mask: a short block at the top)
            if p == P2 or n <= 5000 or k == 1:
                run_case(gpu, oracle, "mask", x, t, k, p, 0.5, check_perm=(k == 1 and p == P2))
            if p == P2 or n <= 5000:
                run_case(gpu, oracle, "mag", x, t, k, p, 0.5, check_perm=False)


# ---- compact (index, value) output of the mask ----------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 7, 64, 100, 400, 1024])
def test_mask_sparse_output(gpu, oracle, n):
    r = np.random.default_rng(600 + n)
    for rows in (1, 41):
        x = r.normal(size=(rows, n)).astype(np.float32)
        if n >= 4:
            x[:, 1] = x[:, 0]
            x[-1] = np.round(x[-1] * 2) / 2
        xd = dev(x)
        for p in (P2, P43):
            for k in sorted({0, 1, max(1, n // 8), n // 2, n}):
                for lam, cap in ((0.05, n), (1.0, n), (1.0, max(1, min(n, k + 2)))):
                    print(f"case shape={x.shape} k={k} p={p:.4f} lam={lam} max_nnz={cap}", flush=True)
                    ref = oracle.topk_mask(x, k, p, lam, want_perm=True)
                    idx, val, nnz = (host(a) for a in gpu.topk_mask_sparse_fwd(xd, k, p, lam, cap))
                    dense = host(gpu.topk_mask_fwd(xd, k, p, lam))
                    for row in range(rows):
                        b = int((ref["out"][row] != 0.0).sum())
                        assert nnz[row] == b
                        m = min(b, cap)
                        assert np.array_equal(idx[row, :m], ref["perm"][row, :m])
                        close(val[row, :m], ref["out"][row, ref["perm"][row, :m]], "sparse values")
                        close(val[row, :m], dense[row, idx[row, :m]], "sparse vs dense")
                        assert np.all(idx[row, m:] == -1) and np.all(val[row, m:] == 0.0)


@pytest.mark.parametrize("rows,n", [(3, 1025), (5, 5000), (2, 8193), (64, 32768), (1, 131072),
                                    (2, 131073), (2, 300001)])
def test_mask_sparse_output_of_longer_rows(gpu, oracle, rows, n):
    """Rows above 1024 elements: the list holds the same (index, value) pairs as the dense output
    has non-zeros; entries of value 1 above the key window come first in index order, the rest
    follows in descending order of theta."""
    r = np.random.default_rng(650 + n)
    x = r.normal(size=(rows, n)).astype(np.float32)
    x[-1] = np.round(x[-1] * 4) / 4
    xd = dev(x)
    for p, lam in ((P2, 0.1), (P43, 0.05)):
        for k in sorted({0, 1, n // 32, n // 3, n}):
            cap = min(n, max(1, 2 * k + 64))
            print(f"case shape={x.shape} k={k} p={p:.4f} lam={lam} max_nnz={cap}", flush=True)
            ref = oracle.topk_mask(x, k, p, lam, want_perm=True)
            idx, val, nnz = (host(a) for a in gpu.topk_mask_sparse_fwd(xd, k, p, lam, cap))
            dense = host(gpu.topk_mask_fwd(xd, k, p, lam))
            for row in range(rows):
                b = int((ref["out"][row] != 0.0).sum())
                assert nnz[row] == b, (row, nnz[row], b)
                m = min(b, cap)
                got_i, got_v = idx[row, :m], val[row, :m]
                assert np.all(idx[row, m:] == -1) and np.all(val[row, m:] == 0.0)
                assert len(np.unique(got_i)) == m and got_i.min(initial=0) >= 0
                if 2048 < n <= 131072:
                    assert np.array_equal(got_v, dense[row, got_i])      # the same values as the dense call
                else:           # another kernel behind the dense call: the same to rounding
                    close(got_v, dense[row, got_i], "sparse vs dense")
                close(got_v, ref["out"][row, got_i], "sparse values")
                ones = int(np.argmax(got_v != 1.0)) if (got_v != 1.0).any() else m
                if m == b:      # the whole list: exactly the oracle's non-zero set
                    assert np.array_equal(np.sort(got_i), np.sort(ref["perm"][row, :b]))
                # after the leading run of ones, the list is the oracle's permutation itself:
                # descending theta, equal values by ascending index
                assert np.array_equal(got_i[ones:], ref["perm"][row, ones:m])


# ---- general non-increasing weights (soft rank / soft sort / partial ranks) -------------------------
@pytest.mark.parametrize("n", [1, 2, 5, 16, 33, 64, 100, 400, 1024, 1025, 3000, 20000])
def test_general_weights(gpu, oracle, n):
    r = np.random.default_rng(500 + n)
    for rows in ((1, 37) if n <= 1024 else (1, 5)):
        x = (r.normal(size=(rows, n)) * 2).astype(np.float32)
        if n >= 4:
            x[:, 1] = x[:, 0]
            x[-1] = np.round(x[-1])                       # many ties
        t = r.normal(size=(rows, n)).astype(np.float32)
        rho = np.arange(n, 0, -1).astype(np.float32)
        k = max(1, n // 3)
        weights = {
            "ones_k": (np.arange(n) < k).astype(np.float32),
            "rank": rho,
            "steps": np.sort(r.choice([0.0, 0.5, 1.0, 2.0, 3.0], size=n))[::-1].astype(np.float32),
            "partial_rank": np.maximum(rho - (n - k), 0.0).astype(np.float32),
            "per_row": -np.sort(-(r.normal(size=(rows, n)) ** 2).astype(np.float32), axis=1),
        }
        xd, td = dev(x), dev(t)
        for wname, w in weights.items():
            wd = dev(w)
            for phi, phic in (("id", gpu.TOPK_PHI_IDENTITY), ("half_sq", gpu.TOPK_PHI_HALF_SQUARE)):
                for p in (P2, P43):
                    lam = float(r.choice([0.1, 1.0, 4.0]))
                    print(f"case shape={x.shape} w={wname} phi={phi} p={p:.4f} lam={lam}", flush=True)
                    xin = -x if wname == "rank" else x            # rank = y(-theta, rho), Sec. 3
                    xin_d = dev(xin)
                    ref = oracle.topk_general(xin, w, p, lam, phi, tangent=t)
                    out1 = host(gpu.topk_general_fwd(xin_d, wd, phic, p, lam))
                    out2, jv = (host(a) for a in gpu.topk_general_jvp(xin_d, wd, td, phic, p, lam))
                    _, jv_only = gpu.topk_general_jvp(xin_d, wd, td, phic, p, lam, want_out=False)
                    assert np.array_equal(out1, out2) and np.array_equal(jv, host(jv_only))
                    close(out1, ref["out"], "general fwd")
                    close(jv, ref["jvp"], "general jvp")
        # w = 1_k through the general path agrees with the top-k kernels
        for phic, fn in ((gpu.TOPK_PHI_IDENTITY, gpu.topk_mask_jvp), (gpu.TOPK_PHI_HALF_SQUARE, gpu.topkmag_jvp)):
            for p in (P2, P43):
                a, b = (host(v) for v in gpu.topk_general_jvp(xd, dev(weights["ones_k"]), td, phic, p, 0.5))
                c, d = (host(v) for v in fn(xd, td, k, p, 0.5))
                close(a, c, "general vs top-k fwd")
                close(b, d, "general vs top-k jvp")
    # soft sort (Sec. 3): input (n, .., 1), weights = the row sorted in descending order
    theta = r.normal(size=(5, n)).astype(np.float32)
    ws = -np.sort(-theta, axis=1)
    if n > 1 and ws.min() < 0:
        ws = ws - ws.min()                                   # keep the weights non-negative
    rho_rows = np.tile(np.arange(n, 0, -1).astype(np.float32), (5, 1))
    ref = oracle.topk_general(rho_rows, ws, P2, 0.3, "id")["out"]
    got = host(gpu.topk_general_fwd(dev(rho_rows), dev(ws), gpu.TOPK_PHI_IDENTITY, P2, 0.3))
    close(got, ref, "soft sort")


def test_general_weights_many_rounds_and_stack_fallback(gpu, oracle):
    """Rows on which the merging rounds remove one boundary at a time (one heavy first weight in
    front of a slowly falling ramp: the pooled block takes in one neighbour per round, some 220 of
    them), so the wavefront hands over to the sequential block stack; and ordinary rows with the
    hand-over forced after 1 and 3 rounds."""
    r = np.random.default_rng(91)
    for n in (300, 1024, 5000):
        x = r.normal(size=(6, n)).astype(np.float32)
        w = -np.sort(-np.abs(r.normal(size=(6, n))).astype(np.float32), axis=1)
        ramp = (10.0 - 0.001 * np.arange(n)).astype(np.float32)
        ramp[0] = 10.0005
        x[1] = ramp[r.permutation(n)]
        w[1] = 0.0
        w[1, 0] = 50.0
        x[4] = x[1]
        w[4] = w[1]
        w[4, 1:n // 2] = 0.25                                 # the same, on top of a step
        t = r.normal(size=(6, n)).astype(np.float32)
        for phi, phic in (("id", gpu.TOPK_PHI_IDENTITY), ("half_sq", gpu.TOPK_PHI_HALF_SQUARE)):
            for p in (P2, P43):
                print(f"ramp n={n} phi={phi} p={p:.3f}", flush=True)
                ref = oracle.topk_general(x, w, p, 1.0, phi, tangent=t)
                for rounds in (0, 1, 3):
                    gpu.set_route(gpu.TOPK_ROUTE_GENERAL_ROUNDS, rounds)
                    try:
                        out, jv = (host(a) for a in gpu.topk_general_jvp(dev(x), dev(w), dev(t), phic, p, 1.0))
                    finally:
                        gpu.set_route(gpu.TOPK_ROUTE_GENERAL_ROUNDS, 0)
                    close(out, ref["out"], f"general fwd rounds={rounds}")
                    close(jv, ref["jvp"], f"general jvp rounds={rounds}")


def test_general_weights_longest_row(gpu, oracle):
    """One row of TOPK_GENERAL_ROW_MAX elements: relaxed ranks (many blocks of every size) and a
    partial-rank weight vector, both p."""
    n = 131072
    r = np.random.default_rng(17)
    x = (r.normal(size=(1, n)) * 3).astype(np.float32)
    t = r.normal(size=(1, n)).astype(np.float32)
    rho = np.arange(n, 0, -1).astype(np.float32)
    for w, lam in ((rho * np.float32(1e-4), 0.5), (np.maximum(rho - (n - 2000), 0.0).astype(np.float32), 0.01)):
        for p in (P2, P43):
            for phi, phic in (("id", gpu.TOPK_PHI_IDENTITY), ("half_sq", gpu.TOPK_PHI_HALF_SQUARE)):
                print(f"longest general row phi={phi} p={p:.3f} lam={lam}", flush=True)
                ref = oracle.topk_general(x, w, p, lam, phi, tangent=t)
                out, jv = (host(a) for a in gpu.topk_general_jvp(dev(x), dev(w), dev(t), phic, p, lam))
                close(out, ref["out"], "general fwd")
                close(jv, ref["jvp"], "general jvp")
    with pytest.raises(gpu.TopkError):
        gpu.topk_general_fwd(dev(np.zeros((1, n + 1), dtype=np.float32)),
                             dev(np.zeros(n + 1, dtype=np.float32)), gpu.TOPK_PHI_IDENTITY, P2, 1.0)


# ---- Dykstra's algorithm with a fixed number of iterations ----------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 16, 63, 64, 100, 400, 1024])
def test_dykstra_iterations(gpu, oracle, n):
    r = np.random.default_rng(400 + n)
    for rows in (1, 50):
        x = r.normal(size=(rows, n)).astype(np.float32)
        if n >= 4:
            x[:, 1] = x[:, 0]
            x[-1] = np.round(x[-1] * 2) / 2
        xd = dev(x)
        for k in sorted({0, 1, max(1, n // 10), n // 2, n}):
            for lam, iters in ((0.1, 100), (1.0, 100), (2.5, 7), (0.5, 0), (1.0, 1)):
                print(f"case shape={x.shape} k={k} lam={lam} iters={iters}", flush=True)
                ref = oracle.topk_mask_dykstra(x, k, lam, iters)
                got = host(gpu.topk_mask_dykstra_fwd(xd, k, lam, iters))
                close(got, ref, "dykstra")
    # the iterates approach the exact operator (how fast depends on the length of the pooled block)
    x = r.normal(size=(20, n)).astype(np.float32)
    k = max(1, n // 10)
    exact = host(gpu.topk_mask_fwd(dev(x), k, P2, 1.0))
    err = [np.abs(exact - host(gpu.topk_mask_dykstra_fwd(dev(x), k, 1.0, it))).max()
           for it in (10, 100, 1000, 20000)]
    assert err[1] <= err[0] + 1e-6 and err[2] <= err[1] + 1e-6 and err[3] <= err[2] + 1e-6, err
    assert err[3] < 1e-2, err


# ---- the operators on |x|: signed mask (phi = |x|) and x o mask(|x|) --------------------------------
@pytest.mark.parametrize("rows,n", [(1, 1), (129, 7), (70, 33), (37, 64), (9, 100), (50, 128),
                                    (5, 300), (40, 512), (7, 1000), (3, 2048), (3, 5000), (1, 200000)])
def test_signed_mask_and_masked_value(gpu, oracle, rows, n):
    r = np.random.default_rng(31 * n + rows)
    x = r.normal(size=(rows, n)).astype(np.float32)
    x[0, 0] = 0.0
    if n >= 8:
        x[:, 3] = -x[:, 2]                                   # equal magnitudes, opposite signs
        x[-1, n // 2:] = np.float32(-0.0)
    t = r.normal(size=(rows, n)).astype(np.float32)
    xd, td = dev(x), dev(t)
    for p in (P2, P43):
        # lambda = 0.05: no truncation at zero; 1.5: the pooled block is truncated for small k;
        # 40: everything is
        for k, lam in ((max(1, n // 10), 0.05), (max(1, n // 3), 1.5), (min(n, 2), 40.0), (n, 0.7),
                       (0, 0.7)):
            if p == P43 and n > 10000 and lam > 1.0 and 0 < k < n:
                continue          # the oracle's p = 4/3 pooling is quadratic in the block length
            print(f"case shape={x.shape} k={k} p={p:.4f} lam={lam}", flush=True)
            for name, ofn in (("topk_signed_mask", oracle.topk_signed_mask),
                              ("topk_masked_value", oracle.topk_masked_value)):
                ref = ofn(x, k, p, lam, tangent=t)
                out1 = host(getattr(gpu, name + "_fwd")(xd, k, p, lam))
                out2, jv = (host(a) for a in getattr(gpu, name + "_jvp")(xd, td, k, p, lam))
                assert np.array_equal(out1, out2), name
                close(out1, ref["out"], name + " fwd")
                close(jv, ref["jvp"], name + " jvp")
                assert np.all(out1[ref["out"] == 0.0] == 0.0)


# ---- paper examples through the GPU path ----------------------------------------------------------
def test_fig1_points(gpu, oracle):
    for lam in (0.25, 1.0):
        for s in (-1.0, 0.0, 1 - lam, 0.9, 1.0, 1.1, 1 + lam, 2.0):
            th = np.array([[3.0, 1.0, -1.0 + s, s]], dtype=np.float32)
            t = np.array([[0.5, -1.0, 2.0, 1.0]], dtype=np.float32)
            for p in (P2, P43):
                run_case(gpu, oracle, "mask", th, t, 2, p, lam)


def test_strict_merge_kinks(gpu, oracle):
    cases = [([2.0, 2.0, 0.0, -1.0], 2, 0.5), ([3.0, 1.5, 1.0, 0.0], 2, 0.5),
             ([3.0, 1.0, 0.75, 0.625], 2, 0.5), ([1.0, 1.0, 1.0, 1.0], 2, 1.0),
             ([0.0, 0.0, 0.0], 1, 0.25),
             # p = 4/3 tie: eight ones pool at exactly 0 = 2 - lambda, so the 2 stays outside
             ([2.0] + [1.0] * 8 + [-5.0], 2, 2.0)]
    for th, k, lam in cases:
        th = np.array([th], dtype=np.float32)
        t = np.arange(1, th.shape[1] + 1, dtype=np.float32)[None, :] * np.float32(0.5)
        for p in (P2, P43):
            run_case(gpu, oracle, "mask", th, t, k, p, lam)
        run_case(gpu, oracle, "mag", th, t, k, P2, lam)


def test_fig2_points_through_the_library(gpu, oracle):
    """Fig. 2 of the paper (phi = x^2/2, k = 2, x = (x1, x2, 1/2, 1), lambda = 0.3), both p."""
    pts = np.linspace(-0.6, 0.6, 7)
    x = np.array([[a, b, 0.5, 1.0] for a in pts for b in pts], dtype=np.float32)
    t = np.tile(np.array([[1.0, -2.0, 0.5, 3.0]], dtype=np.float32), (x.shape[0], 1))
    for p in (P2, P43):
        run_case(gpu, oracle, "mag", x, t, 2, p, 0.3, check_perm=False)


def test_values_closer_than_the_truncated_sort_key(gpu, oracle):
    """Rows whose values differ only in the last few mantissa bits (and mixtures of such clusters
    with exact ties): the permutation must still be the exact stable argsort."""
    r = np.random.default_rng(99)
    for n in (4, 16, 24, 64, 100, 128):
        rows = 37
        ulps = r.permutation(n).astype(np.int64)
        base = np.float32(1.0).view(np.int32)
        x = np.empty((rows, n), dtype=np.float32)
        x[0] = (base + ulps).astype(np.int32).view(np.float32)             # one cluster, all distinct
        x[1] = -x[0]
        x[2] = (base + (ulps // 3)).astype(np.int32).view(np.float32)      # clusters with exact ties
        for i in range(3, rows):
            c = r.normal(size=max(1, n // 8)).astype(np.float32)           # a few cluster centres
            pick = r.integers(0, c.size, size=n)
            off = r.integers(-40, 40, size=n)
            x[i] = (c[pick].view(np.int32) + off).astype(np.int32).view(np.float32)
        t = r.normal(size=(rows, n)).astype(np.float32)
        for k in sorted({1, max(1, n // 4), n - 1}):
            for p in (P2, P43):
                run_case(gpu, oracle, "mask", x, t, k, p, 0.3)
            run_case(gpu, oracle, "mag", x, t, k, P2, 0.05)
            run_case(gpu, oracle, "mag", x, t, k, P43, 0.2)


def test_vjp_against_the_transposed_jacobian_of_the_oracle(gpu, oracle):
    """The oracle's Jacobian, column by column from its JVP on unit tangents, transposed and applied
    to a cotangent, against the library's VJP entry points (which rely on the symmetry)."""
    r = np.random.default_rng(21)
    for op, n, k, p, lam in [("mask", 12, 3, P2, 0.7), ("mask", 20, 5, P43, 1.5), ("mag", 16, 4, P2, 0.4),
                             ("mask", 1500, 40, P2, 0.3), ("mag", 1300, 100, P2, 0.05)]:
        x = r.normal(size=(2, n)).astype(np.float32)
        c = r.normal(size=(2, n)).astype(np.float32)
        ofn = oracle.topk_mask if op == "mask" else oracle.topkmag
        ref = np.zeros((2, n))
        for j in range(n):                               # column j of J: JVP of the j-th unit vector
            e = np.zeros((2, n), dtype=np.float32)
            e[:, j] = 1.0
            col = np.asarray(ofn(x, k, p, lam, tangent=e)["jvp"], dtype=np.float64)
            ref[:, j] = (col * c.astype(np.float64)).sum(axis=1)       # (J^T c)_j = <column j, c>
        fn = gpu.topk_mask_vjp if op == "mask" else gpu.topkmag_vjp
        out, vjp = fn(dev(x), dev(c), k, p, lam)
        close(host(vjp), ref, f"vjp {op} n={n}")
        close(host(out), ofn(x, k, p, lam, tangent=c)["out"], "out")


def test_fenchel_young_loss(gpu, oracle):
    """Smooth top-k loss (Sec. 6) and its gradient against the oracle's value of f (computed from
    the minimisation form of Prop. 2, the library uses the maximisation form)."""
    r = np.random.default_rng(23)
    for rows, n, k, lam in [(64, 10, 3, 0.5), (17, 5, 4, 2.0), (1000, 64, 2, 1.0), (70, 128, 40, 3.0),
                            (300, 100, 3, 1.0), (33, 1000, 5, 0.2), (9, 2048, 300, 0.4), (4, 5000, 50, 0.3),
                            (2, 150000, 100, 0.5)]:
        x = (r.normal(size=(rows, n)) * 2).astype(np.float32)
        t = np.zeros((rows, n), dtype=np.float32)
        t[np.arange(rows), r.integers(0, n, size=rows)] = 1.0          # one-hot classes
        for p in (P2, P43):
            print(f"loss rows={rows} n={n} k={k} p={p:.3f} lam={lam}", flush=True)
            ref_loss, ref_grad = oracle.fenchel_young_loss(x, t, k, p, lam)
            loss, grad = gpu.topk_mask_loss(dev(x), dev(t), k, p, lam)
            close(host(grad), ref_grad, "grad")
            # the loss is summed in float64 from the float32 mask through the Lagrangian of the
            # maximisation form, which is flat at the maximiser: what is left is the float32
            # rounding of the stored value (6e-8 relative; twice that allowed) and 2e-6 absolute
            err = np.abs(host(loss).astype(np.float64) - ref_loss)
            assert (err <= 2e-6 + 1.2e-7 * np.abs(ref_loss)).all(), (rows, n, p, float(err.max()))


def test_small_lambda_against_the_spread_of_the_row(gpu, oracle):
    """lambda a few hundred times smaller than the values: a pooled block's own spread is then far
    below the rounding of row-wide sums of cubes (general weights, p = 4/3), the factors of the
    JVP reach the hundreds (operators on |x|), and the loss sums many terms of either sign."""
    r = np.random.default_rng(77)
    for rows, n in ((60, 66), (70, 449), (40, 963), (30, 1300), (6, 3000)):
        x = (r.normal(size=(rows, n)) * 3).astype(np.float32)
        x[:, : n // 2 : 7] += np.float32(1e-5) * r.normal(size=x[:, : n // 2 : 7].shape).astype(np.float32)
        x[1::2, 1::3] = x[1::2, 0:-1:3][:, : x[1::2, 1::3].shape[1]] + np.float32(8e-6)   # near-ties
        t = r.normal(size=(rows, n)).astype(np.float32)
        weights = {"rank": np.arange(n, 0, -1).astype(np.float32),
                   "per_row": -np.sort(-(r.normal(size=(rows, n)) ** 2).astype(np.float32), axis=1)}
        for wname, w in weights.items():
            for phi, phic in (("id", gpu.TOPK_PHI_IDENTITY), ("half_sq", gpu.TOPK_PHI_HALF_SQUARE)):
                print(f"case shape={x.shape} w={wname} phi={phi}", flush=True)
                ref = oracle.topk_general(x, w, P43, 0.01, phi, tangent=t)
                o, j = (host(a) for a in gpu.topk_general_jvp(dev(x), dev(w), dev(t), phic, P43, 0.01))
                close(o, ref["out"], "general fwd, small lambda")
                close(j, ref["jvp"], "general jvp, small lambda")
        xs = (x * np.float32(0.003)).astype(np.float32)           # |x| around lambda
        for name, ofn in (("topk_signed_mask", oracle.topk_signed_mask),
                          ("topk_masked_value", oracle.topk_masked_value)):
            for k in (n // 10 + 1, n - 1, n):
                ref = ofn(xs, k, P43, 0.01, tangent=t)
                o, j = (host(a) for a in getattr(gpu, name + "_jvp")(dev(xs), dev(t), k, P43, 0.01))
                close(o, ref["out"], name + " fwd, small lambda")
                close(j, ref["jvp"], name + " jvp, small lambda")


def test_binding_rejects_mismatched_tensors(gpu):
    """Shapes, devices, dtypes and aliasing are checked before anything is launched."""
    import torch
    x = dev(np.zeros((4, 64), dtype=np.float32))
    t = dev(np.ones((4, 64), dtype=np.float32))
    small = dev(np.zeros((4, 32), dtype=np.float32))
    host_t = torch.zeros(4, 64)
    E = gpu.TopkError
    with pytest.raises(E):
        gpu.topk_mask_fwd(x, 2, P2, 1.0, out=small)
    with pytest.raises(E):
        gpu.topk_mask_fwd(x, 2, P2, 1.0, out=x)                       # output aliases the input
    with pytest.raises(E):
        gpu.topk_mask_jvp(x, small, 2, P2, 1.0)
    with pytest.raises(E):
        gpu.topk_mask_jvp(x, host_t, 2, P2, 1.0)
    with pytest.raises(E):
        gpu.topk_mask_jvp(x, t, 2, P2, 1.0, jvp_out=t)                # aliases the tangent
    with pytest.raises(E):
        o = torch.empty_like(x)
        gpu.topk_mask_jvp(x, t, 2, P2, 1.0, out=o, jvp_out=o)         # the two outputs overlap
    with pytest.raises(E):
        gpu.topkmag_jvp(x, t, 2, P2, 1.0, jvp_out=small)
    with pytest.raises(E):
        gpu.topk_mask_loss(x, t, 2, P2, 1.0, loss_out=torch.empty(3, device="cuda"))
    with pytest.raises(E):
        gpu.topk_mask_loss(x, small, 2, P2, 1.0)
    with pytest.raises(E):
        gpu.topk_mask_vjp(x, t, 2, P2, 1.0, vjp_out=small)
    with pytest.raises(E):
        gpu.topk_signed_mask_jvp(x, t, 2, P2, 1.0, out=small)
    with pytest.raises(E):
        gpu.topk_general_fwd(x, dev(np.ones(63, dtype=np.float32)), gpu.TOPK_PHI_IDENTITY, P2, 1.0)
    with pytest.raises(E):
        gpu.topk_argsort_desc(x, perm_out=torch.empty((4, 64), dtype=torch.int64, device="cuda"))
    with pytest.raises(E):
        gpu.topk_mask_sparse_fwd(x, 2, P2, 1.0, 8, val_out=small)


def test_workspace_growth_keeps_captured_graphs_valid(gpu, oracle):
    """A larger call between a capture and its replay makes the binding register a bigger
    workspace; the block the captured kernels use must stay alive and untouched."""
    import torch
    r = np.random.default_rng(77)
    x = r.normal(size=(3, 5000)).astype(np.float32)
    t = r.normal(size=(3, 5000)).astype(np.float32)
    xd, td = dev(x), dev(t)
    out, jvp = torch.empty_like(xd), torch.empty_like(xd)
    torch.cuda.synchronize()
    gpu.set_workspace(None)            # whatever earlier tests of this process left registered
    gpu.topk_mask_jvp(xd, td, 200, P2, 0.3, out=out, jvp_out=jvp)      # sizes the workspace
    torch.cuda.synchronize()
    ref_o, ref_j = out.clone(), jvp.clone()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            gpu.topk_mask_jvp(xd, td, 200, P2, 0.3, out=out, jvp_out=jvp, stream=stream)
    # a call that needs more scratch than anything before it in this process
    big = dev(r.normal(size=(1, 3_000_000)).astype(np.float32))
    gpu.topk_mask_fwd(big, 1000, P2, 0.1)
    torch.cuda.synchronize()
    fill = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").fill_(0xAB)   # reuses freed blocks
    for _ in range(2):
        out.zero_()
        jvp.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_o) and torch.equal(jvp, ref_j)
    del fill
    # growing during a capture is refused (nothing can be allocated there)
    huge = dev(r.normal(size=(1, 6_000_000)).astype(np.float32))
    g2 = torch.cuda.CUDAGraph()
    with pytest.raises(gpu.TopkError):
        with torch.cuda.stream(stream):
            with torch.cuda.graph(g2, stream=stream):
                gpu.topk_mask_fwd(huge, 10, P2, 0.1, out=torch.empty_like(huge), stream=stream)


def test_determinism_and_streams(gpu):
    import torch
    from paper_2302_01425_amd.workloads import WORKLOADS
    w = WORKLOADS["moe_router"]
    x, t = w.inputs()
    xd, td = dev(x), dev(t)
    o1, j1 = gpu.topk_mask_jvp(xd, td, w.k, w.p, w.lam)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        o2, j2 = gpu.topk_mask_jvp(xd, td, w.k, w.p, w.lam, stream=st)
    st.synchronize()
    assert torch.equal(o1, o2) and torch.equal(j1, j2)


@pytest.mark.parametrize("rows,n,op", [(1000, 64, "mask"), (4, 5000, "mask"), (1, 300000, "mag")])
def test_hip_graph_replays(gpu, rows, n, op):
    """The calls only enqueue kernels, so they can be captured; every replay, with other work and
    new input contents in between, must give what the eager call gives on the same contents."""
    import torch
    r = np.random.default_rng(1000 + n)
    k, lam = max(1, n // 10), 0.2
    fn = gpu.topk_mask_jvp if op == "mask" else gpu.topkmag_jvp
    xd = torch.empty((rows, n), dtype=torch.float32, device="cuda")
    td = torch.empty_like(xd)
    out, jv = torch.empty_like(xd), torch.empty_like(xd)
    xd.copy_(dev(r.normal(size=(rows, n)).astype(np.float32)))
    td.copy_(dev(r.normal(size=(rows, n)).astype(np.float32)))
    fn(xd, td, k, P2, lam)                                  # registers the workspace before the capture
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(graph, stream=st):
            fn(xd, td, k, P2, lam, out=out, jvp_out=jv, stream=st)
    torch.cuda.synchronize()
    for rep in range(3):
        xd.copy_(dev(r.normal(size=(rows, n)).astype(np.float32)))
        td.copy_(dev(r.normal(size=(rows, n)).astype(np.float32)))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_j = out.clone(), jv.clone()
        ref_o, ref_j = fn(xd, td, k, P2, lam)               # eager, between the replays
        torch.cuda.synchronize()
        assert torch.equal(got_o, ref_o) and torch.equal(got_j, ref_j), rep


def test_rows_zero_and_errors(gpu):
    import torch
    x = torch.zeros((0, 8), device="cuda")
    assert gpu.topk_mask_fwd(x, 2, P2, 1.0).shape == (0, 8)
    y = torch.zeros((2, 8), device="cuda")
    with pytest.raises(gpu.TopkError):
        gpu.topk_mask_fwd(y, 9, P2, 1.0)
    with pytest.raises(gpu.TopkError):
        gpu.topk_mask_fwd(y, 2, 1.7, 1.0)
    with pytest.raises(gpu.TopkError):
        gpu.topkmag_fwd(y, 2, 3.0, 1.0)
