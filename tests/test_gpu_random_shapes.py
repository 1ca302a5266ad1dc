"""Seeded random shapes, parameters and value distributions through every entry point, against the
oracle: row lengths drawn from every kernel family, k from the edges and the middle, lambda over
three decades, normal / quantised (ties) / Laplace / mostly-zero / pre-sorted rows."""
import numpy as np
import pytest

from tests.test_gpu_parity import P2, P43, close, dev, host, gpu  # noqa: F401  (gpu: the fixture)

pytestmark = pytest.mark.gpu


def _row_length(r, upto):
    fam = [(1, 130), (129, 2049), (2049, 8193), (8193, 32769), (32769, 300000), (1, 5000)]
    lo, hi = fam[r.integers(0, len(fam))]
    return int(min(r.integers(lo, hi), upto))


def _values(r, rows, n, dist):
    if dist == 0:
        x = r.normal(size=(rows, n))
    elif dist == 1:
        x = np.round(r.normal(size=(rows, n)) * r.choice([1, 4, 16])) / 4          # ties
    elif dist == 2:
        x = r.laplace(size=(rows, n)) * 0.02
    elif dist == 3:
        x = r.normal(size=(rows, n)) * (r.random((rows, n)) < 0.1)                 # mostly zeros
    else:
        x = np.sort(r.normal(size=(rows, n)), axis=1)[:, ::(1 if r.random() < 0.5 else -1)]
    return np.ascontiguousarray(x, dtype=np.float32)


def test_mask_and_magnitude_on_random_shapes(gpu, oracle):
    for c in range(400):
        r = np.random.default_rng(910000 + c)
        n = _row_length(r, 300000)
        rows = int(max(1, min(r.integers(1, 300), 1500000 // n)))
        p = P2 if r.random() < 0.5 else P43
        # (the oracle's p = 4/3 pooling is quadratic in the block: short blocks on long rows)
        dist = 0 if (p == P43 and n > 3000) else int(r.integers(0, 5))
        x = _values(r, rows, n, dist)
        t = r.normal(size=(rows, n)).astype(np.float32)
        k = int(r.choice([0, 1, max(1, n // 10), n // 2, max(0, n - 1), n, int(r.integers(0, n + 1))]))
        op = "mask" if r.random() < 0.6 else "mag"
        lam = float(r.choice([1e-3, 0.01, 0.1, 0.5, 1.0, 5.0]))
        if p == P43 and n > 3000:
            lam = min(lam, 0.01)
        print(f"case {c}: op={op} rows={rows} n={n} k={k} p={p:.3f} lam={lam} dist={dist}", flush=True)
        ref = (oracle.topk_mask if op == "mask" else oracle.topkmag)(x, k, p, lam, tangent=t)
        o, j = (host(a) for a in (gpu.topk_mask_jvp if op == "mask" else gpu.topkmag_jvp)(dev(x), dev(t), k, p, lam))
        close(o, ref["out"], "fwd")
        close(j, ref["jvp"], "jvp")
        assert np.all(o[ref["out"] == 0.0] == 0.0)


def test_other_entry_points_on_random_shapes(gpu, oracle):
    for c in range(300):
        r = np.random.default_rng(920000 + c)
        what = ["signed", "masked", "loss", "general", "sparse", "vjp", "argsort"][r.integers(0, 7)]
        n = _row_length(r, 3000 if what == "general" else 9000)
        rows = int(max(1, min(r.integers(1, 200), 400000 // n)))
        p = P2 if r.random() < 0.5 else P43
        x = r.normal(size=(rows, n)) * r.choice([0.1, 1.0, 3.0])
        # ties: not for general weights with p = 2 (pooled values that tie only in real arithmetic
        # may be pooled either way) and not beside the kink of the truncation of the operators on |x|
        if r.random() < 0.3 and what not in ("general", "signed", "masked"):
            x = np.round(x * 4) / 4
        x = x.astype(np.float32)
        t = r.normal(size=(rows, n)).astype(np.float32)
        k = int(r.choice([0, 1, max(1, n // 10), n // 2, max(0, n - 1), n]))
        lam = float(r.choice([0.01, 0.1, 0.5, 1.5, 5.0]))
        if p == P43 and n > 3000:
            lam = 0.01
        print(f"case {c}: {what} rows={rows} n={n} k={k} p={p:.3f} lam={lam}", flush=True)
        xd, td = dev(x), dev(t)
        if what in ("signed", "masked"):
            name = "topk_signed_mask" if what == "signed" else "topk_masked_value"
            ref = getattr(oracle, name)(x, k, p, lam, tangent=t)
            o, j = (host(a) for a in getattr(gpu, name + "_jvp")(xd, td, k, p, lam))
            close(o, ref["out"], name + " fwd")
            close(j, ref["jvp"], name + " jvp")
        elif what == "loss":
            tt = np.zeros((rows, n), dtype=np.float32)
            tt[np.arange(rows), r.integers(0, n, size=rows)] = 1.0
            ref_loss, ref_grad = oracle.fenchel_young_loss(x, tt, k, p, lam)
            loss, grad = gpu.topk_mask_loss(xd, dev(tt), k, p, lam)
            close(host(grad), ref_grad, "grad")
            err = np.abs(host(loss).astype(np.float64) - ref_loss)
            assert (err <= 2e-6 + 1.2e-7 * np.abs(ref_loss)).all(), float(err.max())
        elif what == "general":
            wk = r.integers(0, 4)
            if wk == 0:
                w = (np.arange(n) < max(1, k)).astype(np.float32)
            elif wk == 1:
                w = np.arange(n, 0, -1).astype(np.float32)
            elif wk == 2:
                w = np.sort(r.choice([0.0, 0.5, 1.0, 2.0], size=n))[::-1].astype(np.float32)
            else:
                w = -np.sort(-(r.normal(size=(rows, n)) ** 2).astype(np.float32), axis=1)
            phi, phic = (("id", gpu.TOPK_PHI_IDENTITY), ("half_sq", gpu.TOPK_PHI_HALF_SQUARE))[r.integers(0, 2)]
            ref = oracle.topk_general(x, w, p, lam, phi, tangent=t)
            o, j = (host(a) for a in gpu.topk_general_jvp(xd, dev(np.ascontiguousarray(w)), td, phic, p, lam))
            close(o, ref["out"], "general fwd")
            close(j, ref["jvp"], "general jvp")
        elif what == "sparse":
            cap = int(min(n, max(1, r.choice([k + 2, 2 * k + 64, n]))))
            ref = oracle.topk_mask(x, k, p, lam, want_perm=True)
            idx, val, nnz = (host(a) for a in gpu.topk_mask_sparse_fwd(xd, k, p, lam, cap))
            for row in range(rows):
                b = int((ref["out"][row] != 0.0).sum())
                m = min(b, cap)
                gi = idx[row, :m]
                assert nnz[row] == b and np.all(idx[row, m:] == -1) and np.all(val[row, m:] == 0.0)
                assert len(np.unique(gi)) == m
                close(val[row, :m], ref["out"][row, gi], "sparse values")
                if m == b:
                    assert np.array_equal(np.sort(gi), np.sort(ref["perm"][row, :b]))
        elif what == "vjp":
            ref = oracle.topk_mask(x, k, p, lam, tangent=t)
            o, v = (host(a) for a in gpu.topk_mask_vjp(xd, td, k, p, lam))
            close(o, ref["out"], "vjp out")
            close(v, ref["jvp"], "vjp")
        else:
            assert np.array_equal(host(gpu.topk_argsort_desc(xd)), oracle.argsort_desc(x))
