"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU needed).

Every check compares the oracle with something that is not the oracle: values printed in the
paper, closed forms, brute force over KKT patterns, textbook routines, a second algorithm from the
paper (Dykstra), a library routine (isotonic regression), finite differences, or invariants.
"""
import os

import numpy as np
import pytest
from scipy import optimize

from tests import independent as ind

P2, P43 = 2.0, 4.0 / 3.0
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------------------------
# Sec. 3 worked example (printed values) through the lambda -> 0 limit.
def _read_golden():
    d = {}
    with open(os.path.join(GOLDEN, "sec3_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split("=")
            d[key.strip()] = [int(t) for t in val.split()]
    return d


@pytest.mark.parametrize("p", [P2, P43])
def test_sec3_worked_example(oracle, p):
    g = _read_golden()
    x = np.array([0.5, -2.0, 1.0], dtype=np.float32)       # x3 >= x1 >= x2, |x2| >= |x3| >= |x1|
    assert x[2] >= x[0] >= x[1] and abs(x[1]) >= abs(x[2]) >= abs(x[0])
    perm = oracle.argsort_desc(x)
    assert (perm + 1).tolist() == g["argsort"]
    rank = np.empty(3, dtype=int)
    rank[perm] = np.arange(1, 4)
    assert rank.tolist() == g["rank"]
    lam = 1e-4
    m = oracle.topk_mask(x, 2, p, lam)["out"]
    assert np.abs(m - np.array(g["topkmask"])).max() < 1e-9
    topk = x * m
    want = np.array([x[i - 1] if i else 0.0 for i in g["topk_keeps"]])
    assert np.abs(topk - want).max() < 1e-6
    # top-k in magnitude: the relaxed operator tends to x o topkmask(|x|) as lambda -> 0
    mg = oracle.topkmag(x, 2, p, lam)["out"]
    want = np.array([x[i - 1] if i else 0.0 for i in g["topkmag_keeps"]])
    assert np.abs(mg - want).max() <= lam * 2.0 + 1e-12      # error bound of Sec. 5 "Example"


def test_argsort_ties_and_signed_zero(oracle):
    z = np.array([1.0, -0.0, 3.0, 0.0, 1.0, 3.0, -2.0, 0.0], dtype=np.float32)
    perm = oracle.argsort_desc(z)
    assert perm.tolist() == [2, 5, 0, 4, 1, 3, 7, 6]
    r = rng(0)
    for _ in range(50):
        n = int(r.integers(1, 200))
        z = r.integers(-5, 5, size=n).astype(np.float32)       # many ties
        want = np.argsort(-z.astype(np.float64), kind="stable")
        assert np.array_equal(oracle.argsort_desc(z), want)


# ----------------------------------------------------------------------------------------------
# The mask lies in P(1_k) = {y in [0,1]^n, sum y = k}; outside one pooled block it is exactly 0
# or (up to rounding of s - (s - lambda)) 1; its JVP sums to zero because sum y is constant.
@pytest.mark.parametrize("p", [P2, P43])
def test_mask_in_permutahedron(oracle, p):
    r = rng(1)
    for _ in range(200):
        n = int(r.integers(1, 40))
        k = int(r.integers(0, n + 1))
        lam = float(10 ** r.uniform(-3, 1))
        th = r.normal(size=n).astype(np.float32)
        t = r.normal(size=n).astype(np.float32)
        res = oracle.topk_mask(th, k, p, lam, tangent=t, want_perm=True, want_block=True)
        y = res["out"]
        assert abs(y.sum() - k) < 1e-9
        assert y.min() >= 0.0 and y.max() <= 1.0 + 1e-12
        a, b = res["block"]
        ys = y[res["perm"]]
        assert np.all(ys[b:] == 0.0) if b > a else np.all(ys[k:] == 0.0)
        assert np.abs(ys[:a] - 1.0).max(initial=0.0) < 1e-12 if b > a else True
        assert abs(res["jvp"].sum()) < 1e-8 * max(1.0, 1.0 / lam)
        # y is non-increasing along the sorted order
        assert np.all(np.diff(ys) <= 1e-12)


# Brute force over all 3^n active-set patterns of the defining concave program (n <= 6).
@pytest.mark.parametrize("p", [P2, P43])
def test_mask_vs_kkt_bruteforce(oracle, p):
    r = rng(2)
    for trial in range(60):
        n = int(r.integers(1, 7))
        k = int(r.integers(0, n + 1))
        lam = float(r.choice([0.05, 0.3, 1.0, 3.0]))
        th = r.normal(size=n).astype(np.float32)
        if trial % 5 == 0 and n >= 2:
            th[1] = th[0]                                     # a tie
        y = oracle.topk_mask(th, k, p, lam)["out"]
        ref = ind.mask_kkt_bruteforce(th.astype(np.float64), k, p, lam)
        assert np.abs(y - ref).max() < 1e-9, (th, k, lam)


# Threshold form / Euclidean projection onto the capped simplex, found by plain bisection.
@pytest.mark.parametrize("p", [P2, P43])
def test_mask_vs_bisection(oracle, p):
    r = rng(3)
    for _ in range(100):
        n = int(r.integers(2, 300))
        k = int(r.integers(1, n))
        lam = float(10 ** r.uniform(-2, 1))
        th = (r.normal(size=n) * r.uniform(0.5, 3)).astype(np.float32)
        y = oracle.topk_mask(th, k, p, lam)["out"]
        ref = ind.mask_by_bisection(th, k, p, lam)
        assert np.abs(y - ref).max() < 1e-9


# k = 1, p = 2: the mask is the projection of theta/lambda onto the simplex (Fig. 2 of the paper:
# P((1,0,0)) is the probability simplex) -- a textbook routine.  n = 2: closed form.
def test_top1_is_simplex_projection(oracle):
    r = rng(4)
    for _ in range(100):
        n = int(r.integers(2, 50))
        lam = float(10 ** r.uniform(-1, 1))
        th = r.normal(size=n).astype(np.float32)
        y = oracle.topk_mask(th, 1, P2, lam)["out"]
        assert np.abs(y - ind.simplex_projection(th.astype(np.float64) / lam)).max() < 1e-10
    for _ in range(50):
        th = r.normal(size=2).astype(np.float32)
        lam = float(10 ** r.uniform(-1, 1))
        y = oracle.topk_mask(th, 1, P2, lam)["out"]
        y1 = np.clip(0.5 + (float(th[0]) - float(th[1])) / (2 * lam), 0, 1)
        assert abs(y[0] - y1) < 1e-12 and abs(y[1] - (1 - y1)) < 1e-12


# ----------------------------------------------------------------------------------------------
# Fig. 1: theta(s) = (3, 1, -1+s, s), k = 2, curve g(s) = mask_2 + mask_3.
# Around s = 1 the entries "1" and "s" are pooled with one unit of weight between them while "3"
# stays at one and "-1+s" at zero (valid for lambda <= 1 and s <= 3 - lambda):
#   p = 2  : g(s) = clip((1 + lambda - s) / (2 lambda), 0, 1)
#   p = 4/3: g(s) = a^3/lambda^3,  a in [0, lambda] the root of a^3 + (a - (1-s))^3 = lambda^3,
#            for |1 - s| < lambda; 1 to the left, 0 to the right.
@pytest.mark.parametrize("lam", [0.25, 0.5, 1.0])
def test_fig1_curve(oracle, lam):
    svals = np.concatenate([np.linspace(-1.0, 3.0 - lam, 81), [1 - lam, 1.0, 1 + lam]])
    for s in svals:
        th = np.array([3.0, 1.0, -1.0 + s, s], dtype=np.float32)
        s32 = float(np.float32(s))
        sm = float(th[2]) + 1.0                          # the s actually seen through entry 3
        y2 = oracle.topk_mask(th, 2, P2, lam)["out"]
        g2 = np.clip((1 + lam - s32) / (2 * lam), 0, 1)
        assert abs((y2[1] + y2[2]) - g2) < 1e-6, (s, lam)
        y43 = oracle.topk_mask(th, 2, P43, lam)["out"]
        d = 1.0 - s32
        if d >= lam:
            g43 = 1.0
        elif d <= -lam:
            g43 = 0.0
        else:
            a = optimize.brentq(lambda a: a ** 3 + (a - d) ** 3 - lam ** 3, 0.0, lam, xtol=1e-15)
            g43 = a ** 3 / lam ** 3
        assert abs((y43[1] + y43[2]) - g43) < 1e-6, (s, lam, sm)
    # hard operator: 1 for s <= 1 (the tie at s = 1 goes to the smaller index), 0 for 1 < s < 4
    for s, want in [(0.0, 1.0), (1.0, 1.0), (1.5, 0.0), (3.5, 0.0)]:
        th = np.array([3.0, 1.0, -1.0 + s, s], dtype=np.float32)
        perm = oracle.argsort_desc(th)
        hard = np.zeros(4)
        hard[perm[:2]] = 1
        assert hard[1] + hard[2] == want
    # exact sparsity and the symmetric point
    for p in (P2, P43):
        assert oracle.topk_mask(np.array([3, 1, 0.5 + lam, 1.5 + lam], np.float32), 2, p, lam)["out"][1] == 0.0
        mid = oracle.topk_mask(np.array([3, 1, 0, 1], np.float32), 2, p, lam)["out"]
        assert abs(mid[1] - 0.5) < 1e-12 and abs(mid[3] - 0.5) < 1e-12


# ----------------------------------------------------------------------------------------------
# Top-k in magnitude.
# Sec. 5 "Example" + App. remark: without ties and for small lambda every block is a singleton and
# y = 1_k-mask o x / (1 + lambda); error bound ||topkmag_R(x) - topkmag(x)||_inf <= lambda ||x||_inf.
def test_topkmag_small_lambda_closed_form(oracle):
    r = rng(5)
    for _ in range(100):
        n = int(r.integers(2, 60))
        k = int(r.integers(1, n))
        x = r.permutation(np.arange(1, n + 1)).astype(np.float32) * r.choice([-1.0, 1.0], size=n).astype(np.float32)
        lam = 1e-3
        y = oracle.topkmag(x, k, P2, lam)["out"]
        keep = np.zeros(n)
        keep[np.argsort(-np.abs(x), kind="stable")[:k]] = 1
        tol = 4e-16 * float(np.abs(x).max()) / lam          # rounding of (s - v)/lambda
        assert np.abs(y - keep * x / (1 + lam)).max() < tol
        assert np.abs(y - keep * x).max() <= lam * np.abs(x).max() + tol
    for _ in range(100):                                   # the bound also with pooling
        n = int(r.integers(2, 60))
        k = int(r.integers(1, n))
        x = r.normal(size=n).astype(np.float32)
        lam = float(10 ** r.uniform(-4, -2))
        y = oracle.topkmag(x, k, P2, lam)["out"]
        keep = np.zeros(n)
        keep[np.argsort(-np.abs(x), kind="stable")[:k]] = 1
        ax = np.abs(x.astype(np.float64))
        srt = np.sort(ax)[::-1]
        if srt[k - 1] / (1 + lam) >= srt[k]:               # no violation => closed form holds
            tol = 4e-16 * ax.max() / lam
            assert np.abs(y - keep * x / (1 + lam)).max() < tol
            assert np.abs(y - keep * x).max() <= lam * ax.max() + tol


# Fig. 2 (phi = x^2/2, k = 2, x = (x1, x2, 1/2, 1), lambda = 0.3): y1 + y2 is exactly 0 in a central
# region.  From the pooling formula the region is max(|x1|, |x2|) <= (1/2)/(1 + lambda).
@pytest.mark.parametrize("p", [P2, P43])
def test_fig2_zero_region(oracle, p):
    lam = 0.3
    edge = 0.5 / 1.3 if p == P2 else None
    for x1 in np.linspace(-0.6, 0.6, 25):
        for x2 in np.linspace(-0.6, 0.6, 25):
            x = np.array([x1, x2, 0.5, 1.0], dtype=np.float32)
            y = oracle.topkmag(x, 2, p, lam)["out"]
            m = max(abs(float(x[0])), abs(float(x[1])))
            if p == P2:
                if m <= edge - 1e-6:
                    assert y[0] == 0.0 and y[1] == 0.0
                    assert abs(y[2] - 0.5 / 1.3) < 1e-12 and abs(y[3] - 1 / 1.3) < 1e-12
                elif m >= edge + 1e-6 and m < 0.5:
                    assert abs(y[0]) + abs(y[1]) > 0.0
            else:
                # p = 4/3: singleton minimiser g of the kept entry 1/2 solves (g-1/2)^3 + lam^3 g = 0
                g = optimize.brentq(lambda g: (g - 0.5) ** 3 + lam ** 3 * g, 0, 0.5, xtol=1e-16)
                if m <= g - 1e-6:
                    assert y[0] == 0.0 and y[1] == 0.0
                elif m >= g + 1e-6 and m < 0.5:
                    assert abs(y[0]) + abs(y[1]) > 0.0


# The definition itself (Prop. 2): min_u R*(x-u) + sum of k largest u_i^2/2, solved as a smooth
# constrained program over all C(n,k) index sets.
@pytest.mark.parametrize("p", [P2, P43])
def test_topkmag_vs_definition(oracle, p):
    r = rng(6)
    for trial in range(25):
        n = int(r.integers(2, 6))
        k = int(r.integers(1, n + 1))
        lam = float(r.choice([0.1, 0.5, 2.0]))
        x = r.normal(size=n).astype(np.float32)
        y = oracle.topkmag(x, k, p, lam)["out"]
        ref = ind.topkmag_by_definition(x.astype(np.float64), k, p, lam)
        assert np.abs(y - ref).max() < 2e-5, (x, k, lam, y, ref)


# ----------------------------------------------------------------------------------------------
# The isotonic solver alone, general weights.
# p = 2, phi = id: v* is the isotonic (non-increasing) regression of s - lambda*w  (library
# routine); it also equals the limit of Dykstra's alternating projections (Alg. 1).
def test_pav_vs_isotonic_regression_and_dykstra(oracle):
    from sklearn.isotonic import isotonic_regression
    r = rng(7)
    for trial in range(40):
        n = int(r.integers(2, 30))
        s = np.sort(r.normal(size=n))[::-1].copy()
        if trial % 2:
            k = int(r.integers(1, n))
            w = (np.arange(n) < k).astype(np.float64)
        else:
            w = np.sort(r.uniform(0, 2, size=n))[::-1].copy()
        lam = float(r.choice([0.1, 1.0, 4.0]))
        v, _ = oracle.pav(s, w, "id", P2, lam)
        ref = isotonic_regression(s - lam * w, increasing=False)
        assert np.abs(v - ref).max() < 1e-12
        if n <= 12:
            dyk = ind.dykstra_mask_p2(s, w, lam, iters=4000)
            assert np.abs(v - dyk).max() < 1e-6
    # phi = x^2/2, p = 2: minimise sum (s-v)^2/(2 lam) + w v^2/2 = weighted isotonic regression of
    # s/(1+lam w) with weights (1+lam w)/lam.
    for trial in range(40):
        n = int(r.integers(2, 30))
        s = np.sort(np.abs(r.normal(size=n)))[::-1].copy()
        k = int(r.integers(1, n))
        w = (np.arange(n) < k).astype(np.float64)
        lam = float(r.choice([0.1, 1.0, 4.0]))
        v, _ = oracle.pav(s, w, "half_sq", P2, lam)
        ref = isotonic_regression(s / (1 + lam * w), sample_weight=(1 + lam * w) / lam, increasing=False)
        assert np.abs(v - ref).max() < 1e-12


# General convex check of the isotonic solution for p = 4/3 (both phi): KKT of
# min_{v1>=...>=vn} sum h_i(v_i) (App. "Dual of isotonic optimization"): h_i'(v_i) = alpha_i -
# alpha_{i-1} with multipliers alpha_j >= 0 of v_j >= v_{j+1}, so G_j = sum_{i<=j} h_i'(v_i) =
# alpha_j: G_n = 0, G_j >= 0, and G_j = 0 wherever v_j > v_{j+1}.
@pytest.mark.parametrize("phi", ["id", "half_sq"])
def test_pav_p43_kkt(oracle, phi):
    r = rng(8)
    for trial in range(60):
        n = int(r.integers(1, 40))
        s = np.sort(np.abs(r.normal(size=n)) if phi == "half_sq" else r.normal(size=n))[::-1].copy()
        k = int(r.integers(0, n + 1))
        w = (np.arange(n) < k).astype(np.float64)
        lam = float(r.choice([0.2, 1.0, 3.0]))
        v, bid = oracle.pav(s, w, phi, P43, lam)
        assert np.all(np.diff(v) <= 1e-13)
        hp = (v - s) ** 3 / lam ** 3 + (w if phi == "id" else w * v)
        G = np.cumsum(hp)
        assert abs(G[-1]) < 1e-9
        assert np.all(G >= -1e-9)
        strict = np.nonzero(np.diff(v) < -1e-12)[0]
        assert np.all(np.abs(G[strict]) < 1e-9)


# ----------------------------------------------------------------------------------------------
# Invariants of the mask: lambda -> infinity gives k/n (Sec. 7); joint scaling of (theta, lambda);
# shift of theta; permutation equivariance.
@pytest.mark.parametrize("p", [P2, P43])
def test_mask_invariances(oracle, p):
    r = rng(9)
    for _ in range(30):
        n = int(r.integers(2, 64))
        k = int(r.integers(1, n))
        lam = float(10 ** r.uniform(-1, 0.5))
        th = r.normal(size=n).astype(np.float32)
        y = oracle.topk_mask(th, k, p, lam)["out"]
        big = oracle.topk_mask(th, k, p, 1e6)["out"]
        assert np.abs(big - k / n).max() < 1e-4
        y2 = oracle.topk_mask(th * np.float32(4.0), k, p, 4.0 * lam)["out"]       # exact in fp32
        assert np.abs(y - y2).max() < 1e-12
        perm = r.permutation(n)
        y3 = oracle.topk_mask(th[perm], k, p, lam)["out"]
        assert np.abs(y3 - y[perm]).max() < 1e-12
        th64 = th.astype(np.float64)
        y4 = oracle.topk_mask(th64 + 0.375, k, p, lam, f64=True)["out"]
        assert np.abs(y4 - y).max() < 1e-11


# ----------------------------------------------------------------------------------------------
# JVP (Prop. 7) against central finite differences of the float64 forward, away from kinks, and
# the symmetry <a, J b> = <b, J a> that follows from y = grad f (Prop. 2).
def _same_piece(fn, x, t, h, k, p, lam):
    r0 = fn(x, k, p, lam, want_perm=True, want_block=True, f64=True)
    for sgn in (-1.0, 1.0):
        r1 = fn(x + sgn * 4 * h * t, k, p, lam, want_perm=True, want_block=True, f64=True)
        if not np.array_equal(r0["perm"], r1["perm"]) or not np.array_equal(r0["block"], r1["block"]):
            return False
    return True


@pytest.mark.parametrize("op", ["mask", "mag"])
@pytest.mark.parametrize("p", [P2, P43])
def test_jvp_vs_finite_differences(oracle, op, p):
    fn = oracle.topk_mask if op == "mask" else oracle.topkmag
    r = rng(10)
    checked = 0
    for _ in range(200):
        n = int(r.integers(2, 30))
        k = int(r.integers(1, n))
        lam = float(r.choice([0.05, 0.3, 1.0, 2.0]))
        x = r.normal(size=n)
        t = r.normal(size=n)
        h = 1e-6
        if not _same_piece(fn, x, t, h, k, p, lam):
            continue
        jvp = fn(x, k, p, lam, tangent=t, f64=True)["jvp"]
        fd = ind.central_diff_jvp(lambda z: fn(z, k, p, lam, f64=True)["out"], x, t, h)
        scale = max(1.0, np.abs(jvp).max())
        assert np.abs(jvp - fd).max() < 2e-6 * scale / min(1.0, lam), (op, p, n, k, lam)
        checked += 1
    assert checked > 100


@pytest.mark.parametrize("op", ["mask", "mag"])
@pytest.mark.parametrize("p", [P2, P43])
def test_jacobian_symmetric(oracle, op, p):
    fn = oracle.topk_mask if op == "mask" else oracle.topkmag
    r = rng(11)
    for _ in range(50):
        n = int(r.integers(2, 40))
        k = int(r.integers(1, n))
        lam = float(r.choice([0.1, 1.0]))
        x = r.normal(size=n).astype(np.float32)
        a = r.normal(size=n).astype(np.float32)
        b = r.normal(size=n).astype(np.float32)
        Ja = fn(x, k, p, lam, tangent=a)["jvp"]
        Jb = fn(x, k, p, lam, tangent=b)["jvp"]
        lhs, rhs = float(b.astype(np.float64) @ Ja), float(a.astype(np.float64) @ Jb)
        assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))
        # Prop. 7: within a block the weights of d gamma / d s sum to one for phi = id, so a
        # constant tangent is annihilated (shift invariance of the mask)
        if op == "mask":
            assert np.abs(fn(x, k, p, lam, tangent=np.ones(n, np.float32))["jvp"]).max() < 1e-9 / lam


# The strict merge rule decides the JVP at p = 2 kinks: tied entries inside the kept run are not
# pooled (JVP 0 there), an entry exactly at the block value stays outside the block.
def test_strict_merge_convention(oracle):
    th = np.array([2.0, 2.0, 0.0, -1.0], dtype=np.float32)
    res = oracle.topk_mask(th, 2, P2, 0.5, tangent=np.array([1, -1, 3, 5], np.float32), want_block=True)
    assert res["block"].tolist() == [0, 0] or res["block"][0] == res["block"][1]
    assert np.array_equal(res["out"], [1.0, 1.0, 0.0, 0.0]) and np.all(res["jvp"] == 0.0)
    # s_k - lambda == s_{k+1} exactly: not a violation
    th = np.array([3.0, 1.5, 1.0, 0.0], dtype=np.float32)
    res = oracle.topk_mask(th, 2, P2, 0.5, tangent=np.array([1, -1, 3, 5], np.float32), want_block=True)
    assert res["block"][0] == res["block"][1]
    assert np.all(res["jvp"] == 0.0)
    # block {1, 0.75} with gamma = (1.75 - 0.5)/2 = 0.625; entry 0.625 sits exactly at gamma: outside
    th = np.array([3.0, 1.0, 0.75, 0.625], dtype=np.float32)
    res = oracle.topk_mask(th, 2, P2, 0.5, tangent=np.array([0, 1, 2, 7], np.float32), want_block=True)
    assert res["block"].tolist() == [1, 3]
    assert np.allclose(res["out"], [1.0, 0.75, 0.25, 0.0], atol=1e-15)
    assert np.allclose(res["jvp"], [0.0, -1.0, 1.0, 0.0], atol=1e-15)


def test_strict_merge_convention_p43(oracle):
    # p = 4/3, lambda = 2: eight equal values s = 1 carrying one unit of weight pool at
    # gamma = s - lambda (1/8)^(1/3) = 0 exactly (each gets ((1-0)/2)^3 = 1/8, summing to 1).
    # The entry 2 above them has singleton minimiser 2 - lambda = 0 == gamma: a tie, not merged,
    # so it stays at exactly one and its JVP row is zero.
    th = np.array([2.0] + [1.0] * 8 + [-5.0], dtype=np.float32)
    t = np.arange(1, 11, dtype=np.float32)
    res = oracle.topk_mask(th, 2, P43, 2.0, tangent=t, want_block=True)
    assert res["block"].tolist() == [1, 9]
    assert np.allclose(res["out"], [1.0] + [0.125] * 8 + [0.0], atol=1e-15)
    assert res["jvp"][0] == 0.0 and res["jvp"][9] == 0.0
    # inside the block: dy_i = 3 (s_i - gamma)^2 / lambda^3 (t_i - mean t) = (3/8)(t_i - 5.5)
    assert np.allclose(res["jvp"][1:9], 0.375 * (t[1:9] - 5.5), atol=1e-13)


def test_edge_cases(oracle):
    th = np.array([0.3, -1.0, 2.0], dtype=np.float32)
    t = np.ones(3, np.float32)
    for p in (P2, P43):
        r0 = oracle.topk_mask(th, 0, p, 0.7, tangent=t)
        assert np.all(r0["out"] == 0.0) and np.all(r0["jvp"] == 0.0)
        r3 = oracle.topk_mask(th, 3, p, 0.7, tangent=t)
        assert np.abs(r3["out"] - 1.0).max() < 1e-15 and np.abs(r3["jvp"]).max() < 1e-12
    m0 = oracle.topkmag(th, 0, P2, 0.7, tangent=t)
    assert np.all(m0["out"] == 0.0) and np.all(m0["jvp"] == 0.0)
    m3 = oracle.topkmag(th, 3, P2, 0.7, tangent=t)
    assert np.abs(m3["out"] - th / 1.7).max() < 1e-7 and np.abs(m3["jvp"] - 1 / 1.7).max() < 1e-12
    # sign(0) = 0
    z = oracle.topkmag(np.array([0.0, -0.0, 1.0], np.float32), 2, P2, 0.1, tangent=t)
    assert z["out"][0] == 0.0 and z["out"][1] == 0.0
    one = oracle.topk_mask(np.array([5.0], np.float32), 1, P2, 1.0, tangent=np.ones(1, np.float32))
    assert abs(one["out"][0] - 1.0) < 1e-15 and one["jvp"][0] == 0.0


# ----------------------------------------------------------------------------------------------
# The function f_{phi,R}(x, 1_k) itself (Prop. 2) and the Fenchel-Young top-k loss of Sec. 6.
# The oracle evaluates the minimisation form at u*; these checks come from the other side.
@pytest.mark.parametrize("p", [P2, P43])
def test_value_is_the_regularised_lp_over_the_permutahedron(oracle, p):
    """phi = id: f = max_{y in P(1_k)} <y, x> - R(y) with P(1_k) = {0 <= y <= 1, sum y = k}
    (Sec. 4), solved here as a smooth constrained program; and f = <y*, x> - R(y*) at the
    operator's own output (strong duality)."""
    r = rng(40)
    for _ in range(30):
        n = int(r.integers(2, 8))
        k = int(r.integers(1, n + 1))
        lam = float(r.choice([0.2, 1.0, 3.0]))
        x = r.normal(size=n)
        f = float(oracle.value(x, k, p, lam)[0])
        obj = lambda y: -(y @ x - lam / p * np.sum(np.abs(y) ** p))
        res = optimize.minimize(obj, np.full(n, k / n), method="SLSQP", bounds=[(0, 1)] * n,
                                constraints=[{"type": "eq", "fun": lambda y: y.sum() - k}],
                                options={"ftol": 1e-14, "maxiter": 500})
        assert abs(f + res.fun) < 1e-6 * max(1.0, abs(f)), (x, k, lam, f, -res.fun)
        y = oracle.topk_mask(x, k, p, lam, f64=True)["out"]
        assert abs(f - (y @ x - lam / p * np.sum(y ** p))) < 1e-11 * max(1.0, abs(f))


@pytest.mark.parametrize("phi", ["id", "half_sq"])
@pytest.mark.parametrize("p", [P2, P43])
def test_operator_is_the_gradient_of_the_value(oracle, phi, p):
    """y = grad_1 f_{phi,R}(x, 1_k) (Prop. 2): central differences of the value."""
    r = rng(41)
    op = oracle.topk_mask if phi == "id" else oracle.topkmag
    for _ in range(40):
        n = int(r.integers(2, 12))
        k = int(r.integers(1, n))
        lam = float(r.choice([0.3, 1.0]))
        x = r.normal(size=n)
        y = op(x, k, p, lam, f64=True)["out"]
        h = 1e-6
        g = np.array([(oracle.value(x + h * e, k, p, lam, phi)[0] -
                       oracle.value(x - h * e, k, p, lam, phi)[0]) / (2 * h) for e in np.eye(n)])
        assert np.abs(g - y).max() < 5e-6 / min(1.0, lam), (phi, p, x, k, lam)


def test_value_small_lambda_and_loss_lower_bound(oracle):
    r = rng(42)
    for p in (P2, P43):
        x = r.normal(size=(5, 9))
        top = -np.sort(-x, axis=1)[:, :3]
        assert np.abs(oracle.value(x, 3, p, 1e-7) - top.sum(axis=1)).max() < 1e-6
        ax = -np.sort(-np.abs(x), axis=1)[:, :3]
        assert np.abs(oracle.value(x, 3, p, 1e-7, "half_sq") - 0.5 * (ax ** 2).sum(axis=1)).max() < 1e-6
        # Fenchel-Young inequality: f(x) + f*(t) - <x, t> >= 0 with f*(t) = R(t) = k' lambda / p for
        # a 0/1 target with k' <= k ones (t in P(1_k) needs sum t = k: use k ones)
        for lam in (0.3, 2.0):
            t = np.zeros_like(x)
            for i in range(x.shape[0]):
                t[i, r.permutation(9)[:3]] = 1.0
            loss, grad = oracle.fenchel_young_loss(x, t, 3, p, lam)
            assert (loss + 3 * lam / p > -1e-12).all()
            # equality when the target is the hard top-k of a well separated x and lambda is small
        xs = np.array([[10.0, 8.0, 6.0, -5.0, -7.0]])
        ts = np.array([[1.0, 1.0, 1.0, 0.0, 0.0]])
        loss, grad = oracle.fenchel_young_loss(xs, ts, 3, p, 0.5)
        assert abs(loss[0] + 3 * 0.5 / p) < 1e-12 and np.abs(grad).max() < 1e-12


# ----------------------------------------------------------------------------------------------
# The two variants on |x|.  Signed mask (phi = |x|, Sec. 4): the definition of Prop. 2 with the
# OWL norm f_phi(u, 1_k) = sum of the k largest |u_i|, solved as a constrained program; the value
# lambda -> infinity where u* = 0 and y = grad R*(x) exactly; agreement with sign(x) o mask(|x|)
# whenever the truncation at zero is inactive; the JVP by central differences.
@pytest.mark.parametrize("p", [P2, P43])
def test_signed_mask_vs_definition(oracle, p):
    r = rng(21)
    clipped_cases = 0
    for trial in range(30):
        n = int(r.integers(2, 6))
        k = int(r.integers(1, n + 1))
        lam = float(r.choice([0.1, 0.5, 2.0]))
        x = r.normal(size=n).astype(np.float32)
        y = oracle.topk_signed_mask(x, k, p, lam)["out"]
        ref = ind.topkmag_by_definition(x.astype(np.float64), k, p, lam, phi="abs")
        assert np.abs(y - ref).max() < 5e-5, (x, k, lam, y, ref)
        m = oracle.topk_mask(np.abs(x), k, p, lam)["out"]
        clipped_cases += int(np.abs(np.abs(y) - m).max() > 1e-3)
    assert clipped_cases >= 3          # the truncation at zero was exercised


def test_signed_mask_limits_and_jvp(oracle):
    r = rng(22)
    for p, q in ((P2, 2), (P43, 4)):
        x = r.normal(size=(4, 9))
        t = r.normal(size=(4, 9))
        # lambda >= max |x|: every v is truncated to 0, y = grad r*(x), dy = hess r*(x) t
        lam = 5.0
        res = oracle.topk_signed_mask(x, 3, p, lam, tangent=t, f64=True)
        assert np.allclose(res["out"], np.sign(x) * np.abs(x / lam) ** (q - 1), rtol=0, atol=1e-14)
        assert np.allclose(res["jvp"], (q - 1) * np.abs(x / lam) ** (q - 2) / lam * t, rtol=0, atol=1e-14)
        # top-k magnitudes above lambda: no truncation, the signed mask of |x|
        xs = x * 3.0 + np.sign(x) * 2.0
        lam = 0.5
        res = oracle.topk_signed_mask(xs, 3, p, lam, tangent=t, f64=True)
        m = oracle.topk_mask(np.abs(xs), 3, p, lam, tangent=np.sign(xs) * t, f64=True)
        assert np.array_equal(res["out"], np.sign(xs) * m["out"])
        assert np.array_equal(res["jvp"], np.sign(xs) * m["jvp"])
        # hard limit: sign(x) o (top-k mask of |x|)
        hard = oracle.topk_signed_mask(xs, 3, p, 1e-9, f64=True)["out"]
        top = np.argsort(-np.abs(xs), axis=1)[:, :3]
        ref = np.zeros_like(xs)
        np.put_along_axis(ref, top, np.take_along_axis(np.sign(xs), top, 1), 1)
        assert np.abs(hard - ref).max() < 1e-6
    checked = 0
    for _ in range(200):
        p = P2 if r.random() < 0.5 else P43
        n = int(r.integers(2, 20))
        k = int(r.integers(1, n))
        lam = float(r.choice([0.3, 1.0, 2.0]))
        x, t = r.normal(size=n), r.normal(size=n)
        fn = oracle.topk_signed_mask
        if not _same_piece(fn, x, t, 1e-6, k, p, lam):
            continue
        # also stay on one side of the truncation at zero
        o = [fn(x + d * t, k, p, lam, f64=True)["out"] for d in (-4e-6, 0.0, 4e-6)]
        m = [oracle.topk_mask(np.abs(x + d * t), k, p, lam, f64=True)["out"] for d in (-4e-6, 0.0, 4e-6)]
        cl = [np.abs(np.abs(a) - b) > 1e-12 for a, b in zip(o, m)]
        if not (np.array_equal(cl[0], cl[1]) and np.array_equal(cl[1], cl[2])):
            continue
        jvp = fn(x, k, p, lam, tangent=t, f64=True)["jvp"]
        fd = ind.central_diff_jvp(lambda z: fn(z, k, p, lam, f64=True)["out"], x, t, 1e-6)
        assert np.abs(jvp - fd).max() < 2e-6 * max(1.0, np.abs(jvp).max()) / min(1.0, lam)
        checked += 1
    assert checked > 100


# x o mask(|x|) (Sec. 7): lambda -> infinity gives (k / n) x, lambda -> 0 the hard top-k in
# magnitude (both stated in the paper), in between the product with the mask pinned above; the
# JVP by central differences.
def test_masked_value_limits_and_jvp(oracle):
    r = rng(23)
    for p in (P2, P43):
        x = r.normal(size=(5, 12))
        k = 4
        big = oracle.topk_masked_value(x, k, p, 1e8, f64=True)["out"]
        assert np.abs(big - (k / 12) * x).max() < 1e-5
        hard = oracle.topk_masked_value(x, k, p, 1e-9, f64=True)["out"]
        keep = np.argsort(-np.abs(x), axis=1)[:, :k]
        ref = np.zeros_like(x)
        np.put_along_axis(ref, keep, np.take_along_axis(x, keep, 1), 1)
        assert np.abs(hard - ref).max() < 1e-6
        y = oracle.topk_masked_value(x, k, p, 0.4, f64=True)["out"]
        assert np.array_equal(y, x * oracle.topk_mask(np.abs(x), k, p, 0.4, f64=True)["out"])
    checked = 0
    for _ in range(150):
        p = P2 if r.random() < 0.5 else P43
        n = int(r.integers(2, 20))
        k = int(r.integers(1, n))
        lam = float(r.choice([0.3, 1.0, 2.0]))
        x, t = r.normal(size=n), r.normal(size=n)
        if not _same_piece(oracle.topk_signed_mask, x, t, 1e-6, k, p, lam):
            continue
        fn = oracle.topk_masked_value
        jvp = fn(x, k, p, lam, tangent=t, f64=True)["jvp"]
        fd = ind.central_diff_jvp(lambda z: fn(z, k, p, lam, f64=True)["out"], x, t, 1e-6)
        assert np.abs(jvp - fd).max() < 4e-6 * max(1.0, np.abs(jvp).max()) / min(1.0, lam)
        checked += 1
    assert checked > 80


# ----------------------------------------------------------------------------------------------
# Dykstra's algorithm (Alg. 1) with a fixed iteration count: the first iterations of a three-
# element row worked out by hand; the limit is the exact operator (the Euclidean projection onto
# the monotone cone, i.e. the library isotonic regression of s - lambda w); the iterates of a
# separately written numpy version; zero iterations give the hard mask.
def test_dykstra_iterations(oracle):
    # s = (1, 0.8, 0), k = 1, lambda = 1: v0 = (0, 0.8, 0).
    # iteration 1: C1 pair (1,2): 0 < 0.8 -> (0.4, 0.4, 0), p = (-0.4, 0.4, 0); C2 pair (2,3): fine
    #   -> v1 = (0.4, 0.4, 0), q = 0, y = s - v1 = (0.6, 0.4, 0)
    # iteration 2: z = v1 + p = (0, 0.8, 0) -> same projection, v2 = v1: converged after one.
    x = np.array([0.8, 0.0, 1.0], dtype=np.float32)                 # un-sorted on purpose
    a = float(np.float32(0.8))
    for it in (1, 2, 7):
        y = oracle.topk_mask_dykstra(x, 1, 1.0, it)
        assert np.allclose(y, [a - 0.5 * a, 0.0, 1.0 - 0.5 * a], rtol=0, atol=1e-15), (it, y)
    # s = (3, 2, 2.5, 1) sorted (3, 2.5, 2, 1), k = 2, lambda = 2: v0 = (1, 0.5, 2, 1)
    # it 1: C1 pairs (1,2): 1 >= 0.5 ok; (3,4): 2 >= 1 ok -> y = v0, p = 0;
    #       C2 pair (2,3): 0.5 < 2 -> 1.25, 1.25 -> v1 = (1, 1.25, 1.25, 1), q = (0, -0.75, 0.75, 0)
    x = np.array([3.0, 2.0, 2.5, 1.0], dtype=np.float32)
    y1 = oracle.topk_mask_dykstra(x, 2, 2.0, 1)
    assert np.allclose(y1, [(3 - 1) / 2, (2 - 1.25) / 2, (2.5 - 1.25) / 2, 0.0], rtol=0, atol=1e-15)
    # it 2: z = v1 + p = v1: C1 (1,2): 1 < 1.25 -> 1.125 both; (3,4) ok -> y = (1.125, 1.125, 1.25, 1)
    #       p = (-0.125, 0.125, 0, 0); z' = y + q = (1.125, 0.375, 2, 1): C2 (2,3): -> 1.1875 both
    #       v2 = (1.125, 1.1875, 1.1875, 1)
    y2 = oracle.topk_mask_dykstra(x, 2, 2.0, 2)
    assert np.allclose(y2, [(3 - 1.125) / 2, (2 - 1.1875) / 2, (2.5 - 1.1875) / 2, 0.0], rtol=0,
                       atol=1e-15)
    r = rng(31)
    for _ in range(30):
        n = int(r.integers(1, 40))
        k = int(r.integers(0, n + 1))
        lam = float(r.choice([0.1, 1.0, 3.0]))
        x = r.normal(size=n).astype(np.float32)
        hard = oracle.topk_mask_dykstra(x, k, lam, 0)
        ref = np.zeros(n)
        ref[np.argsort(-x, kind="stable")[:k]] = 1.0
        assert np.abs(hard - ref).max() < 1e-12
        exact = oracle.topk_mask(x, k, P2, lam)["out"]
        assert np.abs(oracle.topk_mask_dykstra(x, k, lam, 20000) - exact).max() < 1e-8
        s = np.sort(x.astype(np.float64))[::-1]
        w = (np.arange(n) < k).astype(np.float64)
        for it in (1, 3, 10):
            v = ind.dykstra_mask_p2(s, w, lam, iters=it)
            got = oracle.topk_mask_dykstra(s.astype(np.float32), k, lam, it)
            assert np.abs(got - (s - v) / lam).max() < 1e-13


# ----------------------------------------------------------------------------------------------
# General non-increasing weights (soft rank / soft sort / partial ranks).  phi = identity: the
# regularised LP over the permutahedron P(w) solved as a constrained program; phi = x^2/2: the
# definition of Prop. 2 with f_phi(u, w) as a maximum over permutations; w = 1_k reproduces the
# top-k operators bit for bit; p = 2 is the Euclidean projection of x / lambda onto P(w) computed
# from the library isotonic regression; the JVP by central differences.
@pytest.mark.parametrize("p", [P2, P43])
def test_general_weights_vs_definitions(oracle, p):
    r = rng(41)
    for trial in range(20):
        n = int(r.integers(2, 6))
        lam = float(r.choice([0.2, 1.0, 3.0]))
        x = r.normal(size=n).astype(np.float32) * 2
        w = np.sort(r.choice([0.0, 0.5, 1.0, 2.0, 3.0], size=n))[::-1].astype(np.float32)
        y = oracle.topk_general(x, w, p, lam, "id")["out"]
        ref = ind.general_mask_by_definition(x.astype(np.float64), w, p, lam)
        assert np.abs(y - ref).max() < 1e-4, ("id", x, w, lam, y, ref)
        if n <= 4:
            y = oracle.topk_general(x, w, p, lam, "half_sq")["out"]
            ref = ind.general_mag_by_definition(x.astype(np.float64), w, p, lam)
            assert np.abs(y - ref).max() < 1e-4, ("half_sq", x, w, lam, y, ref)


def test_general_weights_special_cases_and_jvp(oracle):
    from sklearn.isotonic import isotonic_regression
    r = rng(42)
    for _ in range(30):
        n = int(r.integers(1, 50))
        k = int(r.integers(0, n + 1))
        lam = float(r.choice([0.1, 1.0]))
        x = r.normal(size=(3, n)).astype(np.float32)
        t = r.normal(size=(3, n)).astype(np.float32)
        ones_k = (np.arange(n) < k).astype(np.float32)
        for p in (P2, P43):
            for phi, fn in (("id", oracle.topk_mask), ("half_sq", oracle.topkmag)):
                a = oracle.topk_general(x, ones_k, p, lam, phi, tangent=t)
                b = fn(x, k, p, lam, tangent=t)
                assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["jvp"], b["jvp"])
        # soft rank weights: projection onto the permutahedron through isotonic regression
        rho = np.arange(n, 0, -1).astype(np.float32)
        y = oracle.topk_general(x[0], rho, P2, lam, "id")["out"]
        order = np.argsort(-x[0], kind="stable")
        s = x[0].astype(np.float64)[order]
        v = isotonic_regression(s - lam * rho.astype(np.float64), increasing=False)
        ref = np.empty(n)
        ref[order] = (s - v) / lam
        assert np.abs(y - ref).max() < 1e-9
        assert abs(y.sum() - rho.sum()) < 1e-8 * max(1.0, rho.sum())
    checked = 0
    for _ in range(300):
        p = P2 if r.random() < 0.5 else P43
        phi = "id" if r.random() < 0.5 else "half_sq"
        n = int(r.integers(2, 16))
        lam = float(r.choice([0.3, 1.0, 2.0]))
        x, t = r.normal(size=n) * 2, r.normal(size=n)
        w = np.sort(r.choice([0.0, 0.5, 1.0, 2.0, 3.0], size=n))[::-1].astype(np.float32)
        f = lambda z: oracle.topk_general(z, w, p, lam, phi, f64=True)["out"]
        h = 1e-6
        # same piece: second differences vanish when no block changes between x - 4ht and x + 4ht
        a, b, c = f(x - 4 * h * t), f(x), f(x + 4 * h * t)
        if np.abs(a - 2 * b + c).max() > 1e-9:
            continue
        jvp = oracle.topk_general(x, w, p, lam, phi, tangent=t, f64=True)["jvp"]
        fd = ind.central_diff_jvp(f, x, t, h)
        assert np.abs(jvp - fd).max() < 3e-6 * max(1.0, np.abs(jvp).max()) / min(1.0, lam)
        checked += 1
    assert checked > 100
