"""Independent (slow, numpy/scipy) routes to the quantities the oracle computes.

Nothing here imports the oracle or the HIP library.  Each routine goes back to a definition in the
paper (or to a textbook special case of it) and is used to pin the oracle from the outside.
"""
from __future__ import annotations

import itertools

import numpy as np
from scipy import optimize


def q_of(p: float) -> int:
    """Conjugate exponent, 1/p + 1/q = 1 (only p = 2 -> q = 2 and p = 4/3 -> q = 4 are used)."""
    return 2 if abs(p - 2.0) < 1e-9 else 4


# ---------------------------------------------------------------------------------------------
# Relaxed mask by its definition: argmax_{y in P(1_k)} <y, theta> - (lambda/p) sum y^p with
# P(1_k) = {y in [0,1]^n, sum y = k}  (Sec. 3 "LP formulations" + Sec. 4 "Recovering the previous
# framework").  Brute force over the 3^n active-set patterns {at 0, at 1, free}; the KKT system of
# each pattern is one scalar equation in the multiplier tau of the sum constraint.
def mask_kkt_bruteforce(theta, k, p, lam, tol=1e-11):
    theta = np.asarray(theta, dtype=np.float64)
    n = theta.size
    q = q_of(p)
    sols = []
    for pat in itertools.product((0, 1, 2), repeat=n):      # 0: y=0, 1: y=1, 2: free
        pat = np.array(pat)
        ones, free, zeros = pat == 1, pat == 2, pat == 0
        need = k - ones.sum()
        if free.sum() == 0:
            if need != 0:
                continue
            lo = theta[zeros].max() if zeros.any() else -np.inf     # theta_i - tau <= 0
            hi = (theta[ones] - lam).min() if ones.any() else np.inf  # theta_i - lam - tau >= 0
            if lo <= hi + tol:
                sols.append(ones.astype(np.float64))
            continue
        if need < 0 or need > free.sum():
            continue
        tf = theta[free]
        if q == 2:
            tau = (tf.sum() - lam * need) / free.sum()
        else:
            # sum_free ((theta_i - tau)/lam)^3 = need, every term needs theta_i - tau >= 0
            f = lambda t: (((tf - t) / lam) ** 3).sum() - need
            hi_t = tf.min()
            if f(hi_t) > 0:
                continue
            lo_t = tf.min() - lam * 2.0
            while f(lo_t) < 0:
                lo_t -= lam
            tau = optimize.brentq(f, lo_t, hi_t, xtol=1e-15, rtol=1e-15)
        yf = ((tf - tau) / lam)
        if (yf < -tol).any():
            continue
        yf = np.maximum(yf, 0.0) ** (q - 1)
        if (yf > 1 + tol).any():
            continue
        if zeros.any() and (theta[zeros] - tau > tol).any():
            continue
        if ones.any() and (theta[ones] - lam - tau < -tol).any():
            continue
        y = np.zeros(n)
        y[ones] = 1.0
        y[free] = yf
        sols.append(y)
    assert sols, "no KKT point found"
    for y in sols[1:]:
        assert np.abs(y - sols[0]).max() < 1e-7, "KKT points disagree (maximiser is unique)"
    return sols[0]


# Threshold form of the same maximiser: y_i = clip(((theta_i - tau)_+ / lam)^(q-1), 0, 1) with tau
# fixed by sum y = k.  For p = 2 this is the Euclidean projection of theta/lam onto the capped
# simplex.  tau by bisection (a library-free scalar search).
def mask_by_bisection(theta, k, p, lam, iters=200):
    theta = np.asarray(theta, dtype=np.float64)
    q = q_of(p)

    def y_of(tau):
        return np.clip(np.maximum(theta - tau, 0.0) / lam, 0.0, 1.0) ** (q - 1)

    lo, hi = theta.min() - lam - 1.0, theta.max() + 1.0
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if y_of(mid).sum() > k:
            lo = mid
        else:
            hi = mid
    return y_of(0.5 * (lo + hi))


# Textbook Euclidean projection onto the probability simplex (sort-based), i.e. sparsemax.
def simplex_projection(z):
    z = np.asarray(z, dtype=np.float64)
    u = np.sort(z)[::-1]
    css = np.cumsum(u)
    j = np.arange(1, z.size + 1)
    rho = np.nonzero(u - (css - 1.0) / j > 0)[0][-1]
    tau = (css[rho] - 1.0) / (rho + 1.0)
    return np.maximum(z - tau, 0.0)


# ---------------------------------------------------------------------------------------------
# Relaxed top-k in magnitude by its definition (Prop. 2): u* = argmin_u R*(x - u) + f_phi(u, 1_k),
# f_phi(u, 1_k) = sum of the k largest u_i^2/2 = max over index sets I, |I| = k, of sum_I u_i^2/2;
# y* = grad R*(x - u*).  Epigraph form, solved with SLSQP over all C(n, k) sets (n <= 6).
#
# phi = "abs": f_phi(u, 1_k) = sum of the k largest |u_i| (the OWL norm with w = 1_k, Sec. 4) =
# max over index sets and sign patterns of sum_I eps_i u_i: linear constraints.
def topkmag_by_definition(x, k, p, lam, phi="half_sq"):
    x = np.asarray(x, dtype=np.float64)
    n = x.size
    q = q_of(p)
    sets = [np.array(c) for c in itertools.combinations(range(n), k)] if k > 0 else []

    def rstar(t):
        return (np.abs(t) ** q).sum() / (q * lam ** (q - 1))

    def grad_rstar(t):
        return np.sign(t) * np.abs(t) ** (q - 1) / lam ** (q - 1)

    if k == 0:
        return np.zeros(n)

    def obj(z):
        return rstar(x - z[:n]) + z[n]

    def obj_grad(z):
        g = np.zeros(n + 1)
        g[:n] = -grad_rstar(x - z[:n])
        g[n] = 1.0
        return g

    cons = []
    for I in sets:
        if phi == "abs":
            for eps in itertools.product((-1.0, 1.0), repeat=k):
                a = np.zeros(n + 1)
                a[I] = -np.array(eps)
                a[n] = 1.0
                cons.append({"type": "ineq", "fun": lambda z, a=a: a @ z, "jac": lambda z, a=a: a})
            continue

        def c(z, I=I):
            return z[n] - 0.5 * (z[I] ** 2).sum()

        def cj(z, I=I):
            g = np.zeros(n + 1)
            g[I] = -z[I]
            g[n] = 1.0
            return g
        cons.append({"type": "ineq", "fun": c, "jac": cj})

    def f_phi(u):
        a = np.sort(np.abs(u))[::-1][:k]
        return a.sum() if phi == "abs" else 0.5 * (a ** 2).sum()

    best = None
    for start in (x.copy(), x / (1.0 + lam), 0.5 * x):
        z0 = np.concatenate([start, [f_phi(start) + 1e-3]])
        res = optimize.minimize(obj, z0, jac=obj_grad, constraints=cons, method="SLSQP",
                                options={"ftol": 1e-15, "maxiter": 500})
        if best is None or res.fun < best.fun:
            best = res
    u = best.x[:n]
    return grad_rstar(x - u)


# ---------------------------------------------------------------------------------------------
# Dykstra's alternating projections (Alg. 1) for p = 2, phi = identity.  The problem is the
# Euclidean projection of s - lam*w onto the monotone cone C1 ∩ C2; the linear term is applied
# once, to the starting point (applying it inside both projection steps, as the listing prints it,
# would count it twice).
def dykstra_mask_p2(s, w, lam, iters=2000):
    s = np.asarray(s, dtype=np.float64)
    n = s.size
    v = s - lam * np.asarray(w, dtype=np.float64)
    pc = np.zeros(n)
    qc = np.zeros(n)

    def proj_pairs(z, start):
        out = z.copy()
        for i in range(start, n - 1, 2):
            if out[i] < out[i + 1]:
                out[i] = out[i + 1] = 0.5 * (z[i] + z[i + 1])
        return out

    for _ in range(iters):
        y = proj_pairs(v + pc, 0)
        pc = v + pc - y
        v = proj_pairs(y + qc, 1)
        qc = y + qc - v
    return v


def central_diff_jvp(fwd, x, t, h=1e-6):
    """Directional derivative of a float64 forward map by central differences."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    return (fwd(x + h * t) - fwd(x - h * t)) / (2.0 * h)


# ---------------------------------------------------------------------------------------------
# General non-increasing w.  phi = identity (Prop. 2, first line): y* = argmax over the
# permutahedron P(w) of <y, x> - R(y).  P(w) by its inequalities: every subset S of indices has
# sum_S y_i <= w_1 + .. + w_|S|, with equality for the full set (n <= 5: 31 constraints).
def general_mask_by_definition(x, w, p, lam):
    x = np.asarray(x, dtype=np.float64)
    w = np.sort(np.asarray(w, dtype=np.float64))[::-1]
    n = x.size
    cw = np.concatenate([[0.0], np.cumsum(w)])

    def obj(y):
        return -(y @ x) + lam / p * (np.abs(y) ** p).sum()

    def grad(y):
        return -x + lam * np.sign(y) * np.abs(y) ** (p - 1)

    cons = [{"type": "eq", "fun": lambda y: y.sum() - cw[n], "jac": lambda y: np.ones(n)}]
    for m in range(1, n):
        for S in itertools.combinations(range(n), m):
            a = np.zeros(n)
            a[list(S)] = -1.0
            cons.append({"type": "ineq", "fun": lambda y, a=a, m=m: cw[m] + a @ y,
                         "jac": lambda y, a=a: a})
    best = None
    for start in (np.full(n, cw[n] / n), w[np.argsort(np.argsort(-x))].astype(np.float64)):
        res = optimize.minimize(obj, start, jac=grad, constraints=cons, method="SLSQP",
                                options={"ftol": 1e-15, "maxiter": 1000})
        if best is None or res.fun < best.fun:
            best = res
    return best.x


# phi = x^2/2 (Prop. 2, second line): u* = argmin_u R*(x - u) + f_phi(u, w) with
# f_phi(u, w) = max over permutations pi of sum_i w_pi(i) u_i^2 / 2; y* = grad R*(x - u*).
def general_mag_by_definition(x, w, p, lam):
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    n = x.size
    q = q_of(p)

    def rstar(t):
        return (np.abs(t) ** q).sum() / (q * lam ** (q - 1))

    def grad_rstar(t):
        return np.sign(t) * np.abs(t) ** (q - 1) / lam ** (q - 1)

    def obj(z):
        return rstar(x - z[:n]) + z[n]

    def obj_grad(z):
        g = np.zeros(n + 1)
        g[:n] = -grad_rstar(x - z[:n])
        g[n] = 1.0
        return g

    cons = []
    for perm in itertools.permutations(range(n)):
        wp = w[list(perm)]
        cons.append({"type": "ineq", "fun": lambda z, wp=wp: z[n] - 0.5 * (wp * z[:n] ** 2).sum(),
                     "jac": lambda z, wp=wp: np.concatenate([-wp * z[:n], [1.0]])})

    def f_phi(u):
        return 0.5 * (w * np.sort(u ** 2)[::-1]).sum()

    best = None
    for start in (x.copy(), x / (1.0 + lam * w.max()), 0.5 * x):
        z0 = np.concatenate([start, [f_phi(start) + 1e-3]])
        res = optimize.minimize(obj, z0, jac=obj_grad, constraints=cons, method="SLSQP",
                                options={"ftol": 1e-15, "maxiter": 1000})
        if best is None or res.fun < best.fun:
            best = res
    return grad_rstar(x - best.x[:n])
