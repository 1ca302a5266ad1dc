// CPU float64 oracle for the p-norm-regularised top-k mask / top-k-in-magnitude operators.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and the
// benchmark's cpu_baseline leg may call it.  It shares no code with the HIP library.
//
// What it computes (paper: "Fast, Differentiable and Sparse Top-k: a Convex Analysis Perspective"):
//   * descending argsort / sort (Sec. 3 "Review of operators"), ties broken by ascending index;
//   * the relaxed operator y* = grad R*(x - u*) of Prop. 2 (relaxed operator) with
//     R(y) = (lambda/p) ||y||_p^p, p in {2, 4/3}  (Sec. 4 "Differentiable and sparse top-k operators";
//     lambda as in the caption of Fig. 2 and App. "Subproblem derivation");
//   * u* through the reductions to isotonic optimisation: Prop. 5 (phi = identity, top-k mask) and
//     Prop. 6 (phi = x^2/2, top-k in magnitude), with w = 1_k  (Eq. (topk_mask));
//   * the isotonic problem  min_{v1>=...>=vn} sum_i h_i(v_i),  h_i(v) = r*(s_i - v) + w_i phi(v)
//     (Eq. (isotonic_separable)) by the pool-adjacent-violators algorithm of App. "PAV algorithm",
//     written as the usual left-to-right block stack, merging only on a STRICT violation;
//   * the pooling sub-problem (Eq. (pav_subproblem)) in the closed forms of Sec. 5 "Example" and
//     App. "Subproblem derivation";
//   * the Jacobian-vector product from Prop. 7 (differentiation), with lambda restored.
//
// With 1/p + 1/q = 1:  r*(t) = |t|^q / (q lambda^(q-1)),  grad r*(t) = sign(t)|t|^(q-1)/lambda^(q-1).
//   p = 2   -> q = 2,  grad r*(t) = t / lambda
//   p = 4/3 -> q = 4,  grad r*(t) = t^3 / lambda^3
//
// All arithmetic is float64 on the float32 inputs widened exactly.  No blocking, no fusion.
// Parity pins: see tests/test_oracle_*.py (every exported function is pinned).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// phi(x) = x  |  phi(x) = x^2 / 2  |  phi(x) = |x| (the signed top-k mask of Sec. 4, "Connection
// with k-support and OWL norms": on the non-negative cone of Prop. 6 it is the identity, so the
// pooling steps are those of phi(x) = x, followed by the truncation at zero)
enum Phi { PHI_ID = 0, PHI_HALF_SQ = 1, PHI_ABS = 2 };
enum Pcode { P_2 = 0, P_4_3 = 1 };          // p = 2       |   p = 4/3

struct Problem {
  Phi phi;
  Pcode p;
  double lambda;
};

// ---------------------------------------------------------------------------------------------
// Sec. 3, argsort in descending order.  Ties: smaller original index first.  -0.0f == +0.0f
// under the float comparison, so both zeros are one value.
template <class T>
void argsort_desc(const T* z, int64_t n, int32_t* perm) {
  std::iota(perm, perm + n, 0);
  std::sort(perm, perm + n, [z](int32_t a, int32_t b) {
    if (z[a] > z[b]) return true;
    if (z[a] < z[b]) return false;
    return a < b;
  });
}

// ---------------------------------------------------------------------------------------------
// Pooling sub-problem, Eq. (pav_subproblem):  gamma_B = argmin_gamma sum_{i in B} h_i(gamma)
// over the contiguous block B = [lo, hi) of the sorted vector s, W = sum_B w_i, S = sum_B s_i.
//
// p = 2, phi = id    : h_i = (s_i-g)^2/(2 lambda) + w_i g       ->  g = (S - lambda W)/|B|
// p = 2, phi = x^2/2 : Sec. 5 "Example"                          ->  g = S / sum_B(lambda w_i + 1)
// p = 4/3, phi = id  : root of  sum_B (g - s_i)^3 + lambda^3 W = 0          (App. A.5)
// p = 4/3, x^2/2     : root of  sum_B (g - s_i)^3 + lambda^3 g W = 0        (App. A.5, last case)
// Both cubics are strictly increasing in g, so the real root is unique.
double cubic_F(const double* s, int64_t lo, int64_t hi, double g, double lam3W, bool times_g,
               double* dF) {
  double F = 0.0, D = 0.0;
  for (int64_t i = lo; i < hi; ++i) {
    double d = g - s[i];
    F += d * d * d;
    D += 3.0 * d * d;
  }
  if (times_g) {
    F += lam3W * g;
    D += lam3W;
  } else {
    F += lam3W;
  }
  if (dF) *dF = D;
  return F;
}

double cubic_root(const double* s, int64_t lo, int64_t hi, double lambda, double W, bool times_g) {
  double smin = s[lo], smax = s[lo];
  for (int64_t i = lo; i < hi; ++i) {
    smin = std::min(smin, s[i]);
    smax = std::max(smax, s[i]);
  }
  const double lam3W = lambda * lambda * lambda * W;
  const double cnt = double(hi - lo);
  double a, b;   // F(a) <= 0 <= F(b)
  if (times_g) {
    // s >= 0 here (sorted magnitudes):  F(0) = -sum s^3 <= 0,  F(smax) >= 0.
    a = std::min(0.0, smin);
    b = std::max(smax, 0.0);
  } else {
    // At g = smin - delta every term is <= -delta^3, so F <= -|B| delta^3 + lambda^3 W.
    double delta = lambda * std::cbrt(std::max(W, 0.0) / cnt);
    a = smin - delta;
    b = smax;
    if (W < 0.0) b = smax + lambda * std::cbrt(-W / cnt);
  }
  if (a == b) return a;
  double g = 0.5 * (a + b);
  for (int it = 0; it < 200; ++it) {
    double D;
    double F = cubic_F(s, lo, hi, g, lam3W, times_g, &D);
    if (F == 0.0) return g;
    if (F > 0.0) b = g; else a = g;
    double gn = (D > 0.0) ? g - F / D : 0.5 * (a + b);
    if (!(gn > a && gn < b)) gn = 0.5 * (a + b);   // Newton left the bracket: bisect
    bool done = (gn == g) || !(b - a > 0.0) ||
                std::fabs(gn - g) <= 1e-17 * std::max(1.0, std::fabs(g));
    g = gn;
    if (done) break;
  }
  return g;
}

double pool(const Problem& P, const double* s, int64_t lo, int64_t hi, double S, double W) {
  const double cnt = double(hi - lo);
  if (P.p == P_2) {
    if (P.phi != PHI_HALF_SQ) return (S - P.lambda * W) / cnt;
    return S / (P.lambda * W + cnt);
  }
  if (hi - lo == 1) {
    // singleton minimisers by direct solution
    if (P.phi != PHI_HALF_SQ) return s[lo] - P.lambda * std::cbrt(W);
    if (W == 0.0) return s[lo];
  }
  return cubic_root(s, lo, hi, P.lambda, W, P.phi == PHI_HALF_SQ);
}

// ---------------------------------------------------------------------------------------------
// App. "PAV algorithm".  Input: sorted s (descending), weights w (w = 1_k for the top-k
// operators; any non-increasing w works).  Output: v (the isotonic solution, piecewise constant
// on the blocks) and, for every position, the half-open range [blk_lo, blk_hi) of its block.
// A pair of adjacent blocks is merged iff gamma_left < gamma_right strictly.
struct Block {
  int64_t lo, hi;
  double S, W, gamma;
};

// The strict test  gamma_prev < gamma_top  of the PAV loop.  For p = 2 the pooled values are closed
// forms and are compared directly.  For p = 4/3 a pooled value is the root of a strictly increasing
// cubic F (the derivative of the block's strictly convex objective), so
//     gamma_prev < gamma_top  <=>  F_top(gamma_prev) < 0  <=>  F_prev(gamma_top) > 0,
// and when one side is a singleton with a closed-form minimiser the test is made through the other
// side's F at that exact value: an exact tie (F == 0) is then seen as a tie instead of being
// decided by the last bit of a root finder.
bool violates(const Problem& P, const double* s, const Block& prev, const Block& top) {
  if (P.p == P_2) return prev.gamma < top.gamma;
  const bool times_g = (P.phi == PHI_HALF_SQ);
  const double l3 = P.lambda * P.lambda * P.lambda;
  const bool prev_closed = (prev.hi - prev.lo == 1) && (!times_g || prev.W == 0.0);
  const bool top_closed = (top.hi - top.lo == 1) && (!times_g || top.W == 0.0);
  if (prev_closed && top_closed) return prev.gamma < top.gamma;   // two closed forms
  if (prev_closed) return cubic_F(s, top.lo, top.hi, prev.gamma, l3 * top.W, times_g, nullptr) < 0.0;
  if (top_closed) return cubic_F(s, prev.lo, prev.hi, top.gamma, l3 * prev.W, times_g, nullptr) > 0.0;
  return prev.gamma < top.gamma;
}

void pav(const Problem& P, const double* s, const double* w, int64_t n, double* v,
         int64_t* blk_lo, int64_t* blk_hi) {
  std::vector<Block> st;
  st.reserve(64);
  for (int64_t i = 0; i < n; ++i) {
    Block top{i, i + 1, s[i], w[i], 0.0};
    top.gamma = pool(P, s, top.lo, top.hi, top.S, top.W);
    while (!st.empty() && violates(P, s, st.back(), top)) {
      Block& prev = st.back();
      top.lo = prev.lo;
      top.S += prev.S;
      top.W += prev.W;
      st.pop_back();
      top.gamma = pool(P, s, top.lo, top.hi, top.S, top.W);
    }
    st.push_back(top);
  }
  for (const Block& B : st) {
    for (int64_t i = B.lo; i < B.hi; ++i) {
      v[i] = B.gamma;
      blk_lo[i] = B.lo;
      blk_hi[i] = B.hi;
    }
  }
}

// grad r*(t) and its derivative, restricted to what the two exponents need.
inline double grad_rstar(const Problem& P, double t) {
  if (P.p == P_2) return t / P.lambda;
  double l3 = P.lambda * P.lambda * P.lambda;
  return t * t * t / l3;
}
inline double hess_rstar(const Problem& P, double t) {
  if (P.p == P_2) return 1.0 / P.lambda;
  double l3 = P.lambda * P.lambda * P.lambda;
  return 3.0 * t * t / l3;
}

// ---------------------------------------------------------------------------------------------
// One row of the relaxed operator (Prop. 2 + Prop. 5 / Prop. 6) and its JVP (Prop. 7).
//   x        : the row (theta for the mask, the weights for top-k in magnitude)
//   tangent  : direction for the JVP, or nullptr
//   out, jvp : float64 results in the ORIGINAL order
//   perm     : the sorting permutation (0-based), or nullptr
//   ab       : ab[0], ab[1] = 0-based half-open range of the one block with more than one
//              element (lo == hi when every block is a singleton), or nullptr
//   value    : f_{phi,R}(x, 1_k) itself (Prop. 2, second line: min_u R*(x - u) + f_phi(u, 1_k),
//              evaluated at u*, i.e. the optimal value of Eq. (isotonic_separable)), or nullptr
//   weights  : nullptr for w = 1_k, else n non-increasing weights (w_1 >= ... >= w_n), the
//              general second argument of the operators of Sec. 4 (k is then ignored)
template <class T>
void one_row(const Problem& P, const T* x, const T* tangent, int64_t n, int64_t k,
             double* out, double* jvp, int32_t* perm, int64_t* ab, double* value = nullptr,
             const double* weights = nullptr) {
  std::vector<int32_t> sigma(n);
  std::vector<T> z(n);
  std::vector<double> s(n), w(n), v(n), sgn(n);
  std::vector<int64_t> blo(n), bhi(n);

  const bool mag = (P.phi == PHI_HALF_SQ);   // quadratic phi: pooling steps with the w v^2/2 term
  const bool even = (P.phi != PHI_ID);       // even phi: Prop. 6 (sort |x|, sign, v >= 0)
  for (int64_t i = 0; i < n; ++i) z[i] = even ? std::fabs(x[i]) : x[i];
  argsort_desc(z.data(), n, sigma.data());
  for (int64_t i = 0; i < n; ++i) {
    s[i] = double(z[sigma[i]]);
    w[i] = weights ? weights[i] : ((i < k) ? 1.0 : 0.0);   // w = 1_k, Eq. (topk_mask)
    double xv = double(x[sigma[i]]);
    sgn[i] = even ? double((xv > 0.0) - (xv < 0.0)) : 1.0;   // sign(0) = 0
  }
  pav(P, s.data(), w.data(), n, v.data(), blo.data(), bhi.data());
  std::vector<char> clipped(n, 0);
  if (even) {
    // Prop. 6: non-negative monotone cone, handled by truncation of the unconstrained solution.
    for (int64_t i = 0; i < n; ++i) {
      clipped[i] = v[i] < 0.0;
      v[i] = std::max(v[i], 0.0);
    }
  }
  // y* = grad R*(x - u*),  u* = sign(x) o v*_{sigma^-1}
  for (int64_t i = 0; i < n; ++i) out[sigma[i]] = sgn[i] * grad_rstar(P, s[i] - v[i]);
  if (value) {
    // sum_i r*(s_i - v_i) + w_i phi(v_i),  r*(t) = |t|^q / (q lambda^(q-1)),  q = 2 or 4
    const double q = (P.p == P_2) ? 2.0 : 4.0;
    const double lam_qm1 = (P.p == P_2) ? P.lambda : P.lambda * P.lambda * P.lambda;
    double f = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      const double t = std::fabs(s[i] - v[i]);
      f += std::pow(t, q) / (q * lam_qm1) + w[i] * (mag ? 0.5 * v[i] * v[i] : v[i]);
    }
    *value = f;
  }
  if (perm) std::memcpy(perm, sigma.data(), sizeof(int32_t) * size_t(n));
  if (ab) {
    ab[0] = ab[1] = 0;
    for (int64_t i = 0; i < n; ++i)
      if (bhi[i] - blo[i] > 1) { ab[0] = blo[i]; ab[1] = bhi[i]; break; }
  }
  if (!tangent || !jvp) return;

  // Prop. 7 with lambda restored.  tau = tangent in sorted coordinates (times sign for phi even).
  std::vector<double> tau(n);
  for (int64_t i = 0; i < n; ++i) tau[i] = sgn[i] * double(tangent[sigma[i]]);
  const double qm1 = (P.p == P_2) ? 1.0 : 3.0;                       // q - 1
  const double lam_qm1 = (P.p == P_2) ? P.lambda : P.lambda * P.lambda * P.lambda;
  int64_t i = 0;
  while (i < n) {
    const int64_t lo = blo[i], hi = bhi[i];
    const double g = v[lo];
    double dgamma;
    if (hi - lo == 1) {
      // singleton: differentiate the singleton minimiser directly
      if (!mag) {
        dgamma = tau[lo];                                   // gamma = s - lambda w^(1/(q-1))
      } else if (P.p == P_2) {
        dgamma = tau[lo] / (1.0 + P.lambda * w[lo]);        // gamma = s / (1 + lambda w)
      } else if (w[lo] == 0.0) {
        dgamma = tau[lo];                                   // gamma = s
      } else {
        double c = (g - s[lo]) * (g - s[lo]);
        dgamma = 3.0 * c * tau[lo] / (3.0 * c + lam_qm1 * w[lo]);
      }
    } else {
      double num = 0.0, den = 0.0;
      for (int64_t j = lo; j < hi; ++j) {
        double c = (P.p == P_2) ? 1.0 : (g - s[j]) * (g - s[j]);   // |gamma - s_j|^(q-2)
        if (!mag) {
          num += c * tau[j];
          den += c;
        } else {
          num += qm1 * c * tau[j];
          den += qm1 * c + lam_qm1 * w[j];
        }
      }
      dgamma = num / den;
    }
    for (int64_t j = lo; j < hi; ++j) {
      if (clipped[lo])   // v is pinned at 0 there: y = grad r*(x) itself (an odd function of x)
        jvp[sigma[j]] = hess_rstar(P, s[j]) * double(tangent[sigma[j]]);
      else
        jvp[sigma[j]] = sgn[j] * hess_rstar(P, s[j] - v[j]) * (tau[j] - dgamma);
    }
    i = hi;
  }
}

template <class T>
int run_rows(Phi phi, const T* x, const T* tangent, int64_t rows, int64_t n, int64_t k,
             int p_code, double lambda, double* out, double* jvp, int32_t* perm, int64_t* ab) {
  if (!x || !out) return -1;
  if (rows < 0 || n < 1 || k < 0 || k > n) return -2;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return -2;
  if (p_code != P_2 && p_code != P_4_3) return -3;
  Problem P{phi, Pcode(p_code), lambda};
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    one_row<T>(P, x + r * n, tangent ? tangent + r * n : nullptr, n, k, out + r * n,
            jvp ? jvp + r * n : nullptr, perm ? perm + r * n : nullptr, ab ? ab + 2 * r : nullptr);
  }
  return 0;
}

// Sec. 7 ("Advantage of the non-linearity"): the alternative top-k in magnitude that applies the
// relaxed top-k mask to |x| and multiplies the result by x,
//     y = x o m(|x|),      dy = t o m(|x|) + x o J_m(|x|) (sign(x) o t),   sign(0) = 0.
template <class T>
int run_masked_value(const T* x, const T* tangent, int64_t rows, int64_t n, int64_t k, int p_code,
                     double lambda, double* out, double* jvp) {
  if (!x || !out) return -1;
  if (rows < 0 || n < 1 || k < 0 || k > n) return -2;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return -2;
  if (p_code != P_2 && p_code != P_4_3) return -3;
  Problem P{PHI_ID, Pcode(p_code), lambda};
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    const T* xr = x + r * n;
    const T* tr = tangent ? tangent + r * n : nullptr;
    std::vector<T> z(n), st(n);
    std::vector<double> m(n), jm(n);
    for (int64_t i = 0; i < n; ++i) {
      z[i] = std::fabs(xr[i]);
      if (tr) st[i] = T((xr[i] > 0) - (xr[i] < 0)) * tr[i];
    }
    one_row<T>(P, z.data(), tr ? st.data() : nullptr, n, k, m.data(), tr ? jm.data() : nullptr,
               nullptr, nullptr);
    for (int64_t i = 0; i < n; ++i) {
      out[r * n + i] = double(xr[i]) * m[i];
      if (tr && jvp) jvp[r * n + i] = double(tr[i]) * m[i] + double(xr[i]) * jm[i];
    }
  }
  return 0;
}

// General non-increasing weights (see oracle_topk_general below).
template <class T>
int run_general(int phi_code, const T* x, const float* w, int64_t w_stride, const T* tangent,
                int64_t rows, int64_t n, int p_code, double lambda, double* out, double* jvp) {
  if (!x || !w || !out || rows < 0 || n < 1) return -1;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return -2;
  if (phi_code < 0 || phi_code > 1 || p_code < 0 || p_code > 1) return -3;
  if (w_stride != 0 && w_stride != n) return -1;
  Problem P{Phi(phi_code), Pcode(p_code), lambda};
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    std::vector<double> wd(n);
    for (int64_t i = 0; i < n; ++i) wd[i] = double(w[r * w_stride + i]);
    one_row<T>(P, x + r * n, tangent ? tangent + r * n : nullptr, n, 0, out + r * n,
               (tangent && jvp) ? jvp + r * n : nullptr, nullptr, nullptr, nullptr, wd.data());
  }
  return 0;
}
}  // namespace

extern "C" {

// Sec. 3: argsort (descending, ties by ascending index) of every row.  Host pointers.
int oracle_argsort_desc(const float* z, int64_t rows, int64_t n, int32_t* perm) {
  if (!z || !perm || rows < 0 || n < 1) return -1;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) argsort_desc(z + r * n, n, perm + r * n);
  return 0;
}

// Relaxed top-k mask (phi = identity).  tangent/jvp/perm/ab may be null.  p_code 0: p=2, 1: p=4/3.
int oracle_topk_mask(const float* theta, const float* tangent, int64_t rows, int64_t n, int64_t k,
                     int p_code, double lambda, double* out, double* jvp, int32_t* perm,
                     int64_t* ab) {
  return run_rows(PHI_ID, theta, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}

// Relaxed top-k in magnitude (phi = x^2/2).
int oracle_topkmag(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                   int p_code, double lambda, double* out, double* jvp, int32_t* perm,
                   int64_t* ab) {
  return run_rows(PHI_HALF_SQ, x, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}

// The same two operators on float64 inputs (used by the finite-difference pins of the JVP).
int oracle_topk_mask_f64(const double* theta, const double* tangent, int64_t rows, int64_t n,
                         int64_t k, int p_code, double lambda, double* out, double* jvp,
                         int32_t* perm, int64_t* ab) {
  return run_rows(PHI_ID, theta, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}
int oracle_topkmag_f64(const double* x, const double* tangent, int64_t rows, int64_t n, int64_t k,
                       int p_code, double lambda, double* out, double* jvp, int32_t* perm,
                       int64_t* ab) {
  return run_rows(PHI_HALF_SQ, x, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}

// Signed relaxed top-k mask (phi = |x|), float32 and float64 inputs.
int oracle_topk_signed_mask(const float* x, const float* tangent, int64_t rows, int64_t n,
                            int64_t k, int p_code, double lambda, double* out, double* jvp,
                            int32_t* perm, int64_t* ab) {
  return run_rows(PHI_ABS, x, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}
int oracle_topk_signed_mask_f64(const double* x, const double* tangent, int64_t rows, int64_t n,
                                int64_t k, int p_code, double lambda, double* out, double* jvp,
                                int32_t* perm, int64_t* ab) {
  return run_rows(PHI_ABS, x, tangent, rows, n, k, p_code, lambda, out, jvp, perm, ab);
}

// x o mask(|x|); perm and ab are not produced (always pass null).
int oracle_topk_masked_value(const float* x, const float* tangent, int64_t rows, int64_t n,
                             int64_t k, int p_code, double lambda, double* out, double* jvp,
                             int32_t*, int64_t*) {
  return run_masked_value(x, tangent, rows, n, k, p_code, lambda, out, jvp);
}
int oracle_topk_masked_value_f64(const double* x, const double* tangent, int64_t rows, int64_t n,
                                 int64_t k, int p_code, double lambda, double* out, double* jvp,
                                 int32_t*, int64_t*) {
  return run_masked_value(x, tangent, rows, n, k, p_code, lambda, out, jvp);
}

// The relaxed operator y_{phi,R}(x, w) of Prop. 2 for a general non-increasing w (soft rank:
// w = (n, .., 1) on -theta; soft sort: input (n, .., 1), w = sort(theta); partial ranks; Sec. 3
// "LP formulations" and Sec. 4) and its JVP in x.  w: [n] shared by all rows (w_stride = 0) or
// [rows][n] (w_stride = n), float32 like the library's input, widened exactly.  phi_code 0 / 1.
int oracle_topk_general(int phi_code, const float* x, const float* w, int64_t w_stride,
                        const float* tangent, int64_t rows, int64_t n, int p_code, double lambda,
                        double* out, double* jvp) {
  return run_general(phi_code, x, w, w_stride, tangent, rows, n, p_code, lambda, out, jvp);
}
int oracle_topk_general_f64(int phi_code, const double* x, const float* w, int64_t w_stride,
                            const double* tangent, int64_t rows, int64_t n, int p_code,
                            double lambda, double* out, double* jvp) {
  return run_general(phi_code, x, w, w_stride, tangent, rows, n, p_code, lambda, out, jvp);
}

// Sec. 5, Alg. 1: Dykstra's alternating projections for the relaxed top-k mask with p = 2, as an
// approximation with a fixed number of iterations.  Sorted row s, w = 1_k; the problem is the
// Euclidean projection of s - lambda w onto C1 n C2, so the linear term is applied once, to the
// starting point (the listing prints it inside both argmins, which would count it twice).
//   v^0 = s - lambda w,  p^0 = q^0 = 0
//   y^t = P_C1(v^t + p^t),  p^{t+1} = v^t + p^t - y^t,
//   v^{t+1} = P_C2(y^t + q^t),  q^{t+1} = y^t + q^t - v^{t+1}
// P_C1 / P_C2: every pair (1,2),(3,4),.. / (2,3),(4,5),.. that violates z_i >= z_{i+1} is replaced
// by its mean.  Output y = (s - v^iters) / lambda in the original order.
int oracle_topk_mask_dykstra(const float* theta, int64_t rows, int64_t n, int64_t k, double lambda,
                             int64_t iters, double* out) {
  if (!theta || !out || rows < 0 || n < 1 || k < 0 || k > n || iters < 0) return -1;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    const float* x = theta + r * n;
    std::vector<int32_t> sigma(n);
    argsort_desc(x, n, sigma.data());
    std::vector<double> s(n), v(n), p(n, 0.0), q(n, 0.0), z(n), y(n);
    for (int64_t i = 0; i < n; ++i) {
      s[i] = double(x[sigma[i]]);
      v[i] = s[i] - lambda * (i < k ? 1.0 : 0.0);
    }
    auto project = [&](const std::vector<double>& in, std::vector<double>& res, int64_t first) {
      res = in;
      for (int64_t i = first; i + 1 < n; i += 2)
        if (in[i] < in[i + 1]) res[i] = res[i + 1] = 0.5 * (in[i] + in[i + 1]);
    };
    for (int64_t t = 0; t < iters; ++t) {
      for (int64_t i = 0; i < n; ++i) z[i] = v[i] + p[i];
      project(z, y, 0);
      for (int64_t i = 0; i < n; ++i) p[i] = z[i] - y[i];
      for (int64_t i = 0; i < n; ++i) z[i] = y[i] + q[i];
      project(z, v, 1);
      for (int64_t i = 0; i < n; ++i) q[i] = z[i] - v[i];
    }
    for (int64_t i = 0; i < n; ++i) out[r * n + sigma[i]] = (s[i] - v[i]) / lambda;
  }
  return 0;
}

// f_{phi,R}(x, 1_k) of every row (Prop. 2), the function whose gradient in x the operators are;
// the Fenchel-Young top-k loss of Sec. 6 ("Smooth top-k loss") is value - <x, t>.
int oracle_topk_value(int phi_code, const double* x, int64_t rows, int64_t n, int64_t k, int p_code,
                      double lambda, double* value) {
  if (!x || !value || rows < 0 || n < 1 || k < 0 || k > n) return -1;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return -2;
  if (phi_code < 0 || phi_code > 2 || p_code < 0 || p_code > 1) return -3;
  Problem P{Phi(phi_code), Pcode(p_code), lambda};
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < rows; ++r) {
    std::vector<double> out(n);
    one_row<double>(P, x + r * n, nullptr, n, k, out.data(), nullptr, nullptr, nullptr, value + r);
  }
  return 0;
}

// The isotonic solver alone, for any weights w (sorted s, float64):
//   v = argmin_{v1>=...>=vn} sum_i r*(s_i - v_i) + w_i phi(v_i).
// block_id[i] = index of the first element of the block containing i.
int oracle_pav(const double* s, const double* w, int64_t n, int phi_code, int p_code,
               double lambda, double* v, int64_t* block_id) {
  if (!s || !w || !v || n < 1 || !(lambda > 0.0)) return -1;
  if (phi_code < 0 || phi_code > 2 || p_code < 0 || p_code > 1) return -3;
  Problem P{Phi(phi_code), Pcode(p_code), lambda};
  std::vector<int64_t> lo(n), hi(n);
  pav(P, s, w, n, v, lo.data(), hi.data());
  if (block_id) std::copy(lo.begin(), lo.end(), block_id);
  return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int t) {
#ifdef _OPENMP
  if (t > 0) omp_set_num_threads(t);
#else
  (void)t;
#endif
}

}  // extern "C"
