// Pooling arithmetic of the isotonic solve, float64, shared by the short-row and long-row kernels.
//
// With w = 1_k the singleton minimisers of h_i(v) = r*(s_i - v) + w_i phi(v) form two
// non-increasing runs (positions <= k, positions > k), so pool-adjacent-violators can only ever
// grow ONE block [a, b] with a <= k < b, starting from the pair (k, k+1).  The kernels grow that
// block with two monotone predicates, each the exact strict-violation test of the PAV loop
// (paper App. "PAV algorithm") between a singleton and the block next to it:
//
//   right_violates(x = s_j, block [a, j-1]):  gamma_block < s_j            (j > k, w_j = 0)
//   left_violates (x = s_i, block [i+1, b]):  gamma_{i} < gamma_block      (i <= k, w_i = 1)
//
// A block is described by cnt = |B|, m = number of its positions <= k (= sum of w over B) and the
// power sums S1 = sum s, S2 = sum s^2, S3 = sum s^3 over B (S2, S3 only for p = 4/3).
//
// Pooled values (paper Sec. 5 "Example", App. "Subproblem derivation"), with lambda restored:
//   mask, p = 2   : gamma = (S1 - lambda m) / cnt
//   mask, p = 4/3 : root of  F(g) = sum_B (g - s_i)^3 + lambda^3 m
//                              = cnt g^3 - 3 g^2 S1 + 3 g S2 - S3 + lambda^3 m     (increasing in g)
//   mag,  p = 2   : gamma = S1 / (cnt + lambda m)
//   mag,  p = 4/3 : root of  G(g) = sum_B (g - s_i)^3 + lambda^3 m g               (increasing in g)
// Comparisons against a pooled value are made without dividing / without finding the root:
// gamma < x  <=>  F(x) > 0, and for p = 2 by cross-multiplying with the positive denominator.
//
// The mask problem is invariant under a common shift of s and gamma, so its callers pass values
// centred on s_k (all magnitudes below lambda inside the window that can pool), which keeps the
// expanded cubic well conditioned.
#pragma once

#include "common.hpp"

namespace topk {

struct Sums {
  double s1, s2, s3;
};

struct Reg {           // regulariser constants, computed once on the host in float64
  double lambda;       // lambda
  double inv_lambda;   // 1 / lambda
  double lam3;         // lambda^3
  double inv_lam3;     // 1 / lambda^3
  double one_p_lambda; // 1 + lambda
  double inv_1pl;      // 1 / (1 + lambda)
};

// reciprocal of a positive float64 to full precision: hardware estimate + two Newton steps
__device__ __forceinline__ double recip(double c) {
  double r = __builtin_amdgcn_rcp(c);
  r = fma(fma(-c, r, 1.0), r, r);
  r = fma(fma(-c, r, 1.0), r, r);
  return r;
}

// Singleton minimiser of a top-k position of the magnitude operator with p = 4/3: the root g in
// [0, s] of (g - s)^3 + lambda^3 g = 0  (App. "Subproblem derivation", one element, w = 1;
// increasing in g, so safeguarded Newton from the large-s asymptote g = s - lambda s^(1/3)).
__device__ __forceinline__ double singleton_root_mag43(double s, const Reg& R) {
  if (!(s > 0.0)) return 0.0;
  double a = 0.0, b = s;
  double g = s - R.lambda * double(cbrtf(float(s)));
  if (!(g > a && g < b)) g = 0.5 * s;
  // Newton converges quadratically: once a step is below 1e-8 s, the next one lands within
  // rounding of the root (a tolerance at rounding level would never be met reliably)
  const double tol = 1e-8 * s;
  for (int it = 0; it < 64; ++it) {
    const double u = g - s;
    const double F = u * u * u + R.lam3 * g;
    if (F == 0.0) return g;
    if (F > 0.0) b = g; else a = g;
    const double dg = F * recip(3.0 * u * u + R.lam3);
    // a step of rounding size ends the iteration BEFORE the bracket test: at the root the bracket
    // end is g itself, g - dg == g is then "outside", and the bisection that followed threw the
    // converged value away (some forty more iterations to come back)
    if (fabs(dg) <= tol) { g -= dg; break; }
    double gn = g - dg;
    if (!(gn > a && gn < b)) gn = 0.5 * (a + b);
    g = gn;
  }
  const double u = g - s;
  return g - (u * u * u + R.lam3 * g) * recip(3.0 * u * u + R.lam3);
}

// Value arguments of Pool are relative to `center` (s_k) when kCentered, else absolute with
// center = 0.  The mask is shift invariant, so its formulas never see the centre; the magnitude
// operator with p = 4/3 is not (its cubic has the term lambda^3 m gamma), so its formulas add
// the centre back where the absolute value matters.
template <bool MAG, int PC>
struct Pool {
  static constexpr bool kCubic = (PC == kP43);
  static constexpr bool kCentered = !MAG || kCubic;

  // mask:      F(x) = sum_B (x - s_i)^3 + lambda^3 m
  // magnitude: G(x) = sum_B (x - s_i)^3 + lambda^3 m x_abs,   both increasing in x
  __device__ static __forceinline__ double cubic(double x, double cnt, double m, const Sums& S,
                                                 const Reg& R, double center = 0.0) {
    const double lin = MAG ? R.lam3 * m * (x + center) : R.lam3 * m;
    return ((cnt * x - 3.0 * S.s1) * x + 3.0 * S.s2) * x - S.s3 + lin;
  }

  // is the singleton x = s_j (j > k) strictly above the pooled value of the block to its left?
  __device__ static __forceinline__ bool right_violates(double x, double cnt, double m,
                                                        const Sums& S, const Reg& R,
                                                        double center = 0.0) {
    if (kCubic) return cubic(x, cnt, m, S, R, center) > 0.0;
    if (MAG) return x * (cnt + R.lambda * m) > S.s1;
    return x * cnt > S.s1 - R.lambda * m;
  }

  // is the singleton minimiser of s_i = x (i <= k) strictly below the pooled value of the block
  // to its right?
  __device__ static __forceinline__ bool left_violates(double x, double cnt, double m,
                                                       const Sums& S, const Reg& R,
                                                       double center = 0.0) {
    if (kCubic) {
      const double g = MAG ? singleton_root_mag43(x + center, R) - center : x - R.lambda;
      return cubic(g, cnt, m, S, R, center) < 0.0;
    }
    if (MAG) return x * (cnt + R.lambda * m) < S.s1 * R.one_p_lambda;
    return (x - R.lambda) * cnt < S.s1 - R.lambda * m;
  }

  // does the pair (k, k+1) violate at all?  sk, sk1 = s_k, s_{k+1}
  __device__ static __forceinline__ bool seed_violates(double sk, double sk1, const Reg& R,
                                                       double center = 0.0) {
    if (MAG && kCubic) {                       // singleton root of s_k below s_{k+1}
      const double u = sk1 - sk;
      return u * u * u + R.lam3 * (sk1 + center) > 0.0;
    }
    if (MAG) return sk < sk1 * R.one_p_lambda;
    return sk - R.lambda < sk1;
  }

  // Necessary conditions for a position to be able to join the block (they define the value
  // window outside of which nothing can pool).
  __device__ static __forceinline__ bool left_candidate(double x, double sk1, const Reg& R,
                                                        double center = 0.0) {
    if (MAG && kCubic) {
      const double u = sk1 - x;
      return u * u * u + R.lam3 * (sk1 + center) > 0.0;
    }
    if (MAG) return x < sk1 * R.one_p_lambda;
    return x - R.lambda < sk1;
  }
  __device__ static __forceinline__ bool right_candidate(double x, double sk, const Reg& R,
                                                         double center = 0.0) {
    if (MAG && kCubic) {
      const double u = x - sk;
      return u * u * u + R.lam3 * (x + center) > 0.0;
    }
    if (MAG) return x * R.one_p_lambda > sk;
    return x > sk - R.lambda;
  }

  // pooled value of the final block; lo < gamma < hi is known (used to safeguard Newton for the
  // cubic; callers pass lo = singleton minimiser of position a or a lower bound of it, hi = s_b
  // or an upper bound).
  __device__ static __forceinline__ double pooled(double cnt, double m, const Sums& S,
                                                  const Reg& R, double lo, double hi,
                                                  double center = 0.0) {
    if (!kCubic) return MAG ? S.s1 / (cnt + R.lambda * m) : (S.s1 - R.lambda * m) / cnt;
    // Safeguarded Newton.  Inside the block all |s_i| <= ~lambda (centred values), so lambda is
    // the scale of gamma; steps below 1e-13 lambda are rounding noise of the expanded cubic
    // (the outputs need gamma to ~1e-7 lambda only).
    double a = lo, b = hi;
    // start from the root the cubic would have if all s_i sat at their mean:
    // cnt (x - mean)^3 = -lambda^3 m  (float32 cube root: it is only a starting point)
    const double rc = recip(cnt);
    const double scale = MAG ? m * rc * (S.s1 * rc + center) : m * rc;
    double x = S.s1 * rc - R.lambda * double(cbrtf(float(scale)));
    if (!(x > a && x < b)) x = 0.5 * (a + b);
    const double tol = 1e-13 * R.lambda;
    for (int it = 0; it < 64; ++it) {
      const double F = cubic(x, cnt, m, S, R, center);
      if (F == 0.0) break;
      if (F > 0.0) b = x; else a = x;
      const double D = (3.0 * cnt * x - 6.0 * S.s1) * x + 3.0 * S.s2 + (MAG ? R.lam3 * m : 0.0);
      const double dx = F * recip(D);
      // (a step of rounding size ends the iteration before the bracket test, see above)
      if (fabs(dx) <= tol) { x -= dx; break; }
      double xn = x - dx;
      if (!(xn > a && xn < b)) xn = 0.5 * (a + b);   // also catches D <= 0 (inf / nan)
      x = xn;
    }
    return x;
  }

  // y in sorted coordinates for a position inside the block: grad r*(s - gamma)
  __device__ static __forceinline__ double y_in_block(double x, double gamma, const Reg& R) {
    double t = (x - gamma) * R.inv_lambda;
    return kCubic ? t * t * t : t;
  }
  // second derivative of r* at s - gamma
  __device__ static __forceinline__ double hess(double x, double gamma, const Reg& R) {
    if (!kCubic) return R.inv_lambda;
    double t = x - gamma;
    return 3.0 * t * t * R.inv_lam3;
  }
  // Prop. 7 weight (q-1) |gamma - s_j|^(q-2) of position j in d gamma / d s_j (the factor q-1
  // cancels for the mask and is dropped there)
  __device__ static __forceinline__ double jac_weight(double x, double gamma) {
    if (!kCubic) return 1.0;
    double t = gamma - x;
    return MAG ? 3.0 * t * t : t * t;
  }
  // denominator of d gamma: sum of the weights (+ lambda^(q-1) m for phi = x^2/2)
  __device__ static __forceinline__ double jac_denominator(double wsum, double m, const Reg& R) {
    if (MAG) return wsum + (kCubic ? R.lam3 : R.lambda) * m;
    return wsum;
  }

  // y of a top-k position before the block (its own singleton solution), and d y / d tau there
  __device__ static __forceinline__ double above(double x, const Reg& R, double center = 0.0) {
    if (!MAG) return 1.0;
    if (!kCubic) return x * R.inv_1pl;
    return singleton_root_mag43(x + center, R);      // y = (s - g)^3 / lambda^3 = g
  }
  __device__ static __forceinline__ double above_slope(double x, const Reg& R, double center = 0.0) {
    if (!MAG) return 0.0;
    if (!kCubic) return R.inv_1pl;
    const double s = x + center;
    const double u = singleton_root_mag43(s, R) - s;
    return 3.0 * u * u / (3.0 * u * u + R.lam3);
  }
  // both at once (one root for the magnitude operator with p = 4/3)
  __device__ static __forceinline__ void above_both(double x, const Reg& R, double center,
                                                    double* y, double* slope) {
    if (MAG && kCubic) {
      const double s = x + center;
      const double g = singleton_root_mag43(s, R);
      const double u = g - s;
      *y = g;
      *slope = 3.0 * u * u / (3.0 * u * u + R.lam3);
    } else {
      *y = above(x, R, center);
      *slope = above_slope(x, R, center);
    }
  }
};

}  // namespace topk
