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

template <bool MAG, int PC>
struct Pool {
  static constexpr bool kCubic = (PC == kP43);

  __device__ static __forceinline__ double cubic(double x, double cnt, double m, const Sums& S,
                                                 const Reg& R) {
    return ((cnt * x - 3.0 * S.s1) * x + 3.0 * S.s2) * x - S.s3 + R.lam3 * m;
  }

  // is the singleton x = s_j (j > k) strictly above the pooled value of the block to its left?
  __device__ static __forceinline__ bool right_violates(double x, double cnt, double m,
                                                        const Sums& S, const Reg& R) {
    if (MAG) return x * (cnt + R.lambda * m) > S.s1;
    if (kCubic) return cubic(x, cnt, m, S, R) > 0.0;
    return x * cnt > S.s1 - R.lambda * m;
  }

  // is the singleton minimiser of s_i = x (i <= k) strictly below the pooled value of the block
  // to its right?
  __device__ static __forceinline__ bool left_violates(double x, double cnt, double m,
                                                       const Sums& S, const Reg& R) {
    if (MAG) return x * (cnt + R.lambda * m) < S.s1 * R.one_p_lambda;
    if (kCubic) return cubic(x - R.lambda, cnt, m, S, R) < 0.0;
    return (x - R.lambda) * cnt < S.s1 - R.lambda * m;
  }

  // does the pair (k, k+1) violate at all?  sk, sk1 = s_k, s_{k+1}
  __device__ static __forceinline__ bool seed_violates(double sk, double sk1, const Reg& R) {
    if (MAG) return sk < sk1 * R.one_p_lambda;
    return sk - R.lambda < sk1;
  }

  // Necessary conditions for a position to be able to join the block (used to zero everything
  // else before prefix sums, so that far-away large values cannot cancel into the block sums).
  __device__ static __forceinline__ bool left_candidate(double x, double sk1, const Reg& R) {
    if (MAG) return x < sk1 * R.one_p_lambda;
    return x - R.lambda < sk1;
  }
  __device__ static __forceinline__ bool right_candidate(double x, double sk, const Reg& R) {
    if (MAG) return x * R.one_p_lambda > sk;
    return x > sk - R.lambda;
  }

  // pooled value of the final block; lo < gamma < hi is known (lo = singleton minimiser of
  // position a, hi = s_b), used to safeguard Newton for the cubic.
  __device__ static __forceinline__ double pooled(double cnt, double m, const Sums& S,
                                                  const Reg& R, double lo, double hi) {
    if (MAG) return S.s1 / (cnt + R.lambda * m);
    if (!kCubic) return (S.s1 - R.lambda * m) / cnt;
    // Safeguarded Newton.  Inside the block all |s_i| <= ~lambda (centred values), so lambda is
    // the scale of gamma; steps below 1e-13 lambda are rounding noise of the expanded cubic
    // (the outputs need gamma to ~1e-7 lambda only).
    double a = lo, b = hi;
    // start from the root the cubic would have if all s_i sat at their mean:
    // cnt (x - mean)^3 = -lambda^3 m  (float32 cube root: it is only a starting point)
    const double rc = recip(cnt);
    double x = S.s1 * rc - R.lambda * double(cbrtf(float(m * rc)));
    if (!(x > a && x < b)) x = 0.5 * (a + b);
    const double tol = 1e-13 * R.lambda;
    for (int it = 0; it < 64; ++it) {
      const double F = cubic(x, cnt, m, S, R);
      if (F == 0.0) break;
      if (F > 0.0) b = x; else a = x;
      const double D = (3.0 * cnt * x - 6.0 * S.s1) * x + 3.0 * S.s2;
      double xn = x - F * recip(D);
      if (!(xn > a && xn < b)) xn = 0.5 * (a + b);   // also catches D <= 0 (inf / nan)
      const double step = fabs(xn - x);
      x = xn;
      if (step <= tol) break;
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
  // Prop. 7 weight |gamma - s_j|^(q-2) of position j in d gamma / d s_j
  __device__ static __forceinline__ double jac_weight(double x, double gamma) {
    if (!kCubic) return 1.0;
    double t = gamma - x;
    return t * t;
  }
  // denominator of d gamma: sum of the weights (+ lambda^(q-1) m for phi = x^2/2, p = 2)
  __device__ static __forceinline__ double jac_denominator(double wsum, double m, const Reg& R) {
    if (MAG) return wsum + R.lambda * m;
    return wsum;
  }
};

}  // namespace topk
