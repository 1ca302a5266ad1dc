// Pieces of the general-weights solve (Sec. 4 with a general non-increasing w; App. "PAV
// algorithm") shared by the kernel of short rows and the kernel of long rows: the pooled value of
// a block from its sums, the strict violation test between neighbouring blocks, and the
// sequential left-to-right block stack that both kernels hand over to when the merging rounds do
// not settle.
#pragma once

#include "common.hpp"
#include "pooling.hpp"

namespace topk {

// the increasing cubic of a block: sum_B (g - s_i)^3 + lambda^3 W [g] (magnitude: times g).
// shift: the sums are those of s_i - shift and g stands for gamma - shift (matters for the
// magnitude form only, whose last term is lambda^3 W gamma).
template <bool MAG>
__device__ __forceinline__ double block_cubic(double g, double cnt, double W, double S1, double S2,
                                              double S3, const Reg& R, double shift = 0.0) {
  const double lin = MAG ? R.lam3 * W * (g + shift) : R.lam3 * W;
  return ((cnt * g - 3.0 * S1) * g + 3.0 * S2) * g - S3 + lin;
}

// root of the block's cubic inside [lo, hi] (safeguarded Newton; the cubic is increasing)
template <bool MAG>
__device__ double block_root(double cnt, double W, double S1, double S2, double S3, const Reg& R,
                             double lo, double hi, double shift = 0.0) {
  double a = lo, b = hi;
  // start: the root the cubic would have with every s_i at the block's mean
  const double mean = S1 / cnt;
  double x = mean - R.lambda * cbrt(MAG ? W * fmax(mean + shift, 0.0) / cnt : W / cnt);
  if (!(x > a && x < b)) x = 0.5 * (a + b);
  const double scale = fmax(fmax(fabs(a), fabs(b)), R.lambda);
  const double tol = 1e-15 * scale;
  double last = 1e300;
  for (int it = 0; it < 200; ++it) {
    const double F = block_cubic<MAG>(x, cnt, W, S1, S2, S3, R, shift);
    if (F == 0.0) return x;
    if (F > 0.0) b = x; else a = x;
    const double D = (3.0 * cnt * x - 6.0 * S1) * x + 3.0 * S2 + (MAG ? R.lam3 * W : 0.0);
    const double dx = F / D;
    // a step of rounding size ends the iteration before the bracket test: at the root the
    // bracket end is x itself, and bisecting from there would throw the converged value away.
    // Small steps that have stopped shrinking are the rounding noise of the expanded cubic (the
    // block's values lie close together compared with their size): nothing more to gain.
    const double adx = fabs(dx);
    if (adx <= tol || (adx < 1e-7 * scale && adx >= 0.25 * last)) return x - dx;
    last = adx;
    double xn = x - dx;
    if (!(xn > a && xn < b)) xn = 0.5 * (a + b);
    x = xn;
  }
  return x;
}

// Singleton minimiser of the magnitude operator with p = 4/3 and weight W > 0: the root g in
// [0, s] of (g - s)^3 + lambda^3 W g = 0 (App. "Subproblem derivation", one element), evaluated in
// this form: the expanded cubic of block_root loses the small difference g - s.
__device__ double singleton_root_mag(double s, double W, const Reg& R) {
  if (!(s > 0.0)) return 0.0;
  const double L = R.lam3 * W;
  double a = 0.0, b = s;
  double g = s - cbrt(L * s);                  // large-s asymptote
  if (!(g > a && g < b)) g = 0.5 * s;
  const double tol = 1e-8 * s;                 // Newton converges quadratically: the step after
  for (int it = 0; it < 64; ++it) {            // one below tol lands within rounding of the root
    const double u = g - s;
    const double F = u * u * u + L * g;
    if (F == 0.0) return g;
    if (F > 0.0) b = g; else a = g;
    const double dg = F / (3.0 * u * u + L);
    if (fabs(dg) <= tol) { g -= dg; break; }
    double gn = g - dg;
    if (!(gn > a && gn < b)) gn = 0.5 * (a + b);
    g = gn;
  }
  const double u = g - s;
  return g - (u * u * u + L * g) / (3.0 * u * u + L);
}

struct Blk {
  double cnt, W, S1, S2, S3;
};

// pooled value of a block (App. "Subproblem derivation"); smax, smin: its largest / smallest value
template <bool MAG, bool CUBIC>
__device__ __forceinline__ double block_gamma(const Blk& b, double smax, double smin, const Reg& R) {
  if (!CUBIC)
    return MAG ? __ddiv_rn(b.S1, __dadd_rn(__dmul_rn(R.lambda, b.W), b.cnt))
               : __ddiv_rn(__dsub_rn(b.S1, __dmul_rn(R.lambda, b.W)), b.cnt);
  if (b.cnt == 1.0) {
    if (!MAG) return smax - R.lambda * cbrt(b.W);
    return (b.W == 0.0) ? smax : singleton_root_mag(smax, b.W, R);
  }
  return MAG ? block_root<true>(b.cnt, b.W, b.S1, b.S2, b.S3, R, 0.0, smax)
             : block_root<false>(b.cnt, b.W, b.S1, b.S2, b.S3, R,
                                 smin - R.lambda * cbrt(b.W) - 1e-300, smax);
}

// strict violation between the block `p` (pooled value gp) and the block `t` to its right (gt):
// gamma_p < gamma_t.  For p = 4/3 a singleton with a closed-form minimiser is compared through the
// other block's cubic (its sign at that value), as exact as the closed form itself.
template <bool MAG, bool CUBIC>
__device__ __forceinline__ bool blocks_violate(const Blk& p, double gp, const Blk& t, double gt,
                                               const Reg& R) {
  if (!CUBIC) return gp < gt;
  const bool p_closed = (p.cnt == 1.0) && (!MAG || p.W == 0.0);
  const bool t_closed = (t.cnt == 1.0) && (!MAG || t.W == 0.0);
  if (p_closed == t_closed) return gp < gt;
  if (p_closed) return block_cubic<MAG>(gp, t.cnt, t.W, t.S1, t.S2, t.S3, R) < 0.0;
  return block_cubic<MAG>(gt, p.cnt, p.W, p.S1, p.S2, p.S3, R) > 0.0;
}

// The sequential algorithm: one thread walks the sorted row left to right with the block stack
// (columns st_*, slot -> block start in st_lo; the block on top of the stack is kept in
// registers).  ss: sorted values, lw: weights by sorted position, ltau: tangent in sorted
// coordinates (read only when want_jvp).  On return, for every block start lo: st_g[lo] = pooled
// value, DG[lo] = d gamma (Prop. 7), st_lo[lo] = head_mark, and no other entry of st_lo[0, n) has
// that value (stack slots hold starts, which are smaller).  DG may be st_s1.
template <bool MAG, bool CUBIC, typename IdxT>
__device__ void stack_walk(int n, const float* ss, const float* lw, const float* ltau,
                           bool want_jvp, double* st_s1, double* st_w, double* st_g,
                           double* st_s2, double* st_s3, IdxT* st_lo, IdxT head_mark, double* DG,
                           const Reg& R) {
  int top = 0;                           // blocks in LDS below the register-held top
  bool have = false;
  int tlo = 0;
  double tS1 = 0.0, tW = 0.0, tS2 = 0.0, tS3 = 0.0, tg = 0.0;
  float s_next = ss[0], w_next = lw[0];
  for (int i = 0; i < n; ++i) {
    const double si = double(s_next), wi = double(w_next);
    if (i + 1 < n) { s_next = ss[i + 1]; w_next = lw[i + 1]; }
    int lo = i;
    Blk cur{1.0, wi, si, 0.0, 0.0};
    if (CUBIC) { cur.S2 = si * si; cur.S3 = cur.S2 * si; }
    double g = block_gamma<MAG, CUBIC>(cur, si, si, R);
    while (have) {
      const Blk prev{double(lo - tlo), tW, tS1, tS2, tS3};
      if (!blocks_violate<MAG, CUBIC>(prev, tg, cur, g, R)) break;
      // merge the previous block into the current one
      cur.S1 = __dadd_rn(cur.S1, tS1);
      cur.W = __dadd_rn(cur.W, tW);
      if (CUBIC) { cur.S2 += tS2; cur.S3 += tS3; }
      lo = tlo;
      cur.cnt = double(i + 1 - lo);
      // the block below becomes the top
      have = top > 0;
      if (have) {
        --top;
        tlo = st_lo[top]; tS1 = st_s1[top]; tW = st_w[top]; tg = st_g[top];
        if (CUBIC) { tS2 = st_s2[top]; tS3 = st_s3[top]; }
      }
      g = block_gamma<MAG, CUBIC>(cur, double(ss[lo]), si, R);
    }
    if (have) {                          // spill the old top below the new one
      st_lo[top] = IdxT(tlo); st_s1[top] = tS1; st_w[top] = tW; st_g[top] = tg;
      if (CUBIC) { st_s2[top] = tS2; st_s3[top] = tS3; }
      ++top;
    }
    have = true;
    tlo = lo; tS1 = cur.S1; tW = cur.W; tS2 = cur.S2; tS3 = cur.S3; tg = g;
  }
  if (have) {
    st_lo[top] = IdxT(tlo); st_s1[top] = tS1; st_w[top] = tW; st_g[top] = tg;
    if (CUBIC) { st_s2[top] = tS2; st_s3[top] = tS3; }
    ++top;
  }
  // Prop. 7 per block; then everything moves from the stack slot to the block's start (marked
  // in st_lo).  Slots are visited from the top and start >= slot, so nothing that is still to be
  // read gets overwritten.
  int hi = n;
  for (int bk = top - 1; bk >= 0; --bk) {
    const int lo = st_lo[bk];
    const double g = st_g[bk], W = st_w[bk];
    double dg = 0.0;
    if (want_jvp) {
      if (hi - lo == 1) {
        const double tau = double(ltau[lo]);
        if (!MAG) dg = tau;
        else if (!CUBIC) dg = tau / (1.0 + R.lambda * W);
        else if (W == 0.0) dg = tau;
        else {
          const double c = (g - double(ss[lo])) * (g - double(ss[lo]));
          dg = 3.0 * c * tau / (3.0 * c + R.lam3 * W);
        }
      } else {
        double num = 0.0, den = 0.0;
        for (int j = lo; j < hi; ++j) {
          const double d = g - double(ss[j]);
          const double c = CUBIC ? d * d : 1.0;
          const double q = (MAG && CUBIC) ? 3.0 * c : c;
          num += q * double(ltau[j]);
          den += q;
        }
        if (MAG) den += (CUBIC ? R.lam3 : R.lambda) * W;
        dg = num / den;
      }
    }
    st_lo[bk] = 0;
    st_g[lo] = g;
    DG[lo] = dg;
    st_lo[lo] = head_mark;
    hi = lo;
  }
}

}  // namespace topk
