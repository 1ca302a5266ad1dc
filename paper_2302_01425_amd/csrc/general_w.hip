// The relaxed operators y_{phi,R}(x, w) for a GENERAL non-increasing weight vector w (Sec. 4;
// soft rank, soft sort and partial ranks through the LP forms of Sec. 3), rows up to 1024 elements.
//
// With w = 1_k one pooled block suffices and the other kernels exploit that.  For a general w the
// partition of pool-adjacent-violators (App. "PAV algorithm") can have any number of blocks, so
// after the same register sort the partition is built by the usual left-to-right block stack:
// one lane per row runs it (the rows of a wavefront run side by side in different lanes), all the
// per-row state lives in LDS.  Every merge is decided by the strict test gamma_prev < gamma_top;
// block sums are accumulated on the stack in merge order, and the p = 2 pooled values are computed
// without fused multiply-adds, so exact ties are seen as ties.  A second stack walk gives each
// block's d gamma (Prop. 7); the outputs are then written by all lanes, each position finding its
// block by bisection on the block starts.
//
// This is a correctness-first kernel: the stack walk is serial per row (one LDS round trip per
// step), which bounds it far below the memory roofline.
#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "wave.hpp"
#include "sort_network.hpp"

namespace topk {
namespace {

template <int GL, int E, bool CUBIC>
struct GenCfg {
  static constexpr int NP = GL * E;                 // padded row length
  static constexpr int RPW = kWave / GL;            // rows per wavefront
  static constexpr int IDXB = ilog2(NP) + 1;
  static constexpr int ND = CUBIC ? 5 : 3;          // float64 arrays: S1, W, gamma (+ S2, S3)
  // bytes per wavefront: float64 stack arrays, block starts (one extra slot per row), and the
  // float arrays ss (sorted values), lw (weights, later y), lt (tangent, later dy), ltau
  static constexpr int WaveBytes = RPW * (ND * NP * 8 + (NP + 2) * 4 + 4 * NP * 4);
  static constexpr int WPB = (4 * WaveBytes <= 60 * 1024) ? 4 : ((2 * WaveBytes <= 60 * 1024) ? 2 : 1);
};

// the increasing cubic of a block: sum_B (g - s_i)^3 + lambda^3 W [g] (magnitude: times g)
template <bool MAG>
__device__ __forceinline__ double block_cubic(double g, double cnt, double W, double S1, double S2,
                                              double S3, const Reg& R) {
  const double lin = MAG ? R.lam3 * W * g : R.lam3 * W;
  return ((cnt * g - 3.0 * S1) * g + 3.0 * S2) * g - S3 + lin;
}

// root of the block's cubic inside [lo, hi] (safeguarded Newton; the cubic is increasing)
template <bool MAG>
__device__ double block_root(double cnt, double W, double S1, double S2, double S3, const Reg& R,
                             double lo, double hi) {
  double a = lo, b = hi;
  double x = S1 / cnt - (MAG ? 0.0 : R.lambda * cbrt(W / cnt));
  if (!(x > a && x < b)) x = 0.5 * (a + b);
  const double tol = 1e-15 * fmax(fmax(fabs(a), fabs(b)), R.lambda);
  for (int it = 0; it < 200; ++it) {
    const double F = block_cubic<MAG>(x, cnt, W, S1, S2, S3, R);
    if (F == 0.0) return x;
    if (F > 0.0) b = x; else a = x;
    const double D = (3.0 * cnt * x - 6.0 * S1) * x + 3.0 * S2 + (MAG ? R.lam3 * W : 0.0);
    const double dx = F / D;
    // a step of rounding size ends the iteration before the bracket test: at the root the
    // bracket end is x itself, and bisecting from there would throw the converged value away
    if (fabs(dx) <= tol) return x - dx;
    double xn = x - dx;
    if (!(xn > a && xn < b)) xn = 0.5 * (a + b);
    x = xn;
  }
  return x;
}

template <int GL, int E, bool MAG, int PC>
__global__ __launch_bounds__((GenCfg<GL, E, PC == kP43>::WPB * kWave)) void general_rows_kernel(
    const float* __restrict__ x, const float* __restrict__ w_all, int64_t w_stride,
    const float* __restrict__ tangent, float* __restrict__ out, float* __restrict__ jvp,
    int64_t rows, int n, Reg R) {
  constexpr bool CUBIC = (PC == kP43);
  using C = GenCfg<GL, E, CUBIC>;
  constexpr int NP = C::NP, RPW = C::RPW, IDXB = C::IDXB;
  __shared__ __attribute__((aligned(16))) double ldsd[C::WPB][C::ND][RPW * NP];
  __shared__ int lds_lo[C::WPB][RPW * (NP + 2)];
  __shared__ __attribute__((aligned(16))) float ldsf[C::WPB][4][RPW * NP];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int rg = lane / GL;                              // row of the wavefront
  int64_t row = (int64_t(blockIdx.x) * C::WPB + wv) * RPW + rg;
  const bool valid = row < rows;
  if (!valid) row = rows - 1;            // keep the lanes alive for the exchanges; no stores
  const int64_t base = row * n;
  const int e0 = lr * E;
  double* st_s1 = &ldsd[wv][0][rg * NP];                 // stack: sum of s   (later: d gamma)
  double* st_w = &ldsd[wv][1][rg * NP];                  //        sum of w
  double* st_g = &ldsd[wv][2][rg * NP];                  //        pooled value
  double* st_s2 = CUBIC ? &ldsd[wv][C::ND - 2][rg * NP] : nullptr;
  double* st_s3 = CUBIC ? &ldsd[wv][C::ND - 1][rg * NP] : nullptr;
  int* st_lo = &lds_lo[wv][rg * (NP + 2)];               // block starts; [top] = n; [NP + 1] = top
  float* ss = &ldsf[wv][0][rg * NP];                     // sorted values
  float* lw = &ldsf[wv][1][rg * NP];                     // weights by sorted position; later y
  float* lt = &ldsf[wv][2][rg * NP];                     // tangent, original order; later dy
  float* ltau = &ldsf[wv][3][rg * NP];                   // tangent in sorted order (times sign)

  // ---- load, sort ----------------------------------------------------------------------------
  float xin[E], win[E];
  load_elems<E, false>(x, base, e0, n, xin);
  load_elems<E, false>(w_all, row * w_stride, e0, n, win);
  if (jvp != nullptr) {
    float tin[E];
    load_elems<E, false>(tangent, base, e0, n, tin);
#pragma unroll
    for (int r = 0; r < E; ++r) lt[e0 + r] = tin[r];
  }
  double K[E];
  make_keys<E, MAG, IDXB>(xin, e0, n, K);
  SortRuns<GL, E, NP>::run(K, lr);
  float s32[E];
  uint32_t field[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    uint32_t key;
    unpack<IDXB>(K[r], key, field[r]);
    s32[r] = key_to_float(key);
    ss[e0 + r] = s32[r];
    lw[e0 + r] = win[r];
  }
  __builtin_amdgcn_wave_barrier();
  if (jvp != nullptr) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      float tf = 0.0f;
      if (e0 + r < n) tf = lt[MAG ? (field[r] >> 1) : field[r]];
      if (MAG) {
        if (field[r] & 1u) tf = -tf;
        if (s32[r] == 0.0f) tf = 0.0f;         // sign(0) = 0
      }
      ltau[e0 + r] = tf;
    }
  }
  __builtin_amdgcn_wave_barrier();

  // ---- pool adjacent violators, one lane per row ---------------------------------------------
  if (lr == 0) {
    // The block on top of the stack is kept in registers (t*), so the first test of every
    // position needs no LDS read; its copy in LDS is written when the next block is pushed
    // above it.  The next position's value and weight are read one iteration ahead.
    int top = 0;                           // blocks in LDS below the register-held top
    bool have = false;
    int tlo = 0;
    double tS1 = 0.0, tW = 0.0, tS2 = 0.0, tS3 = 0.0, tg = 0.0;
    float s_next = ss[0], w_next = lw[0];
    for (int i = 0; i < n; ++i) {
      const double si = double(s_next), wi = double(w_next);
      if (i + 1 < n) { s_next = ss[i + 1]; w_next = lw[i + 1]; }
      int lo = i;
      double S1 = si, W = wi, S2 = 0.0, S3 = 0.0, g;
      if (CUBIC) { S2 = si * si; S3 = S2 * si; }
      // singleton minimiser
      if (!CUBIC) g = MAG ? __ddiv_rn(S1, __dadd_rn(__dmul_rn(R.lambda, W), 1.0))
                          : __dsub_rn(S1, __dmul_rn(R.lambda, W));
      else if (!MAG) g = si - R.lambda * cbrt(W);
      else g = (W == 0.0) ? si : block_root<true>(1.0, W, S1, S2, S3, R, 0.0, si);
      while (have) {
        bool viol;
        if (!CUBIC) {
          viol = tg < g;
        } else {
          const double pcnt = double(lo - tlo), cnt = double(i + 1 - lo);
          const bool p_closed = (lo - tlo == 1) && (!MAG || tW == 0.0);
          const bool t_closed = (i + 1 - lo == 1) && (!MAG || W == 0.0);
          if (p_closed == t_closed) viol = tg < g;
          else if (p_closed) viol = block_cubic<MAG>(tg, cnt, W, S1, S2, S3, R) < 0.0;
          else viol = block_cubic<MAG>(g, pcnt, tW, tS1, tS2, tS3, R) > 0.0;
        }
        if (!viol) break;
        // merge the previous block into the current one
        S1 = __dadd_rn(S1, tS1);
        W = __dadd_rn(W, tW);
        if (CUBIC) { S2 += tS2; S3 += tS3; }
        lo = tlo;
        // the block below becomes the top
        have = top > 0;
        if (have) {
          --top;
          tlo = st_lo[top]; tS1 = st_s1[top]; tW = st_w[top]; tg = st_g[top];
          if (CUBIC) { tS2 = st_s2[top]; tS3 = st_s3[top]; }
        }
        const double cnt = double(i + 1 - lo);
        if (!CUBIC) {
          g = MAG ? __ddiv_rn(S1, __dadd_rn(__dmul_rn(R.lambda, W), cnt))
                  : __ddiv_rn(__dsub_rn(S1, __dmul_rn(R.lambda, W)), cnt);
        } else {
          const double smax = double(ss[lo]), smin = si;
          g = MAG ? block_root<true>(cnt, W, S1, S2, S3, R, 0.0, smax)
                  : block_root<false>(cnt, W, S1, S2, S3, R, smin - R.lambda * cbrt(W) - 1e-300, smax);
        }
      }
      if (have) {                          // spill the old top below the new one
        st_lo[top] = tlo; st_s1[top] = tS1; st_w[top] = tW; st_g[top] = tg;
        if (CUBIC) { st_s2[top] = tS2; st_s3[top] = tS3; }
        ++top;
      }
      have = true;
      tlo = lo; tS1 = S1; tW = W; tS2 = S2; tS3 = S3; tg = g;
    }
    if (have) {
      st_lo[top] = tlo; st_s1[top] = tS1; st_w[top] = tW; st_g[top] = tg;
      if (CUBIC) { st_s2[top] = tS2; st_s3[top] = tS3; }
      ++top;
    }
    st_lo[top] = n;
    st_lo[NP + 1] = top;
    // ---- Prop. 7: d gamma of every block (overwrites the S1 column of the stack) ---------------
    if (jvp != nullptr) {
      for (int bk = 0; bk < top; ++bk) {
        const int lo = st_lo[bk], hi = st_lo[bk + 1];
        const double g = st_g[bk], W = st_w[bk];
        double dg;
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
        st_s1[bk] = dg;
      }
    }
  }
  __builtin_amdgcn_wave_barrier();

  // ---- outputs: y = sign o grad r*(s - v), dy = sign o hess r*(s - v) (tau - d gamma) ------------
  const int top = st_lo[NP + 1];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos = e0 + r;
    if (pos >= n) continue;
    int lo_b = 0, hi_b = top - 1;                        // last block whose start is <= pos
    while (lo_b < hi_b) {
      const int mid = (lo_b + hi_b + 1) >> 1;
      if (st_lo[mid] <= pos) lo_b = mid; else hi_b = mid - 1;
    }
    const double g = st_g[lo_b];
    const double tt = (double(s32[r]) - g) * R.inv_lambda;
    const bool neg = MAG && (field[r] & 1u);
    const uint32_t orig = MAG ? (field[r] >> 1) : field[r];
    if (out != nullptr) {
      float y = float(CUBIC ? tt * tt * tt : tt);
      if (MAG) y = (y == 0.0f || s32[r] == 0.0f) ? 0.0f : (neg ? -y : y);
      lw[orig] = y;
    }
    if (jvp != nullptr) {
      const double h = CUBIC ? 3.0 * tt * tt * R.inv_lambda : R.inv_lambda;
      float dy = float(h * (double(ltau[pos]) - st_s1[lo_b]));
      if (MAG) dy = (dy == 0.0f || s32[r] == 0.0f) ? 0.0f : (neg ? -dy : dy);
      lt[orig] = dy;
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (!valid) return;
  if (out != nullptr) {
    float yv[E];
#pragma unroll
    for (int r = 0; r < E; ++r) yv[r] = lw[e0 + r];
    store_elems<E, false>(out, base, e0, n, yv);
  }
  if (jvp != nullptr) {
    float jv[E];
#pragma unroll
    for (int r = 0; r < E; ++r) jv[r] = lt[e0 + r];
    store_elems<E, false>(jvp, base, e0, n, jv);
  }
}

template <int GL, int E>
int launch_general_shape(bool mag, int pc, const float* x, const float* w, int64_t w_stride,
                         const float* t, float* out, float* jvp, int64_t rows, int n, const Reg& R,
                         hipStream_t st) {
#define TOPK_GENERAL_CALL(MAGV, PCV)                                                            \
  do {                                                                                          \
    using C = GenCfg<GL, E, PCV == kP43>;                                                       \
    const int64_t waves = (rows + C::RPW - 1) / C::RPW;                                         \
    const int64_t blocks = (waves + C::WPB - 1) / C::WPB;                                       \
    if (blocks > 0x7fffffffLL) return -1;                                                       \
    hipLaunchKernelGGL((general_rows_kernel<GL, E, MAGV, PCV>), dim3((unsigned)blocks),          \
                       dim3(C::WPB * kWave), 0, st, x, w, w_stride, t, out, jvp, rows, n, R);   \
    return 0;                                                                                   \
  } while (0)
  if (!mag && pc == kP2) TOPK_GENERAL_CALL(false, kP2);
  if (!mag && pc == kP43) TOPK_GENERAL_CALL(false, kP43);
  if (mag && pc == kP2) TOPK_GENERAL_CALL(true, kP2);
  if (mag && pc == kP43) TOPK_GENERAL_CALL(true, kP43);
#undef TOPK_GENERAL_CALL
  return -1;
}

}  // namespace

int launch_general_rows(bool mag, int pc, const float* x, const float* w, int64_t w_stride,
                        const float* tangent, float* out, float* jvp, int64_t rows, int n,
                        const Reg& R, hipStream_t st) {
  int np = 2;
  while (np < n) np <<= 1;
#define CALL(GL, E) launch_general_shape<GL, E>(mag, pc, x, w, w_stride, tangent, out, jvp, rows, n, R, st)
  switch (np) {
    case 2: return CALL(1, 2);
    case 4: return CALL(1, 4);
    case 8: return CALL(1, 8);
    case 16: return CALL(2, 8);
    case 32: return CALL(4, 8);
    case 64: return CALL(8, 8);
    case 128: return CALL(16, 8);
    case 256: return CALL(32, 8);
    case 512: return CALL(64, 8);
    case 1024: return CALL(64, 16);
    default: return -1;
  }
#undef CALL
}

}  // namespace topk
