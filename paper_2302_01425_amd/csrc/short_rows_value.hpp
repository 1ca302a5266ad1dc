// Short rows, dense outputs, values only: the kernel of the router workloads (rows of up to 128
// elements, short_rows_select.hip) and of rows of 129 .. 2048 elements (short_rows_select_wide.hip).
//
// The operators' outputs depend on the row only through three numbers: the pooled value gamma of
// the one block [a, b] that pool-adjacent-violators grows around positions k, k+1 (App. "PAV
// algorithm" with w = 1_k), and the values s_a, s_b at its two ends.  An element is
//     above the block   (y = 1, resp. |x| / (1 + lambda))   iff  value >  s_a,
//     inside the block  (y = grad r*(value - gamma))         iff  s_b <= value <= s_a,
//     below the block   (y = 0)                              iff  value <  s_b
// (elements of equal value always pool together: if one of them violates against the block, the
// next one violates against the block that contains the first).  So no permutation is built and
// nothing is scattered: the kernel orders VALUES only, grows the block on them, and then every
// lane computes the outputs of the elements it loaded, in their original places.
//
// Which values have to be ordered.  Every element of the block, and everything above it, is larger
// than s_k - lambda (mask; s_k / (1 + lambda) for the magnitude operator): the pooled value of any
// block holding position k is at least the singleton minimiser of s_k.  For k <= GL (lanes per row)
// the k-th largest of the lanes' maxima is a lower bound of s_k, so
//     T = (k-th largest lane maximum) - lambda        (resp. / (1 + lambda)),  rounded down,
// bounds that window from below without any sort.  The values above T (a handful for a router
// row) are compacted through LDS and sorted by a small network (2 or 4 values per lane); rows
// with more of them, and launches with k > GL, sort the whole row.  The positions 1..cn of the
// row's descending order are then in LDS, and the block growth of the PAV loop runs on them
// (same strict tests, float64, as everywhere else: pooling.hpp).
//
// Order is by value only, with the machine's own float compare-exchange (v_med3_f32 against
// +-inf): ties, and the sign of a zero, cannot matter for values.
#pragma once

#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "wave.hpp"

// wavefronts per workgroup, and single-neighbour growth steps before the chunked growth (p = 2)
#ifndef TOPK_VALUE_WPB
#define TOPK_VALUE_WPB 4
#endif
#ifndef TOPK_VALUE_SINGLE_STEPS
#define TOPK_VALUE_SINGLE_STEPS 3
#endif

namespace topk {
namespace {

__device__ __forceinline__ float med3f(float a, float b, float c) {
  return __builtin_amdgcn_fmed3f(a, b, c);
}
__device__ __forceinline__ float pos_inf() { return __uint_as_float(0x7f800000u); }
__device__ __forceinline__ float neg_inf() { return __uint_as_float(0xff800000u); }

// ---- descending sorting network on floats (mirror-form bitonic, position = lane * E + register) --
template <int GL, int E, int M>
__device__ __forceinline__ void stage_desc(float (&K)[E], int lr) {
  constexpr int RM = M & (E - 1);
  constexpr int LM = M / E;
  if constexpr (LM == 0) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int r2 = r ^ RM;
      if (r < r2) {
        const float hi = med3f(K[r], K[r2], pos_inf());
        const float lo = med3f(K[r], K[r2], neg_inf());
        K[r] = hi;
        K[r2] = lo;
      }
    }
  } else {
    // the lower lane keeps the maximum, the upper one the minimum: the median of (own, other,
    // +inf resp. -inf)
    const float bound = (lr & top_bit(LM)) == 0 ? pos_inf() : neg_inf();
    float O[E];
#pragma unroll
    for (int r = 0; r < E; ++r) O[r] = __uint_as_float(lane_xor<LM>(__float_as_uint(K[r ^ RM])));
#pragma unroll
    for (int r = 0; r < E; ++r) K[r] = med3f(K[r], O[r], bound);
  }
}
template <int GL, int E, int STRIDE>
struct CleanersF {
  static __device__ __forceinline__ void run(float (&K)[E], int lr) {
    stage_desc<GL, E, STRIDE>(K, lr);
    CleanersF<GL, E, STRIDE / 2>::run(K, lr);
  }
};
template <int GL, int E>
struct CleanersF<GL, E, 0> {
  static __device__ __forceinline__ void run(float (&)[E], int) {}
};
template <int GL, int E, int SIZE>
struct SortDesc {
  static __device__ __forceinline__ void run(float (&K)[E], int lr) {
    SortDesc<GL, E, SIZE / 2>::run(K, lr);
    stage_desc<GL, E, SIZE - 1>(K, lr);
    CleanersF<GL, E, SIZE / 4>::run(K, lr);
  }
};
template <int GL, int E>
struct SortDesc<GL, E, 1> {
  static __device__ __forceinline__ void run(float (&)[E], int) {}
};

// inclusive prefix sum of one int per lane over the GL lanes of a row (DPP moves inside a row of
// 16 lanes, shuffles across such rows)
template <int GL>
__device__ __forceinline__ int row_scan_i32(int v, int lr) {
  if constexpr (GL >= 2) { const int o = int(dpp_mov<0x111>(uint32_t(v))); v += ((lr & 15) >= 1) ? o : 0; }
  if constexpr (GL >= 4) { const int o = int(dpp_mov<0x112>(uint32_t(v))); v += ((lr & 15) >= 2) ? o : 0; }
  if constexpr (GL >= 8) { const int o = int(dpp_mov<0x114>(uint32_t(v))); v += ((lr & 15) >= 4) ? o : 0; }
  if constexpr (GL >= 16) { const int o = int(dpp_mov<0x118>(uint32_t(v))); v += ((lr & 15) >= 8) ? o : 0; }
  if constexpr (GL >= 32) { const int o = __shfl_up(v, (lr & 15) + 1, GL); v += (lr & 16) ? o : 0; }
  if constexpr (GL >= 64) {
    const int o = __shfl(v, 31, GL);             // total of the first two rows of 16
    v += (lr & 32) ? o : 0;
  }
  return v;
}

// inclusive prefix sum over groups of H consecutive lanes (H a power of two up to 32, the group
// aligned to H lanes); t = lane index inside the group
template <int H>
__device__ __forceinline__ void half_scan(double& v, int t) {
  if constexpr (H >= 2) { const double o = row_shr_f64<1>(v); v = ((t & 15) >= 1) ? v + o : v; }
  if constexpr (H >= 4) { const double o = row_shr_f64<2>(v); v = ((t & 15) >= 2) ? v + o : v; }
  if constexpr (H >= 8) { const double o = row_shr_f64<4>(v); v = ((t & 15) >= 4) ? v + o : v; }
  if constexpr (H >= 16) { const double o = row_shr_f64<8>(v); v = ((t & 15) >= 8) ? v + o : v; }
  if constexpr (H >= 32) {
    const double o = __shfl_up(v, (t & 15) + 1, 32);   // the last lane of the row of 16 before mine
    v = (t & 16) ? v + o : v;
  }
}

template <int GL, int E>
struct SelCfg {
  static constexpr int NP = GL * E;
  static constexpr int RPW = kWave / GL;
  static constexpr int RS = NP + 4;       // row stride in LDS (floats): rows start 4 banks apart
};

// Sorts the GL * E2 values in ls[0 .. GL * E2) in place, descending (the list, filled up with -inf).
template <int GL, int E2>
__device__ __forceinline__ void sort_listed(float* ls, int lr) {
  float K[E2];
#pragma unroll
  for (int j = 0; j < E2; ++j) K[j] = ls[j * GL + lr];
  SortDesc<GL, E2, GL * E2>::run(K, lr);
  __builtin_amdgcn_wave_barrier();
  lds_store<E2>(ls + lr * E2, K);
}

// VEC: rows are 16-byte aligned and n % 4 == 0 (float4 loads and stores, rows dealt to the lanes
// float4 by float4).  FULL: additionally n == GL * E, so there is no padding and no bounds test.
// MODE: 0 forward only, 1 JVP only, 2 forward + JVP.
// SELECT: 1 <= k <= GL and k < n (checked by the launcher): order only the values above T.
// VAR: what is made of the mask (MAG = false only; kVarPlain: the operator itself):
//   kVarSigned  signed mask, phi = |x| (Sec. 4 on the OWL norm): the mask m of |x| with the
//               tangent sign(x) t, then y = sign(x) min(m, cap), cap = grad r*(|x|): the truncation
//               v >= 0 of Prop. 6 is active exactly where m > cap, and there dy = hess r*(|x|) t;
//   kVarMasked  x o mask(|x|) (Sec. 7): y = x m, dy = t m + x J_m (sign(x) o t);
//   kVarLoss    Fenchel-Young loss of Sec. 6 (MODE 0; `tangent` is the target t): out = y - t
//               and loss[row] = sum_i y_i x_i - (lambda / p) y_i^p - x_i t_i, the maximisation
//               form of Prop. 2 at its maximiser y.
constexpr int kVarPlain = 0, kVarSigned = 1, kVarMasked = 2, kVarLoss = 3;

template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE, bool SELECT, int WPB,
          int VAR = kVarPlain>
__global__ __launch_bounds__(WPB * kWave) void short_rows_value_kernel(
    const float* __restrict__ x, const float* __restrict__ tangent, float* __restrict__ out,
    float* __restrict__ jvp, int64_t rows, int n, int k, Reg R, float inv_lambda32,
    float inv_1pl32, float* __restrict__ loss = nullptr, double lam_over_p = 0.0) {
  static_assert(VAR == kVarPlain || !MAG, "the variants are built on the mask");
  static_assert(VAR != kVarLoss || MODE == 0, "the loss is a forward quantity");
  constexpr bool ABS = MAG || VAR == kVarSigned || VAR == kVarMasked;   // values ordered: |x|
  constexpr bool LOSS = VAR == kVarLoss;
  using P = Pool<MAG, PC>;
  using C = SelCfg<GL, E>;
  constexpr int NP = C::NP, RS = C::RS;
  constexpr bool CUBIC = (PC == kP43);
  constexpr bool CHUNKED = GL >= 4;
  constexpr bool want_out = (MODE == 0 || MODE == 2), want_jvp = (MODE == 1 || MODE == 2);
  __shared__ __attribute__((aligned(16))) float lds[WPB][C::RPW * RS];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int64_t row_raw = (int64_t(blockIdx.x) * WPB + wv) * C::RPW + lane / GL;
  const bool valid = row_raw < rows;
  const int64_t row = valid ? row_raw : rows - 1;   // lanes stay alive for the exchanges; no stores
  const int64_t base = row * n;
  float* ls = &lds[wv][(lane / GL) * RS];            // the row's ordered values
  const int nn = FULL ? NP : n;

  // ---- load ------------------------------------------------------------------------------------
  // (lanes with 16 or more elements fetch the tangent only when the block is known: registers)
  constexpr bool LATE_TANGENT = E >= 16;
  float xin[E], tin[E];
  load_row<GL, E, VEC, true>(x, base, lr, nn, xin);
  if ((want_jvp || LOSS) && !LATE_TANGENT) load_row<GL, E, VEC, true>(tangent, base, lr, nn, tin);
  float v[E];                                        // the values that are ordered; padding -inf
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const float a = ABS ? fabsf(xin[r]) : xin[r];
    v[r] = (FULL || elem_of<GL, E, VEC>(lr, r) < nn) ? a : neg_inf();
  }

  // ---- order the values that can matter ------------------------------------------------------------
  int cn = nn;                   // ls[0 .. cn) = sorted positions 1 .. cn of the row
  float T32 = neg_inf();         // everything that can pool, and all of the top k, is above T32
  const bool solve = (k >= 1 && k < nn);             // uniform; k = 0 and k = n pool nothing
  bool whole = solve;            // sort the whole row
  if constexpr (SELECT) {
    float lm = v[0];
#pragma unroll
    for (int r = 1; r < E; ++r) lm = med3f(lm, v[r], pos_inf());
    float K1[1] = {lm};
    SortDesc<GL, 1, GL>::run(K1, lr);
    const float lb = bcast_lane<GL>(K1[0], k - 1);   // k-th largest lane maximum <= s_k
    const double Td = MAG ? double(lb) * R.inv_1pl : double(lb) - R.lambda;
    T32 = float(Td);
    T32 = T32 - (fabsf(T32) * 2.4e-7f + 1.2e-38f);   // rounded down with room to spare
    int pos[E];
    int c = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      pos[r] = c;
      c += (v[r] > T32) ? 1 : 0;
    }
    const int inc = row_scan_i32<GL>(c, lr);
    const int pre = inc - c;
    cn = bcast_lane<GL>(inc, GL - 1);
    constexpr int kTier2 = (4 * GL < NP) ? 4 * GL : 0;   // 0: no second tier (it would be the whole row)
    constexpr int kListMax = kTier2 > 0 ? kTier2 : ((2 * GL < NP) ? 2 * GL : 0);
    whole = kListMax == 0 || __any(cn > kListMax);
    if (!whole) {
      // the list area starts as -inf; every lane then drops its values above T32 at their places
      // in the list (the others go to a spare word of the lane: no branch per element)
      constexpr int kPerLane = kListMax > 0 ? kListMax / GL : 1;   // 2 or 4
      float fill[kPerLane];
#pragma unroll
      for (int j = 0; j < kPerLane; ++j) fill[j] = neg_inf();
      lds_store<kPerLane>(ls + lr * kPerLane, fill);
      __builtin_amdgcn_wave_barrier();
      const int spare = kListMax + lr;
#pragma unroll
      for (int r = 0; r < E; ++r) ls[(v[r] > T32) ? pre + pos[r] : spare] = v[r];
      __builtin_amdgcn_wave_barrier();
      if (kTier2 > 0 && __any(cn > 2 * GL)) sort_listed<GL, 4>(ls, lr);
      else sort_listed<GL, 2>(ls, lr);
    } else {
      cn = nn;
    }
  }
  if (whole) {
    float s[E];
#pragma unroll
    for (int r = 0; r < E; ++r) s[r] = v[r];
    SortDesc<GL, E, NP>::run(s, lr);
    lds_store<E>(ls + lr * E, s);
  }
  __builtin_amdgcn_wave_barrier();

  // ---- isotonic solve: grow the one pooled block outwards from (k, k+1) ----------------------
  // All lanes of a row carry the same (a, b, sums).  A step tests the two neighbours of the block
  // with the strict violation tests of the PAV loop and takes in whichever violates; both may
  // join in one step (the right one raises the pooled value, the left one lowers it, so each
  // still violates after the other has joined).  Straight-line selects, one branch per step.
  int a = k + 1, b = k;                  // 1-based inclusive block [a, b]; empty when a > b
  double center = 0.0, gamma = 0.0, cnt = 0.0, m = 0.0;
  float c32 = 0.0f;                      // s_k: the outputs are computed on values relative to it
  float one_gt = (k == 0) ? pos_inf() : neg_inf();   // above the block iff value > one_gt
  float blk_ge = pos_inf();                           // else inside it iff value >= blk_ge
  if (solve) {                           // uniform
    c32 = ls[k - 1];
    const float fk1 = ls[k];             // -inf when the row has only k listed values
    float nl = ls[k >= 2 ? k - 2 : 0];       // value left of the block (position a-1)
    float nr = ls[k + 1 < cn ? k + 1 : k];   // value right of the block (position b+1)
    const double sk = double(c32), sk1 = double(fk1);
    if (!MAG) center = sk;
    const double dk = sk - center, dk1 = sk1 - center;
    const bool grew = (cn > k) & P::seed_violates(dk, dk1, R);
    // nothing pools: the top k are ones; s_k > s_{k+1} strictly, and an unlisted s_{k+1} is <= T32
    one_gt = cn > k ? fk1 : T32;
    if (__any(grew)) {
      Sums S{dk + dk1, 0.0, 0.0};
      if (CUBIC) {
        S.s2 = dk * dk + dk1 * dk1;
        S.s3 = dk * dk * dk + dk1 * dk1 * dk1;
      }
      a = grew ? k : a;
      b = grew ? k + 1 : b;
      cnt = 2.0;
      m = 1.0;
      // (1) a few single-neighbour steps: the usual p = 2 block has 2-5 positions
      constexpr int kSingleSteps = CUBIC ? 0 : TOPK_VALUE_SINGLE_STEPS;
      bool pending = true;               // some row of the wavefront may still grow
      for (int step = 0; step < kSingleSteps || !CHUNKED; ++step) {
        const double dj = double(nr) - center, di = double(nl) - center;
        const bool add_r = grew & (b < cn) & P::right_violates(dj, cnt, m, S, R);
        const bool add_l = grew & (a > 1) & P::left_violates(di, cnt, m, S, R);
        if (!__any(add_r | add_l)) { pending = false; break; }
        b += add_r ? 1 : 0;
        a -= add_l ? 1 : 0;
        nr = ls[b < cn ? b : cn - 1];
        nl = ls[a >= 2 ? a - 2 : 0];
        const double ar = add_r ? dj : 0.0, al = add_l ? di : 0.0;
        S.s1 += ar + al;
        if (CUBIC) {
          S.s2 += ar * ar + al * al;
          S.s3 += ar * ar * ar + al * al * al;
        }
        cnt = double(b - a + 1);
        m = double(k - a + 1);
      }
      // (2) larger blocks: every step tests GL/2 positions on each side at once.  The lower half
      // of the row's lanes takes the positions b+1, b+2, .. and the upper half a-1, a-2, ..; an
      // exclusive scan of the power sums inside each half gives every lane the block it would
      // join (all candidates before it included), and the violation tests hold on a prefix of
      // each half, whose length is read off a ballot.
      if constexpr (CHUNKED) {
        constexpr int H = GL / 2;
        const int t = lr & (H - 1);
        const bool left = lr >= H;
        bool first_chunk = true;
        while (pending) {
          if (!first_chunk) {
            // the tests are monotone along each side: if neither immediate neighbour of the block
            // violates now, no position does, and the growth is over
            const double dj = double(ls[b < cn ? b : cn - 1]) - center;
            const double di = double(ls[a >= 2 ? a - 2 : 0]) - center;
            const bool add_r = grew & (b < cn) & P::right_violates(dj, cnt, m, S, R);
            const bool add_l = grew & (a > 1) & P::left_violates(di, cnt, m, S, R);
            if (!__any(add_r | add_l)) break;
          }
          first_chunk = false;
          const int q = left ? a - 2 - t : b + t;            // 0-based sorted position
          const bool ok = grew & (left ? q >= 0 : q < cn);
          const float val = ls[ok ? q : 0];
          const double d = ok ? double(val) - center : 0.0;
          Sums own{d, CUBIC ? d * d : 0.0, CUBIC ? d * d * d : 0.0};
          Sums pre = own;                                    // inclusive scan over the half
          half_scan<H>(pre.s1, t);
          if (CUBIC) { half_scan<H>(pre.s2, t); half_scan<H>(pre.s3, t); }
          Sums blk{S.s1 + (pre.s1 - own.s1), S.s2 + (pre.s2 - own.s2), S.s3 + (pre.s3 - own.s3)};
          const double cnt_t = cnt + double(t), m_t = m + (left ? double(t) : 0.0);
          const bool viol = left ? P::left_violates(d, cnt_t, m_t, blk, R)
                                 : P::right_violates(d, cnt_t, m_t, blk, R);
          const unsigned long long bal = __ballot(ok & viol);
          const unsigned long long rowbits = bal >> (lane & ~(GL - 1));   // my row's lanes from bit 0
          // number of leading candidates that join, per side (the tests are monotone)
          constexpr unsigned long long kHalfMask = (1ull << H) - 1ull;
          const int n_r = __builtin_ctzll(~(rowbits & kHalfMask) | (1ull << H));
          const int n_l = __builtin_ctzll(~((rowbits >> H) & kHalfMask) | (1ull << H));
          if (!__any((n_r | n_l) != 0)) break;
          const bool take = t < (left ? n_l : n_r);
          Sums add{take ? own.s1 : 0.0, take ? own.s2 : 0.0, take ? own.s3 : 0.0};
          S.s1 += group_sum_f64<GL>(add.s1);
          if (CUBIC) {
            S.s2 += group_sum_f64<GL>(add.s2);
            S.s3 += group_sum_f64<GL>(add.s3);
          }
          b += n_r;
          a -= n_l;
          cnt = double(b - a + 1);
          m = double(k - a + 1);
        }
      }
      const float fa = ls[a - 1], fb = ls[b - 1];
      const double da = double(fa) - center, db = double(fb) - center;
      if (MAG) gamma = S.s1 * recip(cnt + R.lambda * m);
      else if (!CUBIC) gamma = (S.s1 - R.lambda * m) * recip(cnt);
      else if (grew) gamma = P::pooled(cnt, m, S, R, da - R.lambda, db);   // (rows without a
      // block skip the Newton solve: their sums may hold the -inf of an unlisted s_{k+1})
      gamma = grew ? gamma : 0.0;
      one_gt = grew ? fa : one_gt;
      blk_ge = grew ? fb : blk_ge;
    }
  }

  // ---- outputs, element by element in the original places -----------------------------------------
  if ((want_jvp || LOSS) && LATE_TANGENT) load_row<GL, E, VEC, true>(tangent, base, lr, nn, tin);
  const bool have = a <= b;
  const float g32 = float(MAG ? gamma - double(c32) : gamma);   // pooled value relative to s_k
  bool abv[E], inb[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    abv[r] = v[r] > one_gt;
    inb[r] = (!abv[r]) & (v[r] >= blk_ge);
  }
  float tau[E];                                      // tangent in sorted-value coordinates
  if (want_jvp) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      float t = tin[r];
      if (ABS) {
        t = (__float_as_uint(xin[r]) >> 31) ? -t : t;
        t = (v[r] == 0.0f) ? 0.0f : t;               // sign(0) = 0
      }
      tau[r] = t;
    }
  }
  double dgamma = 0.0;
  if (want_jvp && __any(have)) {
    // Prop. 7: d gamma = sum_B c_j tau_j / (sum_B c_j [+ lambda m])
    double num = 0.0, wsum = 0.0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      if (CUBIC) {
        const double w = inb[r] ? P::jac_weight(double(v[r]) - center, gamma) : 0.0;
        num += w * double(tau[r]);
        wsum += w;
      } else {
        num += double(inb[r] ? tau[r] : 0.0f);
      }
    }
    num = group_sum_f64<GL>(num);
    if (CUBIC) wsum = group_sum_f64<GL>(wsum);
    else wsum = cnt;
    const double den = P::jac_denominator(wsum, m, R);
    dgamma = have ? num * recip(den) : 0.0;
  }
  float yv[E], jv[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const bool neg = MAG && (__float_as_uint(xin[r]) >> 31);
    const float t = ((v[r] - c32) - g32) * inv_lambda32;       // (s - gamma) / lambda
    if (want_out) {
      float y;
      if (MAG) {
        const double yd = inb[r] ? P::y_in_block(double(v[r]), gamma, R) : double(v[r]) * R.inv_1pl;
        y = (abv[r] | inb[r]) ? float(yd) : 0.0f;
        y = (y == 0.0f) ? 0.0f : (neg ? -y : y);
      } else {
        y = inb[r] ? (CUBIC ? t * t * t : t) : (abv[r] ? 1.0f : 0.0f);
      }
      yv[r] = y;
    }
    if (want_jvp) {
      const double diff = double(tau[r]) - dgamma;
      float dyb;
      if (CUBIC) {
        // (float64: the factor 3 t^2 / lambda reaches the hundreds for small lambda, and three
        // float32 roundings would show against a bar of one float32 ulp)
        const double td = ((double(v[r]) - double(c32)) - double(MAG ? gamma - double(c32) : gamma)) * R.inv_lambda;
        dyb = float(3.0 * td * td * R.inv_lambda * diff);
      } else {
        dyb = float(diff * R.inv_lambda);
      }
      float dy = inb[r] ? dyb : ((MAG && abv[r]) ? tau[r] * inv_1pl32 : 0.0f);
      if (MAG) dy = (dy == 0.0f || v[r] == 0.0f) ? 0.0f : (neg ? -dy : dy);
      jv[r] = dy;
    }
    // ---- what the variants make of the mask (element-wise; float64 for the values: with a small
    // lambda the factors reach the hundreds, and two or three float32 roundings would show
    // against a bar of one float32 ulp) --------------------------------------------------------
    if (VAR == kVarSigned) {
      const float xv = xin[r];
      const float sg = float((xv > 0.0f) - (xv < 0.0f));
      const double u = double(v[r]) * R.inv_lambda;
      const float cap = float(CUBIC ? u * u * u : u);
      // the truncation v >= 0 is active where the mask exceeds the cap: inside the block
      // ((s - gamma) / lambda against s / lambda) exactly when gamma < 0, above it (the literal 1)
      // when s < lambda, below it never -- decided on gamma and s themselves, so that a pooled
      // value of exactly zero is the tie it is and not the last bit of two float32 roundings
      const bool clipped = inb[r] ? (double(c32) + gamma < 0.0)
                                  : (abv[r] && double(v[r]) < R.lambda);
      if (want_jvp) {
        const double hess = CUBIC ? 3.0 * u * u * R.inv_lambda : R.inv_lambda;
        float jm = clipped ? float(hess * double(tin[r])) : sg * jv[r];
        jv[r] = (jm == 0.0f) ? 0.0f : jm;
      }
      const float y = sg * (clipped ? cap : yv[r]);
      yv[r] = (y == 0.0f) ? 0.0f : y;
    } else if (VAR == kVarMasked) {
      if (want_jvp) jv[r] = float(double(tin[r]) * double(yv[r]) + double(xin[r]) * double(jv[r]));
      yv[r] = xin[r] * yv[r];
    }
  }
  if (LOSS) {
    // f(x) = max_y <y, x> - (lambda / p) sum y^p over the capped simplex, evaluated at the float32
    // mask through its Lagrangian, <y, x> - (lambda / p) sum y^p - gamma (sum y - k): the same
    // value at the maximiser, and flat there -- x_i - lambda y_i^(p-1) = gamma on the block -- so
    // that the rounding of the y_i does not enter in first order
    double acc = 0.0, ysum = 0.0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const bool real = FULL || elem_of<GL, E, VEC>(lr, r) < nn;
      const double yd = double(yv[r]);
      double yp = yd * yd;                           // y^p: p = 2, or the exact ends of p = 4/3
      if (CUBIC && __any(yv[r] != 0.0f && yv[r] != 1.0f)) {
        const double c = cbrt(yd);                   // y^(4/3), y in [0, 1]
        yp = c * c * c * c;
      }
      if (real) {
        acc += yd * double(xin[r]) - lam_over_p * yp - double(xin[r]) * double(tin[r]);
        ysum += yd;
      }
      yv[r] = yv[r] - tin[r];                        // the gradient y - t
    }
    acc = group_sum_f64<GL>(acc);
    ysum = group_sum_f64<GL>(ysum);
    // (without a block every y is a literal 0 or 1 and sum y = k exactly)
    if (have) acc -= (double(c32) + gamma) * (ysum - double(k));
    if (valid && lr == 0) loss[row] = float(acc);
  }
  if (!valid) return;
  if (want_out) store_row<GL, E, VEC, true>(out, base, lr, nn, yv);
  if (want_jvp) store_row<GL, E, VEC, true>(jvp, base, lr, nn, jv);
}

}  // namespace
}  // namespace topk
