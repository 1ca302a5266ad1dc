// The relaxed operators y_{phi,R}(x, w) for a GENERAL non-increasing weight vector w (Sec. 4;
// soft rank, soft sort and partial ranks through the LP forms of Sec. 3), rows up to 1024 elements.
//
// With w = 1_k one pooled block suffices and the other kernels exploit that.  For a general w the
// partition of pool-adjacent-violators (App. "PAV algorithm") can have any number of blocks.  After
// the same register sort, the lanes of a row build the partition together, in ROUNDS:
//
//   * float64 prefix sums of (s, w [, s^2, s^3]) over the sorted positions live in LDS, so the sums
//     of any block [lo, hi) are two reads and a subtraction;
//   * every lane owns E consecutive positions and keeps the block starts among them as a bit mask;
//     a suffix-minimum / prefix-maximum over the lanes tells each block where its neighbours start;
//   * a round computes the pooled value of every block that changed since the last round, then
//     tests every boundary with the strict test of the PAV loop (gamma_left < gamma_right) and
//     removes ALL violating boundaries at once.
//
// Removing several violating boundaries together is legal: a violating pair of neighbours stays
// violating whatever else is merged first (merging the right block with a block that violates
// against it raises its pooled value, merging the left block with one on its left lowers it), so
// every such pair ends in one block of the sequential algorithm as well, and the partition in
// which no strict violation is left is unique.  Typical rows need a handful of rounds.  A row
// built so that only one boundary violates at a time (a low value followed by a slowly falling
// ramp) needs one round per element: after 32 + n / 4 rounds (p = 2) the wavefront gives up and one
// lane per row walks the usual left-to-right block stack instead.
//
// Pooled values of p = 2 are computed without fused multiply-adds, from sums that are exact
// whenever the float32 inputs span fewer than ~2^19 in magnitude, so exact ties are seen as ties.
// d gamma of every block (Prop. 7) comes from two more prefix sums (weights c_j and c_j tau_j);
// the outputs are then written by all lanes, each position looking up its block's start.
#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "wave.hpp"
#include "sort_network.hpp"
#include "general_pav.hpp"

namespace topk {
namespace {

constexpr int kMinRounds = 32;

template <int GL, int E, bool CUBIC>
struct GenCfg {
  static constexpr int NP = GL * E;                 // padded row length
  static constexpr int NQ = NP + 1;                 // entries of a prefix array
  static constexpr int RPW = kWave / GL;            // rows per wavefront
  static constexpr int IDXB = ilog2(NP) + 1;
  // float64 arrays per row: prefix S1, prefix W, gamma per block start (+ prefix S2, S3)
  static constexpr int ND = CUBIC ? 5 : 3;
  // bytes per wavefront: the float64 arrays, the cached block ends (16 bits) and their round
  // stamps (8 bits), and the float arrays ss (sorted values), lw (weights, later y), ltau
  static constexpr int WaveBytes = RPW * (ND * NQ * 8 + (NP + 2) * 2 + NP + 3 * NP * 4);
  // wavefronts per workgroup: rows of 1024 elements take 40 KB (p = 2), one wavefront each, so that
  // four workgroups fit the 160 KB of a compute unit
  static constexpr int WPB = (4 * WaveBytes <= 60 * 1024) ? 4 : ((2 * WaveBytes <= 60 * 1024) ? 2 : 1);
};

// first block start in the lanes after this one / last block start in the lanes before it
template <int GL>
__device__ __forceinline__ int lanes_after_min(int v, int lr, int none) {
#pragma unroll
  for (int off = 1; off < GL; off <<= 1) {
    const int o = __shfl_down(v, off, GL);
    if (lr + off < GL) v = min(v, o);
  }
  const int nx = __shfl_down(v, 1, GL);
  return lr + 1 < GL ? nx : none;
}
template <int GL>
__device__ __forceinline__ int lanes_before_max(int v, int lr, int none) {
#pragma unroll
  for (int off = 1; off < GL; off <<= 1) {
    const int o = __shfl_up(v, off, GL);
    if (lr >= off) v = max(v, o);
  }
  const int pv = __shfl_up(v, 1, GL);
  return lr >= 1 ? pv : none;
}

template <int GL, int E, bool MAG, int PC>
__global__ __launch_bounds__((GenCfg<GL, E, PC == kP43>::WPB * kWave)) void general_rows_kernel(
    const float* __restrict__ x, const float* __restrict__ w_all, int64_t w_stride,
    const float* __restrict__ tangent, float* __restrict__ out, float* __restrict__ jvp,
    int64_t rows, int n, Reg R, int max_rounds) {
  constexpr bool CUBIC = (PC == kP43);
  using C = GenCfg<GL, E, CUBIC>;
  constexpr int NP = C::NP, NQ = C::NQ, RPW = C::RPW, IDXB = C::IDXB;
  static_assert(E <= 16, "the block starts of a lane are kept in a 32-bit mask");
  static_assert(NP < 0xffff, "block ends are kept in 16 bits");
  __shared__ __attribute__((aligned(16))) double ldsd[C::WPB][C::ND][RPW * NQ];
  __shared__ uint16_t lds_hi[C::WPB][RPW * (NP + 2)];
  __shared__ uint8_t lds_ver[C::WPB][RPW * NP];
  __shared__ __attribute__((aligned(16))) float ldsf[C::WPB][3][RPW * NP];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int rg = lane / GL;                              // row of the wavefront
  int64_t row = (int64_t(blockIdx.x) * C::WPB + wv) * RPW + rg;
  const bool valid = row < rows;
  if (!valid) row = rows - 1;            // keep the lanes alive for the exchanges; no stores
  const int64_t base = row * n;
  const int e0 = lr * E;
  // float64 arrays of the row.  P*: prefix sums over sorted positions, P[i] = sum of j < i.
  double* P1 = &ldsd[wv][0][rg * NQ];    // of s; after the rounds: of c_j tau_j (Prop. 7)
  double* PW = &ldsd[wv][1][rg * NQ];    // of w
  double* G = &ldsd[wv][2][rg * NQ];     // pooled value by block start; at the very end d gamma
  double* P2 = CUBIC ? &ldsd[wv][3][rg * NQ] : nullptr;   // of s^2; after the rounds: of c_j
  double* P3 = CUBIC ? &ldsd[wv][4][rg * NQ] : nullptr;   // of s^3
  uint16_t* hi_of = &lds_hi[wv][rg * (NP + 2)];  // end of the block that G[lo] was computed for
  uint8_t* ver = &lds_ver[wv][rg * NP];          // round (mod 256) in which that last changed
  float* ss = &ldsf[wv][0][rg * NP];                     // sorted values
  float* lw = &ldsf[wv][1][rg * NP];                     // weights by sorted position; later y
  float* ltau = &ldsf[wv][2][rg * NP];                   // tangent in sorted order (times sign)
  float* lt = reinterpret_cast<float*>(G);               // tangent, original order; later dy

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
    hi_of[e0 + r] = 0xffff;
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

  // ---- prefix sums of the sorted row --------------------------------------------------------------
  {
    double t1 = 0.0, tw = 0.0, t2 = 0.0, t3 = 0.0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const bool real = e0 + r < n;
      const double sd = real ? double(s32[r]) : 0.0, wd = real ? double(win[r]) : 0.0;
      t1 += sd;
      tw += wd;
      if (CUBIC) { t2 += sd * sd; t3 += sd * sd * sd; }
    }
    double r1 = group_exclusive_scan_f64<GL>(t1, lr), rw = group_exclusive_scan_f64<GL>(tw, lr);
    double r2 = 0.0, r3 = 0.0;
    if (CUBIC) { r2 = group_exclusive_scan_f64<GL>(t2, lr); r3 = group_exclusive_scan_f64<GL>(t3, lr); }
#pragma unroll
    for (int r = 0; r < E; ++r) {
      P1[e0 + r] = r1;
      PW[e0 + r] = rw;
      if (CUBIC) { P2[e0 + r] = r2; P3[e0 + r] = r3; }
      const bool real = e0 + r < n;
      const double sd = real ? double(s32[r]) : 0.0, wd = real ? double(win[r]) : 0.0;
      r1 += sd;
      rw += wd;
      if (CUBIC) { r2 += sd * sd; r3 += sd * sd * sd; }
    }
    if (lr == GL - 1) {
      P1[NP] = r1;
      PW[NP] = rw;
      if (CUBIC) { P2[NP] = r2; P3[NP] = r3; }
    }
  }
  __builtin_amdgcn_wave_barrier();               // (also: the tangent in G's place has been read)

  auto block_sums = [&](int lo, int hi) -> Blk {
    Blk b;
    b.cnt = double(hi - lo);
    b.S2 = b.S3 = 0.0;
    if (hi - lo == 1) {                      // a singleton: its own value and weight, exactly
      b.S1 = double(ss[lo]);
      b.W = double(lw[lo]);
      if (CUBIC) { b.S2 = b.S1 * b.S1; b.S3 = b.S2 * b.S1; }
    } else {
      b.S1 = P1[hi] - P1[lo];
      b.W = PW[hi] - PW[lo];
      if (CUBIC) { b.S2 = P2[hi] - P2[lo]; b.S3 = P3[hi] - P3[lo]; }
    }
    return b;
  };

  // ---- pool adjacent violators in rounds ------------------------------------------------------------
  uint32_t hm = 0;                           // block starts among my positions (bit r: e0 + r)
#pragma unroll
  for (int r = 0; r < E; ++r)
    if (e0 + r < n) hm |= 1u << r;
  bool gave_up = false;
  for (int round = 0;; ++round) {
    const uint8_t now = uint8_t(round);
    const int first = hm ? e0 + __builtin_ctz(hm) : n;
    const int last = hm ? e0 + 31 - __builtin_clz(hm) : -1;
    const int nxt = lanes_after_min<GL>(first, lr, n);
    const int prv = lanes_before_max<GL>(last, lr, -1);
    // pooled value of every block that is not the one of the last round
    for (uint32_t m = hm; m != 0;) {
      const int r = __builtin_ctz(m);
      m &= m - 1;
      const int lo = e0 + r, hi = m ? e0 + __builtin_ctz(m) : nxt;
      if (int(hi_of[lo]) != hi) {
        hi_of[lo] = uint16_t(hi);
        ver[lo] = now;
        G[lo] = block_gamma<MAG, CUBIC>(block_sums(lo, hi), double(ss[lo]), double(ss[hi - 1]), R);
      }
    }
    __builtin_amdgcn_wave_barrier();
    // every boundary whose two blocks violate goes; a boundary between two blocks that are both
    // those of the last round was tested then
    uint32_t keep = hm;
    for (uint32_t m = hm; m != 0;) {
      const int r = __builtin_ctz(m);
      m &= m - 1;
      const int lo = e0 + r, hi = m ? e0 + __builtin_ctz(m) : nxt;
      const uint32_t below = hm & ((1u << r) - 1u);
      const int p = below ? e0 + 31 - __builtin_clz(below) : prv;
      if (p < 0) continue;                   // the first block of the row
      if (ver[p] != now && ver[lo] != now) continue;
      bool viol;
      if (!CUBIC) viol = G[p] < G[lo];
      else viol = blocks_violate<MAG, CUBIC>(block_sums(p, lo), G[p], block_sums(lo, hi), G[lo], R);
      if (viol) keep &= ~(1u << r);
    }
    const bool changed = keep != hm;
    hm = keep;
    if (!__any(changed)) break;
    if (round + 1 >= max_rounds) { gave_up = true; break; }
    __builtin_amdgcn_wave_barrier();
  }
  __builtin_amdgcn_wave_barrier();

  double* DG = G;                            // d gamma by block start
  float yv[E];
  double tt[E];                              // (s - gamma) / lambda
  if (!gave_up) {
    const int last = hm ? e0 + 31 - __builtin_clz(hm) : -1;
    const int prv = lanes_before_max<GL>(last, lr, -1);
    if (CUBIC) {
      // ---- the roots once more, from sums of the blocks' own spread.  A block's sums so far are
      // differences of prefix sums over the whole row: their rounding is that of the row's values
      // cubed, while the cubic of a block whose values lie within a small lambda of each other
      // needs that of the spread cubed.  With the partition final, every position is taken
      // relative to the first value c of its own block: the prefix sums of d = s - c, d^2, d^3
      // stay as small as the blocks are narrow (a block's sums involve its own positions only),
      // and the safeguarded Newton solve of the rounds, on sum (g - d_i)^3 + lambda^3 W [c + g] = 0
      // with the same bracket, gives gamma = c + g to the rounding of the spread -----------------
      double dd[E];
      double t1 = 0.0, t2 = 0.0, t3 = 0.0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const uint32_t upto = hm & ((2u << r) - 1u);
        int b = upto ? e0 + 31 - __builtin_clz(upto) : prv;
        if (b < 0) b = 0;
        dd[r] = (e0 + r < n) ? double(s32[r]) - double(ss[b]) : 0.0;
        t1 += dd[r];
        t2 += dd[r] * dd[r];
        t3 += dd[r] * dd[r] * dd[r];
      }
      double r1 = group_exclusive_scan_f64<GL>(t1, lr), r2 = group_exclusive_scan_f64<GL>(t2, lr);
      double r3 = group_exclusive_scan_f64<GL>(t3, lr);
      __builtin_amdgcn_wave_barrier();           // the prefix sums of the rounds have been read
#pragma unroll
      for (int r = 0; r < E; ++r) {
        P1[e0 + r] = r1;
        P2[e0 + r] = r2;
        P3[e0 + r] = r3;
        r1 += dd[r];
        r2 += dd[r] * dd[r];
        r3 += dd[r] * dd[r] * dd[r];
      }
      if (lr == GL - 1) {
        P1[NP] = r1;
        P2[NP] = r2;
        P3[NP] = r3;
      }
      __builtin_amdgcn_wave_barrier();
      const int first = hm ? e0 + __builtin_ctz(hm) : n;
      const int nxt = lanes_after_min<GL>(first, lr, n);
      for (uint32_t m = hm; m != 0;) {
        const int r = __builtin_ctz(m);
        m &= m - 1;
        const int lo = e0 + r, hi = m ? e0 + __builtin_ctz(m) : nxt;
        if (hi - lo == 1) continue;              // (singletons have closed forms)
        const double cnt = double(hi - lo), c = double(ss[lo]);
        const double S1 = P1[hi] - P1[lo], S2 = P2[hi] - P2[lo], S3 = P3[hi] - P3[lo];
        const double W = PW[hi] - PW[lo];
        // the bracket of the first solve, relative to c: [smin - lambda cbrt(W), smax] (mask), [0, smax]
        const double dmin = double(ss[hi - 1]) - c;
        const double g = MAG ? block_root<true>(cnt, W, S1, S2, S3, R, -c, 0.0, c)
                             : block_root<false>(cnt, W, S1, S2, S3, R,
                                                 dmin - R.lambda * cbrt(W) - 1e-300, 0.0);
        G[lo] = c + g;
      }
      __builtin_amdgcn_wave_barrier();
    }
    // ---- y; then Prop. 7: d gamma of every block from prefix sums of c_j tau_j and c_j --------------
    double cq[E], cc[E];
    double tq = 0.0, tc = 0.0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const uint32_t upto = hm & ((2u << r) - 1u);
      int b = upto ? e0 + 31 - __builtin_clz(upto) : prv;
      if (b < 0) b = 0;
      const double g = G[b];
      tt[r] = (double(s32[r]) - g) * R.inv_lambda;
      double c = 1.0;
      if (CUBIC) {
        const double d = g - double(s32[r]);
        c = MAG ? 3.0 * d * d : d * d;
      }
      const bool real = e0 + r < n;
      cc[r] = real ? c : 0.0;
      cq[r] = (real && jvp != nullptr) ? c * double(ltau[e0 + r]) : 0.0;
      tq += cq[r];
      tc += cc[r];
    }
    if (jvp != nullptr) {
      double rq = group_exclusive_scan_f64<GL>(tq, lr);
      double rc = CUBIC ? group_exclusive_scan_f64<GL>(tc, lr) : 0.0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        P1[e0 + r] = rq;
        if (CUBIC) P2[e0 + r] = rc;
        rq += cq[r];
        rc += cc[r];
      }
      if (lr == GL - 1) {
        P1[NP] = rq;
        if (CUBIC) P2[NP] = rc;
      }
      __builtin_amdgcn_wave_barrier();
      const int first = hm ? e0 + __builtin_ctz(hm) : n;
      const int nxt = lanes_after_min<GL>(first, lr, n);
      for (uint32_t m = hm; m != 0;) {
        const int r = __builtin_ctz(m);
        m &= m - 1;
        const int lo = e0 + r, hi = m ? e0 + __builtin_ctz(m) : nxt;
        double dg;
        if (hi - lo == 1) {
          const double tau = double(ltau[lo]), W = double(lw[lo]);
          if (!MAG) dg = tau;
          else if (!CUBIC) dg = tau / (1.0 + R.lambda * W);
          else if (W == 0.0) dg = tau;
          else {
            const double d = G[lo] - double(ss[lo]);
            dg = 3.0 * d * d * tau / (3.0 * d * d + R.lam3 * W);
          }
        } else {
          const double num = P1[hi] - P1[lo];
          double den = CUBIC ? P2[hi] - P2[lo] : double(hi - lo);
          if (MAG) den += (CUBIC ? R.lam3 : R.lambda) * (PW[hi] - PW[lo]);
          dg = num / den;
        }
        DG[lo] = dg;                         // G[lo] is read by this lane only, above
      }
    }
  } else {
    // ---- too many rounds: the left-to-right block stack, one lane per row ---------------------------
    // (stack columns in the arrays of the rounds, block starts in hi_of; the block on top of the
    // stack is kept in registers)
    double* st_s1 = P1;
    double* st_w = PW;
    double* st_g = G;
    double* st_s2 = P2;
    double* st_s3 = P3;
    uint16_t* st_lo = hi_of;
    DG = P1;
    __builtin_amdgcn_wave_barrier();
    if (lr == 0)
      stack_walk<MAG, CUBIC, uint16_t>(n, ss, lw, ltau, jvp != nullptr, st_s1, st_w, st_g, st_s2,
                                       st_s3, st_lo, uint16_t(0xffff), DG, R);
    __builtin_amdgcn_wave_barrier();
    hm = 0;
#pragma unroll
    for (int r = 0; r < E; ++r)
      if (e0 + r < n && hi_of[e0 + r] == 0xffff) hm |= 1u << r;
    const int last = hm ? e0 + 31 - __builtin_clz(hm) : -1;
    const int prv = lanes_before_max<GL>(last, lr, -1);
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const uint32_t upto = hm & ((2u << r) - 1u);
      int b = upto ? e0 + 31 - __builtin_clz(upto) : prv;
      if (b < 0) b = 0;
      tt[r] = (double(s32[r]) - G[b]) * R.inv_lambda;
    }
  }
  __builtin_amdgcn_wave_barrier();

  // ---- outputs: y = sign o grad r*(s - v), dy = sign o hess r*(s - v) (tau - d gamma) ------------
  {
    const int last = hm ? e0 + 31 - __builtin_clz(hm) : -1;
    const int prv = lanes_before_max<GL>(last, lr, -1);
    float dv[E];
    uint32_t orig[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const uint32_t upto = hm & ((2u << r) - 1u);
      int b = upto ? e0 + 31 - __builtin_clz(upto) : prv;
      if (b < 0) b = 0;                                    // padding of an empty tail
      const bool neg = MAG && (field[r] & 1u);
      orig[r] = MAG ? (field[r] >> 1) : field[r];
      float y = float(CUBIC ? tt[r] * tt[r] * tt[r] : tt[r]);
      if (MAG) y = (y == 0.0f || s32[r] == 0.0f) ? 0.0f : (neg ? -y : y);
      yv[r] = y;
      dv[r] = 0.0f;
      if (jvp != nullptr) {
        const double h = CUBIC ? 3.0 * tt[r] * tt[r] * R.inv_lambda : R.inv_lambda;
        float dy = float(h * (double(ltau[e0 + r]) - DG[b]));
        if (MAG) dy = (dy == 0.0f || s32[r] == 0.0f) ? 0.0f : (neg ? -dy : dy);
        dv[r] = dy;
      }
    }
    __builtin_amdgcn_wave_barrier();             // lw and G's place are free: everything was read
#pragma unroll
    for (int r = 0; r < E; ++r) {
      if (e0 + r >= n) continue;
      if (out != nullptr) lw[orig[r]] = yv[r];
      if (jvp != nullptr) lt[orig[r]] = dv[r];
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (!valid) return;
  if (out != nullptr) {
    float ov[E];
#pragma unroll
    for (int r = 0; r < E; ++r) ov[r] = lw[e0 + r];
    store_elems<E, false>(out, base, e0, n, ov);
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
                         hipStream_t st, int max_rounds) {
#define TOPK_GENERAL_CALL(MAGV, PCV)                                                            \
  do {                                                                                          \
    using C = GenCfg<GL, E, PCV == kP43>;                                                       \
    const int64_t waves = (rows + C::RPW - 1) / C::RPW;                                         \
    const int64_t blocks = (waves + C::WPB - 1) / C::WPB;                                       \
    if (blocks > 0x7fffffffLL) return -1;                                                       \
    hipLaunchKernelGGL((general_rows_kernel<GL, E, MAGV, PCV>), dim3((unsigned)blocks),          \
                       dim3(C::WPB * kWave), 0, st, x, w, w_stride, t, out, jvp, rows, n, R,   \
                       max_rounds);                                                             \
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
  // Rounds before the hand-over to the sequential walk.  A round costs about as much as four
  // steps of the walk for p = 2; for p = 4/3 every step of the walk solves a cubic, and the rounds
  // (n - 1 of them at most: each removes a boundary) always win.
  const int forced = routes().general_rounds;            // test control
  const int max_rounds = forced > 0 ? forced : (pc == kP43 ? n + 1 : kMinRounds + n / 4);
#define CALL(GL, E) \
  launch_general_shape<GL, E>(mag, pc, x, w, w_stride, tangent, out, jvp, rows, n, R, st, max_rounds)
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
