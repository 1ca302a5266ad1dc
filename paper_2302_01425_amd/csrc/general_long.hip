// General weights (Sec. 4 with a general non-increasing w; App. "PAV algorithm"), rows of
// 1025 .. kGeneralLongMax elements: after a complete sort of the row (radix_sort.hip; sorted keys
// and the index payload in the scratch arrays), ONE workgroup per row builds the PAV partition in
// the same merging rounds as the short-row kernel (general_w.hip), with
//   * the float64 prefix sums of (s, w [, s^2, s^3]) and the per-block values in global scratch
//     (a row of 131072 elements needs 5 MB of them: they stay in the L2),
//   * every thread owning SEG = ceil(n / 1024) consecutive sorted positions, the block starts among
//     them as a 128-bit mask in registers,
//   * the "first block start after my positions" / "last one before" of a round from a
//     suffix-minimum / prefix-maximum over the 1024 threads.
// The strict test, the legality of removing all violating boundaries at once and the hand-over to
// the sequential block stack (thread 0) are those of general_w.hip.  The outputs are scattered
// through the sort's index payload.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "general_pav.hpp"

namespace topk {
namespace {

constexpr int kGT = 1024;                      // threads of the workgroup
constexpr int kGW = kGT / kWave;               // wavefronts
constexpr uint32_t kHiBits = 18;               // block ends are kept in 18 bits, a round stamp above
constexpr uint32_t kHiMask = (1u << kHiBits) - 1u;
static_assert(kGeneralLongMax < (1 << kHiBits) - 1, "block ends must fit their bit field");
static_assert(kGeneralLongMax <= 128 * kGT, "a thread keeps its block starts in 128 bits");

struct Mask128 {
  unsigned long long lo, hi;
};
__device__ __forceinline__ int mask_first(const Mask128& m) {
  if (m.lo) return __builtin_ctzll(m.lo);
  if (m.hi) return 64 + __builtin_ctzll(m.hi);
  return -1;
}
__device__ __forceinline__ int mask_last(const Mask128& m) {
  if (m.hi) return 127 - __builtin_clzll(m.hi);
  if (m.lo) return 63 - __builtin_clzll(m.lo);
  return -1;
}
// smallest set bit above j / largest set bit below j, -1 when there is none
__device__ __forceinline__ int mask_next(const Mask128& m, int j) {
  const unsigned long long a = j < 63 ? (m.lo & (~0ull << (j + 1))) : 0ull;
  if (a) return __builtin_ctzll(a);
  const unsigned long long b = j < 64 ? m.hi : (j < 127 ? (m.hi & (~0ull << (j - 63))) : 0ull);
  if (b) return 64 + __builtin_ctzll(b);
  return -1;
}
__device__ __forceinline__ int mask_prev(const Mask128& m, int j) {
  const unsigned long long b = j > 64 ? (m.hi & ((1ull << (j - 64)) - 1ull)) : 0ull;
  if (b) return 127 - __builtin_clzll(b);
  const unsigned long long a = j >= 64 ? m.lo : (j > 0 ? (m.lo & ((1ull << j) - 1ull)) : 0ull);
  if (a) return 63 - __builtin_clzll(a);
  return -1;
}
__device__ __forceinline__ void mask_clear(Mask128& m, int j) {
  if (j < 64) m.lo &= ~(1ull << j);
  else m.hi &= ~(1ull << (j - 64));
}
__device__ __forceinline__ bool mask_test(const Mask128& m, int j) {
  return j < 64 ? ((m.lo >> j) & 1ull) != 0 : ((m.hi >> (j - 64)) & 1ull) != 0;
}

// A prefix sum over 131072 values is five orders of magnitude larger than the sum over a small
// block, which is the difference of two of them: in plain float64 that difference would carry the
// rounding of the large numbers (1e-9 where the block's cubic needs 1e-13 to decide near-ties as
// the direct summation does).  So the prefix sums are kept as unevaluated pairs h + l (h the
// rounded sum, l its error), added with the error-free two-sum, and a block's sum is
// (h_hi - h_lo) + (l_hi - l_lo).
__device__ __forceinline__ DD dd_add(const DD& a, const DD& b) {
  const double s = a.h + b.h;
  const double bb = s - a.h;
  double e = (a.h - (s - bb)) + (b.h - bb);
  e += a.l + b.l;
  const double h = s + e;
  return DD{h, e - (h - s)};
}
__device__ __forceinline__ DD dd_add(const DD& a, double b) { return dd_add(a, DD{b, 0.0}); }
__device__ __forceinline__ double dd_diff(const DD& hi, const DD& lo) {
  return (hi.h - lo.h) + (hi.l - lo.l);
}

struct ScanShared {
  DD d[4][kGW];
  double q[2][kGW];
  int first[kGW], last[kGW];
};

// exclusive prefix sum over the threads of the workgroup (one value per thread)
__device__ __forceinline__ DD block_exclusive_scan(const DD& v, DD* wave_tot) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  DD inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const DD o{__shfl_up(inc.h, off, kWave), __shfl_up(inc.l, off, kWave)};
    if (lane >= off) inc = dd_add(o, inc);
  }
  DD prev{__shfl_up(inc.h, 1, kWave), __shfl_up(inc.l, 1, kWave)};
  if (lane == 0) prev = DD{0.0, 0.0};
  if (lane == kWave - 1) wave_tot[w] = inc;
  __syncthreads();
  DD before{0.0, 0.0};
#pragma unroll
  for (int q = 0; q < kGW; ++q)
    if (q < w) before = dd_add(before, wave_tot[q]);
  __syncthreads();
  return dd_add(before, prev);
}
__device__ __forceinline__ double block_exclusive_scan(double v, double* wave_tot) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  double inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const double o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  if (lane == kWave - 1) wave_tot[w] = inc;
  __syncthreads();
  double before = 0.0;
#pragma unroll
  for (int q = 0; q < kGW; ++q)
    if (q < w) before += wave_tot[q];
  __syncthreads();
  return before + inc - v;
}

// first block start in the threads after this one (n when there is none) and last block start in
// the threads before it (-1 when there is none), from each thread's own first / last
__device__ __forceinline__ void block_neighbours(int first, int last, int n, ScanShared& sm,
                                                 int* nxt, int* prv) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  int mn = first, mx = last;                  // inclusive suffix minimum / prefix maximum
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int a = __shfl_down(mn, off, kWave);
    const int b = __shfl_up(mx, off, kWave);
    if (lane + off < kWave) mn = min(mn, a);
    if (lane >= off) mx = max(mx, b);
  }
  if (lane == 0) sm.first[w] = mn;
  if (lane == kWave - 1) sm.last[w] = mx;
  const int mn1 = __shfl_down(mn, 1, kWave), mx1 = __shfl_up(mx, 1, kWave);
  __syncthreads();
  int after = n, before = -1;
#pragma unroll
  for (int q = 0; q < kGW; ++q) {
    if (q > w) after = min(after, sm.first[q]);
    if (q < w) before = max(before, sm.last[q]);
  }
  *nxt = lane + 1 < kWave ? min(mn1, after) : after;
  *prv = lane >= 1 ? max(mx1, before) : before;
  __syncthreads();
}

template <bool MAG, int PC>
__global__ __launch_bounds__(kGT) void general_long_kernel(
    uint32_t* keys_all, const uint32_t* __restrict__ idx_all, const float* __restrict__ x_all,
    const float* __restrict__ w_all, int64_t w_stride, const float* __restrict__ tangent_all,
    float* __restrict__ out_all, float* __restrict__ jvp_all, GeneralBuffers gb, int n, Reg R,
    int max_rounds) {
  constexpr bool CUBIC = (PC == kP43);
  __shared__ ScanShared sm;
  const int64_t row = blockIdx.x;
  const int64_t base = row * int64_t(n);
  const int64_t qbase = row * int64_t(n + 1);
  const int t = threadIdx.x;
  const int seg = (n + kGT - 1) / kGT;         // sorted positions per thread (at most 128)
  const int p0 = t * seg;
  const int own = max(0, min(seg, n - p0));    // my positions: p0 .. p0 + own - 1
  float* ss = reinterpret_cast<float*>(keys_all + base);   // keys now, sorted values from step 1 on
  const uint32_t* keys = keys_all + base;
  const uint32_t* idx = idx_all + base;
  const float* lw = w_all + row * w_stride;    // weights by sorted position
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
  DD* P1 = gb.p1 + qbase;                      // prefix sums, P[i] = sum over sorted positions j < i
  DD* PW = gb.pw + qbase;
  DD* P2 = CUBIC ? gb.p2 + qbase : nullptr;
  DD* P3 = CUBIC ? gb.p3 + qbase : nullptr;
  // after the rounds the same memory holds plain float64 arrays: prefix sums of c_j tau_j and c_j
  // (Prop. 7), and the columns of the sequential walk's stack
  double* Q1 = reinterpret_cast<double*>(P1);
  double* Q2 = CUBIC ? reinterpret_cast<double*>(P2) : nullptr;
  double* QW = reinterpret_cast<double*>(PW);
  double* Q3 = CUBIC ? reinterpret_cast<double*>(P3) : nullptr;
  double* G = gb.g + qbase;                    // pooled value by block start
  double* DG = gb.dg + qbase;                  // d gamma by block start
  uint32_t* hi_of = gb.hi_of + base;           // (round stamp, end of the block G[lo] was computed for)
  float* ltau = gb.ltau + base;                // tangent in sorted coordinates

  // ---- 1. prefix sums; keys -> values; tangent into sorted coordinates ----------------------------
  {
    DD t1{0.0, 0.0}, tw{0.0, 0.0}, t2{0.0, 0.0}, t3{0.0, 0.0};
    for (int j = 0; j < own; ++j) {
      const double sd = double(key_to_float(keys[p0 + j])), wd = double(lw[p0 + j]);
      t1 = dd_add(t1, sd);
      tw = dd_add(tw, wd);
      if (CUBIC) { t2 = dd_add(t2, sd * sd); t3 = dd_add(t3, sd * sd * sd); }
    }
    DD r1 = block_exclusive_scan(t1, sm.d[0]), rw = block_exclusive_scan(tw, sm.d[1]);
    DD r2{0.0, 0.0}, r3{0.0, 0.0};
    if (CUBIC) { r2 = block_exclusive_scan(t2, sm.d[2]); r3 = block_exclusive_scan(t3, sm.d[3]); }
    for (int j = 0; j < own; ++j) {
      const int pos = p0 + j;
      const float sv = key_to_float(keys[pos]);
      P1[pos] = r1;
      PW[pos] = rw;
      if (CUBIC) { P2[pos] = r2; P3[pos] = r3; }
      const double sd = double(sv), wd = double(lw[pos]);
      r1 = dd_add(r1, sd);
      rw = dd_add(rw, wd);
      if (CUBIC) { r2 = dd_add(r2, sd * sd); r3 = dd_add(r3, sd * sd * sd); }
      ss[pos] = sv;
      if (jvp != nullptr) {
        const uint32_t id = idx[pos];
        float tf = tangent[MAG ? (id >> 1) : id];
        if (MAG) {
          if (id & 1u) tf = -tf;
          if (sv == 0.0f) tf = 0.0f;           // sign(0) = 0
        }
        ltau[pos] = tf;
      }
    }
    if (own > 0 && p0 + own == n) {
      P1[n] = r1;
      PW[n] = rw;
      if (CUBIC) { P2[n] = r2; P3[n] = r3; }
    }
  }
  __syncthreads();

  auto block_sums = [&](int lo, int hi) -> Blk {
    Blk b;
    b.cnt = double(hi - lo);
    b.S2 = b.S3 = 0.0;
    if (hi - lo == 1) {                        // a singleton: its own value and weight, exactly
      b.S1 = double(ss[lo]);
      b.W = double(lw[lo]);
      if (CUBIC) { b.S2 = b.S1 * b.S1; b.S3 = b.S2 * b.S1; }
    } else {
      b.S1 = dd_diff(P1[hi], P1[lo]);
      b.W = dd_diff(PW[hi], PW[lo]);
      if (CUBIC) { b.S2 = dd_diff(P2[hi], P2[lo]); b.S3 = dd_diff(P3[hi], P3[lo]); }
    }
    return b;
  };

  // ---- 2. pool adjacent violators in rounds ----------------------------------------------------------
  Mask128 hm{0ull, 0ull};                      // block starts among my positions (bit j: p0 + j)
  if (own >= 64) {
    hm.lo = ~0ull;
    hm.hi = own >= 128 ? ~0ull : ((1ull << (own - 64)) - 1ull);
  } else {
    hm.lo = (1ull << own) - 1ull;
  }
  bool gave_up = false;
  for (int round = 0;; ++round) {
    const uint32_t stamp = uint32_t(round) & ((1u << (32 - kHiBits)) - 1u);
    const int jf = mask_first(hm), jl = mask_last(hm);
    int nxt, prv;
    block_neighbours(jf >= 0 ? p0 + jf : n, jl >= 0 ? p0 + jl : -1, n, sm, &nxt, &prv);
    // pooled value of every block that is not the one of the last round
    for (int j = jf; j >= 0;) {
      const int jn = mask_next(hm, j);
      const int lo = p0 + j, hi = jn >= 0 ? p0 + jn : nxt;
      if (round == 0 || int(hi_of[lo] & kHiMask) != hi) {
        hi_of[lo] = (stamp << kHiBits) | uint32_t(hi);
        G[lo] = block_gamma<MAG, CUBIC>(block_sums(lo, hi), double(ss[lo]), double(ss[hi - 1]), R);
      }
      j = jn;
    }
    __syncthreads();
    // every boundary whose two blocks violate goes; a boundary between two blocks that are both
    // those of the last round was tested then
    Mask128 keep = hm;
    for (int j = jf; j >= 0;) {
      const int jn = mask_next(hm, j);
      const int lo = p0 + j, hi = jn >= 0 ? p0 + jn : nxt;
      const int jp = mask_prev(hm, j);
      const int p = jp >= 0 ? p0 + jp : prv;
      if (p >= 0 && ((hi_of[p] >> kHiBits) == stamp || (hi_of[lo] >> kHiBits) == stamp)) {
        bool viol;
        if (!CUBIC) viol = G[p] < G[lo];
        else viol = blocks_violate<MAG, CUBIC>(block_sums(p, lo), G[p], block_sums(lo, hi), G[lo], R);
        if (viol) mask_clear(keep, j);
      }
      j = jn;
    }
    const bool changed = keep.lo != hm.lo || keep.hi != hm.hi;
    hm = keep;
    if (!__syncthreads_or(changed)) break;
    if (round + 1 >= max_rounds) { gave_up = true; break; }
  }

  if (gave_up) {
    // ---- too many rounds: the left-to-right block stack, one thread ---------------------------------
    __syncthreads();
    if (t == 0)
      stack_walk<MAG, CUBIC, uint32_t>(n, ss, lw, ltau, jvp != nullptr, Q1, QW, G, Q2, Q3, hi_of,
                                       0xffffffffu, DG, R);
    __syncthreads();
    hm = Mask128{0ull, 0ull};
    for (int j = 0; j < own; ++j)
      if (hi_of[p0 + j] == 0xffffffffu) {
        if (j < 64) hm.lo |= 1ull << j;
        else hm.hi |= 1ull << (j - 64);
      }
  }
  const int jf = mask_first(hm), jl = mask_last(hm);
  int nxt, prv;
  block_neighbours(jf >= 0 ? p0 + jf : n, jl >= 0 ? p0 + jl : -1, n, sm, &nxt, &prv);

  // ---- 2b. p = 4/3: the roots once more, from sums of the blocks' own spread.  The expanded cubic
  // of a block carries the rounding of its values cubed, while a block whose values lie within a
  // small lambda of each other needs that of the spread cubed.  With the partition final, every
  // position is taken relative to the first value c of its own block: plain float64 prefix sums
  // of d = s - c, d^2, d^3 are as small as the blocks are narrow, and the safeguarded Newton solve
  // of the rounds, on sum (g - d_i)^3 + lambda^3 W [c + g] = 0 with the same bracket, gives
  // gamma = c + g to the rounding of the spread ----------------------------------------------------
  if (CUBIC && !gave_up) {
    double t1 = 0.0, t2 = 0.0, t3 = 0.0;
    {
      double c = double(ss[prv >= 0 ? prv : 0]);
      for (int j = 0; j < own; ++j) {
        if (mask_test(hm, j)) c = double(ss[p0 + j]);
        const double d = double(ss[p0 + j]) - c;
        t1 += d;
        t2 += d * d;
        t3 += d * d * d;
      }
    }
    double r1 = block_exclusive_scan(t1, sm.q[0]), r2 = block_exclusive_scan(t2, sm.q[1]);
    double r3 = block_exclusive_scan(t3, sm.q[0]);
    __syncthreads();                           // (the prefix sums of the rounds have been read)
    {
      double c = double(ss[prv >= 0 ? prv : 0]);
      for (int j = 0; j < own; ++j) {
        if (mask_test(hm, j)) c = double(ss[p0 + j]);
        const double d = double(ss[p0 + j]) - c;
        Q1[p0 + j] = r1;
        Q2[p0 + j] = r2;
        Q3[p0 + j] = r3;
        r1 += d;
        r2 += d * d;
        r3 += d * d * d;
      }
      if (own > 0 && p0 + own == n) {
        Q1[n] = r1;
        Q2[n] = r2;
        Q3[n] = r3;
      }
    }
    __syncthreads();
    for (int j = jf; j >= 0;) {
      const int jn = mask_next(hm, j);
      const int lo = p0 + j, hi = jn >= 0 ? p0 + jn : nxt;
      j = jn;
      if (hi - lo == 1) continue;              // (singletons have closed forms)
      const double cnt = double(hi - lo), c = double(ss[lo]);
      const double S1 = Q1[hi] - Q1[lo], S2 = Q2[hi] - Q2[lo], S3 = Q3[hi] - Q3[lo];
      const double W = dd_diff(PW[hi], PW[lo]);
      // the bracket of the first solve, relative to c: [smin - lambda cbrt(W), smax] (mask), [0, smax]
      const double dmin = double(ss[hi - 1]) - c;
      const double g = MAG ? block_root<true>(cnt, W, S1, S2, S3, R, -c, 0.0, c)
                           : block_root<false>(cnt, W, S1, S2, S3, R,
                                               dmin - R.lambda * cbrt(W) - 1e-300, 0.0);
      G[lo] = c + g;
    }
    __syncthreads();
  }

  // ---- 3. Prop. 7: d gamma of every block from prefix sums of c_j tau_j and c_j ------------------------
  if (!gave_up && jvp != nullptr) {
    double tq = 0.0, tc = 0.0;
    {
      int b = prv >= 0 ? prv : 0;
      double g = G[b];
      for (int j = 0; j < own; ++j) {
        if (mask_test(hm, j)) { b = p0 + j; g = G[b]; }
        double c = 1.0;
        if (CUBIC) {
          const double d = g - double(ss[p0 + j]);
          c = MAG ? 3.0 * d * d : d * d;
        }
        tq += c * double(ltau[p0 + j]);
        tc += c;
      }
    }
    double rq = block_exclusive_scan(tq, sm.q[0]);
    double rc = CUBIC ? block_exclusive_scan(tc, sm.q[1]) : 0.0;
    __syncthreads();
    {
      int b = prv >= 0 ? prv : 0;
      double g = G[b];
      for (int j = 0; j < own; ++j) {
        if (mask_test(hm, j)) { b = p0 + j; g = G[b]; }
        double c = 1.0;
        if (CUBIC) {
          const double d = g - double(ss[p0 + j]);
          c = MAG ? 3.0 * d * d : d * d;
        }
        Q1[p0 + j] = rq;                       // (the prefix sums of s and s^2 are not needed any more)
        if (CUBIC) Q2[p0 + j] = rc;
        rq += c * double(ltau[p0 + j]);
        rc += c;
      }
      if (own > 0 && p0 + own == n) {
        Q1[n] = rq;
        if (CUBIC) Q2[n] = rc;
      }
    }
    __syncthreads();
    for (int j = jf; j >= 0;) {
      const int jn = mask_next(hm, j);
      const int lo = p0 + j, hi = jn >= 0 ? p0 + jn : nxt;
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
        const double num = Q1[hi] - Q1[lo];
        double den = CUBIC ? Q2[hi] - Q2[lo] : double(hi - lo);
        if (MAG) den += (CUBIC ? R.lam3 : R.lambda) * dd_diff(PW[hi], PW[lo]);
        dg = num / den;
      }
      DG[lo] = dg;
      j = jn;
    }
  }
  __syncthreads();

  // ---- 4. outputs: y = sign o grad r*(s - v), dy = sign o hess r*(s - v) (tau - d gamma) -----------
  {
    int b = prv >= 0 ? prv : 0;
    double g = G[b], dg = jvp != nullptr ? DG[b] : 0.0;
    for (int j = 0; j < own; ++j) {
      const int pos = p0 + j;
      if (mask_test(hm, j)) {
        b = pos;
        g = G[b];
        if (jvp != nullptr) dg = DG[b];
      }
      const float sv = ss[pos];
      const uint32_t id = idx[pos];
      const bool neg = MAG && (id & 1u);
      const uint32_t orig = MAG ? (id >> 1) : id;
      const double tt = (double(sv) - g) * R.inv_lambda;
      if (out != nullptr) {
        float y = float(CUBIC ? tt * tt * tt : tt);
        if (MAG) y = (y == 0.0f || sv == 0.0f) ? 0.0f : (neg ? -y : y);
        out[orig] = y;
      }
      if (jvp != nullptr) {
        const double h = CUBIC ? 3.0 * tt * tt * R.inv_lambda : R.inv_lambda;
        float dy = float(h * (double(ltau[pos]) - dg));
        if (MAG) dy = (dy == 0.0f || sv == 0.0f) ? 0.0f : (neg ? -dy : dy);
        jvp[orig] = dy;
      }
    }
  }
}

}  // namespace

size_t general_long_bytes(int64_t rows, int64_t n, int pc) {
  const size_t q = size_t(rows) * size_t(n + 1) * 8, e = size_t(rows) * size_t(n) * 4;
  auto up = [](size_t v) { return (v + 255) & ~size_t(255); };
  return (pc == kP43 ? 4 : 2) * up(2 * q) + 2 * up(q) + 2 * up(e);
}

GeneralBuffers general_long_carve(void* ptr, int64_t rows, int64_t n, int pc) {
  const size_t q = size_t(rows) * size_t(n + 1) * 8, e = size_t(rows) * size_t(n) * 4;
  auto up = [](size_t v) { return (v + 255) & ~size_t(255); };
  char* c = static_cast<char*>(ptr);
  GeneralBuffers gb{};
  gb.p1 = reinterpret_cast<DD*>(c); c += up(2 * q);
  gb.pw = reinterpret_cast<DD*>(c); c += up(2 * q);
  gb.g = reinterpret_cast<double*>(c); c += up(q);
  gb.dg = reinterpret_cast<double*>(c); c += up(q);
  if (pc == kP43) {
    gb.p2 = reinterpret_cast<DD*>(c); c += up(2 * q);
    gb.p3 = reinterpret_cast<DD*>(c); c += up(2 * q);
  }
  gb.hi_of = reinterpret_cast<uint32_t*>(c); c += up(e);
  gb.ltau = reinterpret_cast<float*>(c);
  return gb;
}

// The rows are sorted already: B.keys_a holds the sorted keys (overwritten with the sorted values),
// B.idx_a the index payload (index * 2 + sign bit for the magnitude form).
int launch_general_long(bool mag, int pc, const SortBuffers& B, const GeneralBuffers& gb,
                        const float* x, const float* w, int64_t w_stride, const float* tangent,
                        float* out, float* jvp, int64_t rows, int64_t n, const Reg& R,
                        hipStream_t st) {
  if (n <= 1024 || n > kGeneralLongMax || rows > 0x7fffffffLL) return -1;
  const int forced = routes().general_rounds;          // test control
  const int max_rounds = forced > 0 ? forced : (pc == kP43 ? int(n) + 1 : 32 + int(n) / 4);
#define TOPK_GENERAL_LONG(M, P)                                                                   \
  hipLaunchKernelGGL((general_long_kernel<M, P>), dim3(unsigned(rows)), dim3(kGT), 0, st, B.keys_a, \
                     B.idx_a, x, w, w_stride, tangent, out, jvp, gb, int(n), R, max_rounds)
  if (!mag && pc == kP2) TOPK_GENERAL_LONG(false, kP2);
  else if (!mag && pc == kP43) TOPK_GENERAL_LONG(false, kP43);
  else if (mag && pc == kP2) TOPK_GENERAL_LONG(true, kP2);
  else if (mag && pc == kP43) TOPK_GENERAL_LONG(true, kP43);
  else return -1;
#undef TOPK_GENERAL_LONG
  return 0;
}

}  // namespace topk
