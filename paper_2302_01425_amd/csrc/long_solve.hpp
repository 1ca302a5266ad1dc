// Isotonic solve of one long row by one workgroup of NT threads, on the row's sorted keys (or
// on its sorted candidate list) in global memory.
//
// The single pooled block [a, b] grows outwards from (k, k+1) in chunks of 4*NT sorted positions
// per side: a block-wide exclusive scan of the float64 power sums (centred on s_k for the mask)
// gives every position the block "up to me", the monotone strict-violation tests of pooling.hpp
// are evaluated for all positions of the chunk at once, and the sweep stops at the first chunk
// that is not taken entirely.  Then gamma, d gamma (paper Prop. 7) through a gather of the
// tangent, and the value window of the block widened over ties.
#pragma once

#include "common.hpp"
#include "launch.hpp"
#include "pooling.hpp"
#include "wave.hpp"

#ifndef TOPK_SOLVE_MARK
#define TOPK_SOLVE_MARK(i) do { } while (0)
#endif

namespace topk {

struct Acc {
  double s1, s2, s3;
  int c;
};

template <int NT>
struct SolveShared {
  Sums sums[NT / kWave];
  Acc acc[NT / kWave];
  struct {
    int64_t a, b;
    Sums S;
    int done;
  } hand;                 // state of the block after the single-wavefront phase
};

__device__ __forceinline__ double readlane_f64(double v, int src_lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
  return __hiloint2double(hi, lo);
}

// inclusive prefix sum over the 64 lanes of a wavefront: DPP shifts inside the rows of 16 lanes
// (vacated lanes read 0), then the totals of the rows before this one
__device__ __forceinline__ double wave_inclusive_scan_f64(double v) {
  v += row_shr_f64<1>(v);
  v += row_shr_f64<2>(v);
  v += row_shr_f64<4>(v);
  v += row_shr_f64<8>(v);
  const double t0 = readlane_f64(v, 15), t1 = readlane_f64(v, 31), t2 = readlane_f64(v, 47);
  const int row = (threadIdx.x & (kWave - 1)) >> 4;
  double before = 0.0;
  if (row >= 1) before = t0;
  if (row >= 2) before += t1;
  if (row >= 3) before += t2;
  return v + before;
}

// Block growth by ONE wavefront, both sides per step, 128 sorted positions per side and step
// (lane l looks at positions 2l and 2l+1 of each side's traversal).  Tests as in the sweeps
// below; accepting both sides' prefixes in the same step is valid because additions on one side
// only make the other side's tests more true.  Returns true when neither side can grow any
// further, false when `max_steps` steps were not enough (the caller continues with block-wide
// sweeps from the state left in a, b, S).  Called by all 64 lanes of one wavefront; no barriers.
template <bool MAG, int PC>
__device__ bool wave_grow(const uint32_t* __restrict__ skeys, int64_t n, int64_t k, double center,
                          const Reg& R, int64_t& a, int64_t& b, Sums& S, int max_steps) {
  using P = Pool<MAG, PC>;
  constexpr bool CUBIC = (PC == kP43);
  const int lane = threadIdx.x & (kWave - 1);
  for (int step = 0; step < max_steps; ++step) {
    const int64_t rem_r = n - b, rem_l = a - 1;
    double dr[2], dl[2];
    bool vr[2], vl[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t q = 2 * lane + i;
      vr[i] = q < rem_r;
      vl[i] = q < rem_l;
      dr[i] = vr[i] ? double(key_to_float(skeys[b + q])) - center : 0.0;          // position b+1+q
      dl[i] = vl[i] ? double(key_to_float(skeys[a - 2 - q])) - center : 0.0;      // position a-1-q
    }
    // inclusive scans of the lane totals; exclusive prefix of a position = inclusive - what follows
    Sums ir, il;
    ir.s1 = wave_inclusive_scan_f64(dr[0] + dr[1]);
    il.s1 = wave_inclusive_scan_f64(dl[0] + dl[1]);
    ir.s2 = ir.s3 = il.s2 = il.s3 = 0.0;
    if (CUBIC) {
      ir.s2 = wave_inclusive_scan_f64(dr[0] * dr[0] + dr[1] * dr[1]);
      ir.s3 = wave_inclusive_scan_f64(dr[0] * dr[0] * dr[0] + dr[1] * dr[1] * dr[1]);
      il.s2 = wave_inclusive_scan_f64(dl[0] * dl[0] + dl[1] * dl[1]);
      il.s3 = wave_inclusive_scan_f64(dl[0] * dl[0] * dl[0] + dl[1] * dl[1] * dl[1]);
    }
    // prefix[j] = sums of this side's positions before position 2*lane + j, j = 0, 1, 2
    Sums pr[3], pl[3];
    pr[2] = ir;
    pr[1] = Sums{ir.s1 - dr[1], ir.s2 - dr[1] * dr[1], ir.s3 - dr[1] * dr[1] * dr[1]};
    pr[0] = Sums{pr[1].s1 - dr[0], pr[1].s2 - dr[0] * dr[0], pr[1].s3 - dr[0] * dr[0] * dr[0]};
    pl[2] = il;
    pl[1] = Sums{il.s1 - dl[1], il.s2 - dl[1] * dl[1], il.s3 - dl[1] * dl[1] * dl[1]};
    pl[0] = Sums{pl[1].s1 - dl[0], pl[1].s2 - dl[0] * dl[0], pl[1].s3 - dl[0] * dl[0] * dl[0]};
    const double cnt0 = double(b - a + 1), m0 = double(k - a + 1);
    unsigned long long okr[2], okl[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const double q = double(2 * lane + i);
      const Sums run_r{S.s1 + pr[i].s1, S.s2 + pr[i].s2, S.s3 + pr[i].s3};
      const Sums run_l{S.s1 + pl[i].s1, S.s2 + pl[i].s2, S.s3 + pl[i].s3};
      const bool tr = vr[i] & P::right_violates(dr[i], cnt0 + q, m0, run_r, R);
      const bool tl = vl[i] & P::left_violates(dl[i], cnt0 + q, m0 + q, run_l, R);
      okr[i] = __ballot(tr);
      okl[i] = __ballot(tl);
    }
    // length of the leading run of accepted positions in traversal order 0, 1, 2, ...
    auto leading = [](unsigned long long ok0, unsigned long long ok1) -> int {
      const int f0 = (~ok0 == 0ull) ? 128 : 2 * (__ffsll((long long)~ok0) - 1);
      const int f1 = (~ok1 == 0ull) ? 128 : 2 * (__ffsll((long long)~ok1) - 1) + 1;
      return f0 < f1 ? f0 : f1;
    };
    const int nr = leading(okr[0], okr[1]);
    const int nl = leading(okl[0], okl[1]);
    if (nr == 0 && nl == 0) return true;
    // sums of the first nr (nl) positions: prefix[j] of lane nr/2 with j = nr%2 (128: lane 63, j = 2)
    auto take = [&](const Sums (&pre)[3], int cnt) -> Sums {
      const int src = cnt >= 128 ? 63 : (cnt >> 1);
      const int j = cnt >= 128 ? 2 : (cnt & 1);
      Sums pick = pre[0];
      if (j == 1) pick = pre[1];
      if (j == 2) pick = pre[2];
      Sums out;
      out.s1 = readlane_f64(pick.s1, src);
      out.s2 = CUBIC ? readlane_f64(pick.s2, src) : 0.0;
      out.s3 = CUBIC ? readlane_f64(pick.s3, src) : 0.0;
      return out;
    };
    const Sums ar = take(pr, nr), al = take(pl, nl);
    S.s1 += ar.s1 + al.s1;
    S.s2 += ar.s2 + al.s2;
    S.s3 += ar.s3 + al.s3;
    b += nr;
    a -= nl;
  }
  return false;
}

template <int NT>
struct RowSolver {
  static constexpr int kWaves = NT / kWave;
  static constexpr int kPer = 4;
  static constexpr int kChunk = NT * kPer;

  // Block-wide exclusive scan (in thread order) of the power sums.
  template <bool CUBIC>
  __device__ static __forceinline__ Sums exclusive_scan_sums(const Sums& v, Sums* wave_tot) {
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    Sums inc = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const double o1 = __shfl_up(inc.s1, off, kWave);
      const double o2 = CUBIC ? __shfl_up(inc.s2, off, kWave) : 0.0;
      const double o3 = CUBIC ? __shfl_up(inc.s3, off, kWave) : 0.0;
      if (lane >= off) { inc.s1 += o1; inc.s2 += o2; inc.s3 += o3; }
    }
    __syncthreads();
    if (lane == kWave - 1) wave_tot[w] = inc;
    __syncthreads();
    Sums before{0.0, 0.0, 0.0};
    for (int q = 0; q < w; ++q) {
      const Sums t = wave_tot[q];
      before.s1 += t.s1; before.s2 += t.s2; before.s3 += t.s3;
    }
    // exclusive value inside the wave: the inclusive value of the lane before
    double e1 = __shfl_up(inc.s1, 1, kWave);
    double e2 = CUBIC ? __shfl_up(inc.s2, 1, kWave) : 0.0;
    double e3 = CUBIC ? __shfl_up(inc.s3, 1, kWave) : 0.0;
    if (lane == 0) { e1 = 0.0; e2 = 0.0; e3 = 0.0; }
    return Sums{before.s1 + e1, before.s2 + e2, before.s3 + e3};
  }

  // Block-wide sum of (s1, s2, s3, c).
  __device__ static __forceinline__ Acc sum_acc(Acc v, Acc* wave_tot) {
#pragma unroll
    for (int off = kWave >> 1; off >= 1; off >>= 1) {
      v.s1 += __shfl_xor(v.s1, off, kWave);
      v.s2 += __shfl_xor(v.s2, off, kWave);
      v.s3 += __shfl_xor(v.s3, off, kWave);
      v.c += __shfl_xor(v.c, off, kWave);
    }
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) wave_tot[threadIdx.x / kWave] = v;
    __syncthreads();
    Acc r{0.0, 0.0, 0.0, 0};
    for (int q = 0; q < kWaves; ++q) {
      r.s1 += wave_tot[q].s1; r.s2 += wave_tot[q].s2; r.s3 += wave_tot[q].s3; r.c += wave_tot[q].c;
    }
    return r;
  }

  // One sweep in one direction.  Traversal step q visits sorted position (1-based)
  // start + dir*q.  The predicate holds on a prefix of the traversal; the sweep stops at its end.
  // RIGHT: positions > k joining [a, pos-1]; LEFT: positions <= k joining [pos+1, b].
  template <bool MAG, int PC, bool RIGHT>
  __device__ static int64_t sweep(const uint32_t* __restrict__ skeys, int64_t n, int64_t k,
                                  double center, const Reg& R, int64_t& a, int64_t& b, Sums& S,
                                  SolveShared<NT>& sm) {
    using P = Pool<MAG, PC>;
    constexpr bool CUBIC = (PC == kP43);
    int64_t added = 0;
    for (;;) {
      const int64_t start = RIGHT ? b + 1 : a - 1;
      const int64_t remaining = RIGHT ? (n - b) : (a - 1);
      if (remaining <= 0) break;
      double d[kPer];
      bool valid[kPer];
      Sums mine{0.0, 0.0, 0.0};
#pragma unroll
      for (int i = 0; i < kPer; ++i) {
        const int64_t q = int64_t(threadIdx.x) * kPer + i;
        valid[i] = q < remaining;
        const int64_t pos1 = RIGHT ? start + q : start - q;
        d[i] = valid[i] ? double(key_to_float(skeys[pos1 - 1])) - center : 0.0;
        mine.s1 += d[i];
        if (CUBIC) { mine.s2 += d[i] * d[i]; mine.s3 += d[i] * d[i] * d[i]; }
      }
      const Sums ex = exclusive_scan_sums<CUBIC>(mine, sm.sums);
      Acc acc{0.0, 0.0, 0.0, 0};
      Sums run{S.s1 + ex.s1, S.s2 + ex.s2, S.s3 + ex.s3};
#pragma unroll
      for (int i = 0; i < kPer; ++i) {
        const int64_t q = int64_t(threadIdx.x) * kPer + i;
        const int64_t pos1 = RIGHT ? start + q : start - q;
        bool pred = false;
        if (valid[i]) {
          if (RIGHT) pred = P::right_violates(d[i], double(pos1 - a), double(k - a + 1), run, R);
          else pred = P::left_violates(d[i], double(b - pos1), double(k - pos1), run, R);
        }
        if (pred) {
          acc.s1 += d[i];
          if (CUBIC) { acc.s2 += d[i] * d[i]; acc.s3 += d[i] * d[i] * d[i]; }
          acc.c += 1;
        }
        run.s1 += d[i];
        if (CUBIC) { run.s2 += d[i] * d[i]; run.s3 += d[i] * d[i] * d[i]; }
      }
      const Acc got = sum_acc(acc, sm.acc);
      S.s1 += got.s1; S.s2 += got.s2; S.s3 += got.s3;
      if (RIGHT) b += got.c; else a -= got.c;
      added += got.c;
      const int64_t visited = remaining < kChunk ? remaining : kChunk;
      if (got.c < visited) break;
    }
    return added;
  }

  // Length of the run of sorted keys equal to `key` that starts at 1-based position `start` and
  // extends upwards (UP) or downwards, counted by the whole workgroup in chunks.
  template <bool UP>
  __device__ static int64_t count_equal_run(const uint32_t* __restrict__ skeys, int64_t n,
                                            int64_t start, uint32_t key, SolveShared<NT>& sm) {
    int64_t total = 0;
    for (;;) {
      const int64_t from = UP ? start + total : start - total;
      const int64_t remaining = UP ? (n - from + 1) : from;
      if (remaining <= 0) break;
      Acc acc{0.0, 0.0, 0.0, 0};
      // equal keys are contiguous, so counting matches inside the chunk gives the run length
#pragma unroll
      for (int i = 0; i < kPer; ++i) {
        const int64_t q = int64_t(threadIdx.x) * kPer + i;
        if (q < remaining) {
          const int64_t pos1 = UP ? from + q : from - q;
          acc.c += (skeys[pos1 - 1] == key) ? 1 : 0;
        }
      }
      const Acc got = sum_acc(acc, sm.acc);
      total += got.c;
      const int64_t visited = remaining < kChunk ? remaining : kChunk;
      if (got.c < visited) break;
    }
    return total;
  }

  // The whole solve of one row.  skeys/sidx: the n sorted (key, index payload) pairs the block
  // can draw from, k the number of them that belong to the top-k; tangent: the row's tangent in
  // original order, or null.  Every thread returns the same RowInfo (positions relative to
  // skeys).
  template <bool MAG, int PC>
  __device__ static RowInfo solve(const uint32_t* __restrict__ skeys,
                                  const uint32_t* __restrict__ sidx,
                                  const float* __restrict__ tangent, int64_t n, int64_t k,
                                  const Reg& R, SolveShared<NT>& sm) {
    using P = Pool<MAG, PC>;
    int64_t a = k + 1, b = k;
    double gamma = 0.0, center = 0.0, dgamma = 0.0;
    bool grow = false;
    if (k >= 1 && k < n) {
      const double sk = double(key_to_float(skeys[k - 1]));
      const double sk1 = double(key_to_float(skeys[k]));
      if (!MAG) center = sk;
      const double dk = sk - center, dk1 = sk1 - center;
      grow = P::seed_violates(dk, dk1, R);
      TOPK_SOLVE_MARK(7);
      if (grow) {
        a = k;
        b = k + 1;
        Sums S{dk + dk1, dk * dk + dk1 * dk1, dk * dk * dk + dk1 * dk1 * dk1};
        // small blocks (the common case) are finished by the first wavefront alone, in short
        // steps without barriers; blocks that are still growing after that continue with
        // sweeps of the whole workgroup
        if (threadIdx.x < kWave) {
          const bool done = wave_grow<MAG, PC>(skeys, n, k, center, R, a, b, S, 12);
          if (threadIdx.x == 0) {
            sm.hand.a = a;
            sm.hand.b = b;
            sm.hand.S = S;
            sm.hand.done = done ? 1 : 0;
          }
        }
        __syncthreads();
        a = sm.hand.a;
        b = sm.hand.b;
        S = sm.hand.S;
        const bool done = sm.hand.done != 0;
        if (!done) {
          bool first = true;
          for (;;) {
            const int64_t r = sweep<MAG, PC, true>(skeys, n, k, center, R, a, b, S, sm);
            if (r == 0 && !first) break;
            const int64_t l = sweep<MAG, PC, false>(skeys, n, k, center, R, a, b, S, sm);
            if (l == 0) break;
            first = false;
          }
        }
        TOPK_SOLVE_MARK(8);
        const double da = double(key_to_float(skeys[a - 1])) - center;
        const double db = double(key_to_float(skeys[b - 1])) - center;
        gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, da - R.lambda, db);
      }
    }
    TOPK_SOLVE_MARK(9);
    if (grow && tangent != nullptr) {
      // Prop. 7: d gamma = sum_B c_j tau_j / (sum_B c_j [+ lambda m]),  c_j = |gamma - s_j|^(q-2)
      Acc acc{0.0, 0.0, 0.0, 0};
      for (int64_t pos1 = a + threadIdx.x; pos1 <= b; pos1 += NT) {
        const uint32_t key = skeys[pos1 - 1];
        const uint32_t id = sidx[pos1 - 1];
        const float sv = key_to_float(key);
        double t = double(tangent[MAG ? (id >> 1) : id]);
        if (MAG) {
          if (id & 1u) t = -t;
          if (sv == 0.0f) t = 0.0;
        }
        const double w = P::jac_weight(double(sv) - center, gamma);
        acc.s1 += w * t;
        acc.s2 += w;
      }
      const Acc got = sum_acc(acc, sm.acc);
      dgamma = got.s1 / P::jac_denominator(got.s2, double(k - a + 1), R);
    }
    TOPK_SOLVE_MARK(10);
    // ---- value window of the block, widened over ties at both ends -----------------------------
    RowInfo ri;
    ri.a = a;
    ri.b = b;
    ri.gamma = gamma;
    ri.center = center;
    ri.dgamma = dgamma;
    if (grow) {
      const uint32_t key_a = skeys[a - 1], key_b = skeys[b - 1];
      ri.hi_incl = key_to_float(key_a);
      ri.lo_incl = key_to_float(key_b);
      ri.wa = a - count_equal_run<false>(skeys, n, a - 1, key_a, sm);
      ri.wb = b + count_equal_run<true>(skeys, n, b + 1, key_b, sm);
    } else if (k >= 1 && k < n) {
      // no violation: s_k > s_{k+1} strictly; "above hi" = the top k, "below lo" = the rest
      ri.hi_incl = key_to_float(skeys[k]);        // s_{k+1}
      ri.lo_incl = key_to_float(skeys[k - 1]);    // s_k
      ri.wa = k + 1;
      ri.wb = k;
    } else {
      // k == 0: everything is below; k == n: everything is above
      ri.hi_incl = (k == 0) ? __uint_as_float(0x7f800000u) : __uint_as_float(0xff800000u);
      ri.lo_incl = ri.hi_incl;
      ri.wa = k + 1;
      ri.wb = k;
    }
    return ri;
  }
};

// y and dy of sorted position pos1 (value sv, index payload id) given the row's solve; writes
// through the payload's index.  Shared by the window passes of the long and medium rows.
template <bool MAG, int PC>
__device__ __forceinline__ void emit_window_position(const RowInfo& ri, int64_t pos1, float sv,
                                                     uint32_t id, const float* __restrict__ tangent,
                                                     float* __restrict__ out,
                                                     float* __restrict__ jvp, const Reg& R) {
  using P = Pool<MAG, PC>;
  const int64_t o = MAG ? (id >> 1) : id;
  const bool neg = MAG && (id & 1u);
  const double v = double(sv) - ri.center;
  const bool before = pos1 < ri.a, after = pos1 > ri.b;
  if (out != nullptr) {
    double y = before ? (MAG ? v * R.inv_1pl : 1.0) : P::y_in_block(v, ri.gamma, R);
    if (after) y = 0.0;
    const float yf = float(y);
    out[o] = (MAG && yf == 0.0f) ? 0.0f : (neg ? -yf : yf);
  }
  if (jvp != nullptr) {
    double t = double(tangent[o]);
    if (neg) t = -t;
    if (MAG && sv == 0.0f) t = 0.0;
    double dy = before ? (MAG ? t * R.inv_1pl : 0.0) : P::hess(v, ri.gamma, R) * (t - ri.dgamma);
    if (after) dy = 0.0;
    float df = float(dy);
    if (MAG && sv == 0.0f) df = 0.0f;
    jvp[o] = (df == 0.0f) ? 0.0f : (neg ? -df : df);
  }
}

// Dense part of the output for one element outside the value window of the block:
// mask: 1 above, 0 below; magnitude: x/(1+lambda) above, 0 below; JVP 0 resp. t/(1+lambda).
// Returns false (and writes nothing) for an element inside the window.
template <bool MAG>
__device__ __forceinline__ bool emit_dense_element(const RowInfo& ri, float xv, int64_t e,
                                                   const float* __restrict__ tangent,
                                                   float* __restrict__ out, float* __restrict__ jvp,
                                                   float inv_1pl) {
  const bool empty = ri.wa > ri.wb;
  const float v = MAG ? fabsf(xv) : xv;
  // empty window: hi_incl = s_{k+1} < lo_incl = s_k, every value is > hi or < lo
  const bool above = v > ri.hi_incl;
  const bool below = v < ri.lo_incl;
  if (!empty && !above && !below) return false;
  if (out != nullptr) out[e] = above ? (MAG ? xv * inv_1pl : 1.0f) : 0.0f;
  if (jvp != nullptr) {
    float d = 0.0f;
    if (MAG && above && xv != 0.0f) d = tangent[e] * inv_1pl;
    jvp[e] = d;
  }
  return true;
}

}  // namespace topk
