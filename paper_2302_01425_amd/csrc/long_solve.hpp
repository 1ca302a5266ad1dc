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

namespace topk {

struct Acc {
  double s1, s2, s3;
  int c;
};

template <int NT>
struct GrowShared {
  Sums wave_r[NT / kWave], wave_l[NT / kWave];   // wavefront totals of the scans
  int first_r[NT / kWave], first_l[NT / kWave];  // leading accepted run inside each wavefront
  Sums take_r, take_l;                           // sums of the accepted runs
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
  GrowShared<NT> grow;
  GrowShared<kWave> grow1;
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

// Block growth by W = 1 wavefront or by the whole workgroup of NT threads (W = NT / 64), both
// sides per step, 2 sorted positions per thread, side and step (thread t looks at positions 2t
// and 2t+1 of each side's traversal, counted from the block outwards).
//
// Per step: inclusive scans of the float64 power sums over the traversal give every position the
// sums of its side's positions before it; the strict-violation tests of pooling.hpp are evaluated
// for all positions at once; each side takes its leading run of accepted positions (the tests are
// monotone along the traversal), and the sums of that run are read off the scan.  Accepting both
// sides' runs in the same step is valid because additions on one side only make the other
// side's tests more true.
//
// Returns true when neither side can grow any further.  With `max_steps` > 0 it gives up (false)
// after that many steps, or after three steps that took a whole chunk on one side: the block is
// large, and the caller continues with the whole workgroup from the state left in a, b, S.
// W = 1: called by the 64 lanes of one wavefront, no barriers; else by all NT threads.
template <int NT, bool MAG, int PC>
__device__ __forceinline__ bool grow_block(const uint32_t* __restrict__ skeys, int64_t n, int64_t k, double center,
                           const Reg& R, int64_t& a, int64_t& b, Sums& S, int max_steps,
                           GrowShared<NT>& gs) {
  using P = Pool<MAG, PC>;
  constexpr bool CUBIC = (PC == kP43);
  constexpr int W = NT / kWave;
  constexpr int kSide = 2 * NT;                  // positions per side and step
  const int lane = threadIdx.x & (kWave - 1);
  const int w = (W == 1) ? 0 : int(threadIdx.x) / kWave;
  const int t = (W == 1) ? lane : int(threadIdx.x);
  int full_steps = 0;
  for (int step = 0; max_steps <= 0 || (step < max_steps && full_steps < 3); ++step) {
    const int64_t rem_r = n - b, rem_l = a - 1;
    double dr[2], dl[2];
    bool vr[2], vl[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t q = 2 * t + i;
      vr[i] = q < rem_r;
      vl[i] = q < rem_l;
      dr[i] = vr[i] ? double(key_to_float(skeys[b + q])) - center : 0.0;          // position b+1+q
      dl[i] = vl[i] ? double(key_to_float(skeys[a - 2 - q])) - center : 0.0;      // position a-1-q
    }
    // inclusive scans of the thread totals
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
    if constexpr (W > 1) {
      __syncthreads();                           // the previous step's readers are done
      if (lane == kWave - 1) {
        gs.wave_r[w] = ir;
        gs.wave_l[w] = il;
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < W; ++q) {
        if (q < w) {
          const Sums tr = gs.wave_r[q], tl = gs.wave_l[q];
          ir.s1 += tr.s1; il.s1 += tl.s1;
          if (CUBIC) { ir.s2 += tr.s2; ir.s3 += tr.s3; il.s2 += tl.s2; il.s3 += tl.s3; }
        }
      }
    }
    // sums of this side's positions before position 2t + j  =  inclusive scan - tail[j], where
    // tail[0] = both positions of this thread, tail[1] = the second one, tail[2] = nothing
    // (plain variables and selects: indexable arrays would end up in scratch memory)
    const Sums tr0{dr[0] + dr[1], dr[0] * dr[0] + dr[1] * dr[1],
                   dr[0] * dr[0] * dr[0] + dr[1] * dr[1] * dr[1]};
    const Sums tr1{dr[1], dr[1] * dr[1], dr[1] * dr[1] * dr[1]};
    const Sums tl0{dl[0] + dl[1], dl[0] * dl[0] + dl[1] * dl[1],
                   dl[0] * dl[0] * dl[0] + dl[1] * dl[1] * dl[1]};
    const Sums tl1{dl[1], dl[1] * dl[1], dl[1] * dl[1] * dl[1]};
    const double cnt0 = double(b - a + 1), m0 = double(k - a + 1);
    unsigned long long okr[2], okl[2];
    {
      const double q = double(2 * t);
      const Sums run_r{S.s1 + (ir.s1 - tr0.s1), S.s2 + (ir.s2 - tr0.s2), S.s3 + (ir.s3 - tr0.s3)};
      const Sums run_l{S.s1 + (il.s1 - tl0.s1), S.s2 + (il.s2 - tl0.s2), S.s3 + (il.s3 - tl0.s3)};
      okr[0] = __ballot(vr[0] & P::right_violates(dr[0], cnt0 + q, m0, run_r, R, center));
      okl[0] = __ballot(vl[0] & P::left_violates(dl[0], cnt0 + q, m0 + q, run_l, R, center));
    }
    {
      const double q = double(2 * t + 1);
      const Sums run_r{S.s1 + (ir.s1 - tr1.s1), S.s2 + (ir.s2 - tr1.s2), S.s3 + (ir.s3 - tr1.s3)};
      const Sums run_l{S.s1 + (il.s1 - tl1.s1), S.s2 + (il.s2 - tl1.s2), S.s3 + (il.s3 - tl1.s3)};
      okr[1] = __ballot(vr[1] & P::right_violates(dr[1], cnt0 + q, m0, run_r, R, center));
      okl[1] = __ballot(vl[1] & P::left_violates(dl[1], cnt0 + q, m0 + q, run_l, R, center));
    }
    // length of the leading run of accepted positions of this wavefront's 128 positions
    auto leading = [](unsigned long long ok0, unsigned long long ok1) -> int {
      const int f0 = (~ok0 == 0ull) ? 128 : 2 * (__ffsll((long long)~ok0) - 1);
      const int f1 = (~ok1 == 0ull) ? 128 : 2 * (__ffsll((long long)~ok1) - 1) + 1;
      return f0 < f1 ? f0 : f1;
    };
    int nr = leading(okr[0], okr[1]);
    int nl = leading(okl[0], okl[1]);
    if constexpr (W > 1) {
      if (lane == 0) {
        gs.first_r[w] = nr;
        gs.first_l[w] = nl;
      }
      __syncthreads();
      // the run of the workgroup ends in the first wavefront whose own run is not complete
      int tot_r = kSide, tot_l = kSide;
#pragma unroll
      for (int q = W - 1; q >= 0; --q) {
        if (gs.first_r[q] < 128) tot_r = q * 128 + gs.first_r[q];
        if (gs.first_l[q] < 128) tot_l = q * 128 + gs.first_l[q];
      }
      nr = tot_r;
      nl = tot_l;
    }
    if (nr == 0 && nl == 0) return true;
    // sums of the first nr (nl) positions: those before position nr, held by thread nr/2 with
    // j = nr%2 (a whole chunk: the last thread's inclusive value)
    const int src_r = nr >= kSide ? NT - 1 : (nr >> 1), jr = nr >= kSide ? 2 : (nr & 1);
    const int src_l = nl >= kSide ? NT - 1 : (nl >> 1), jl = nl >= kSide ? 2 : (nl & 1);
    auto before = [](const Sums& inc, const Sums& t0, const Sums& t1, int j) -> Sums {
      const double c1 = j == 0 ? t0.s1 : (j == 1 ? t1.s1 : 0.0);
      const double c2 = j == 0 ? t0.s2 : (j == 1 ? t1.s2 : 0.0);
      const double c3 = j == 0 ? t0.s3 : (j == 1 ? t1.s3 : 0.0);
      return Sums{inc.s1 - c1, inc.s2 - c2, inc.s3 - c3};
    };
    const Sums mine_r = before(ir, tr0, tr1, jr), mine_l = before(il, tl0, tl1, jl);
    Sums ar, al;
    if constexpr (W == 1) {
      ar.s1 = readlane_f64(mine_r.s1, src_r);
      al.s1 = readlane_f64(mine_l.s1, src_l);
      ar.s2 = CUBIC ? readlane_f64(mine_r.s2, src_r) : 0.0;
      ar.s3 = CUBIC ? readlane_f64(mine_r.s3, src_r) : 0.0;
      al.s2 = CUBIC ? readlane_f64(mine_l.s2, src_l) : 0.0;
      al.s3 = CUBIC ? readlane_f64(mine_l.s3, src_l) : 0.0;
    } else {
      if (t == src_r) gs.take_r = mine_r;
      if (t == src_l) gs.take_l = mine_l;
      __syncthreads();
      ar = gs.take_r;
      al = gs.take_l;
    }
    S.s1 += ar.s1 + al.s1;
    S.s2 += ar.s2 + al.s2;
    S.s3 += ar.s3 + al.s3;
    b += nr;
    a -= nl;
    if (nr == kSide || nl == kSide) ++full_steps;
  }
  return false;
}

template <int NT>
struct RowSolver {
  static constexpr int kWaves = NT / kWave;
  static constexpr int kPer = 4;
  static constexpr int kChunk = NT * kPer;

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
  // VALUE_ONLY: the caller computes the outputs from values (thresholds hi_incl, lo_incl) and adds
  // up the tangent itself: no index payload is read and the tie runs are not counted (wa, wb are
  // then just a, b).
  template <bool MAG, int PC, bool VALUE_ONLY = false>
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
      if (P::kCentered) center = sk;
      const double dk = sk - center, dk1 = sk1 - center;
      grow = P::seed_violates(dk, dk1, R, center);
      if (grow) {
        a = k;
        b = k + 1;
        Sums S{dk + dk1, dk * dk + dk1 * dk1, dk * dk * dk + dk1 * dk1 * dk1};
        // small blocks (the common case) are finished by the first wavefront alone, in short
        // steps without barriers; blocks that are still growing after that continue with
        // sweeps of the whole workgroup
        if (threadIdx.x < kWave) {
          const bool done = grow_block<kWave, MAG, PC>(skeys, n, k, center, R, a, b, S, 12, sm.grow1);
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
        if (sm.hand.done == 0) grow_block<NT, MAG, PC>(skeys, n, k, center, R, a, b, S, 0, sm.grow);
        const double da = double(key_to_float(skeys[a - 1])) - center;
        const double db = double(key_to_float(skeys[b - 1])) - center;
        // bracket of the pooled value: above the singleton minimiser of position a (mask:
        // s_a - lambda; magnitude: at least 0), below s_b (magnitude: below s_a)
        gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, MAG ? -center : da - R.lambda,
                          MAG ? da : db, center);
      }
    }
    if (!VALUE_ONLY && grow && tangent != nullptr) {
      // Prop. 7: d gamma = sum_B c_j tau_j / (sum_B c_j [+ lambda m]),  c_j = |gamma - s_j|^(q-2)
      Acc acc{0.0, 0.0, 0.0, 0};
      for (int64_t p0 = a + threadIdx.x; p0 <= b; p0 += 4 * NT) {
        uint32_t id[4];
        float sv[4], tv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int64_t pos1 = p0 + int64_t(i) * NT;
          id[i] = pos1 <= b ? sidx[pos1 - 1] : 0u;
          sv[i] = pos1 <= b ? key_to_float(skeys[pos1 - 1]) : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          tv[i] = (p0 + int64_t(i) * NT <= b) ? tangent[MAG ? (id[i] >> 1) : id[i]] : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (p0 + int64_t(i) * NT > b) continue;
          double t = double(tv[i]);
          if (MAG) {
            if (id[i] & 1u) t = -t;
            if (sv[i] == 0.0f) t = 0.0;
          }
          const double w = P::jac_weight(double(sv[i]) - center, gamma);
          acc.s1 += w * t;
          acc.s2 += w;
        }
      }
      const Acc got = sum_acc(acc, sm.acc);
      dgamma = got.s1 / P::jac_denominator(got.s2, double(k - a + 1), R);
    }
    // ---- value window of the block, widened over ties at both ends -----------------------------
    RowInfo ri;
    ri.src = 0;
    ri.pad = 0;
    ri.a = a;
    ri.b = b;
    ri.gamma = gamma;
    ri.center = center;
    ri.dgamma = dgamma;
    if (grow) {
      const uint32_t key_a = skeys[a - 1], key_b = skeys[b - 1];
      ri.hi_incl = key_to_float(key_a);
      ri.lo_incl = key_to_float(key_b);
      ri.wa = VALUE_ONLY ? a : a - count_equal_run<false>(skeys, n, a - 1, key_a, sm);
      ri.wb = VALUE_ONLY ? b : b + count_equal_run<true>(skeys, n, b + 1, key_b, sm);
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
    double y = before ? P::above(v, R, ri.center) : P::y_in_block(v, ri.gamma, R);
    if (after) y = 0.0;
    const float yf = float(y);
    out[o] = (MAG && yf == 0.0f) ? 0.0f : (neg ? -yf : yf);
  }
  if (jvp != nullptr) {
    double t = double(tangent[o]);
    if (neg) t = -t;
    if (MAG && sv == 0.0f) t = 0.0;
    double dy = before ? P::above_slope(v, R, ri.center) * t
                       : P::hess(v, ri.gamma, R) * (t - ri.dgamma);
    if (after) dy = 0.0;
    float df = float(dy);
    if (MAG && sv == 0.0f) df = 0.0f;
    jvp[o] = (df == 0.0f) ? 0.0f : (neg ? -df : df);
  }
}

// Dense part of the output for one element outside the value window of the block:
// mask: 1 above, 0 below; magnitude: the element's own singleton solution above (x/(1+lambda)
// for p = 2, sign(x) times the root of the one-element cubic for p = 4/3), 0 below; JVP 0 resp.
// the slope of that solution times the tangent.
// Returns false (and writes nothing) for an element inside the window.
template <bool MAG, int PC>
__device__ __forceinline__ bool emit_dense_element(const RowInfo& ri, float xv, int64_t e,
                                                   const float* __restrict__ tangent,
                                                   float* __restrict__ out, float* __restrict__ jvp,
                                                   const Reg& R) {
  using P = Pool<MAG, PC>;
  const bool empty = ri.wa > ri.wb;
  const float v = MAG ? fabsf(xv) : xv;
  // empty window: hi_incl = s_{k+1} < lo_incl = s_k, every value is > hi or < lo
  const bool above = v > ri.hi_incl;
  const bool below = v < ri.lo_incl;
  if (!empty && !above && !below) return false;
  // dense outputs are written once and the tangent is read once: streaming accesses
  if constexpr (MAG && PC == kP43) {
    float y = 0.0f, d = 0.0f;
    if (above && xv != 0.0f) {
      double g, slope;
      P::above_both(double(v), R, 0.0, &g, &slope);
      y = float(xv < 0.0f ? -g : g);
      if (jvp != nullptr) d = float(slope * double(load_stream(tangent + e)));
    }
    if (out != nullptr) store_stream(out + e, y);
    if (jvp != nullptr) store_stream(jvp + e, d);
  } else {
    const float inv_1pl = float(R.inv_1pl);
    if (out != nullptr) store_stream(out + e, above ? (MAG ? xv * inv_1pl : 1.0f) : 0.0f);
    if (jvp != nullptr) {
      float d = 0.0f;
      if (MAG && above && xv != 0.0f) d = load_stream(tangent + e) * inv_1pl;
      store_stream(jvp + e, d);
    }
  }
  return true;
}

}  // namespace topk
