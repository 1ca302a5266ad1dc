// Long rows, after the segmented sort: isotonic solve on the sorted keys, then the sparse
// un-sort scatter and the JVP.
//
//   solve    : one workgroup per row grows the single pooled block [a, b] outwards from (k, k+1)
//              in chunks of 1024 sorted positions, keeping float64 power sums of the block
//              (centred on s_k for the mask); writes (a, b, gamma, d gamma) per row.
//   fill     : dense zero fill of the outputs (everything below the block is exactly 0).
//   epilogue : positions 1..b only: y (and dy) from (a, b, gamma), scattered through sigma.
#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPer = 4;
constexpr int kChunk = kThreads * kPer;

struct Acc {
  double s1, s2, s3;
  int c;
};

// Block-wide exclusive scan (in thread order) of the power sums; `tot` receives the block total.
template <bool CUBIC>
__device__ __forceinline__ Sums block_exclusive_scan_sums(const Sums& v, Sums* wave_tot, Sums* tot) {
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
  Sums before{0.0, 0.0, 0.0}, all{0.0, 0.0, 0.0};
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const Sums t = wave_tot[q];
    if (q < w) { before.s1 += t.s1; before.s2 += t.s2; before.s3 += t.s3; }
    all.s1 += t.s1; all.s2 += t.s2; all.s3 += t.s3;
  }
  *tot = all;
  // exclusive value inside the wave: the inclusive value of the lane before
  double e1 = __shfl_up(inc.s1, 1, kWave);
  double e2 = CUBIC ? __shfl_up(inc.s2, 1, kWave) : 0.0;
  double e3 = CUBIC ? __shfl_up(inc.s3, 1, kWave) : 0.0;
  if (lane == 0) { e1 = 0.0; e2 = 0.0; e3 = 0.0; }
  Sums ex{before.s1 + e1, before.s2 + e2, before.s3 + e3};
  return ex;
}

// Block-wide sum of (s1, s2, s3, c).
__device__ __forceinline__ Acc block_sum_acc(Acc v, Acc* wave_tot) {
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
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    r.s1 += wave_tot[q].s1; r.s2 += wave_tot[q].s2; r.s3 += wave_tot[q].s3; r.c += wave_tot[q].c;
  }
  return r;
}

// One sweep in one direction.  Traversal step q visits sorted position (1-based)
// start + dir*q.  The predicate holds on a prefix of the traversal; the sweep stops at its end.
// RIGHT: positions > k joining [a, pos-1]; LEFT: positions <= k joining [pos+1, b].
template <bool MAG, int PC, bool RIGHT>
__device__ int64_t sweep(const uint32_t* __restrict__ skeys, int64_t n, int64_t k, double center,
                         const Reg& R, int64_t& a, int64_t& b, Sums& S, Sums* sm_sums,
                         Acc* sm_acc) {
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
    Sums tot;
    Sums ex = block_exclusive_scan_sums<CUBIC>(mine, sm_sums, &tot);
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
    const Acc got = block_sum_acc(acc, sm_acc);
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
__device__ int64_t count_equal_run(const uint32_t* __restrict__ skeys, int64_t n, int64_t start,
                                   uint32_t key, Acc* sm_acc) {
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
    const Acc got = block_sum_acc(acc, sm_acc);
    total += got.c;
    const int64_t visited = remaining < kChunk ? remaining : kChunk;
    if (got.c < visited) break;
  }
  return total;
}

template <bool MAG, int PC>
__global__ __launch_bounds__(kThreads) void long_solve_kernel(
    const uint32_t* __restrict__ skeys_all, const uint32_t* __restrict__ sidx_all,
    const float* __restrict__ tangent_all, RowInfo* __restrict__ info, int64_t n, int64_t k,
    Reg R) {
  using P = Pool<MAG, PC>;
  constexpr bool CUBIC = (PC == kP43);
  __shared__ Sums sm_sums[kWaves];
  __shared__ Acc sm_acc[kWaves];
  const int64_t row = blockIdx.x;
  const uint32_t* skeys = skeys_all + row * n;
  const uint32_t* sidx = sidx_all + row * n;

  int64_t a = k + 1, b = k;
  double gamma = 0.0, center = 0.0, dgamma = 0.0;
  bool grow = false;
  if (k >= 1 && k < n) {
    const double sk = double(key_to_float(skeys[k - 1]));
    const double sk1 = double(key_to_float(skeys[k]));
    if (!MAG) center = sk;
    const double dk = sk - center, dk1 = sk1 - center;
    grow = P::seed_violates(dk, dk1, R);
    if (grow) {
      a = k;
      b = k + 1;
      Sums S{dk + dk1, dk * dk + dk1 * dk1, dk * dk * dk + dk1 * dk1 * dk1};
      bool first = true;
      for (;;) {
        const int64_t r = sweep<MAG, PC, true>(skeys, n, k, center, R, a, b, S, sm_sums, sm_acc);
        if (r == 0 && !first) break;
        const int64_t l = sweep<MAG, PC, false>(skeys, n, k, center, R, a, b, S, sm_sums, sm_acc);
        if (l == 0) break;
        first = false;
      }
      const double da = double(key_to_float(skeys[a - 1])) - center;
      const double db = double(key_to_float(skeys[b - 1])) - center;
      gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, da - R.lambda, db);
    }
  }
  if (grow && tangent_all != nullptr) {
    // Prop. 7: d gamma = sum_B c_j tau_j / (sum_B c_j [+ lambda m]),  c_j = |gamma - s_j|^(q-2)
    const float* tangent = tangent_all + row * n;
    Acc acc{0.0, 0.0, 0.0, 0};
    for (int64_t pos1 = a + threadIdx.x; pos1 <= b; pos1 += kThreads) {
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
    const Acc got = block_sum_acc(acc, sm_acc);
    dgamma = got.s1 / P::jac_denominator(got.s2, double(k - a + 1), R);
  }
  // ---- value window of the block, widened over ties at both ends -------------------------------
  int64_t wa = a, wb = b;
  float hi_incl, lo_incl;
  if (grow) {
    const uint32_t key_a = skeys[a - 1], key_b = skeys[b - 1];
    hi_incl = key_to_float(key_a);
    lo_incl = key_to_float(key_b);
    wa = a - count_equal_run<false>(skeys, n, a - 1, key_a, sm_acc);
    wb = b + count_equal_run<true>(skeys, n, b + 1, key_b, sm_acc);
  } else if (k >= 1 && k < n) {
    // no violation: s_k > s_{k+1} strictly; "above hi" = the top k, "below lo" = the rest
    hi_incl = key_to_float(skeys[k]);        // s_{k+1}
    lo_incl = key_to_float(skeys[k - 1]);    // s_k
    wa = k + 1;
    wb = k;
  } else {
    // k == 0: everything is below; k == n: everything is above
    hi_incl = (k == 0) ? __uint_as_float(0x7f800000u) : __uint_as_float(0xff800000u);
    lo_incl = hi_incl;
    wa = k + 1;
    wb = k;
  }
  if (threadIdx.x == 0) {
    RowInfo ri;
    ri.a = a;
    ri.b = b;
    ri.wa = wa;
    ri.wb = wb;
    ri.gamma = gamma;
    ri.center = center;
    ri.dgamma = dgamma;
    ri.hi_incl = hi_incl;
    ri.lo_incl = lo_incl;
    info[row] = ri;
  }
  (void)CUBIC;
}

// Dense pass in original order: everything whose value lies outside the block's value window.
// mask: 1 above, 0 below; magnitude: x/(1+lambda) above, 0 below; JVP 0 resp. t/(1+lambda).
// Elements inside the window are left to long_window_kernel.
template <bool MAG>
__global__ __launch_bounds__(kThreads) void long_dense_kernel(
    const float* __restrict__ x_all, const float* __restrict__ tangent_all,
    const RowInfo* __restrict__ info, float* __restrict__ out_all, float* __restrict__ jvp_all,
    int64_t n, int chunks, float inv_1pl) {
  const int64_t row = blockIdx.x / chunks;
  const int64_t chunk = blockIdx.x % chunks;
  const RowInfo ri = info[row];
  const bool empty = ri.wa > ri.wb;
  const int64_t base = row * n;
  const int64_t first = chunk * int64_t(kThreads * 8);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t e = first + int64_t(i) * kThreads + threadIdx.x;
    if (e >= n) continue;
    const float xv = x_all[base + e];
    const float v = MAG ? fabsf(xv) : xv;
    // empty window: hi_incl = s_{k+1} < lo_incl = s_k, every value is > hi or < lo
    const bool above = v > ri.hi_incl;
    const bool below = v < ri.lo_incl;
    if (!empty && !above && !below) continue;          // inside the window
    if (out_all != nullptr) out_all[base + e] = above ? (MAG ? xv * inv_1pl : 1.0f) : 0.0f;
    if (jvp_all != nullptr) {
      float d = 0.0f;
      if (MAG && above && xv != 0.0f) d = tangent_all[base + e] * inv_1pl;
      jvp_all[base + e] = d;
    }
  }
}

// Sorted positions wa..wb of every row: y and dy from (a, b, gamma), scattered through sigma.
template <bool MAG, int PC>
__global__ __launch_bounds__(kThreads) void long_window_kernel(
    const uint32_t* __restrict__ skeys_all, const uint32_t* __restrict__ sidx_all,
    const float* __restrict__ tangent_all, const RowInfo* __restrict__ info,
    float* __restrict__ out_all, float* __restrict__ jvp_all, int64_t n, int blocks_per_row,
    Reg R) {
  using P = Pool<MAG, PC>;
  const int64_t row = blockIdx.x / blocks_per_row;
  const int64_t part = blockIdx.x % blocks_per_row;
  const RowInfo ri = info[row];
  const int64_t base = row * n;
  for (int64_t pos1 = ri.wa + part * kThreads + threadIdx.x; pos1 <= ri.wb;
       pos1 += int64_t(blocks_per_row) * kThreads) {
    const uint32_t id = sidx_all[base + pos1 - 1];
    const float sv = key_to_float(skeys_all[base + pos1 - 1]);
    const int64_t o = base + (MAG ? (id >> 1) : id);
    const bool neg = MAG && (id & 1u);
    const double v = double(sv) - ri.center;
    const bool before = pos1 < ri.a, after = pos1 > ri.b;
    if (out_all != nullptr) {
      double y = before ? (MAG ? v * R.inv_1pl : 1.0) : P::y_in_block(v, ri.gamma, R);
      if (after) y = 0.0;
      const float yf = float(y);
      out_all[o] = (MAG && yf == 0.0f) ? 0.0f : (neg ? -yf : yf);
    }
    if (jvp_all != nullptr) {
      double t = double(tangent_all[o]);
      if (neg) t = -t;
      if (MAG && sv == 0.0f) t = 0.0;
      double dy = before ? (MAG ? t * R.inv_1pl : 0.0) : P::hess(v, ri.gamma, R) * (t - ri.dgamma);
      if (after) dy = 0.0;
      float df = float(dy);
      if (MAG && sv == 0.0f) df = 0.0f;
      jvp_all[o] = (df == 0.0f) ? 0.0f : (neg ? -df : df);
    }
  }
}

template <bool MAG, int PC>
void launch_tail(const SortBuffers& B, const float* x, const float* tangent, float* out,
                 float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  hipLaunchKernelGGL((long_solve_kernel<MAG, PC>), dim3(unsigned(rows)), dim3(kThreads), 0, st,
                     B.keys_a, B.idx_a, jvp ? tangent : nullptr, B.info, n, k, R);
  const int chunks = int((n + kThreads * 8 - 1) / (kThreads * 8));
  hipLaunchKernelGGL((long_dense_kernel<MAG>), dim3(unsigned(rows * chunks)), dim3(kThreads), 0, st,
                     x, tangent, B.info, out, jvp, n, chunks, float(R.inv_1pl));
  const int64_t tiles = (n + kChunk - 1) / kChunk;
  const int bpr = int(tiles < 64 ? tiles : 64);
  hipLaunchKernelGGL((long_window_kernel<MAG, PC>), dim3(unsigned(rows * bpr)), dim3(kThreads), 0,
                     st, B.keys_a, B.idx_a, tangent, B.info, out, jvp, n, bpr, R);
}

}  // namespace

int launch_long_tail(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                     float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                     hipStream_t st) {
  const int64_t chunks = (n + kThreads * 8 - 1) / (kThreads * 8);
  if (rows * chunks > 0x7fffffffLL) return -1;
  if (!mag && pc == kP2) launch_tail<false, kP2>(B, x, tangent, out, jvp, rows, n, k, R, st);
  else if (!mag && pc == kP43) launch_tail<false, kP43>(B, x, tangent, out, jvp, rows, n, k, R, st);
  else if (mag && pc == kP2) launch_tail<true, kP2>(B, x, tangent, out, jvp, rows, n, k, R, st);
  else return -1;
  return 0;
}

}  // namespace topk
