// Short rows (n <= 1024): one row per group of GL lanes of a wavefront, E elements per lane,
// everything after the load kept in registers.
//
//   load -> (key, index) bitonic sort -> float64 windowed prefix sums -> block growth
//        -> pooled value -> y in sorted order -> un-sort scatter (+ JVP of Prop. 7)
//
// Layout: lane l of a row group holds the elements l*E .. l*E+E-1 of the row (so a lane's loads
// are contiguous) and, after the sort, the sorted positions l*E .. l*E+E-1.
#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"

namespace topk {
namespace {

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask, int width) {
  uint32_t lo = uint32_t(v), hi = uint32_t(v >> 32);
  lo = __shfl_xor(lo, mask, width);
  hi = __shfl_xor(hi, mask, width);
  return (uint64_t(hi) << 32) | lo;
}

// Bitonic sorting network over the GL*E composites of one row, ascending.
// Strides below E are compare-exchanges between registers of one lane; strides of E and above
// are exchanges with the lane at distance stride/E.
template <int GL, int E>
__device__ __forceinline__ void bitonic_sort(uint64_t (&K)[E], int lr) {
  constexpr int NP = GL * E;
#pragma unroll
  for (int size = 2; size <= NP; size <<= 1) {
#pragma unroll
    for (int stride = size >> 1; stride >= 1; stride >>= 1) {
      if (stride < E) {
#pragma unroll
        for (int r = 0; r < E; ++r) {
          if ((r & stride) == 0) {
            const bool up = (((lr * E + r) & size) == 0);
            uint64_t lo = K[r], hi = K[r | stride];
            const bool sw = (lo > hi) == up;
            K[r] = sw ? hi : lo;
            K[r | stride] = sw ? lo : hi;
          }
        }
      } else {
        const int ls = stride / E;
        const bool low = (lr & ls) == 0;
#pragma unroll
        for (int r = 0; r < E; ++r) {
          const bool up = (((lr * E + r) & size) == 0);
          const uint64_t o = shfl_xor_u64(K[r], ls, GL);
          const bool keep_min = (low == up);
          const bool o_lt = o < K[r];
          K[r] = (keep_min == o_lt) ? o : K[r];
        }
      }
    }
  }
}

// value of per-lane array v[] at sorted position pos0 (0-based) of this lane's row
template <int GL, int E, class T>
__device__ __forceinline__ T at_pos(const T (&v)[E], int pos0) {
  const int r = pos0 & (E - 1);
  T sel = v[0];
#pragma unroll
  for (int q = 1; q < E; ++q) sel = (r == q) ? v[q] : sel;
  return group_bcast<GL>(sel, pos0 / E);
}

// Load one row into composites.  Index field: original index (mask) or 2*index + signbit (mag).
template <int GL, int E, bool MAG>
__device__ __forceinline__ void load_row(const float* __restrict__ x, int64_t base, int n, int lr,
                                         uint64_t (&K)[E]) {
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = lr * E + r;
    uint32_t key = kSentinelKey, idx = 0xffffffffu;
    if (e < n) {
      float v = x[base + e];
      if (MAG) {
        idx = (uint32_t(e) << 1) | (__float_as_uint(v) >> 31);
        v = fabsf(v);
      } else {
        idx = uint32_t(e);
      }
      key = desc_key(v);
    }
    K[r] = (uint64_t(key) << 32) | idx;
  }
}

template <int GL, int E>
__global__ __launch_bounds__(256) void short_argsort_kernel(const float* __restrict__ x,
                                                            int32_t* __restrict__ perm,
                                                            int64_t rows, int n) {
  constexpr int RPW = kWave / GL;
  const int lr = lane_in_group<GL>();
  const int64_t wave = int64_t(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
  int64_t row = wave * RPW + ((threadIdx.x & (kWave - 1)) / GL);
  const bool valid = row < rows;
  if (!valid) row = rows - 1;
  uint64_t K[E];
  load_row<GL, E, false>(x, row * n, n, lr, K);
  bitonic_sort<GL, E>(K, lr);
  if (!valid) return;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos = lr * E + r;
    if (pos < n) perm[row * n + pos] = int32_t(uint32_t(K[r]));
  }
}

template <int GL, int E, bool MAG, int PC>
__global__ __launch_bounds__(256) void short_rows_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ tangent,
                                                         float* __restrict__ out,
                                                         float* __restrict__ jvp, int64_t rows,
                                                         int n, int k, Reg R) {
  using P = Pool<MAG, PC>;
  constexpr int RPW = kWave / GL;
  constexpr bool CUBIC = (PC == kP43);
  const int lr = lane_in_group<GL>();
  const int64_t wave = int64_t(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
  int64_t row = wave * RPW + ((threadIdx.x & (kWave - 1)) / GL);
  const bool valid = row < rows;
  if (!valid) row = rows - 1;            // keep the lanes alive for the shuffles; no stores
  const int64_t base = row * n;

  // ---- load + sort -------------------------------------------------------------------------
  uint64_t K[E];
  load_row<GL, E, MAG>(x, base, n, lr, K);
  bitonic_sort<GL, E>(K, lr);

  float s32[E];
  uint32_t idx[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    s32[r] = key_to_float(uint32_t(K[r] >> 32));
    idx[r] = uint32_t(K[r]);
  }

  // ---- window of positions that can pool, centred values ------------------------------------
  // mask: values relative to s_k (shift invariance); magnitude: the values themselves.
  double d[E];
  bool cand[E];
  int a = k + 1, b = k;                  // 1-based inclusive block [a, b]; empty when a > b
  bool grow = false;
  double center = 0.0;
  if (k >= 1 && k < n) {
    const double sk = double(at_pos<GL, E>(s32, k - 1));
    const double sk1 = double(at_pos<GL, E>(s32, k));
    if (!MAG) center = sk;
    const double ck = sk - center, ck1 = sk1 - center;
    grow = P::seed_violates(ck, ck1, R);
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = lr * E + r + 1;
      const double v = double(s32[r]) - center;
      cand[r] = grow && (pos1 <= n) && (pos1 <= k ? P::left_candidate(v, ck1, R)
                                                    : P::right_candidate(v, ck, R));
      d[r] = cand[r] ? v : 0.0;
    }
    if (grow) { a = k; b = k + 1; }
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) { d[r] = 0.0; cand[r] = false; }
  }

  double gamma = 0.0;                    // pooled value (centred for the mask)
  if (__any(grow)) {
    // ---- exclusive prefix sums of d, d^2, d^3 over the sorted positions --------------------
    double X1[E], X2[E], X3[E];
    {
      double t1 = 0.0, t2 = 0.0, t3 = 0.0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        X1[r] = t1; t1 += d[r];
        if (CUBIC) {
          X2[r] = t2; t2 += d[r] * d[r];
          X3[r] = t3; t3 += d[r] * d[r] * d[r];
        }
      }
      const double p1 = group_exclusive_scan<GL>(t1, lr);
      double p2 = 0.0, p3 = 0.0;
      if (CUBIC) {
        p2 = group_exclusive_scan<GL>(t2, lr);
        p3 = group_exclusive_scan<GL>(t3, lr);
      }
#pragma unroll
      for (int r = 0; r < E; ++r) {
        X1[r] += p1;
        if (CUBIC) { X2[r] += p2; X3[r] += p3; }
      }
    }
    double I1[E], I2[E], I3[E];          // inclusive prefixes
#pragma unroll
    for (int r = 0; r < E; ++r) {
      I1[r] = X1[r] + d[r];
      if (CUBIC) {
        I2[r] = X2[r] + d[r] * d[r];
        I3[r] = X3[r] + d[r] * d[r] * d[r];
      }
    }

    // ---- grow the block: right run, then left run, until neither moves ---------------------
    bool active = grow;
    while (__any(active)) {
      // right: positions j > k with  s_j > gamma([a, j-1])  form a prefix of the tail
      Sums A;                             // exclusive prefix at position a
      A.s1 = at_pos<GL, E>(X1, a - 1);
      A.s2 = CUBIC ? at_pos<GL, E>(X2, a - 1) : 0.0;
      A.s3 = CUBIC ? at_pos<GL, E>(X3, a - 1) : 0.0;
      const double mR = double(k - a + 1);
      int cntR = 0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pos1 = lr * E + r + 1;
        Sums S{X1[r] - A.s1, CUBIC ? X2[r] - A.s2 : 0.0, CUBIC ? X3[r] - A.s3 : 0.0};
        const bool pr = active && cand[r] && pos1 > k &&
                        P::right_violates(d[r], double(pos1 - a), mR, S, R);
        cntR += group_count<GL>(pr);
      }
      const int b_new = max(b, k + cntR);
      // left: positions i <= k with  gamma_i < gamma([i+1, b])  form a suffix of the head
      Sums B;                             // inclusive prefix at position b_new
      B.s1 = at_pos<GL, E>(I1, b_new - 1);
      B.s2 = CUBIC ? at_pos<GL, E>(I2, b_new - 1) : 0.0;
      B.s3 = CUBIC ? at_pos<GL, E>(I3, b_new - 1) : 0.0;
      int cntL = 0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pos1 = lr * E + r + 1;
        Sums S{B.s1 - I1[r], CUBIC ? B.s2 - I2[r] : 0.0, CUBIC ? B.s3 - I3[r] : 0.0};
        const bool pl = active && cand[r] && pos1 <= k &&
                        P::left_violates(d[r], double(b_new - pos1), double(k - pos1), S, R);
        cntL += group_count<GL>(pl);
      }
      const int a_new = min(a, k + 1 - cntL);
      if (active) {
        active = (a_new != a) || (b_new != b);
        a = a_new;
        b = b_new;
      }
    }

    // ---- pooled value of the final block -----------------------------------------------------
    if (grow) {
      Sums S;
      S.s1 = at_pos<GL, E>(I1, b - 1) - at_pos<GL, E>(X1, a - 1);
      S.s2 = CUBIC ? at_pos<GL, E>(I2, b - 1) - at_pos<GL, E>(X2, a - 1) : 0.0;
      S.s3 = CUBIC ? at_pos<GL, E>(I3, b - 1) - at_pos<GL, E>(X3, a - 1) : 0.0;
      const double da = at_pos<GL, E>(d, a - 1), db = at_pos<GL, E>(d, b - 1);
      gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, da - R.lambda, db);
    }
  }

  // ---- y in sorted order, un-sort scatter ------------------------------------------------------
  // Positions before the block keep their singleton solution (mask: exactly 1; magnitude:
  // s/(1+lambda)); positions after it are exactly 0.
  double ys[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos1 = lr * E + r + 1;
    const double v = double(s32[r]) - center;
    double y;
    if (pos1 < a) y = MAG ? v * R.inv_1pl : 1.0;
    else if (pos1 <= b) y = P::y_in_block(v, gamma, R);
    else y = 0.0;
    ys[r] = y;
  }
  if (out != nullptr && valid) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = lr * E + r + 1;
      if (pos1 <= n) {
        if (MAG) {
          const uint32_t o = idx[r] >> 1;
          const float yv = float(ys[r]);
          out[base + o] = (yv == 0.0f) ? 0.0f : ((idx[r] & 1u) ? -yv : yv);
        } else {
          out[base + idx[r]] = float(ys[r]);
        }
      }
    }
  }
  if (jvp == nullptr) return;

  // ---- JVP (Prop. 7): d gamma = weighted block average of the sorted tangent --------------------
  double tau[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos1 = lr * E + r + 1;
    double t = 0.0;
    if (pos1 <= n) {
      if (MAG) {
        t = double(tangent[base + (idx[r] >> 1)]);
        if (idx[r] & 1u) t = -t;
        if (s32[r] == 0.0f) t = 0.0;         // sign(0) = 0
      } else {
        t = double(tangent[base + idx[r]]);
      }
    }
    tau[r] = t;
  }
  double dgamma = 0.0;
  if (__any(a <= b)) {
    double num = 0.0, wsum = 0.0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = lr * E + r + 1;
      if (pos1 >= a && pos1 <= b) {
        const double w = P::jac_weight(double(s32[r]) - center, gamma);
        num += w * tau[r];
        wsum += w;
      }
    }
    num = group_sum<GL>(num);
    wsum = group_sum<GL>(wsum);
    if (a <= b) dgamma = num / P::jac_denominator(wsum, double(k - a + 1), R);
  }
  if (!valid) return;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos1 = lr * E + r + 1;
    if (pos1 > n) continue;
    double dy;
    if (pos1 < a) dy = MAG ? tau[r] * R.inv_1pl : 0.0;
    else if (pos1 <= b) dy = P::hess(double(s32[r]) - center, gamma, R) * (tau[r] - dgamma);
    else dy = 0.0;
    if (MAG) {
      const float v = (s32[r] == 0.0f) ? 0.0f : float(dy);
      jvp[base + (idx[r] >> 1)] = (v == 0.0f) ? 0.0f : ((idx[r] & 1u) ? -v : v);
    } else {
      jvp[base + idx[r]] = float(dy);
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <int GL, int E>
int launch_shape(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                 int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  constexpr int RPW = kWave / GL;
  const int64_t waves = (rows + RPW - 1) / RPW;
  const int64_t blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffLL) return -1;
  dim3 grid((unsigned)blocks), block(256);
  if (!mag && pc == kP2)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, false, kP2>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R);
  else if (!mag && pc == kP43)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, false, kP43>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R);
  else if (mag && pc == kP2)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, true, kP2>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R);
  else
    return -1;
  return 0;
}

template <int GL, int E>
int launch_argsort_shape(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st) {
  constexpr int RPW = kWave / GL;
  const int64_t waves = (rows + RPW - 1) / RPW;
  const int64_t blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffLL) return -1;
  hipLaunchKernelGGL((short_argsort_kernel<GL, E>), dim3((unsigned)blocks), dim3(256), 0, st, x,
                     perm, rows, n);
  return 0;
}

}  // namespace

#define TOPK_SHAPE_SWITCH(CALL)                      \
  if (n <= 2) return CALL(2, 1);                     \
  if (n <= 4) return CALL(4, 1);                     \
  if (n <= 8) return CALL(8, 1);                     \
  if (n <= 16) return CALL(16, 1);                   \
  if (n <= 32) return CALL(32, 1);                   \
  if (n <= 64) return CALL(64, 1);                   \
  if (n <= 128) return CALL(64, 2);                  \
  if (n <= 256) return CALL(64, 4);                  \
  if (n <= 512) return CALL(64, 8);                  \
  if (n <= 1024) return CALL(64, 16);                \
  return -1;

int launch_short_rows(bool mag, int pc, const float* x, const float* tangent, float* out,
                      float* jvp, int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
#define CALL(GL, E) launch_shape<GL, E>(mag, pc, x, tangent, out, jvp, rows, n, k, R, st)
  TOPK_SHAPE_SWITCH(CALL)
#undef CALL
}

int launch_short_argsort(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st) {
#define CALL(GL, E) launch_argsort_shape<GL, E>(x, perm, rows, n, st)
  TOPK_SHAPE_SWITCH(CALL)
#undef CALL
}

}  // namespace topk
