// Rows of 8193 .. 32768 elements, dense outputs: the whole operator for one row in ONE workgroup
// of 1024 threads, one launch; the outputs are computed from values, so no permutation is built.
// A thread holds 32 elements of the row in registers from the histogram to the compaction.
//
//   1. histogram of the leading key bits of the row (LDS atomics)
//   2. the bins of sorted positions k and k+1 give the key window that holds every element able
//      to pool (radix.hpp: key_window)
//   3. compaction of those candidates: keys into LDS, (key, index) pairs into the row's scratch
//   4. keys-only sort and block growth on prefix sums, in LDS (sort_solve.hpp) -> gamma and the
//      block's value window; d gamma (Prop. 7) from the pairs whose value lies inside it
//   5. one pass over the row: every output from its element's value
// The row is read twice (HBM once, then L2).  Lists that do not fit the LDS buffers (the
// window holds more than kMedCap elements: rare) go through the scratch arrays.
#include "sort_solve.hpp"

namespace topk {
namespace {

constexpr int kMedCap = 8192;                  // keys of a list sorted in LDS
constexpr int kItems = 32;                     // elements of the row per thread
constexpr int kMed2RowMax = kWT * kItems;      // 32768

template <bool MAG, int PC>
__global__ __launch_bounds__(kWT) void medium2_kernel(
    const float* __restrict__ x_all, const float* __restrict__ tangent_all,
    float* __restrict__ out_all, float* __restrict__ jvp_all, uint32_t* keys_a, uint32_t* tau_a,
    uint32_t* keys_b, uint32_t* idx_b, int n, int k_row, Reg R) {
  using P = Pool<MAG, PC>;
  __shared__ ListShared<kMedCap> sm;
  __shared__ uint32_t found[2];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t base = int64_t(blockIdx.x) * n;
  const float* x = x_all + base;
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
  const bool want_jvp = jvp != nullptr;
  uint32_t* ka = keys_a + base;                // the row's list: keys
  uint32_t* pa = tau_a + base;                 //                 tangent bits

  RowInfo ri;
  ri.src = 0;
  ri.pad = 0;
  ri.a = int64_t(k_row) + 1;
  ri.b = k_row;
  ri.wa = ri.a;
  ri.wb = ri.b;
  ri.gamma = ri.center = ri.dgamma = 0.0;
  // k = 0: everything is below the window; k = n: everything above
  ri.hi_incl = k_row == 0 ? __uint_as_float(0x7f800000u) : __uint_as_float(0xff800000u);
  ri.lo_incl = ri.hi_incl;
  if (k_row >= 1 && k_row < n) {
    // ---- 1. histogram of the leading key bits ---------------------------------------------------
    uint32_t* hist = sm.keys_b;                // kSelBins words; the buffer is free until the sort
    static_assert(kSelBins <= kMedCap, "the histogram uses a sort buffer");
    for (int i = threadIdx.x; i < kSelBins; i += kWT) hist[i] = 0;
    __syncthreads();
    // element i of lane l of wavefront w is e = w * 2048 + i * 64 + l: wavefronts read contiguous
    // spans, and the order (wavefront, item, lane) is the element order
    float xv[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int e = w * (kItems * kWave) + i * kWave + lane;
      xv[i] = e < n ? x[e] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int e = w * (kItems * kWave) + i * kWave + lane;
      const uint32_t bin = first_key<MAG>(xv[i]) >> (32 - kSelBits);
      if (e < n) atomicAdd(&hist[bin], 1u);
    }
    __syncthreads();
    // ---- 2. bins of positions k and k+1, key window ---------------------------------------------
    constexpr int kPerThread = kSelBins / kWT;
    uint32_t c[kPerThread], mine = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      c[i] = hist[threadIdx.x * kPerThread + i];
      mine += c[i];
    }
    uint32_t run = wide_exclusive_scan(mine, sm.wave_tot, nullptr);
    const uint32_t q0 = uint32_t(k_row), q1 = uint32_t(k_row) + 1u;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const uint32_t next = run + c[i];
      if (run < q0 && q0 <= next) found[0] = threadIdx.x * kPerThread + i;
      if (run < q1 && q1 <= next) found[1] = threadIdx.x * kPerThread + i;
      run = next;
    }
    __syncthreads();
    uint32_t klo, khi;
    key_window<MAG>(found[0], found[1], R, PC == kP43, &klo, &khi);

    // ---- 3. compaction of the candidates ----------------------------------------------------------
    // the window in value space (key order is reversed value order, -0 == +0 either way; keys
    // beyond the infinities are clamped, they would decode to NaN)
    const float v_top = float(bound_value(klo)), v_bot = float(bound_value(khi));
    // list order: thread by thread, a thread's candidates in item order (any fixed order will do:
    // the list is sorted by value afterwards); one scan of the threads' counts places them
    uint32_t cn = 0, above = 0;
    {
      uint32_t cmask = 0u;                 // bit i: item i of this thread is a candidate
#pragma unroll
      for (int i = 0; i < kItems; ++i) {
        const int e = w * (kItems * kWave) + i * kWave + lane;
        const bool valid = e < n;
        const float v = MAG ? fabsf(xv[i]) : xv[i];
        const bool cand = valid && v <= v_top && v >= v_bot;
        above += (valid && v > v_top) ? 1u : 0u;
        cmask |= cand ? (1u << i) : 0u;
      }
      uint64_t total;
      const uint64_t ex = wide_exclusive_scan64(uint64_t(__popc(cmask)) | (uint64_t(above) << 32),
                                                sm.wave_tot64, &total);
      cn = uint32_t(total);
      above = uint32_t(total >> 32);       // now the whole row's count
      uint32_t j = uint32_t(ex);
      if (cmask != 0u) {
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
          if ((cmask >> i) & 1u) {
            const int e = w * (kItems * kWave) + i * kWave + lane;
            const uint32_t key = first_key<MAG>(xv[i]);
            ka[j] = key;
            if (j < uint32_t(kMedCap)) sm.keys_a[j] = key;
            // payload: the element's index, with its sign for the magnitude operator
            if (want_jvp)
              pa[j] = MAG ? ((uint32_t(e) << 1) | (__float_as_uint(xv[i]) >> 31)) : uint32_t(e);
            ++j;
          }
        }
      }
    }
    const int64_t k = int64_t(k_row) - int64_t(above);
    __syncthreads();                       // the list (LDS and scratch) is complete

    // ---- 4. sort, block, d gamma ------------------------------------------------------------------
    if (cn <= uint32_t(kMedCap)) {
      ri = solve_lds_list<MAG, PC, kMedCap>(cn, k, klo, khi, R, sm);
    } else {
      ri = solve_unsorted_list<MAG, PC, kMedCap>(ka, pa, cn, k, klo, khi, R, false, sm);
    }
    // d gamma (Prop. 7): the tangent of the list's elements whose value lies inside the block's
    // window, gathered through their indices
    if (ri.a <= ri.b && want_jvp) {
      double num = 0.0, den = 0.0;
      for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 4 * kWT) {
        uint32_t id[4];
        float sv[4], tv[4];
        bool in[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t j = j0 + uint32_t(i) * kWT;
          sv[i] = j < cn ? key_to_float(ka[j]) : 0.0f;
          id[i] = j < cn ? pa[j] : 0u;
          in[i] = j < cn && sv[i] >= ri.lo_incl && sv[i] <= ri.hi_incl;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) tv[i] = in[i] ? tangent[MAG ? (id[i] >> 1) : id[i]] : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (!in[i]) continue;
          double t = double(tv[i]);
          if (MAG) {
            if (id[i] & 1u) t = -t;
            if (sv[i] == 0.0f) t = 0.0;
          }
          const double wgt = P::jac_weight(double(sv[i]) - ri.center, ri.gamma);
          num += wgt * t;
          den += wgt;
        }
      }
      wide_sum2(num, den, sm);
      ri.dgamma = num / P::jac_denominator(den, double(k - ri.a + 1), R);
    }
  }

  // ---- 5. outputs: every element from its own value ------------------------------------------------
  const bool have_block = ri.a <= ri.b;
  const float inv_1pl = float(R.inv_1pl);
  constexpr int kOut = 16;
  for (int e0 = threadIdx.x; e0 < n; e0 += kOut * kWT) {
    float xv[kOut], tv[kOut];
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
      const int e = e0 + i * kWT;
      xv[i] = e < n ? load_stream(x + e) : 0.0f;
      // the mask's JVP is zero outside the block: only the magnitude operator streams the tangent
      tv[i] = (MAG && e < n && want_jvp) ? load_stream(tangent + e) : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
      const int e = e0 + i * kWT;
      const float v = MAG ? fabsf(xv[i]) : xv[i];
      const bool is_above = e < n && v > ri.hi_incl;
      const bool inside = e < n && have_block && !is_above && v >= ri.lo_incl;
      const bool neg = MAG && (__float_as_uint(xv[i]) >> 31);
      float y = 0.0f, d = 0.0f;
      if (is_above) {
        if constexpr (MAG && PC == kP43) {
          if (xv[i] != 0.0f) {
            double g, slope;
            P::above_both(double(v), R, 0.0, &g, &slope);
            y = float(neg ? -g : g);
            if (want_jvp) d = float(slope * double(tv[i]));
          }
        } else if (MAG) {
          y = xv[i] * inv_1pl;
          if (want_jvp && xv[i] != 0.0f) d = tv[i] * inv_1pl;
        } else {
          y = 1.0f;
        }
      }
      if (__any(inside)) {                 // few wavefronts hold an element of the block
        if (inside) {
          const double cv = double(v) - ri.center;
          y = float(P::y_in_block(cv, ri.gamma, R));
          if (MAG) y = (y == 0.0f) ? 0.0f : (neg ? -y : y);
          if (want_jvp) {
            double t = double(MAG ? tv[i] : tangent[e]);
            if (neg) t = -t;
            if (MAG && v == 0.0f) t = 0.0;
            float df = float(P::hess(cv, ri.gamma, R) * (t - ri.dgamma));
            if (MAG && v == 0.0f) df = 0.0f;
            d = (df == 0.0f) ? 0.0f : (neg ? -df : df);
          }
        }
      }
      if (e < n) {
        if (out != nullptr) store_stream(out + e, y);
        if (want_jvp) store_stream(jvp + e, d);
      }
    }
  }
}

}  // namespace

int launch_medium_rows2(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                        float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                        hipStream_t st) {
  if (n > kMed2RowMax || rows > 0x7fffffffLL) return -1;
#define TOPK_MED2(M, P)                                                                          \
  hipLaunchKernelGGL((medium2_kernel<M, P>), dim3(unsigned(rows)), dim3(kWT), 0, st, x, tangent, \
                     out, jvp, B.keys_a, B.idx_a, B.keys_b, B.idx_b, int(n), int(k), R)
  if (!mag && pc == kP2) TOPK_MED2(false, kP2);
  else if (!mag && pc == kP43) TOPK_MED2(false, kP43);
  else if (mag && pc == kP2) TOPK_MED2(true, kP2);
  else if (mag && pc == kP43) TOPK_MED2(true, kP43);
  else return -1;
#undef TOPK_MED2
  return 0;
}

}  // namespace topk
