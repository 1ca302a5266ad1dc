// Pieces shared by the radix-sort passes and the candidate selection of the long and medium rows.
#pragma once

#include "common.hpp"
#include "launch.hpp"
#include "pooling.hpp"

namespace topk {

constexpr int kRadix = 256;

// lanes (among `valid`) that hold the same 8-bit digit as this lane
__device__ __forceinline__ unsigned long long match_digit(uint32_t d, unsigned long long valid) {
  unsigned long long peers = valid;
#pragma unroll
  for (int bit = 0; bit < 8; ++bit) {
    const bool one = (d >> bit) & 1u;
    const unsigned long long bal = __ballot(one);
    peers &= one ? bal : ~bal;
  }
  return peers;
}

__device__ __forceinline__ unsigned long long lanemask_lt() {
  const int lane = threadIdx.x & (kWave - 1);
  return (1ull << lane) - 1ull;
}

// Key of element e of a row in the first pass (from the float input), later passes read keys.
template <bool MAG>
__device__ __forceinline__ uint32_t first_key(float v) {
  return desc_key(MAG ? fabsf(v) : v);
}

// Count one digit per valid lane into this wavefront's private counters.  The digit of the first
// valid lane is counted once for all lanes that share it (this keeps skewed digits, e.g. the
// exponent byte, from serialising); the other lanes add 1 each.
__device__ __forceinline__ void count_digit(uint32_t* __restrict__ wave_cnt, uint32_t d, bool valid,
                                            int lane) {
  const unsigned long long vm = __ballot(valid);
  if (vm == 0) return;
  const int first = __ffsll((long long)vm) - 1;
  const uint32_t d0 = uint32_t(__builtin_amdgcn_readlane(int(d), first));
  const bool same = valid && d == d0;
  const unsigned long long m0 = __ballot(same);
  if (lane == first) wave_cnt[d0] += __popcll(m0);
  if (valid && !same) atomicAdd(&wave_cnt[d], 1u);
}

// Keys of all finite values and the infinities lie in [key(+inf), key(-inf)].
__device__ __forceinline__ double bound_value(uint32_t key) {
  const uint32_t lo = 0x007fffffu, hi = 0xff800000u;
  key = key < lo ? lo : (key > hi ? hi : key);
  return double(key_to_float(key));
}


// Key window [klo, khi] of the candidates of one row, from the histogram bins (leading BITS
// key bits) that hold sorted positions k and k+1.  s_k is at least the smallest value of its bin
// and s_{k+1} at most the largest value of its bin; the window holds both bins and every element
// that passes the necessary conditions for joining the block (pooling.hpp: left_candidate,
// right_candidate) for ANY s_k, s_{k+1} inside those bins.
// cubic: p = 4/3 (matters for the magnitude operator only: the mask's conditions do not depend on p).
template <bool MAG, int BITS = kSelBits>
__device__ __forceinline__ void key_window(uint32_t bin_k, uint32_t bin_k1, const Reg& R, bool cubic,
                                           uint32_t* klo_out, uint32_t* khi_out) {
  constexpr int kShift = 32 - BITS;
  const uint32_t low_bits = (1u << kShift) - 1u;
  const uint32_t first_k = bin_k << kShift;                       // largest value of s_k's bin
  const uint32_t last_k1 = (bin_k1 << kShift) | low_bits;         // smallest value of s_{k+1}'s bin
  const double lo_k = bound_value(first_k | low_bits);            // s_k >= lo_k
  const double hi_k1 = bound_value(bin_k1 << kShift);             // s_{k+1} <= hi_k1
  // right candidates: x > s_k - lambda (mask), x (1 + lambda) > s_k (magnitude);
  // left candidates: x - lambda < s_{k+1}, x < s_{k+1} (1 + lambda).  Two keys of slack cover
  // the rounding of the float conversions.
  double right_lim = MAG ? lo_k * R.inv_1pl : lo_k - R.lambda;
  double left_lim = MAG ? hi_k1 * R.one_p_lambda : hi_k1 + R.lambda;
  if (MAG && cubic) {
    // right: x above the singleton root of s_k (increasing in s_k, taken a little low);
    // left: the singleton root of x below s_{k+1}  <=>  x < s_{k+1} + lambda s_{k+1}^(1/3)
    right_lim = singleton_root_mag43(lo_k > 0.0 ? lo_k : 0.0, R) * (1.0 - 1e-6);
    left_lim = hi_k1 > 0.0 ? hi_k1 + R.lambda * cbrt(hi_k1) * (1.0 + 1e-6) : R.lambda;
  }
  uint32_t khi = desc_key(float(right_lim));
  khi = khi > 0xfffffffdu ? 0xffffffffu : khi + 2u;
  uint32_t klo = desc_key(float(left_lim));
  klo = klo < 2u ? 0u : klo - 2u;
  klo = klo < first_k ? klo : first_k;
  // 0x80000000 would be the key of -0.0, which desc_key folds onto +0.0 (0x7fffffff): start the
  // window at the zeros, so that "key >= klo" and "value <= value(klo)" select the same elements
  if (klo == 0x80000000u) klo = 0x7fffffffu;
  *klo_out = klo;
  *khi_out = khi > last_k1 ? khi : last_k1;
}

}  // namespace topk
