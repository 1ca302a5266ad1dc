// Shared device helpers of the gfx950 kernels: order-preserving keys and row-group wavefront
// primitives.  A "row group" is GL consecutive lanes of a 64-wide wavefront that own one row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace topk {

constexpr int kWave = 64;

enum PCode : int { kP2 = 0, kP43 = 1 };

// Sorting is descending in value with ascending original index on ties (paper Sec. 3 sorts in
// descending order; the tie rule makes the permutation unique).  Keys are mapped so that an
// ASCENDING unsigned order of (key, index) is that order: key = ~ord(f), ord = the usual
// order-preserving map of IEEE-754 floats to unsigned.  -0.0f is folded onto +0.0f first.
__device__ __forceinline__ uint32_t desc_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return ~ord;
}

__device__ __forceinline__ float key_to_float(uint32_t key) {
  uint32_t ord = ~key;
  uint32_t b = (ord & 0x80000000u) ? (ord & 0x7fffffffu) : ~ord;
  return __uint_as_float(b);
}

constexpr uint32_t kSentinelKey = 0xffffffffu;   // sorts after every finite value and -inf

template <int GL>
__device__ __forceinline__ int lane_in_group() {
  return int(threadIdx.x) & (GL - 1);
}

template <int GL, class T>
__device__ __forceinline__ T group_bcast(T v, int src) {
  return __shfl(v, src, GL);
}

// Number of lanes of this lane's row group whose predicate is set.
template <int GL>
__device__ __forceinline__ int group_count(bool pred) {
  unsigned long long b = __ballot(pred);
  if (GL < kWave) {
    int base = (int(threadIdx.x) & (kWave - 1)) & ~(GL - 1);
    b = (b >> base) & ((1ull << (GL & 63)) - 1ull);
  }
  return __popcll(b);
}

template <int GL>
__device__ __forceinline__ double group_sum(double v) {
#pragma unroll
  for (int off = GL >> 1; off >= 1; off >>= 1) v += __shfl_xor(v, off, GL);
  return v;
}

// Exclusive prefix sum across the lanes of a row group (lane totals in, exclusive prefix out).
template <int GL>
__device__ __forceinline__ double group_exclusive_scan(double tot, int lr) {
  double inc = tot;
#pragma unroll
  for (int off = 1; off < GL; off <<= 1) {
    double o = __shfl_up(inc, off, GL);
    if (lr >= off) inc += o;
  }
  double prev = __shfl_up(inc, 1, GL);
  return lr == 0 ? 0.0 : prev;
}

}  // namespace topk
