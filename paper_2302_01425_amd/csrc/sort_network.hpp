// The register-resident sorting network of the short-row kernels and the packing of
// (descending-order key, index field) into one float64 (see short_rows.hip for the layout).
#pragma once

#include "common.hpp"
#include "wave.hpp"

namespace topk {

// ---- the sorting network ---------------------------------------------------------------------
// One stage: every position p is compared with p ^ M; the lower position keeps the minimum.
// p = lane*E + r, so M splits into a register mask (M mod E) and a lane mask (M / E).
template <int GL, int E, int M>
__device__ __forceinline__ void sort_stage(double (&K)[E], int lr) {
  constexpr int RM = M & (E - 1);
  constexpr int LM = M / E;
  if constexpr (LM == 0) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int r2 = r ^ RM;
      if (r < r2) {
        const double lo = min_f64(K[r], K[r2]);
        const double hi = max_f64(K[r], K[r2]);
        K[r] = lo;
        K[r2] = hi;
      }
    }
  } else {
    const bool low = (lr & top_bit(LM)) == 0;
    double O[E];
#pragma unroll
    for (int r = 0; r < E; ++r) O[r] = lane_xor_f64<LM>(K[r ^ RM]);
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const bool o_lt = O[r] < K[r];
      K[r] = (o_lt == low) ? O[r] : K[r];
    }
  }
}

template <int GL, int E, int STRIDE>
struct HalfCleaners {
  static __device__ __forceinline__ void run(double (&K)[E], int lr) {
    sort_stage<GL, E, STRIDE>(K, lr);
    HalfCleaners<GL, E, STRIDE / 2>::run(K, lr);
  }
};
template <int GL, int E>
struct HalfCleaners<GL, E, 0> {
  static __device__ __forceinline__ void run(double (&)[E], int) {}
};

// Bitonic merge sort in its "mirror" form: merging two sorted runs of SIZE/2 starts with the
// comparison p <-> p ^ (SIZE-1), then half-cleaners of stride SIZE/4 .. 1; every compare-exchange
// is ascending.
template <int GL, int E, int SIZE>
struct SortRuns {
  static __device__ __forceinline__ void run(double (&K)[E], int lr) {
    SortRuns<GL, E, SIZE / 2>::run(K, lr);
    sort_stage<GL, E, SIZE - 1>(K, lr);
    HalfCleaners<GL, E, SIZE / 4>::run(K, lr);
  }
};
template <int GL, int E>
struct SortRuns<GL, E, 1> {
  static __device__ __forceinline__ void run(double (&)[E], int) {}
};

// ---- packing -----------------------------------------------------------------------------------
template <int IDXB>
__device__ __forceinline__ double pack(uint32_t key, uint32_t field) {
  const uint32_t lo = (key << IDXB) | field;
  const uint32_t hi = 0x43300000u | (key >> (32 - IDXB));
  return __hiloint2double(int(hi), int(lo));
}
template <int IDXB>
__device__ __forceinline__ void unpack(double c, uint32_t& key, uint32_t& field) {
  const uint32_t lo = uint32_t(__double2loint(c)), hi = uint32_t(__double2hiint(c));
  key = (hi << (32 - IDXB)) | (lo >> IDXB);
  field = lo & ((1u << IDXB) - 1u);
}

// the same for a row dealt to the lanes by elem_of<GL, E, VEC>
template <int GL, int E, bool VEC, bool MAG, int IDXB>
__device__ __forceinline__ void make_keys_row(const float (&v)[E], int lr, int n, double (&K)[E]) {
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = elem_of<GL, E, VEC>(lr, r);
    uint32_t key = kSentinelKey, field = (1u << IDXB) - 1u;
    if (e < n) {
      if (MAG) {
        field = (uint32_t(e) << 1) | (__float_as_uint(v[r]) >> 31);
        key = desc_key(fabsf(v[r]));
      } else {
        field = uint32_t(e);
        key = desc_key(v[r]);
      }
    }
    K[r] = pack<IDXB>(key, field);
  }
}

template <int E, bool MAG, int IDXB>
__device__ __forceinline__ void make_keys(const float (&v)[E], int e0, int n, double (&K)[E]) {
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = e0 + r;
    uint32_t key = kSentinelKey, field = (1u << IDXB) - 1u;
    if (e < n) {
      if (MAG) {
        field = (uint32_t(e) << 1) | (__float_as_uint(v[r]) >> 31);
        key = desc_key(fabsf(v[r]));
      } else {
        field = uint32_t(e);
        key = desc_key(v[r]);
      }
    }
    K[r] = pack<IDXB>(key, field);
  }
}


}  // namespace topk
