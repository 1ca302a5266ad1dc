// Wavefront-level building blocks of the short-row kernels (gfx950): DPP lane exchanges,
// row-group sums and scans, vectorised row loads/stores.  A "row group" is GL consecutive
// lanes (a power of two, at most 64) that own one row.
#pragma once

#include "common.hpp"

namespace topk {

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }
constexpr int top_bit(int v) { return 1 << ilog2(v); }

// ---- cross-lane exchanges -------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
  return uint32_t(__builtin_amdgcn_mov_dpp(int(v), CTRL, 0xF, 0xF, true));
}

// value of lane (l ^ LM).  LM is one of the masks a bitonic network on <= 64 lanes needs:
// strides 1,2,4,8,16,32 and mirrors 3,7,15,31,63.  Within a row of 16 lanes these are DPP moves.
template <int LM>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
  if constexpr (LM == 1) return dpp_mov<0xB1>(v);            // quad_perm [1,0,3,2]
  else if constexpr (LM == 2) return dpp_mov<0x4E>(v);       // quad_perm [2,3,0,1]
  else if constexpr (LM == 3) return dpp_mov<0x1B>(v);       // quad_perm [3,2,1,0]
  else if constexpr (LM == 7) return dpp_mov<0x141>(v);      // row_half_mirror
  else if constexpr (LM == 15) return dpp_mov<0x140>(v);     // row_mirror
  else if constexpr (LM == 8) return dpp_mov<0x128>(v);      // row_ror:8
  else if constexpr (LM == 4) {
    // banks 0 and 2 (lanes 0-3, 8-11) read lane+4, banks 1 and 3 read lane-4
    int t = __builtin_amdgcn_update_dpp(int(v), int(v), 0x104, 0xF, 0x5, false);   // row_shl:4
    t = __builtin_amdgcn_update_dpp(t, int(v), 0x114, 0xF, 0xA, false);            // row_shr:4
    return uint32_t(t);
  } else if constexpr (LM == 16) {
    return uint32_t(__builtin_amdgcn_ds_swizzle(int(v), (16 << 10) | 0x1F));       // swap rows
  } else if constexpr (LM == 31) {
    return lane_xor<16>(lane_xor<15>(v));
  } else if constexpr (LM == 32) {
    return uint32_t(__shfl_xor(int(v), 32, kWave));
  } else {
    static_assert(LM == 63, "unsupported lane mask");
    return lane_xor<32>(lane_xor<31>(v));
  }
}

template <int LM>
__device__ __forceinline__ double lane_xor_f64(double v) {
  const uint32_t lo = lane_xor<LM>(uint32_t(__double2loint(v)));
  const uint32_t hi = lane_xor<LM>(uint32_t(__double2hiint(v)));
  return __hiloint2double(int(hi), int(lo));
}

// plain machine min / max: the operands are never NaN, so no canonicalisation is wanted
__device__ __forceinline__ double min_f64(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ double max_f64(double a, double b) {
  double r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// ---- row-group collectives --------------------------------------------------------------------
template <int GL, class T>
__device__ __forceinline__ T bcast_lane(T v, int src) {
  if constexpr (GL == 1) return v;
  else return __shfl(v, src, GL);
}

// value of the per-lane array v[] at sorted position pos0 (0-based) of this lane's row
template <int GL, int E, class T>
__device__ __forceinline__ T at_pos(const T (&v)[E], int pos0) {
  const int r = pos0 & (E - 1);
  T sel = v[0];
#pragma unroll
  for (int q = 1; q < E; ++q) sel = (r == q) ? v[q] : sel;
  return bcast_lane<GL>(sel, pos0 / E);
}

template <int GL, int LM>
struct XorSum {
  static __device__ __forceinline__ double f64(double v) {
    v = XorSum<GL, LM / 2>::f64(v);
    return v + lane_xor_f64<LM>(v);
  }
  static __device__ __forceinline__ uint32_t u32(uint32_t v) {
    v = XorSum<GL, LM / 2>::u32(v);
    return v + lane_xor<LM>(v);
  }
};
template <int GL>
struct XorSum<GL, 0> {
  static __device__ __forceinline__ double f64(double v) { return v; }
  static __device__ __forceinline__ uint32_t u32(uint32_t v) { return v; }
};
// sums over the GL lanes of the row group, result in every lane
template <int GL>
__device__ __forceinline__ double group_sum_f64(double v) { return XorSum<GL, GL / 2>::f64(v); }
template <int GL>
__device__ __forceinline__ uint32_t group_sum_u32(uint32_t v) { return XorSum<GL, GL / 2>::u32(v); }

// value of lane l - OFF of the same DPP row (0 when that lane does not exist)
template <int OFF>
__device__ __forceinline__ double row_shr_f64(double v) {
  const uint32_t lo = dpp_mov<0x110 + OFF>(uint32_t(__double2loint(v)));
  const uint32_t hi = dpp_mov<0x110 + OFF>(uint32_t(__double2hiint(v)));
  return __hiloint2double(int(hi), int(lo));
}

template <int GL, int OFF>
struct ScanSteps {
  static __device__ __forceinline__ double run(double inc, int lr) {
    inc = ScanSteps<GL, OFF / 2>::run(inc, lr);
    double o;
    if constexpr (GL <= 16) o = row_shr_f64<OFF>(inc);   // the group lies inside one DPP row
    else o = __shfl_up(inc, OFF, GL);
    return (lr >= OFF) ? inc + o : inc;
  }
};
template <int GL>
struct ScanSteps<GL, 0> {
  static __device__ __forceinline__ double run(double inc, int) { return inc; }
};
// exclusive prefix (over the lanes of the row group) of one value per lane
template <int GL>
__device__ __forceinline__ double group_exclusive_scan_f64(double tot, int lr) {
  if constexpr (GL == 1) return 0.0;
  else {
    const double inc = ScanSteps<GL, GL / 2>::run(tot, lr);
    double prev;
    if constexpr (GL <= 16) prev = row_shr_f64<1>(inc);
    else prev = __shfl_up(inc, 1, GL);
    return lr == 0 ? 0.0 : prev;
  }
}

// 16-byte loads and stores with the non-temporal hint, for data that is touched once (inputs
// read once, final outputs): they do not displace cache lines that will be used again, and
// measured 17 % faster than plain accesses on the 16384 x 64 router workload (8 elements per
// lane).  Not for lanes that own 16 CONSECUTIVE elements (load_elems / store_elems): there one
// cache line is shared by the four accesses of a lane, and the hinted accesses each go to the L2
// again (measured twice as slow on 65536 x 256); rows dealt float4 by float4 (load_row) are fine.
typedef float float4_raw __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load4_stream(const float* p) {
  const float4_raw v = __builtin_nontemporal_load(reinterpret_cast<const float4_raw*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store4_stream(float* p, float4 v) {
  const float4_raw w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<float4_raw*>(p));
}
__device__ __forceinline__ float load_stream(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(float* p, float v) { __builtin_nontemporal_store(v, p); }

template <int E, bool VEC>
__device__ __forceinline__ void load_elems(const float* __restrict__ p, int64_t base, int e0, int n,
                                           float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e0 + 4 * c < n) q = *reinterpret_cast<const float4*>(p + base + e0 + 4 * c);
      v[4 * c + 0] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) v[r] = (e0 + r < n) ? p[base + e0 + r] : 0.0f;
  }
}

template <int E, bool VEC>
__device__ __forceinline__ void store_elems(float* __restrict__ p, int64_t base, int e0, int n,
                                            const float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c)
      if (e0 + 4 * c < n)
        *reinterpret_cast<float4*>(p + base + e0 + 4 * c) =
            make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r)
      if (e0 + r < n) p[base + e0 + r] = v[r];
  }
}

// ---- rows dealt to the lanes float4 by float4 ---------------------------------------------------
// For vectorisable rows (VEC) register r of lane lr holds element ((r/4) * GL + lr) * 4 + r % 4
// instead of lr * E + r: every load / store instruction of a row group then covers one
// contiguous span of the row.  Which elements a lane holds is immaterial to the sort, the index
// travels with the key.  STREAM adds the non-temporal hint.
template <int GL, int E, bool VEC>
__device__ __forceinline__ int elem_of(int lr, int r) {
  if constexpr (VEC) return (((r >> 2) * GL + lr) << 2) + (r & 3);
  else return lr * E + r;
}
template <int GL, int E, bool VEC, bool STREAM>
__device__ __forceinline__ void load_row(const float* __restrict__ p, int64_t base, int lr, int n,
                                         float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      const int off = (c * GL + lr) * 4;
      float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
      if (off < n) q = STREAM ? load4_stream(p + base + off) : *reinterpret_cast<const float4*>(p + base + off);
      v[4 * c + 0] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
    }
  } else {
    load_elems<E, false>(p, base, lr * E, n, v);
  }
}
template <int GL, int E, bool VEC, bool STREAM>
__device__ __forceinline__ void store_row(float* __restrict__ p, int64_t base, int lr, int n,
                                          const float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      const int off = (c * GL + lr) * 4;
      const float4 q = make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
      if (off < n) {
        if (STREAM) store4_stream(p + base + off, q);
        else *reinterpret_cast<float4*>(p + base + off) = q;
      }
    }
  } else {
    store_elems<E, false>(p, base, lr * E, n, v);
  }
}
// the same registers to / from a row staged in LDS in original element order
template <int GL, int E, bool VEC>
__device__ __forceinline__ void lds_store_row(float* row, int lr, const float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c)
      *reinterpret_cast<float4*>(row + (c * GL + lr) * 4) =
          make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) row[lr * E + r] = v[r];
  }
}
template <int GL, int E, bool VEC>
__device__ __forceinline__ void lds_load_row(const float* row, int lr, float (&v)[E]) {
  if constexpr (VEC) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      const float4 q = *reinterpret_cast<const float4*>(row + (c * GL + lr) * 4);
      v[4 * c] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) v[r] = row[lr * E + r];
  }
}

// E consecutive floats to / from LDS (16-byte aligned when E >= 4)
template <int E>
__device__ __forceinline__ void lds_store(float* p, const float (&v)[E]) {
  if constexpr (E % 4 == 0) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c)
      *reinterpret_cast<float4*>(p + 4 * c) = make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) p[r] = v[r];
  }
}
template <int E>
__device__ __forceinline__ void lds_load(const float* p, float (&v)[E]) {
  if constexpr (E % 4 == 0) {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      const float4 q = *reinterpret_cast<const float4*>(p + 4 * c);
      v[4 * c] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < E; ++r) v[r] = p[r];
  }
}

}  // namespace topk
