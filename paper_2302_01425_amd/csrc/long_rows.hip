// Long rows, after the sort of the row (or of its candidate list): the launches that use it.
//
//   solve  : one workgroup per row grows the single pooled block [a, b] outwards from (k, k+1)
//            (long_solve.hpp) and writes (a, b, gamma, d gamma, value window) per row; rows whose
//            short candidate list was sorted and solved by one workgroup are skipped.
//   dense  : one coalesced pass in original order for everything outside the block's value
//            window: literal 1 (mask) or x/(1+lambda) (magnitude) above it, literal 0 below it.
//   window : the sorted positions inside the window: y (and dy) from (a, b, gamma, d gamma),
//            scattered through sigma.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "long_solve.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kSolveThreads = 1024;
using Solver = RowSolver<kSolveThreads>;

template <bool MAG, int PC>
__global__ __launch_bounds__(kSolveThreads) void long_solve_kernel(
    const uint32_t* __restrict__ skeys_all, const uint32_t* __restrict__ sidx_all,
    const float* __restrict__ tangent_all, RowInfo* __restrict__ info,
    const RowSel* __restrict__ sel, int64_t row_len, int64_t k_row, Reg R) {
  __shared__ SolveShared<kSolveThreads> sm;
  const int64_t row = blockIdx.x;
  // With a candidate list the sorted arrays hold sorted positions above+1 .. above+cn of the
  // row; all positions below are relative to that list (it contains positions k and k+1 and
  // every position that can pool, so the block never stops growing because the list ends).
  int64_t n = row_len, k = k_row;
  if (sel != nullptr) {
    n = int64_t(sel[row].cn);
    k = k_row - sel[row].above;
    if (n <= kFinishMax) return;          // solved together with the sort of its short list
  }
  const RowInfo ri = Solver::solve<MAG, PC>(
      skeys_all + row * row_len, sidx_all + row * row_len,
      tangent_all != nullptr ? tangent_all + row * row_len : nullptr, n, k, R, sm);
  if (threadIdx.x == 0) info[row] = ri;
}

// Dense pass in original order: everything whose value lies outside the block's value window.
// Elements inside the window are left to long_window_kernel.
template <bool MAG, int PC>
__global__ __launch_bounds__(kThreads) void long_dense_kernel(
    const float* __restrict__ x_all, const float* __restrict__ tangent_all,
    const RowInfo* __restrict__ info, float* __restrict__ out_all, float* __restrict__ jvp_all,
    int64_t n, int chunks, Reg R) {
  const int64_t row = blockIdx.x / chunks;
  const int64_t chunk = blockIdx.x % chunks;
  const RowInfo ri = info[row];
  const int64_t base = row * n;
  const int64_t first = chunk * int64_t(kThreads * 8);
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t e = first + int64_t(i) * kThreads + threadIdx.x;
    if (e >= n) continue;
    emit_dense_element<MAG, PC>(ri, load_stream(x_all + base + e), e, tangent, out, jvp, R);
  }
}

// Sorted positions wa..wb of every row: y and dy from (a, b, gamma), scattered through sigma.
template <bool MAG, int PC>
__global__ __launch_bounds__(kThreads) void long_window_kernel(
    const uint32_t* __restrict__ keys_a, const uint32_t* __restrict__ idx_a,
    const uint32_t* __restrict__ keys_b, const uint32_t* __restrict__ idx_b,
    const float* __restrict__ tangent_all, const RowInfo* __restrict__ info,
    float* __restrict__ out_all, float* __restrict__ jvp_all, int64_t n, int blocks_per_row,
    Reg R) {
  const int64_t row = blockIdx.x / blocks_per_row;
  const int64_t part = blockIdx.x % blocks_per_row;
  const RowInfo ri = info[row];
  const int64_t base = row * n;
  const uint32_t* skeys_all = ri.src == 0 ? keys_a : keys_b;
  const uint32_t* sidx_all = ri.src == 0 ? idx_a : idx_b;
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
  for (int64_t pos1 = ri.wa + part * kThreads + threadIdx.x; pos1 <= ri.wb;
       pos1 += int64_t(blocks_per_row) * kThreads) {
    emit_window_position<MAG, PC>(ri, pos1, key_to_float(skeys_all[base + pos1 - 1]),
                                  sidx_all[base + pos1 - 1], tangent, out, jvp, R);
  }
}


// Wide route: the whole output of a row in one pass in original order, every element from its own
// value: above the block's value window the literal 1 (mask) or its own singleton solution
// (magnitude), below it 0, inside it (lo_incl <= value <= hi_incl: exactly the block, elements of
// equal value pool together) the pooled formula with the row's gamma and d gamma.
// VEC (rows that start 16-byte aligned in all four arrays, n a multiple of 4): 16-byte loads and
// stores, element i of a thread is first + ((i / 4) * kThreads + thread) * 4 + i % 4.
template <bool MAG, int PC, bool VEC>
__global__ __launch_bounds__(kThreads) void wide_dense_kernel(
    const float* __restrict__ x_all, const float* __restrict__ tangent_all,
    const RowInfo* __restrict__ info, float* __restrict__ out_all, float* __restrict__ jvp_all,
    int64_t n, int chunks, Reg R) {
  using P = Pool<MAG, PC>;
  const int64_t row = blockIdx.x / chunks;
  const int64_t chunk = blockIdx.x % chunks;
  const RowInfo ri = info[row];
  const int64_t base = row * n;
  const int64_t first = chunk * int64_t(kThreads * 8);
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
  const bool have_block = ri.a <= ri.b;
  auto elem = [&](int i) -> int64_t {
    return VEC ? first + (int64_t(i / 4) * kThreads + threadIdx.x) * 4 + (i % 4)
               : first + int64_t(i) * kThreads + threadIdx.x;
  };
  float xv[8], tv[8];
  // (the mask's JVP is zero outside the block: only the magnitude operator streams the tangent)
  const bool stream_t = MAG && jvp != nullptr;
  if (VEC) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int64_t e = elem(4 * q);
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
      if (e < n) {
        a = load4_stream(x_all + base + e);
        if (stream_t) b = load4_stream(tangent + e);
      }
      xv[4 * q] = a.x; xv[4 * q + 1] = a.y; xv[4 * q + 2] = a.z; xv[4 * q + 3] = a.w;
      tv[4 * q] = b.x; tv[4 * q + 1] = b.y; tv[4 * q + 2] = b.z; tv[4 * q + 3] = b.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t e = elem(i);
      xv[i] = e < n ? load_stream(x_all + base + e) : 0.0f;
      tv[i] = (stream_t && e < n) ? load_stream(tangent + e) : 0.0f;
    }
  }
  float yo[8], dout[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t e = elem(i);
    yo[i] = dout[i] = 0.0f;
    if (e >= n) continue;
    const float v = MAG ? fabsf(xv[i]) : xv[i];
    const bool above = v > ri.hi_incl;
    const bool inside = have_block && !above && v >= ri.lo_incl;
    const bool neg = MAG && (__float_as_uint(xv[i]) >> 31);
    float y = 0.0f, d = 0.0f;
    if (inside) {
      const double c = double(v) - ri.center;
      y = float(P::y_in_block(c, ri.gamma, R));
      if (MAG) y = (y == 0.0f) ? 0.0f : (neg ? -y : y);
      if (jvp != nullptr) {
        double t = double(MAG ? tv[i] : tangent[e]);
        if (neg) t = -t;
        if (MAG && v == 0.0f) t = 0.0;
        float df = float(P::hess(c, ri.gamma, R) * (t - ri.dgamma));
        if (MAG && v == 0.0f) df = 0.0f;
        d = (df == 0.0f) ? 0.0f : (neg ? -df : df);
      }
    } else if (above) {
      if constexpr (MAG && PC == kP43) {
        if (xv[i] != 0.0f) {
          double g, slope;
          P::above_both(double(v), R, 0.0, &g, &slope);
          y = float(neg ? -g : g);
          if (jvp != nullptr) d = float(slope * double(tv[i]));
        }
      } else if (MAG) {
        const float inv_1pl = float(R.inv_1pl);
        y = xv[i] * inv_1pl;
        if (jvp != nullptr && xv[i] != 0.0f) d = tv[i] * inv_1pl;
      } else {
        y = 1.0f;
      }
    }
    yo[i] = y;
    dout[i] = d;
  }
  if (VEC) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int64_t e = elem(4 * q);
      if (e >= n) continue;
      if (out != nullptr)
        store4_stream(out + e, make_float4(yo[4 * q], yo[4 * q + 1], yo[4 * q + 2], yo[4 * q + 3]));
      if (jvp != nullptr)
        store4_stream(jvp + e, make_float4(dout[4 * q], dout[4 * q + 1], dout[4 * q + 2], dout[4 * q + 3]));
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t e = elem(i);
      if (e >= n) continue;
      if (out != nullptr) store_stream(out + e, yo[i]);
      if (jvp != nullptr) store_stream(jvp + e, dout[i]);
    }
  }
}

template <bool MAG, int PC>
void launch_wide_dense_t(const SortBuffers& B, const float* x, const float* tangent, float* out,
                         float* jvp, int64_t rows, int64_t n, const Reg& R, hipStream_t st) {
  const int chunks = int((n + kThreads * 8 - 1) / (kThreads * 8));
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(out) |
                         reinterpret_cast<uintptr_t>(jvp) |
                         reinterpret_cast<uintptr_t>(jvp ? tangent : nullptr);
  // (measured: the mask, which does not stream the tangent, is faster with 4-byte accesses:
  // 34.7 against 41.0 us on 2^24 elements; the magnitude operator with 16-byte ones: 42.4 against 44.1)
  if (MAG && (bits & 15u) == 0 && n % 4 == 0)
    hipLaunchKernelGGL((wide_dense_kernel<MAG, PC, true>), dim3(unsigned(rows * chunks)),
                       dim3(kThreads), 0, st, x, jvp ? tangent : nullptr, B.info, out, jvp, n, chunks, R);
  else
    hipLaunchKernelGGL((wide_dense_kernel<MAG, PC, false>), dim3(unsigned(rows * chunks)),
                       dim3(kThreads), 0, st, x, jvp ? tangent : nullptr, B.info, out, jvp, n, chunks, R);
}

template <bool MAG, int PC>
void launch_tail(bool selected, const SortBuffers& B, const float* x, const float* tangent,
                 float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                 hipStream_t st) {
  hipLaunchKernelGGL((long_solve_kernel<MAG, PC>), dim3(unsigned(rows)), dim3(kSolveThreads), 0, st,
                     B.keys_a, B.idx_a, jvp ? tangent : nullptr, B.info,
                     selected ? B.sel : nullptr, n, k, R);
  const int chunks = int((n + kThreads * 8 - 1) / (kThreads * 8));
  hipLaunchKernelGGL((long_dense_kernel<MAG, PC>), dim3(unsigned(rows * chunks)), dim3(kThreads), 0,
                     st, x, tangent, B.info, out, jvp, n, chunks, R);
  const int64_t tiles = (n + 1023) / 1024;
  const int bpr = int(tiles < 64 ? tiles : 64);
  hipLaunchKernelGGL((long_window_kernel<MAG, PC>), dim3(unsigned(rows * bpr)), dim3(kThreads), 0,
                     st, B.keys_a, B.idx_a, B.keys_b, B.idx_b, tangent, B.info, out, jvp, n, bpr, R);
}

}  // namespace

int launch_wide_dense(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                      float* out, float* jvp, int64_t rows, int64_t n, const Reg& R,
                      hipStream_t st) {
  const int64_t chunks = (n + kThreads * 8 - 1) / (kThreads * 8);
  if (rows * chunks > 0x7fffffffLL) return -1;
  if (!mag && pc == kP2) launch_wide_dense_t<false, kP2>(B, x, tangent, out, jvp, rows, n, R, st);
  else if (!mag && pc == kP43) launch_wide_dense_t<false, kP43>(B, x, tangent, out, jvp, rows, n, R, st);
  else if (mag && pc == kP2) launch_wide_dense_t<true, kP2>(B, x, tangent, out, jvp, rows, n, R, st);
  else if (mag && pc == kP43) launch_wide_dense_t<true, kP43>(B, x, tangent, out, jvp, rows, n, R, st);
  else return -1;
  return 0;
}

int launch_long_solve(bool mag, int pc, bool selected, const SortBuffers& B, const float* tangent,
                      int64_t rows, int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  if (rows > 0x7fffffffLL) return -1;
#define TOPK_LONG_SOLVE(M, P)                                                                      \
  hipLaunchKernelGGL((long_solve_kernel<M, P>), dim3(unsigned(rows)), dim3(kSolveThreads), 0, st,  \
                     B.keys_a, B.idx_a, tangent, B.info, selected ? B.sel : nullptr, n, k, R)
  if (!mag && pc == kP2) TOPK_LONG_SOLVE(false, kP2);
  else if (!mag && pc == kP43) TOPK_LONG_SOLVE(false, kP43);
  else if (mag && pc == kP2) TOPK_LONG_SOLVE(true, kP2);
  else if (mag && pc == kP43) TOPK_LONG_SOLVE(true, kP43);
  else return -1;
#undef TOPK_LONG_SOLVE
  return 0;
}

int launch_long_tail(bool mag, int pc, bool selected, const SortBuffers& B, const float* x,
                     const float* tangent, float* out, float* jvp, int64_t rows, int64_t n,
                     int64_t k, const Reg& R, hipStream_t st) {
  const int64_t chunks = (n + kThreads * 8 - 1) / (kThreads * 8);
  if (rows * chunks > 0x7fffffffLL) return -1;
  if (!mag && pc == kP2)
    launch_tail<false, kP2>(selected, B, x, tangent, out, jvp, rows, n, k, R, st);
  else if (!mag && pc == kP43)
    launch_tail<false, kP43>(selected, B, x, tangent, out, jvp, rows, n, k, R, st);
  else if (mag && pc == kP2)
    launch_tail<true, kP2>(selected, B, x, tangent, out, jvp, rows, n, k, R, st);
  else if (mag && pc == kP43)
    launch_tail<true, kP43>(selected, B, x, tangent, out, jvp, rows, n, k, R, st);
  else return -1;
  return 0;
}

}  // namespace topk
