// Launchers of the values-only short-row kernel (short_rows_value.hpp) for rows of 129 .. 2048
// elements: 32 or 64 lanes per row with 8, 16 or 32 elements per lane; one row (two for 256
// elements) per wavefront.  With k <= lanes per row only the values above the threshold T are
// ordered; otherwise the whole row goes through the float network in registers.
#include "short_rows_value.hpp"

namespace topk {
namespace {

template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE>
int launch_wide_mode(const float* x, const float* t, float* out, float* jvp, int64_t rows, int n, int k,
                     const Reg& R, hipStream_t st) {
  using C = SelCfg<GL, E>;
  constexpr int WPB = (C::NP >= 2048) ? 2 : 4;           // LDS: 8 KB per row of 2048
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + WPB - 1) / WPB;
  if (blocks > 0x7fffffffLL) return -1;
  const float il = float(R.inv_lambda), i1 = float(R.inv_1pl);
  if (k >= 1 && k <= GL && k < n)
    hipLaunchKernelGGL((short_rows_value_kernel<GL, E, MAG, PC, VEC, FULL, MODE, true, WPB>),
                       dim3((unsigned)blocks), dim3(WPB * kWave), 0, st, x, t, out, jvp, rows, n, k, R,
                       il, i1, nullptr, 0.0);
  else
    hipLaunchKernelGGL((short_rows_value_kernel<GL, E, MAG, PC, VEC, FULL, MODE, false, WPB>),
                       dim3((unsigned)blocks), dim3(WPB * kWave), 0, st, x, t, out, jvp, rows, n, k, R,
                       il, i1, nullptr, 0.0);
  return 0;
}

// mask: p = 2 and p = 4/3; magnitude: p = 2
template <int GL, int E, bool VEC, bool FULL>
int launch_wide_shape2(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                       int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  const int mode = (jvp == nullptr) ? 0 : (out == nullptr ? 1 : 2);
#define TOPK_MODE_CALL(MAGV, PCV, M) \
  return launch_wide_mode<GL, E, MAGV, PCV, VEC, FULL, M>(x, t, out, jvp, rows, n, k, R, st)
  if (!mag && pc == kP2) {
    if (mode == 0) TOPK_MODE_CALL(false, kP2, 0);
    if (mode == 1) TOPK_MODE_CALL(false, kP2, 1);
    TOPK_MODE_CALL(false, kP2, 2);
  }
  if (!mag && pc == kP43) {
    if (mode == 0) TOPK_MODE_CALL(false, kP43, 0);
    if (mode == 1) TOPK_MODE_CALL(false, kP43, 1);
    TOPK_MODE_CALL(false, kP43, 2);
  }
  if (mag && pc == kP2) {
    if (mode == 0) TOPK_MODE_CALL(true, kP2, 0);
    if (mode == 1) TOPK_MODE_CALL(true, kP2, 1);
    TOPK_MODE_CALL(true, kP2, 2);
  }
#undef TOPK_MODE_CALL
  return -2;
}

template <int GL, int E>
int launch_wide_shape(bool vec, bool mag, int pc, const float* x, const float* t, float* out,
                      float* jvp, int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  if (vec && n == GL * E)
    return launch_wide_shape2<GL, E, true, true>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
  if (vec) return launch_wide_shape2<GL, E, true, false>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
  return launch_wide_shape2<GL, E, false, false>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
}

}  // namespace

// np: the row length padded to a power of two, 256 .. 2048.  Returns -2 for other lengths and for
// the magnitude operator with p = 4/3 (the caller then uses the kernels that build the
// permutation).
int launch_short_rows_value_wide(int np, bool vec, bool mag, int pc, const float* x,
                                 const float* tangent, float* out, float* jvp, int64_t rows, int n,
                                 int k, const Reg& R, hipStream_t st) {
  switch (np) {
    case 256: return launch_wide_shape<32, 8>(vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    case 512: return launch_wide_shape<64, 8>(vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    case 1024: return launch_wide_shape<64, 16>(vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    case 2048: return launch_wide_shape<64, 32>(vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    default: return -2;
  }
}

}  // namespace topk
