// Launchers of the values-only short-row kernel (short_rows_value.hpp) for rows of up to 128
// elements: 1 .. 16 lanes per row, 4 or 8 elements per lane; also the operators built on the mask.
#include "short_rows_value.hpp"

namespace topk {
namespace {

template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE, bool SELECT, int WPB,
          int VAR = kVarPlain>
int launch_value_wpb(const float* x, const float* t, float* out, float* jvp, int64_t rows, int n,
                     int k, const Reg& R, hipStream_t st, float* loss = nullptr,
                     double lam_over_p = 0.0) {
  using C = SelCfg<GL, E>;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + WPB - 1) / WPB;
  if (blocks > 0x7fffffffLL) return -1;
  const float il = float(R.inv_lambda), i1 = float(R.inv_1pl);
  hipLaunchKernelGGL((short_rows_value_kernel<GL, E, MAG, PC, VEC, FULL, MODE, SELECT, WPB, VAR>),
                     dim3((unsigned)blocks), dim3(WPB * kWave), 0, st, x, t, out, jvp, rows, n, k, R,
                     il, i1, loss, lam_over_p);
  return 0;
}

template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE, int VAR = kVarPlain>
int launch_value_mode(const float* x, const float* t, float* out, float* jvp, int64_t rows, int n,
                      int k, const Reg& R, hipStream_t st, float* loss = nullptr,
                      double lam_over_p = 0.0) {
  constexpr int WPB = TOPK_VALUE_WPB;
  if (k >= 1 && k <= GL && k < n)
    return launch_value_wpb<GL, E, MAG, PC, VEC, FULL, MODE, true, WPB, VAR>(x, t, out, jvp, rows, n,
                                                                            k, R, st, loss, lam_over_p);
  return launch_value_wpb<GL, E, MAG, PC, VEC, FULL, MODE, false, WPB, VAR>(x, t, out, jvp, rows, n,
                                                                           k, R, st, loss, lam_over_p);
}

// the operators built on the mask (see VAR): forward, or forward + JVP (out is always written)
template <int GL, int E, bool VEC, bool FULL>
int launch_variant_shape2(int var, int pc, const float* x, const float* t, float* out, float* jvp,
                          float* loss, double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                          hipStream_t st) {
#define TOPK_VAR_CALL(PCV, M, V) \
  return launch_value_mode<GL, E, false, PCV, VEC, FULL, M, V>(x, t, out, jvp, rows, n, k, R, st, loss, lam_over_p)
  if (var == kVarLoss) {
    if (pc == kP2) TOPK_VAR_CALL(kP2, 0, kVarLoss);
    if (pc == kP43) TOPK_VAR_CALL(kP43, 0, kVarLoss);
    return -2;
  }
  const bool with_jvp = jvp != nullptr;
  if (var == kVarSigned) {
    if (pc == kP2 && !with_jvp) TOPK_VAR_CALL(kP2, 0, kVarSigned);
    if (pc == kP2) TOPK_VAR_CALL(kP2, 2, kVarSigned);
    if (pc == kP43 && !with_jvp) TOPK_VAR_CALL(kP43, 0, kVarSigned);
    if (pc == kP43) TOPK_VAR_CALL(kP43, 2, kVarSigned);
  }
  if (var == kVarMasked) {
    if (pc == kP2 && !with_jvp) TOPK_VAR_CALL(kP2, 0, kVarMasked);
    if (pc == kP2) TOPK_VAR_CALL(kP2, 2, kVarMasked);
    if (pc == kP43 && !with_jvp) TOPK_VAR_CALL(kP43, 0, kVarMasked);
    if (pc == kP43) TOPK_VAR_CALL(kP43, 2, kVarMasked);
  }
#undef TOPK_VAR_CALL
  return -2;
}

template <int GL, int E, bool VEC>
int launch_variant_shape(int var, int pc, const float* x, const float* t, float* out, float* jvp,
                         float* loss, double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                         hipStream_t st) {
  if (VEC && n == GL * E)
    return launch_variant_shape2<GL, E, true, true>(var, pc, x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st);
  return launch_variant_shape2<GL, E, VEC, false>(var, pc, x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st);
}

// mask: p = 2 and p = 4/3; magnitude: p = 2
template <int GL, int E, bool VEC, bool FULL>
int launch_value_shape2(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                        int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  const int mode = (jvp == nullptr) ? 0 : (out == nullptr ? 1 : 2);
#define TOPK_MODE_CALL(MAGV, PCV, M) \
  return launch_value_mode<GL, E, MAGV, PCV, VEC, FULL, M>(x, t, out, jvp, rows, n, k, R, st)
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

template <int GL, int E, bool VEC>
int launch_value_shape(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                       int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  if (VEC && n == GL * E)
    return launch_value_shape2<GL, E, true, true>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
  return launch_value_shape2<GL, E, VEC, false>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
}

}  // namespace

// Shapes: rows of 4..128 padded elements, at most 16 lanes per row (one DPP row), 4 or 8 elements
// per lane.  Returns -2 when (np, lg) is not one of them, or for the magnitude operator with
// p = 4/3 (the caller then uses the general kernels).
int launch_short_rows_value(int np, int lg, bool vec, bool mag, int pc, const float* x,
                            const float* tangent, float* out, float* jvp, int64_t rows, int n,
                            int k, const Reg& R, hipStream_t st) {
#define TOPK_VALUE_SHAPE(GL, E)                                                                  \
  if (np == (GL) * (E) && lg == ilog2(GL))                                                       \
    return vec ? launch_value_shape<GL, E, true>(mag, pc, x, tangent, out, jvp, rows, n, k, R, st) \
               : launch_value_shape<GL, E, false>(mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
  TOPK_VALUE_SHAPE(1, 4) TOPK_VALUE_SHAPE(1, 8) TOPK_VALUE_SHAPE(2, 4) TOPK_VALUE_SHAPE(2, 8)
  TOPK_VALUE_SHAPE(4, 4) TOPK_VALUE_SHAPE(4, 8) TOPK_VALUE_SHAPE(8, 4) TOPK_VALUE_SHAPE(8, 8)
  TOPK_VALUE_SHAPE(16, 4) TOPK_VALUE_SHAPE(16, 8)
#undef TOPK_VALUE_SHAPE
  return -2;
}

// The operators built on the mask, fused into the same kernel: var = 1 signed mask, 2 x o mask(|x|)
// (tangent / jvp may be null: forward only), 3 Fenchel-Young loss (tangent = target, out = the
// gradient y - target, loss[rows]).  Returns -2 when the shape is not one of the kernel's.
int launch_short_rows_variant(int np, int lg, bool vec, int var, int pc, const float* x,
                              const float* tangent, float* out, float* jvp, float* loss,
                              double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                              hipStream_t st) {
#define TOPK_VARIANT_SHAPE(GL, E)                                                               \
  if (np == (GL) * (E) && lg == ilog2(GL))                                                      \
    return vec ? launch_variant_shape<GL, E, true>(var, pc, x, tangent, out, jvp, loss,         \
                                                   lam_over_p, rows, n, k, R, st)               \
               : launch_variant_shape<GL, E, false>(var, pc, x, tangent, out, jvp, loss,        \
                                                    lam_over_p, rows, n, k, R, st);
  TOPK_VARIANT_SHAPE(1, 4) TOPK_VARIANT_SHAPE(1, 8) TOPK_VARIANT_SHAPE(2, 4) TOPK_VARIANT_SHAPE(2, 8)
  TOPK_VARIANT_SHAPE(4, 4) TOPK_VARIANT_SHAPE(4, 8) TOPK_VARIANT_SHAPE(8, 4) TOPK_VARIANT_SHAPE(8, 8)
  TOPK_VARIANT_SHAPE(16, 4) TOPK_VARIANT_SHAPE(16, 8)
#undef TOPK_VARIANT_SHAPE
  return -2;
}

}  // namespace topk
