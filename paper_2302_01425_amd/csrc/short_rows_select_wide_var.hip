// The operators built on the mask (signed mask, x o mask(|x|), Fenchel-Young loss; VAR of
// short_rows_value.hpp) for rows of 129 .. 2048 elements: the shapes of short_rows_select_wide.hip.
#include "short_rows_value.hpp"

namespace topk {
namespace {

template <int GL, int E, int PC, bool VEC, bool FULL, int MODE, int VAR>
int launch_var_mode(const float* x, const float* t, float* out, float* jvp, float* loss,
                    double lam_over_p, int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  using C = SelCfg<GL, E>;
  constexpr int WPB = (C::NP >= 2048) ? 2 : 4;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + WPB - 1) / WPB;
  if (blocks > 0x7fffffffLL) return -1;
  const float il = float(R.inv_lambda), i1 = float(R.inv_1pl);
  if (k >= 1 && k <= GL && k < n)
    hipLaunchKernelGGL((short_rows_value_kernel<GL, E, false, PC, VEC, FULL, MODE, true, WPB, VAR>),
                       dim3((unsigned)blocks), dim3(WPB * kWave), 0, st, x, t, out, jvp, rows, n, k, R,
                       il, i1, loss, lam_over_p);
  else
    hipLaunchKernelGGL((short_rows_value_kernel<GL, E, false, PC, VEC, FULL, MODE, false, WPB, VAR>),
                       dim3((unsigned)blocks), dim3(WPB * kWave), 0, st, x, t, out, jvp, rows, n, k, R,
                       il, i1, loss, lam_over_p);
  return 0;
}

template <int GL, int E, bool VEC, bool FULL>
int launch_var_shape2(int var, int pc, const float* x, const float* t, float* out, float* jvp,
                      float* loss, double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                      hipStream_t st) {
#define TOPK_VAR_CALL(PCV, M, V) \
  return launch_var_mode<GL, E, PCV, VEC, FULL, M, V>(x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st)
  const bool with_jvp = jvp != nullptr;
  if (var == kVarLoss) {
    if (pc == kP2) TOPK_VAR_CALL(kP2, 0, kVarLoss);
    if (pc == kP43) TOPK_VAR_CALL(kP43, 0, kVarLoss);
  }
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

template <int GL, int E>
int launch_var_shape(bool vec, int var, int pc, const float* x, const float* t, float* out, float* jvp,
                     float* loss, double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                     hipStream_t st) {
  if (vec && n == GL * E)
    return launch_var_shape2<GL, E, true, true>(var, pc, x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st);
  if (vec)
    return launch_var_shape2<GL, E, true, false>(var, pc, x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st);
  return launch_var_shape2<GL, E, false, false>(var, pc, x, t, out, jvp, loss, lam_over_p, rows, n, k, R, st);
}

}  // namespace

// var: 1 signed mask, 2 x o mask(|x|) (tangent / jvp may be null: forward only), 3 Fenchel-Young
// loss (tangent = target, out = the gradient y - target, loss[rows]).  np = 256 .. 2048.
int launch_short_rows_variant_wide(int np, bool vec, int var, int pc, const float* x,
                                   const float* tangent, float* out, float* jvp, float* loss,
                                   double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                                   hipStream_t st) {
  switch (np) {
    case 256: return launch_var_shape<32, 8>(vec, var, pc, x, tangent, out, jvp, loss, lam_over_p, rows, n, k, R, st);
    case 512: return launch_var_shape<64, 8>(vec, var, pc, x, tangent, out, jvp, loss, lam_over_p, rows, n, k, R, st);
    case 1024: return launch_var_shape<64, 16>(vec, var, pc, x, tangent, out, jvp, loss, lam_over_p, rows, n, k, R, st);
    case 2048: return launch_var_shape<64, 32>(vec, var, pc, x, tangent, out, jvp, loss, lam_over_p, rows, n, k, R, st);
    default: return -2;
  }
}

}  // namespace topk
