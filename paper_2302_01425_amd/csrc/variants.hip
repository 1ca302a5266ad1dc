// The two operators built on the relaxed top-k mask of |x|: element-wise passes around the mask
// kernels.
//
//   signed mask (phi(x) = |x|, Sec. 4 on the OWL norm; reduction of Prop. 6): on the non-negative
//   cone phi is the identity, so v* is the mask's isotonic solution on s = sort(|x|) truncated at
//   zero, and y = sign(x) o grad r*(s - max(v, 0)).  With m the mask of |x| this is, per element,
//       y = sign(x) min(m, cap),  cap = grad r*(|x|) = (|x| / lambda)^(q-1),
//   the truncation being active exactly where m > cap (v < 0); there y = grad r*(x) and
//   dy = hess r*(|x|) t, elsewhere dy = sign(x) (J_m (sign(x) o t)).
//
//   masked value (Sec. 7, "Advantage of the non-linearity"): y = x o m, dy = t o m + x o J_m (sign(x) o t).
#include <initializer_list>

#include "common.hpp"
#include "launch.hpp"

namespace topk {
namespace {

constexpr int kVT = 256;
constexpr int kVItems = 4;     // float4 per thread and step

__device__ __forceinline__ float sign_of(float v) { return float((v > 0.0f) - (v < 0.0f)); }

// ax = |x|, st = sign(x) t (t, st may be null)
__global__ __launch_bounds__(kVT) void abs_prepare_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ t,
                                                          float* __restrict__ ax,
                                                          float* __restrict__ st, int64_t count,
                                                          bool vec) {
  const int64_t stride = int64_t(gridDim.x) * kVT * kVItems;
  for (int64_t e0 = (int64_t(blockIdx.x) * kVT + threadIdx.x) * kVItems; e0 < count; e0 += stride) {
    if (vec && e0 + kVItems <= count) {
      const float4 v = *reinterpret_cast<const float4*>(x + e0);
      *reinterpret_cast<float4*>(ax + e0) = make_float4(fabsf(v.x), fabsf(v.y), fabsf(v.z), fabsf(v.w));
      if (t != nullptr) {
        const float4 tv = *reinterpret_cast<const float4*>(t + e0);
        *reinterpret_cast<float4*>(st + e0) = make_float4(sign_of(v.x) * tv.x, sign_of(v.y) * tv.y,
                                                          sign_of(v.z) * tv.z, sign_of(v.w) * tv.w);
      }
    } else {
      for (int64_t e = e0; e < count && e < e0 + kVItems; ++e) {
        ax[e] = fabsf(x[e]);
        if (t != nullptr) st[e] = sign_of(x[e]) * t[e];
      }
    }
  }
}

// in place: out holds m, jvp holds J_m (sign o t) on entry (jvp, t may be null)
// (float64 for the values: with a small lambda the factors reach the hundreds, and two or three
// float32 roundings would show against a bar of one float32 ulp)
template <bool SIGNED, int PC>
__device__ __forceinline__ void finish_element(float xv, float tv, float& m, float& jm, bool want_jvp,
                                               double inv_lambda) {
  const float sg = sign_of(xv);
  if (SIGNED) {
    const double u = double(fabsf(xv)) * inv_lambda;
    const float cap = float(PC == kP43 ? u * u * u : u);
    const bool clipped = m > cap;
    if (want_jvp) {
      const double hess = PC == kP43 ? 3.0 * u * u * inv_lambda : inv_lambda;
      jm = clipped ? float(hess * double(tv)) : sg * jm;
      jm = (jm == 0.0f) ? 0.0f : jm;
    }
    const float y = sg * (clipped ? cap : m);
    m = (y == 0.0f) ? 0.0f : y;
  } else {
    if (want_jvp) jm = float(double(tv) * double(m) + double(xv) * double(jm));
    m = xv * m;
  }
}

template <bool SIGNED, int PC>
__global__ __launch_bounds__(kVT) void abs_finish_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ t, float* out,
                                                         float* jvp, int64_t count,
                                                         double inv_lambda, bool vec) {
  const bool want_jvp = jvp != nullptr;
  const int64_t stride = int64_t(gridDim.x) * kVT * kVItems;
  for (int64_t e0 = (int64_t(blockIdx.x) * kVT + threadIdx.x) * kVItems; e0 < count; e0 += stride) {
    if (vec && e0 + kVItems <= count) {
      const float4 xv = *reinterpret_cast<const float4*>(x + e0);
      float4 m = *reinterpret_cast<const float4*>(out + e0);
      float4 tv = make_float4(0.f, 0.f, 0.f, 0.f), jm = tv;
      if (want_jvp) {
        tv = *reinterpret_cast<const float4*>(t + e0);
        jm = *reinterpret_cast<const float4*>(jvp + e0);
      }
      finish_element<SIGNED, PC>(xv.x, tv.x, m.x, jm.x, want_jvp, inv_lambda);
      finish_element<SIGNED, PC>(xv.y, tv.y, m.y, jm.y, want_jvp, inv_lambda);
      finish_element<SIGNED, PC>(xv.z, tv.z, m.z, jm.z, want_jvp, inv_lambda);
      finish_element<SIGNED, PC>(xv.w, tv.w, m.w, jm.w, want_jvp, inv_lambda);
      *reinterpret_cast<float4*>(out + e0) = m;
      if (want_jvp) *reinterpret_cast<float4*>(jvp + e0) = jm;
    } else {
      for (int64_t e = e0; e < count && e < e0 + kVItems; ++e) {
        float m = out[e], jm = want_jvp ? jvp[e] : 0.0f;
        finish_element<SIGNED, PC>(x[e], want_jvp ? t[e] : 0.0f, m, jm, want_jvp, inv_lambda);
        out[e] = m;
        if (want_jvp) jvp[e] = jm;
      }
    }
  }
}

unsigned grid_for(int64_t count) {
  const int64_t per_block = int64_t(kVT) * kVItems;
  int64_t blocks = (count + per_block - 1) / per_block;
  if (blocks > 8192) blocks = 8192;          // grid-stride beyond that
  return unsigned(blocks < 1 ? 1 : blocks);
}

// float4 accesses need 16-byte aligned arrays (null pointers count as aligned)
bool aligned16(std::initializer_list<const void*> ps) {
  for (const void* p : ps)
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return false;
  return true;
}

}  // namespace

int launch_abs_prepare(const float* x, const float* t, float* ax, float* st, int64_t count,
                       hipStream_t stream) {
  if (count <= 0) return 0;
  hipLaunchKernelGGL(abs_prepare_kernel, dim3(grid_for(count)), dim3(kVT), 0, stream, x, t, ax,
                     t != nullptr ? st : nullptr, count, aligned16({x, t, ax, st}));
  return 0;
}

int launch_abs_finish(bool signed_mask, int pc, const float* x, const float* t, float* out,
                      float* jvp, int64_t count, const Reg& R, hipStream_t stream) {
  if (count <= 0) return 0;
  const dim3 grid(grid_for(count)), block(kVT);
  const double il = R.inv_lambda;
  if (jvp == nullptr) t = nullptr;
  const bool vec = aligned16({x, t, out, jvp});
#define TOPK_VARIANT_CALL(S, P) \
  hipLaunchKernelGGL((abs_finish_kernel<S, P>), grid, block, 0, stream, x, t, out, jvp, count, il, vec)
  if (signed_mask && pc == kP2) TOPK_VARIANT_CALL(true, kP2);
  else if (signed_mask && pc == kP43) TOPK_VARIANT_CALL(true, kP43);
  else if (pc == kP2) TOPK_VARIANT_CALL(false, kP2);
  else if (pc == kP43) TOPK_VARIANT_CALL(false, kP43);
  else return -1;
#undef TOPK_VARIANT_CALL
  return 0;
}

}  // namespace topk
