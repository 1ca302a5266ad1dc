// Smooth top-k loss (paper Sec. 6, "Smooth top-k loss"): the Fenchel-Young loss
//   l(x, t) = f_{phi,R}(x, 1_k) - <x, t>,   phi = identity,
// and its gradient in x, y - t, from the relaxed top-k mask y of x.  By Prop. 2 (first line, the
// maximisation form) f_{phi,R}(x, 1_k) = <y, x> - R(y) at the maximiser y, which is the mask, so
// after the forward pass the loss is one reduction per row:
//   l = sum_i  y_i x_i - (lambda / p) y_i^p - x_i t_i .
// `grad` holds y on entry and y - t on exit.
#include "common.hpp"
#include "launch.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;

template <int PC>
__device__ __forceinline__ double term(float x, float t, float y, double lam_over_p) {
  const double yd = double(y);
  double yp;
  if (PC == kP2) {
    yp = yd * yd;
  } else {
    const double c = cbrt(yd);            // y^(4/3), y in [0, 1]
    yp = c * c * c * c;
  }
  return yd * double(x) - lam_over_p * yp - double(x) * double(t);
}

// GROUP lanes per row (a power of two <= 64), or the whole workgroup per row (GROUP == 0).
template <int PC, int GROUP>
__global__ __launch_bounds__(kThreads) void loss_kernel(const float* __restrict__ x,
                                                        const float* __restrict__ target,
                                                        float* __restrict__ grad,
                                                        float* __restrict__ loss, int64_t rows,
                                                        int64_t n, double lam_over_p) {
  __shared__ double wave_sum[kThreads / kWave];
  constexpr int kLanes = GROUP == 0 ? kThreads : GROUP;
  constexpr int kRowsPerBlock = GROUP == 0 ? 1 : kThreads / GROUP;
  const int64_t row = int64_t(blockIdx.x) * kRowsPerBlock + (GROUP == 0 ? 0 : threadIdx.x / GROUP);
  const int l = GROUP == 0 ? threadIdx.x : threadIdx.x % GROUP;
  double acc = 0.0;
  if (row < rows) {
    const int64_t base = row * n;
    for (int64_t e = l; e < n; e += kLanes) {
      const float xv = x[base + e], tv = target[base + e], yv = grad[base + e];
      acc += term<PC>(xv, tv, yv, lam_over_p);
      grad[base + e] = yv - tv;
    }
  }
  if constexpr (GROUP != 0) {
#pragma unroll
    for (int off = GROUP >> 1; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, GROUP);
    if (l == 0 && row < rows) loss[row] = float(acc);
  } else {
#pragma unroll
    for (int off = kWave >> 1; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wave_sum[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      double s = 0.0;
      for (int q = 0; q < kThreads / kWave; ++q) s += wave_sum[q];
      loss[row] = float(s);
    }
  }
}

template <int PC>
int launch(const float* x, const float* target, float* grad, float* loss, int64_t rows, int64_t n,
           double lam_over_p, hipStream_t st) {
#define TOPK_LOSS(G)                                                                        \
  {                                                                                         \
    constexpr int rpb = (G) == 0 ? 1 : kThreads / ((G) == 0 ? 1 : (G));                     \
    const int64_t blocks = (rows + rpb - 1) / rpb;                                          \
    if (blocks > 0x7fffffffLL) return -1;                                                   \
    hipLaunchKernelGGL((loss_kernel<PC, (G)>), dim3(unsigned(blocks)), dim3(kThreads), 0, st, x, \
                       target, grad, loss, rows, n, lam_over_p);                            \
    return 0;                                                                               \
  }
  if (n <= 16) TOPK_LOSS(8)
  if (n <= 128) TOPK_LOSS(16)
  if (n <= 1024) TOPK_LOSS(64)
  TOPK_LOSS(0)
#undef TOPK_LOSS
}

}  // namespace

int launch_mask_loss(int pc, const float* x, const float* target, float* grad, float* loss,
                     int64_t rows, int64_t n, double lambda, double p, hipStream_t st) {
  if (pc == kP2) return launch<kP2>(x, target, grad, loss, rows, n, lambda / p, st);
  if (pc == kP43) return launch<kP43>(x, target, grad, loss, rows, n, lambda / p, st);
  return -1;
}

}  // namespace topk
