// Smooth top-k loss (paper Sec. 6, "Smooth top-k loss"): the Fenchel-Young loss
//   l(x, t) = f_{phi,R}(x, 1_k) - <x, t>,   phi = identity,
// and its gradient in x, y - t, from the relaxed top-k mask y of x.  By Prop. 2 (first line, the
// maximisation form) f_{phi,R}(x, 1_k) = <y, x> - R(y) at the maximiser y, which is the mask, so
// after the forward pass the loss is one reduction per row.  The float32 mask is not exactly the
// maximiser; the sum is therefore taken of the Lagrangian
//   l = sum_i ( y_i x_i - (lambda / p) y_i^p - x_i t_i )  -  gamma ( sum_i y_i - k ),
// which has the same value at the maximiser and is flat there (on the block
// x_i - lambda y_i^(p-1) = gamma, elsewhere y_i is a literal 0 or 1), so that the rounding of the
// y_i does not enter in first order.  gamma is taken from the block's elements themselves: the
// mean of x_i - lambda y_i^(p-1) over 0 < y_i < 1.
// `grad` holds y on entry and y - t on exit.
#include "common.hpp"
#include "launch.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;

struct Acc4 {
  double f, ysum, gsum, cnt;
};

template <int PC>
__device__ __forceinline__ void add_term(Acc4& a, float x, float t, float y, double lam_over_p,
                                         double lambda) {
  const double yd = double(y);
  double yp, ypm1;                       // y^p, y^(p-1)
  if (PC == kP2) {
    yp = yd * yd;
    ypm1 = yd;
  } else {
    const double c = cbrt(yd);            // y in [0, 1]
    yp = c * c * c * c;
    ypm1 = c;
  }
  a.f += yd * double(x) - lam_over_p * yp - double(x) * double(t);
  a.ysum += yd;
  if (y > 0.0f && y < 1.0f) {
    a.gsum += double(x) - lambda * ypm1;
    a.cnt += 1.0;
  }
}

__device__ __forceinline__ float finish_loss(const Acc4& a, double k) {
  const double gamma = a.cnt > 0.0 ? a.gsum / a.cnt : 0.0;
  return float(a.f - gamma * (a.ysum - k));
}

// GROUP lanes per row (a power of two <= 64), or the whole workgroup per row (GROUP == 0).
template <int PC, int GROUP>
__global__ __launch_bounds__(kThreads) void loss_kernel(const float* __restrict__ x,
                                                        const float* __restrict__ target,
                                                        float* __restrict__ grad,
                                                        float* __restrict__ loss, int64_t rows,
                                                        int64_t n, double k, double lam_over_p,
                                                        double lambda) {
  __shared__ Acc4 wave_sum[kThreads / kWave];
  constexpr int kLanes = GROUP == 0 ? kThreads : GROUP;
  constexpr int kRowsPerBlock = GROUP == 0 ? 1 : kThreads / GROUP;
  const int64_t row = int64_t(blockIdx.x) * kRowsPerBlock + (GROUP == 0 ? 0 : threadIdx.x / GROUP);
  const int l = GROUP == 0 ? threadIdx.x : threadIdx.x % GROUP;
  Acc4 acc{0.0, 0.0, 0.0, 0.0};
  if (row < rows) {
    const int64_t base = row * n;
    for (int64_t e = l; e < n; e += kLanes) {
      const float xv = x[base + e], tv = target[base + e], yv = grad[base + e];
      add_term<PC>(acc, xv, tv, yv, lam_over_p, lambda);
      grad[base + e] = yv - tv;
    }
  }
  constexpr int kWidth = GROUP != 0 ? GROUP : kWave;
#pragma unroll
  for (int off = kWidth >> 1; off >= 1; off >>= 1) {
    acc.f += __shfl_xor(acc.f, off, kWidth);
    acc.ysum += __shfl_xor(acc.ysum, off, kWidth);
    acc.gsum += __shfl_xor(acc.gsum, off, kWidth);
    acc.cnt += __shfl_xor(acc.cnt, off, kWidth);
  }
  if constexpr (GROUP != 0) {
    if (l == 0 && row < rows) loss[row] = finish_loss(acc, k);
  } else {
    if ((threadIdx.x & (kWave - 1)) == 0) wave_sum[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      Acc4 s{0.0, 0.0, 0.0, 0.0};
      for (int q = 0; q < kThreads / kWave; ++q) {
        s.f += wave_sum[q].f;
        s.ysum += wave_sum[q].ysum;
        s.gsum += wave_sum[q].gsum;
        s.cnt += wave_sum[q].cnt;
      }
      loss[row] = finish_loss(s, k);
    }
  }
}

template <int PC>
int launch(const float* x, const float* target, float* grad, float* loss, int64_t rows, int64_t n,
           int64_t k, double lam_over_p, double lambda, hipStream_t st) {
#define TOPK_LOSS(G)                                                                        \
  {                                                                                         \
    constexpr int rpb = (G) == 0 ? 1 : kThreads / ((G) == 0 ? 1 : (G));                     \
    const int64_t blocks = (rows + rpb - 1) / rpb;                                          \
    if (blocks > 0x7fffffffLL) return -1;                                                   \
    hipLaunchKernelGGL((loss_kernel<PC, (G)>), dim3(unsigned(blocks)), dim3(kThreads), 0, st, x, \
                       target, grad, loss, rows, n, double(k), lam_over_p, lambda);         \
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
                     int64_t rows, int64_t n, int64_t k, double lambda, double p, hipStream_t st) {
  if (pc == kP2) return launch<kP2>(x, target, grad, loss, rows, n, k, lambda / p, lambda, st);
  if (pc == kP43) return launch<kP43>(x, target, grad, loss, rows, n, k, lambda / p, lambda, st);
  return -1;
}

}  // namespace topk
